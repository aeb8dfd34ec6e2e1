// tf_spec_accept: Verify / Correct / bonus token of Algorithm 1 -- the standard lossless
// speculative-sampling rule (Sec. 4.2 "Correctness") -- over the vocabulary.
//
// Latency-bound (about 1 MB of logits per sequence), and the cost is fp64 exponentials:
// probabilities are computed in fp64 on the GPU because the accept decision and the sampled
// token are integers decided by floating point, and fp64 keeps them identical to an fp64
// reference unless a comparison is within ~1e-13 of a tie. To keep the latency down the
// vocabulary of every logits row is cut into segments of 4096 entries, one workgroup each, so
// a sequence's work spreads over many CUs. Three kernels on one stream:
//   rowstats  per (row, segment): maximum (with its first index) and sum of exponentials;
//   mass      per (sequence, segment): combines the segment records into the statistics of all
//             2G-1 rows (32 lanes per row), replays the accept walk (cheap), then computes the
//             per-thread partial sums of the distribution to draw from -- the residual
//             max(p-q,0) of the rejected position, or p of the bonus position -- in index order;
//   decide    per sequence: the same row statistics and accept walk, prefix sums over segment and
//             thread partials, and the owner thread walks its 4 entries for the inverse-CDF draw.
//             A plain whole-row path in the same kernel covers the rare cases (all-zero residual,
//             rounding at a cell edge).
#include "tf_common.hpp"

namespace tf {

constexpr int kAccThreads = 1024;
constexpr int kAccPer = 4;                           // vocabulary entries per thread of a segment
constexpr int kAccSeg = kAccThreads * kAccPer;       // entries per segment
constexpr int kNone = 0x7fffffff;

struct AcceptParams {
    const float *tl, *dl;
    const int32_t *toks;
    const int32_t *n_draft;  // [B] drafted tokens per sequence (<= G-1), or nullptr = G-1 for all
    int32_t B, G, V, S;  // S = segments per row
    double T;
    const float *ua, *us;
    int32_t *n_acc, *out;
    double *seg_stats;  // [B][2G-1][S][4]: {max logit, sum exp((x-max)/T), first arg-max, -}
    double *part;       // [B][S][kAccThreads]: per-thread partial sums of the draw distribution
    double *seg_sum;    // [B][S]
};

// drafted tokens of sequence b (array strides stay G-1 whatever this count is)
__device__ __forceinline__ int drafted(const AcceptParams &p, int b) {
    return p.n_draft ? min(max(p.n_draft[b], 0), p.G - 1) : p.G - 1;
}

__device__ __forceinline__ const float *logits_row(const AcceptParams &p, int b, int rr) {
    return rr < p.G ? p.tl + ((int64_t)b * p.G + rr) * p.V
                    : p.dl + ((int64_t)b * (p.G - 1) + (rr - p.G)) * p.V;
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kAccThreads) void accept_rowstats_kernel(const AcceptParams p) {
    __shared__ double red_d[kAccThreads / 64];
    __shared__ float red_f[kAccThreads / 64];
    __shared__ int red_i[kAccThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rows = 2 * p.G - 1;
    const int seg = blockIdx.x % p.S;
    const int br = blockIdx.x / p.S;
    const int b = br / rows, rr = br - b * rows;
    const float *x = logits_row(p, b, rr);

    // this thread's strided share of the segment, all loads in flight together
    float xs[kAccPer];
#pragma unroll
    for (int j = 0; j < kAccPer; ++j) {
        const int v = seg * kAccSeg + tid + j * kAccThreads;
        xs[j] = v < p.V ? x[v] : -INFINITY;
    }
    float mx = -INFINITY;
    int mi = kNone;
#pragma unroll
    for (int j = 0; j < kAccPer; ++j) {
        const int v = seg * kAccSeg + tid + j * kAccThreads;
        if (v < p.V && (xs[j] > mx || (xs[j] == mx && v < mi))) {
            mx = xs[j];
            mi = v;
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float om = __shfl_xor(mx, off, kWave);
        const int oi = __shfl_xor(mi, off, kWave);
        if (om > mx || (om == mx && oi < mi)) {
            mx = om;
            mi = oi;
        }
    }
    if (lane == 0) {
        red_f[wave] = mx;
        red_i[wave] = mi;
    }
    __syncthreads();
    mx = red_f[0];
    mi = red_i[0];
    for (int w = 1; w < kAccThreads / 64; ++w) {
        const float om = red_f[w];
        const int oi = red_i[w];
        if (om > mx || (om == mx && oi < mi)) {
            mx = om;
            mi = oi;
        }
    }
    double sum = 0.0;
    if (p.T != 0.0 && mx != -INFINITY) {  // a segment of masked (-inf) logits contributes nothing
        const double zmax = (double)mx / p.T;
#pragma unroll
        for (int j = 0; j < kAccPer; ++j)
            if (seg * kAccSeg + tid + j * kAccThreads < p.V) sum += exp((double)xs[j] / p.T - zmax);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, kWave);
        if (lane == 0) red_d[wave] = sum;
        __syncthreads();
        sum = 0.0;
        for (int w = 0; w < kAccThreads / 64; ++w) sum += red_d[w];
    }
    if (tid == 0) {
        double *st = p.seg_stats + (((int64_t)b * rows + rr) * p.S + seg) * 4;
        st[0] = (double)mx;
        st[1] = sum;
        st[2] = (double)(mi == kNone ? 0 : mi);
        st[3] = 0.0;
    }
}

// statistics of a whole row from its segments: zmax = max(x)/T, sum = sum exp(x/T - zmax),
// arg = first arg-max
struct RowStats {
    double zmax, sum;
    int arg;
};
constexpr int kMaxRows = 2 * TF_MAX_SPEC - 1;  // target rows 0..G-1, then draft rows

// All 2G-1 rows of sequence b at once, by the whole workgroup: 32 lanes per row, a lane takes
// every 32nd segment (one fp64 exponential each at V <= 131072) and shuffles finish the row.
// A thread that walked a row's segments alone would spend 2 x S dependent exponentials per row,
// which was most of the latency of the two kernels below. Every workgroup that calls this gets
// bit-identical values (same inputs, same order), so they all take the same decisions.
// Ends with a barrier; rows[] is then valid for every thread.
__device__ __forceinline__ void combine_rows(const AcceptParams &p, int b, RowStats *rows /* LDS [kMaxRows] */) {
    const int n_rows = 2 * p.G - 1;
    const int rr = threadIdx.x >> 5, l = threadIdx.x & 31;  // 1024 threads = 32 rows x 32 lanes
    if (rr < n_rows) {
        const double *st = p.seg_stats + ((int64_t)b * n_rows + rr) * p.S * 4;
        double mx = -INFINITY;
        int arg = kNone;
        for (int s = l; s < p.S; s += 32) {
            const double m = st[s * 4];
            const int a = (int)st[s * 4 + 2];
            if (m > mx || (m == mx && a < arg)) {  // ties: the lower vocabulary index
                mx = m;
                arg = a;
            }
        }
#pragma unroll
        for (int off = 16; off > 0; off >>= 1) {
            const double om = __shfl_xor(mx, off, kWave);
            const int oa = __shfl_xor(arg, off, kWave);
            if (om > mx || (om == mx && oa < arg)) {
                mx = om;
                arg = oa;
            }
        }
        double sum = 0.0, zmax = 0.0;
        if (p.T != 0.0) {
            zmax = mx / p.T;
            for (int s = l; s < p.S; s += 32) {
                const double m = st[s * 4];
                if (m != -INFINITY) sum += st[s * 4 + 1] * exp(m / p.T - zmax);
            }
#pragma unroll
            for (int off = 16; off > 0; off >>= 1) sum += __shfl_xor(sum, off, kWave);
        }
        if (l == 0) {
            rows[rr].zmax = zmax;
            rows[rr].sum = sum;
            rows[rr].arg = arg == kNone ? 0 : arg;
        }
    }
    __syncthreads();
}

// Accept walk of sequence b by the first wave: lane i tests drafted position i, a ballot finds
// the first rejection. Returns n (valid in every lane of the calling wave).
__device__ __forceinline__ int accept_walk(const AcceptParams &p, int b, int lane, const RowStats *rows) {
    const int gamma = p.G - 1, mine = drafted(p, b);
    bool ok = true;
    if (lane < mine) {
        const int tok = p.toks[(int64_t)b * gamma + lane];
        ok = tok >= 0 && tok < p.V;
        if (ok) {
            const RowStats t = rows[lane];
            if (p.T == 0.0) {
                ok = tok == t.arg;
            } else {
                const RowStats d = rows[p.G + lane];
                const double pt = exp((double)logits_row(p, b, lane)[tok] / p.T - t.zmax) / t.sum;
                const double qt = exp((double)logits_row(p, b, p.G + lane)[tok] / p.T - d.zmax) / d.sum;
                ok = (double)p.ua[(int64_t)b * gamma + lane] * qt < pt;
            }
        }
    }
    const unsigned long long rej = __builtin_amdgcn_ballot_w64(!ok);
    return rej ? __builtin_ctzll(rej) : mine;
}

// mass of vocabulary entry with target logit t and draft logit dq in the distribution drawn from
struct DrawDist {
    double T, tz, ts, dz, ds;
    bool use_p;
    __device__ __forceinline__ double mass(float t, float dq) const {
        const double pv = exp((double)t / T - tz) / ts;
        if (use_p) return pv;
        const double qv = exp((double)dq / T - dz) / ds;
        return pv - qv > 0.0 ? pv - qv : 0.0;
    }
};

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kAccThreads) void accept_mass_kernel(const AcceptParams p) {
    __shared__ int s_n;
    __shared__ double wtot[kAccThreads / 64];
    __shared__ RowStats rows[kMaxRows];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int seg = blockIdx.x % p.S, b = blockIdx.x / p.S;
    const int gamma = p.G - 1;
    combine_rows(p, b, rows);
    if (tid < 64) {
        const int n = accept_walk(p, b, lane, rows);
        if (tid == 0) s_n = n;
    }
    __syncthreads();
    const int n = s_n;
    const bool rejected = n < drafted(p, b);
    const RowStats ts = rows[n];
    RowStats ds = ts;
    if (rejected) ds = rows[p.G + n];
    const DrawDist dist{p.T, ts.zmax, ts.sum, ds.zmax, ds.sum, !rejected};
    const float *tl = logits_row(p, b, n);
    const float *dl = rejected ? logits_row(p, b, p.G + n) : tl;

    // thread t owns the contiguous entries [seg*4096 + 4t, +4): partial sums are in index order
    const int v0 = seg * kAccSeg + tid * kAccPer;
    float t4[kAccPer], d4[kAccPer];
#pragma unroll
    for (int j = 0; j < kAccPer; ++j) {
        t4[j] = v0 + j < p.V ? tl[v0 + j] : -INFINITY;
        d4[j] = v0 + j < p.V ? dl[v0 + j] : -INFINITY;
    }
    double local = 0.0;
#pragma unroll
    for (int j = 0; j < kAccPer; ++j)
        if (v0 + j < p.V) local += dist.mass(t4[j], d4[j]);
    p.part[((int64_t)b * p.S + seg) * kAccThreads + tid] = local;
    double tot = local;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) tot += __shfl_xor(tot, off, kWave);
    if (lane == 0) wtot[wave] = tot;
    __syncthreads();
    if (tid == 0) {
        double z = 0.0;
        for (int w = 0; w < kAccThreads / 64; ++w) z += wtot[w];
        p.seg_sum[(int64_t)b * p.S + seg] = z;
    }
}

// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kAccThreads) void accept_decide_kernel(const AcceptParams p) {
    __shared__ int s_n, s_tok, s_last;
    __shared__ double wtot[kAccThreads / 64];
    __shared__ RowStats rows[kMaxRows];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    const int gamma = p.G - 1;
    const int32_t *x = p.toks + (int64_t)b * gamma;
    int32_t *out = p.out + (int64_t)b * p.G;

    combine_rows(p, b, rows);
    if (tid < 64) {
        const int n = accept_walk(p, b, lane, rows);
        if (tid == 0) {
            s_n = n;
            s_tok = kNone;
            s_last = -1;
        }
    }
    __syncthreads();
    const int n = s_n;
    const bool rejected = n < drafted(p, b);
    const RowStats ts = rows[n];

    if (p.T == 0.0) {
        if (tid == 0) {
            for (int i = 0; i < p.G; ++i) out[i] = i < n ? x[i] : -1;
            out[n] = ts.arg;
            p.n_acc[b] = n;
        }
        return;
    }
    RowStats ds = ts;
    if (rejected) ds = rows[p.G + n];
    DrawDist dist{p.T, ts.zmax, ts.sum, ds.zmax, ds.sum, !rejected};
    const float *tl = logits_row(p, b, n);
    const float *dl = rejected ? logits_row(p, b, p.G + n) : tl;

    // fast path: segment sums -> segment holding u*Z -> thread partials of that segment -> owner
    const double *seg_sum = p.seg_sum + (int64_t)b * p.S;
    double Z = 0.0;
    for (int s = 0; s < p.S; ++s) Z += seg_sum[s];
    bool need_slow = !(Z > 0.0);  // an all-zero residual: draw from p itself (whole-row path)
    if (!need_slow) {
        const double target = (double)p.us[b] * Z;
        int seg = -1;
        double cum_seg = 0.0;
        for (int s = 0; s < p.S; ++s) {
            if (cum_seg + seg_sum[s] > target) {
                seg = s;
                break;
            }
            cum_seg += seg_sum[s];
        }
        if (seg >= 0) {  // uniform over the workgroup
            const double local = p.part[((int64_t)b * p.S + seg) * kAccThreads + tid];
            double incl = local;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const double u = __shfl_up(incl, off, kWave);
                if (lane >= off) incl += u;
            }
            if (lane == 63) wtot[wave] = incl;
            __syncthreads();
            double before = cum_seg;
            for (int w = 0; w < wave; ++w) before += wtot[w];
            double cum = before + incl - local;
            if (cum + local > target) {  // the owner, and threads behind it (first positive entry)
                const int v0 = seg * kAccSeg + tid * kAccPer;
                int found = kNone;
#pragma unroll
                for (int j = 0; j < kAccPer; ++j)
                    if (found == kNone && v0 + j < p.V) {
                        const double mv = dist.mass(tl[v0 + j], dl[v0 + j]);
                        cum += mv;
                        if (cum > target && mv > 0.0) found = v0 + j;  // never a zero-mass entry
                    }
                if (found != kNone) atomicMin(&s_tok, found);
            }
            __syncthreads();
            need_slow = s_tok == kNone;  // rounding at a cell edge: settle it on the whole row
        } else {
            need_slow = true;  // u*Z beyond the last cell by rounding
        }
    }

    if (need_slow) {
        // Whole-row path: thread t owns [t*per, (t+1)*per); two passes (sum, then walk).
        const int per = (p.V + kAccThreads - 1) / kAccThreads;
        const int v_lo = min(tid * per, p.V), v_hi = min(p.V, v_lo + per);
        for (int round = 0; round < 2; ++round) {
            double local = 0.0;
            int lastpos = -1;
            for (int v = v_lo; v < v_hi; ++v) {
                const double mv = dist.mass(tl[v], dl[v]);
                local += mv;
                if (mv > 0.0) lastpos = v;
            }
            double incl = local;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const double u = __shfl_up(incl, off, kWave);
                if (lane >= off) incl += u;
            }
            __syncthreads();
            if (lane == 63) wtot[wave] = incl;
            __syncthreads();
            double before = 0.0, Zs = 0.0;
            for (int w = 0; w < kAccThreads / 64; ++w) {
                if (w < wave) before += wtot[w];
                Zs += wtot[w];
            }
            if (!dist.use_p && !(Zs > 0.0)) {  // uniform over the workgroup
                dist.use_p = true;
                continue;
            }
            const double target = (double)p.us[b] * Zs;
            double cum = before + incl - local;
            int found = kNone;
            if (cum + local > target)
                for (int v = v_lo; v < v_hi; ++v) {
                    const double mv = dist.mass(tl[v], dl[v]);
                    cum += mv;
                    if (cum > target && mv > 0.0) {  // never a zero-mass entry
                        found = v;
                        break;
                    }
                }
            if (found != kNone) atomicMin(&s_tok, found);
            if (lastpos >= 0) atomicMax(&s_last, lastpos);  // if no cell lies above the target
            break;
        }
        __syncthreads();
    }
    if (tid == 0) {
        const int tok = s_tok != kNone ? s_tok : max(s_last, 0);
        for (int i = 0; i < p.G; ++i) out[i] = i < n ? x[i] : -1;
        out[n] = tok;
        p.n_acc[b] = n;
    }
}

static int segments_of(int32_t V) { return (V + kAccSeg - 1) / kAccSeg; }

size_t accept_workspace_bytes(int32_t B, int32_t G, int32_t V) {
    if (B <= 0 || G <= 0 || V <= 0) return 0;
    const size_t S = (size_t)segments_of(V);
    return ((size_t)B * (2 * (size_t)G - 1) * S * 4 + (size_t)B * S * kAccThreads + (size_t)B * S) * sizeof(double);
}

int accept_launch(const float *target_logits, const float *draft_logits, const int32_t *draft_tokens, int32_t B,
                  int32_t G, int32_t V, float temperature, const float *u_accept, const float *u_sample,
                  int32_t *n_accepted, int32_t *out_tokens, void *ws, size_t ws_bytes, void *stream,
                  const int32_t *n_draft) {
    if (B < 1 || G < 1 || V < 1) return TF_ERR_INVALID_ARG;
    if (G > TF_MAX_SPEC) return TF_ERR_UNSUPPORTED;
    if (!target_logits || !u_sample || !n_accepted || !out_tokens) return TF_ERR_INVALID_ARG;
    if (G > 1 && (!draft_logits || !draft_tokens || !u_accept)) return TF_ERR_INVALID_ARG;
    if (!(temperature >= 0.f) || temperature - temperature != 0.f) return TF_ERR_INVALID_ARG;
    const int S = segments_of(V);
    if ((int64_t)B * (2 * G - 1) * S >= (int64_t)1 << 31) return TF_ERR_UNSUPPORTED;
    if (!ws || !aligned(ws, 256) || ws_bytes < accept_workspace_bytes(B, G, V)) return TF_ERR_WORKSPACE;
    AcceptParams p;
    p.tl = target_logits;
    p.dl = draft_logits;
    p.toks = draft_tokens;
    p.n_draft = n_draft;
    p.B = B;
    p.G = G;
    p.V = V;
    p.S = S;
    p.T = (double)temperature;
    p.ua = u_accept;
    p.us = u_sample;
    p.n_acc = n_accepted;
    p.out = out_tokens;
    p.seg_stats = static_cast<double *>(ws);
    p.part = p.seg_stats + (size_t)B * (2 * (size_t)G - 1) * S * 4;
    p.seg_sum = p.part + (size_t)B * S * kAccThreads;
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(accept_rowstats_kernel, dim3((unsigned)(B * (2 * G - 1) * S)), dim3(kAccThreads), 0, st, p);
    if (temperature > 0.f)
        hipLaunchKernelGGL(accept_mass_kernel, dim3((unsigned)(B * S)), dim3(kAccThreads), 0, st, p);
    hipLaunchKernelGGL(accept_decide_kernel, dim3((unsigned)B), dim3(kAccThreads), 0, st, p);
    return hip_status(hipGetLastError());
}

}  // namespace tf
