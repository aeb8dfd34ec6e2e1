// tf_spec_accept: Verify / Correct / bonus token of Algorithm 1 -- the standard lossless
// speculative-sampling rule (Sec. 4.2 "Correctness") -- over the vocabulary.
//
// Latency-bound (about 1 MB of logits per sequence). Probabilities are computed in fp64 on the
// GPU: the accept decision and the sampled token are integers decided by floating point, and
// fp64 keeps them identical to an fp64 reference unless a comparison is within ~1e-13 of a tie.
// Two kernels: (1) one workgroup per logits row: maximum and sum of exponentials (or first
// arg-max at temperature 0); (2) one workgroup per sequence: accept walk, then the residual /
// bonus distribution is scanned in index order (block prefix sums) for the inverse-CDF draw.
#include "tf_common.hpp"

namespace tf {

constexpr int kAccThreads = 1024;

struct AcceptParams {
    const float *tl, *dl;
    const int32_t *toks;
    int32_t B, G, V;
    double T;
    const float *ua, *us;
    int32_t *n_acc, *out;
    double *stats;  // [B][2G-1][2]: rows 0..G-1 target, G..2G-2 draft; {max of l/T, sum exp} or {argmax, 0}
};

__device__ __forceinline__ const float *logits_row(const AcceptParams &p, int b, int rr) {
    return rr < p.G ? p.tl + ((int64_t)b * p.G + rr) * p.V
                    : p.dl + ((int64_t)b * (p.G - 1) + (rr - p.G)) * p.V;
}

constexpr int kAccReg = 32;  // logits per thread kept in registers (covers V <= 32768)

__global__ __launch_bounds__(kAccThreads) void accept_rowstats_kernel(const AcceptParams p) {
    __shared__ double red_d[kAccThreads / 64];
    __shared__ float red_f[kAccThreads / 64];
    __shared__ int red_i[kAccThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rows = 2 * p.G - 1;
    const int b = blockIdx.x / rows, rr = blockIdx.x - b * rows;
    const float *x = logits_row(p, b, rr);
    const bool in_regs = p.V <= kAccReg * kAccThreads;  // uniform

    // one round trip to memory: every thread's strided share of the row, all loads in flight
    float xs[kAccReg];
    if (in_regs) {
#pragma unroll
        for (int j = 0; j < kAccReg; ++j) {
            const int v = tid + j * kAccThreads;
            xs[j] = v < p.V ? x[v] : -INFINITY;
        }
    }
    // maximum logit and its first index
    float mx = -INFINITY;
    int mi = 0x7fffffff;
    if (in_regs) {
#pragma unroll
        for (int j = 0; j < kAccReg; ++j) {
            const int v = tid + j * kAccThreads;
            if (v < p.V && (xs[j] > mx || (xs[j] == mx && v < mi))) {
                mx = xs[j];
                mi = v;
            }
        }
    } else {
        for (int v = tid; v < p.V; v += kAccThreads) {
            const float f = x[v];
            if (f > mx || (f == mx && v < mi)) {
                mx = f;
                mi = v;
            }
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
    double *st = p.stats + ((int64_t)b * rows + rr) * 2;
    if (p.T == 0.0) {
        if (tid == 0) {
            st[0] = (double)(mi == 0x7fffffff ? 0 : mi);
            st[1] = 0.0;
        }
        return;
    }
    const double zmax = (double)mx / p.T;
    double sum = 0.0;
    if (in_regs) {
#pragma unroll
        for (int j = 0; j < kAccReg; ++j)
            if (tid + j * kAccThreads < p.V) sum += exp((double)xs[j] / p.T - zmax);
    } else {
        for (int v = tid; v < p.V; v += kAccThreads) sum += exp((double)x[v] / p.T - zmax);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, kWave);
    if (lane == 0) red_d[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        double tot = 0.0;
        for (int w = 0; w < kAccThreads / 64; ++w) tot += red_d[w];
        st[0] = zmax;
        st[1] = tot;
    }
}

__global__ __launch_bounds__(kAccThreads) void accept_decide_kernel(const AcceptParams p) {
    __shared__ int s_n, s_rej, s_tok, s_last;
    __shared__ double wtot[kAccThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    const int gamma = p.G - 1, rows = 2 * p.G - 1;
    const double *st = p.stats + (int64_t)b * rows * 2;
    const int32_t *x = p.toks + (int64_t)b * gamma;
    int32_t *out = p.out + (int64_t)b * p.G;

    // accept walk: lane i of the first wave evaluates drafted position i, a ballot finds the
    // first rejection
    if (tid < 64) {
        bool ok = true;
        if (tid < gamma) {
            const int tok = x[tid];
            ok = tok >= 0 && tok < p.V;
            if (ok) {
                if (p.T == 0.0) {
                    ok = tok == (int)st[tid * 2];
                } else {
                    const double pt = exp((double)logits_row(p, b, tid)[tok] / p.T - st[tid * 2]) / st[tid * 2 + 1];
                    const double qt = exp((double)logits_row(p, b, p.G + tid)[tok] / p.T - st[(p.G + tid) * 2]) /
                                      st[(p.G + tid) * 2 + 1];
                    ok = (double)p.ua[(int64_t)b * gamma + tid] * qt < pt;
                }
            }
        }
        const unsigned long long rej = __builtin_amdgcn_ballot_w64(!ok);
        if (tid == 0) {
            const int n = rej ? __builtin_ctzll(rej) : gamma;
            s_n = n;
            s_rej = n < gamma;
            s_tok = 0x7fffffff;
            s_last = -1;
        }
    }
    __syncthreads();
    const int n = s_n, rejected = s_rej;

    if (p.T == 0.0) {
        if (tid == 0) {
            for (int i = 0; i < p.G; ++i) out[i] = i < n ? x[i] : -1;
            out[n] = (int)st[n * 2];
            p.n_acc[b] = n;
        }
        return;
    }

    // distribution to draw from: residual of row n if rejected, else target row gamma (= n).
    // Thread t owns the contiguous index range [t*per, (t+1)*per) so the scan is in index order.
    const float *tl = logits_row(p, b, n);
    const float *dl = rejected ? logits_row(p, b, p.G + n) : tl;
    const double tz = st[n * 2], ts = st[n * 2 + 1];
    const double dz = rejected ? st[(p.G + n) * 2] : 0.0, ds = rejected ? st[(p.G + n) * 2 + 1] : 1.0;
    const int per = (p.V + kAccThreads - 1) / kAccThreads;
    const int v_lo = min(tid * per, p.V), v_hi = min(p.V, v_lo + per);

    bool use_p = !rejected;  // second round only if the residual is identically zero
    auto mass_of = [&](float t, float dq) -> double {
        const double pv = exp((double)t / p.T - tz) / ts;
        if (use_p) return pv;
        const double qv = exp((double)dq / p.T - dz) / ds;
        return pv - qv > 0.0 ? pv - qv : 0.0;
    };
    // logits are fetched 8 at a time so that the loads of a group are in flight together
    auto load8 = [&](int v0, float(&t8)[8], float(&d8)[8]) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int v = v0 + j;
            t8[j] = v < v_hi ? tl[v] : -INFINITY;
            d8[j] = (rejected && v < v_hi) ? dl[v] : -INFINITY;
        }
    };
    for (int round = 0; round < 2; ++round) {
        double local = 0.0;
        int lastpos = -1;  // last index of this range with positive mass
#pragma unroll 1
        for (int v0 = v_lo; v0 < v_hi; v0 += 8) {
            float t8[8], d8[8];
            load8(v0, t8, d8);
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (v0 + j < v_hi) {
                    const double mv = mass_of(t8[j], d8[j]);
                    local += mv;
                    if (mv > 0.0) lastpos = v0 + j;
                }
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
        double before = 0.0, Z = 0.0;
        for (int w = 0; w < kAccThreads / 64; ++w) {
            if (w < wave) before += wtot[w];
            Z += wtot[w];
        }
        if (!use_p && !(Z > 0.0)) {  // uniform over the workgroup: fall back to p itself
            use_p = true;
            continue;
        }
        const double target = (double)p.us[b] * Z;
        double cum = before + incl - local;
        // only ranges whose end lies above the target are walked: the one holding the answer
        // and those behind it (which stop at their first positive entry)
        int found = 0x7fffffff;
        if (cum + local > target) {
#pragma unroll 1
            for (int v0 = v_lo; v0 < v_hi && found == 0x7fffffff; v0 += 8) {
                float t8[8], d8[8];
                load8(v0, t8, d8);
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (found == 0x7fffffff && v0 + j < v_hi) {
                        const double mv = mass_of(t8[j], d8[j]);
                        cum += mv;
                        if (cum > target) found = v0 + j;
                    }
            }
        }
        if (found != 0x7fffffff) atomicMin(&s_tok, found);
        // used only when rounding leaves no cell above the target: the last positive entry
        if (lastpos >= 0) atomicMax(&s_last, lastpos);
        break;
    }
    __syncthreads();
    if (tid == 0) {
        const int tok = s_tok != 0x7fffffff ? s_tok : max(s_last, 0);
        for (int i = 0; i < p.G; ++i) out[i] = i < n ? x[i] : -1;
        out[n] = tok;
        p.n_acc[b] = n;
    }
}

size_t accept_workspace_bytes(int32_t B, int32_t G, int32_t V) {
    if (B <= 0 || G <= 0 || V <= 0) return 0;
    return (size_t)B * (2 * (size_t)G - 1) * 2 * sizeof(double);
}

int accept_launch(const float *target_logits, const float *draft_logits, const int32_t *draft_tokens, int32_t B,
                  int32_t G, int32_t V, float temperature, const float *u_accept, const float *u_sample,
                  int32_t *n_accepted, int32_t *out_tokens, void *ws, size_t ws_bytes, void *stream) {
    if (B < 1 || G < 1 || V < 1) return TF_ERR_INVALID_ARG;
    if (G > TF_MAX_SPEC) return TF_ERR_UNSUPPORTED;
    if (!target_logits || !u_sample || !n_accepted || !out_tokens) return TF_ERR_INVALID_ARG;
    if (G > 1 && (!draft_logits || !draft_tokens || !u_accept)) return TF_ERR_INVALID_ARG;
    if (!(temperature >= 0.f) || temperature - temperature != 0.f) return TF_ERR_INVALID_ARG;
    if ((int64_t)B * (2 * G - 1) >= (int64_t)1 << 31) return TF_ERR_UNSUPPORTED;
    if (!ws || !aligned(ws, 256) || ws_bytes < accept_workspace_bytes(B, G, V)) return TF_ERR_WORKSPACE;
    AcceptParams p;
    p.tl = target_logits;
    p.dl = draft_logits;
    p.toks = draft_tokens;
    p.B = B;
    p.G = G;
    p.V = V;
    p.T = (double)temperature;
    p.ua = u_accept;
    p.us = u_sample;
    p.n_acc = n_accepted;
    p.out = out_tokens;
    p.stats = static_cast<double *>(ws);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(accept_rowstats_kernel, dim3((unsigned)(B * (2 * G - 1))), dim3(kAccThreads), 0, st, p);
    hipLaunchKernelGGL(accept_decide_kernel, dim3((unsigned)B), dim3(kAccThreads), 0, st, p);
    return hip_status(hipGetLastError());
}

}  // namespace tf
