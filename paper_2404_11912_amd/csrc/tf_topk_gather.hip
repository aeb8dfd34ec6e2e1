// tf_chunk_topk_gather: retrieval-cache construction (Sec. 4.1 / Sec. 4.3): score every
// chunk by query . average-key, keep the k best in descending order, gather their K/V.
//
// Three kernels on one stream:
//   score   HBM streaming over the fp32 average-key table (512 B per chunk). A wave takes 16
//           chunk rows at a time; lane (r,s) holds dims {16j+4s..+4} of row r, does 32 fp32
//           FMAs against the resident query and two wave shuffles finish the dot product.
//   select  one 1024-thread workgroup per (b,h): exact radix select (4 x 8 bits, LDS
//           histograms) of the k-th largest order-preserving key, ordered compaction of the
//           winners (ties toward the lower chunk index), bitonic sort of the <= 2048 winners
//           on (score desc, index asc) in LDS.
//   gather  one wave per selected chunk copies its rows (256 B each) of K and V with 16-byte
//           loads and stores.
#include "tf_common.hpp"

namespace tf {

constexpr int kScoreIters = 4;
constexpr int kScoreRowsPerWg = 4 * 16 * kScoreIters;  // 4 waves x 16 rows x iters
constexpr int kSelThreads = 1024;

struct ScoreParams {
    const uint16_t *q_r;
    const float *Kmean;
    int64_t M_cap;
    const int32_t *n_chunks;
    int32_t n_all, H;
    int32_t blocks_per_bh;
    float *scores;
    int64_t score_stride;
};

__global__ __launch_bounds__(256) void chunk_score_kernel(const ScoreParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, s = lane >> 4;
    const int blk = blockIdx.x % p.blocks_per_bh;
    const int64_t bh = blockIdx.x / p.blocks_per_bh;
    const int b = (int)(bh / p.H);
    int n = p.n_chunks ? p.n_chunks[b] : p.n_all;
    n = min(max(n, 0), p.n_all);

    float q[8][4];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint2 w = *reinterpret_cast<const uint2 *>(p.q_r + bh * kHeadDim + 16 * j + 4 * s);
        q[j][0] = bf16lo(w.x);
        q[j][1] = bf16hi(w.x);
        q[j][2] = bf16lo(w.y);
        q[j][3] = bf16hi(w.y);
    }
    const float *base = p.Kmean + bh * p.M_cap * kHeadDim + 4 * s;
#pragma unroll 1
    for (int it = 0; it < kScoreIters; ++it) {
        const int m = blk * kScoreRowsPerWg + (wave * kScoreIters + it) * 16 + r;
        if (blk * kScoreRowsPerWg + (wave * kScoreIters + it) * 16 >= p.n_all) break;  // wave-uniform
        const int m_ld = min(m, max(n - 1, 0));
        const float *row = base + (int64_t)m_ld * kHeadDim;
        float4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = ldf4_stream(row + 16 * j);
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            acc = fmaf(q[j][0], v[j].x, acc);
            acc = fmaf(q[j][1], v[j].y, acc);
            acc = fmaf(q[j][2], v[j].z, acc);
            acc = fmaf(q[j][3], v[j].w, acc);
        }
        acc += __shfl_xor(acc, 16, kWave);
        acc += __shfl_xor(acc, 32, kWave);
        if (s == 0 && m < p.n_all) p.scores[bh * p.score_stride + m] = m < n ? acc : -INFINITY;
    }
}

// ascending order of keys == ascending order of the floats (-0 < +0, NaNs at the ends)
__device__ __forceinline__ uint32_t score_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// exclusive scan of one value per thread over a 1024-thread workgroup; *total = sum of all
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *wave_tot /*[16]*/, uint32_t *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t u = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += u;
    }
    __syncthreads();  // wave_tot may still be read from a previous scan
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kSelThreads / 64; ++w) {
        const uint32_t t = wave_tot[w];
        if (w < wave) before += t;
        all += t;
    }
    *total = all;
    return before + incl - v;
}

__global__ __launch_bounds__(kSelThreads) void topk_select_kernel(const float *__restrict__ scores,
                                                                  int64_t score_stride,
                                                                  const int32_t *__restrict__ n_chunks, int n_all,
                                                                  int H, int k, int32_t *__restrict__ out_idx,
                                                                  float *__restrict__ out_score) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wtot[16];
    __shared__ uint32_t s_digit, s_remaining;
    __shared__ unsigned long long cand[TF_MAX_K_CHUNKS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bh = blockIdx.x;
    const int b = (int)(bh / H);
    int n = n_chunks ? n_chunks[b] : n_all;
    n = min(max(n, 0), n_all);
    const int k_eff = min(k, n);
    const float *sc = scores + bh * score_stride;

    // ---- radix select: key of the k_eff-th largest score -------------------------------
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)k_eff;
    if (k_eff > 0) {
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (int i = tid; i < n; i += kSelThreads) {
                const uint32_t key = score_key(sc[i]);
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            // waves 0..3: suffix sums over the 256 bins (bin = tid)
            uint32_t hv = 0, incl = 0;
            if (tid < 256) {
                hv = hist[tid];
                incl = hv;
#pragma unroll
                for (int off = 1; off < 64; off <<= 1) {
                    const uint32_t u = __shfl_down(incl, off, kWave);
                    if (lane + off < 64) incl += u;
                }
                if (lane == 0) wtot[wave] = incl;
            }
            __syncthreads();
            if (tid < 256) {
                uint32_t above = 0;  // elements in the bins of higher waves
                for (int w = wave + 1; w < 4; ++w) above += wtot[w];
                const uint32_t sfx = incl + above;   // elements in bins >= tid
                const uint32_t sfx_excl = sfx - hv;  // elements in bins  > tid
                if (sfx >= remaining && sfx_excl < remaining) {
                    s_digit = (uint32_t)tid;
                    s_remaining = remaining - sfx_excl;
                }
            }
            __syncthreads();
            prefix |= s_digit << shift;
            mask |= 0xffu << shift;
            remaining = s_remaining;
            __syncthreads();
        }
    }
    const uint32_t T = prefix;                        // key of the k_eff-th largest
    const uint32_t n_gt = (uint32_t)k_eff - remaining;  // keys strictly above T (all kept)

    // ---- ordered compaction: thread t owns the contiguous index range [t*per, (t+1)*per) --
    int per = (n + kSelThreads - 1) / kSelThreads;
    per = (per + 3) & ~3;
    const int i_lo = tid * per, i_hi = min(n, i_lo + per);
    uint32_t c_gt = 0, c_eq = 0;
    if (k_eff > 0) {
        for (int i = i_lo; i < i_hi; i += 4) {
            const float4 f = *reinterpret_cast<const float4 *>(sc + i);
            const float fv[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i + u < i_hi) {
                    const uint32_t key = score_key(fv[u]);
                    c_gt += key > T;
                    c_eq += key == T;
                }
        }
    }
    uint32_t tot_gt, tot_eq;
    uint32_t p_gt = block_excl_scan(c_gt, wtot, &tot_gt);
    uint32_t p_eq = block_excl_scan(c_eq, wtot, &tot_eq);
    if (k_eff > 0) {
        for (int i = i_lo; i < i_hi; i += 4) {
            const float4 f = *reinterpret_cast<const float4 *>(sc + i);
            const float fv[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (i + u < i_hi) {
                    const uint32_t key = score_key(fv[u]);
                    const unsigned long long comp =
                        ((unsigned long long)key << 32) | (unsigned long long)(0xffffffffu - (uint32_t)(i + u));
                    if (key > T) {
                        cand[p_gt++] = comp;
                    } else if (key == T) {
                        if (p_eq < remaining) cand[n_gt + p_eq] = comp;
                        ++p_eq;
                    }
                }
        }
    }
    int kp = 1;
    while (kp < k_eff) kp <<= 1;
    for (int j = k_eff + tid; j < kp; j += kSelThreads) cand[j] = 0ull;  // below every real entry

    // ---- bitonic sort, descending on (key, ~index) ---------------------------------------
    for (int size = 2; size <= kp; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int t = tid; t < (kp >> 1); t += kSelThreads) {
                const int lo = 2 * t - (t & (stride - 1));
                const int hi = lo + stride;
                const bool desc = (lo & size) == 0;
                const unsigned long long a = cand[lo], c = cand[hi];
                if ((a < c) == desc) {
                    cand[lo] = c;
                    cand[hi] = a;
                }
            }
        }
    }
    __syncthreads();
    for (int j = tid; j < k; j += kSelThreads) {
        int32_t idx = -1;
        float val = -INFINITY;
        if (j < k_eff) {
            idx = (int32_t)(0xffffffffu - (uint32_t)(cand[j] & 0xffffffffull));
            val = sc[idx];
        }
        out_idx[bh * k + j] = idx;
        if (out_score) out_score[bh * k + j] = val;
    }
}

struct GatherParams {
    const uint16_t *K, *V;
    uint16_t *Kr, *Vr;
    int64_t sb, sh, st;     // source strides
    int64_t rb, rh, rt;     // retrieval-cache strides
    const int32_t *idx;
    int32_t H, k, chunk, jblocks;
};

__global__ __launch_bounds__(256) void chunk_gather_kernel(const GatherParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = (blockIdx.x % p.jblocks) * 4 + wave;
    const int64_t bh = blockIdx.x / p.jblocks;
    if (j >= p.k) return;
    const int m = p.idx[bh * p.k + j];
    if (m < 0) return;
    const int b = (int)(bh / p.H), h = (int)(bh - (int64_t)b * p.H);
    const int64_t src = (int64_t)b * p.sb + (int64_t)h * p.sh + (int64_t)m * p.chunk * p.st + (lane & 15) * 8;
    const int64_t dst = (int64_t)b * p.rb + (int64_t)h * p.rh + (int64_t)j * p.chunk * p.rt + (lane & 15) * 8;
#pragma unroll 2
    for (int i = lane >> 4; i < p.chunk; i += 4) {
        const uint4 kv = ld16_stream(p.K + src + (int64_t)i * p.st);
        const uint4 vv = ld16_stream(p.V + src + (int64_t)i * p.st);
        st16(p.Kr + dst + (int64_t)i * p.rt, kv);
        st16(p.Vr + dst + (int64_t)i * p.rt, vv);
    }
}

static int64_t score_stride_of(int64_t n_all) { return (n_all + 3) & ~(int64_t)3; }

size_t topk_workspace_bytes(int32_t batch, int32_t heads, int64_t n_chunks_all, int32_t k_chunks) {
    if (batch <= 0 || heads <= 0 || n_chunks_all <= 0 || k_chunks <= 0) return 0;
    // scores [BH][stride] fp32 (+ one float4 of slack for the vector loads of the last row)
    return ((size_t)batch * heads * score_stride_of(n_chunks_all) + 4) * sizeof(float);
}

int topk_gather_launch(const void *q_r, const float *Kmean, int64_t M_cap, const void *K, const void *V,
                       const tf_kv_desc *kd, int32_t chunk, const int32_t *n_chunks, int64_t n_chunks_all,
                       int32_t k_chunks, int32_t *out_idx, float *out_score, void *Kr, void *Vr,
                       const tf_kv_desc *rd, void *ws, size_t ws_bytes, void *stream) {
    if (!q_r || !Kmean || !out_idx) return TF_ERR_INVALID_ARG;
    int rc = check_desc(kd);
    if (rc != TF_OK) return rc;
    const bool do_gather = Kr != nullptr || Vr != nullptr;
    if (do_gather) {
        if (!Kr || !Vr || !K || !V) return TF_ERR_INVALID_ARG;
        rc = check_desc(rd);
        if (rc != TF_OK) return rc;
        if (rd->batch != kd->batch || rd->heads != kd->heads) return TF_ERR_INVALID_ARG;
        if ((int64_t)k_chunks * chunk > rd->capacity) return TF_ERR_INVALID_ARG;
        if (!aligned(K, 16) || !aligned(V, 16) || !aligned(Kr, 16) || !aligned(Vr, 16)) return TF_ERR_INVALID_ARG;
    }
    if (chunk < 1 || k_chunks < 1 || n_chunks_all < 1 || M_cap < 1) return TF_ERR_INVALID_ARG;
    if (chunk > 64 || k_chunks > TF_MAX_K_CHUNKS) return TF_ERR_UNSUPPORTED;
    if (n_chunks_all > M_cap || k_chunks > n_chunks_all) return TF_ERR_INVALID_ARG;
    if (n_chunks_all > ((int64_t)1 << 30)) return TF_ERR_UNSUPPORTED;
    if (n_chunks_all * chunk > kd->capacity) return TF_ERR_INVALID_ARG;
    if (!aligned(q_r, 8) || !aligned(Kmean, 16)) return TF_ERR_INVALID_ARG;
    if (!ws || !aligned(ws, 256) ||
        ws_bytes < topk_workspace_bytes(kd->batch, kd->heads, n_chunks_all, k_chunks))
        return TF_ERR_WORKSPACE;

    const int64_t BH = (int64_t)kd->batch * kd->heads;
    hipStream_t st = static_cast<hipStream_t>(stream);

    ScoreParams sp;
    sp.q_r = static_cast<const uint16_t *>(q_r);
    sp.Kmean = Kmean;
    sp.M_cap = M_cap;
    sp.n_chunks = n_chunks;
    sp.n_all = (int32_t)n_chunks_all;
    sp.H = kd->heads;
    sp.blocks_per_bh = (int32_t)((n_chunks_all + kScoreRowsPerWg - 1) / kScoreRowsPerWg);
    sp.scores = static_cast<float *>(ws);
    sp.score_stride = score_stride_of(n_chunks_all);
    if (sp.blocks_per_bh * BH >= (int64_t)1 << 31) return TF_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(chunk_score_kernel, dim3((unsigned)(sp.blocks_per_bh * BH)), dim3(256), 0, st, sp);

    hipLaunchKernelGGL(topk_select_kernel, dim3((unsigned)BH), dim3(kSelThreads), 0, st, sp.scores,
                       sp.score_stride, n_chunks, (int)n_chunks_all, (int)kd->heads, (int)k_chunks, out_idx,
                       out_score);

    if (do_gather) {
        GatherParams gp;
        gp.K = static_cast<const uint16_t *>(K);
        gp.V = static_cast<const uint16_t *>(V);
        gp.Kr = static_cast<uint16_t *>(Kr);
        gp.Vr = static_cast<uint16_t *>(Vr);
        gp.sb = kd->stride_b;
        gp.sh = kd->stride_h;
        gp.st = kd->stride_t;
        gp.rb = rd->stride_b;
        gp.rh = rd->stride_h;
        gp.rt = rd->stride_t;
        gp.idx = out_idx;
        gp.H = kd->heads;
        gp.k = k_chunks;
        gp.chunk = chunk;
        gp.jblocks = (k_chunks + 3) / 4;
        hipLaunchKernelGGL(chunk_gather_kernel, dim3((unsigned)(gp.jblocks * BH)), dim3(256), 0, st, gp);
    }
    return hip_status(hipGetLastError());
}

}  // namespace tf
