// tf_chunk_summarize: the average key of every KV chunk (Sec. 4.1: the keys of a chunk are
// averaged), fp32 output (or, as a variant, the fp32 mean rounded to bf16).
//
// Pure HBM streaming: K is read once (256 B per token), 512 B are written per chunk. A wave
// owns 4 chunks at a time: lane (r,s) accumulates dims 8r..8r+8 of chunk s over the chunk's
// rows, so every load instruction reads four whole 256-byte rows and no cross-lane
// reduction is needed. Rows of a chunk are added in token order in fp32.
#include "tf_common.hpp"

namespace tf {

constexpr int kSumWaves = 2;                                  // waves per workgroup
constexpr int kSumIters = 1;                                  // chunk groups per wave (1 measured best)
constexpr int kSumChunksPerWg = kSumWaves * 4 * kSumIters;    // waves x 4 chunks x iters

struct SumParams {
    const uint16_t *K;
    int64_t sb, sh, st;
    int32_t H, chunk;
    int64_t first_chunk, n_chunks;
    int64_t blocks_per_bh;
    void *Kmean;  // fp32 or bf16 [BH][M_cap][128]
    int64_t M_cap;
};

template <bool kBf16Out>
__global__ __launch_bounds__(kSumWaves * 64) void chunk_summarize_kernel(const SumParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 15, s = lane >> 4;
    const int64_t blk = blockIdx.x % p.blocks_per_bh;
    const int64_t bh = blockIdx.x / p.blocks_per_bh;
    const int b = (int)(bh / p.H), h = (int)(bh - (int64_t)b * p.H);
    const uint16_t *Kb = p.K + (int64_t)b * p.sb + (int64_t)h * p.sh + r * 8;
    const int c = p.chunk;

#pragma unroll 1
    for (int it = 0; it < kSumIters; ++it) {
        const int64_t local = blk * kSumChunksPerWg + (int64_t)(wave * kSumIters + it) * 4 + s;
        if (local >= p.n_chunks) continue;
        const int64_t m = p.first_chunk + local;
        const uint16_t *src = Kb + m * c * p.st;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int i0 = 0; i0 < c; i0 += 8) {
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (i0 + u < c) v[u] = ld16_stream(src + (int64_t)(i0 + u) * p.st);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (i0 + u < c) {
                    acc[0] += bf16lo(v[u].x);
                    acc[1] += bf16hi(v[u].x);
                    acc[2] += bf16lo(v[u].y);
                    acc[3] += bf16hi(v[u].y);
                    acc[4] += bf16lo(v[u].z);
                    acc[5] += bf16hi(v[u].z);
                    acc[6] += bf16lo(v[u].w);
                    acc[7] += bf16hi(v[u].w);
                }
        }
        const int64_t off = (bh * p.M_cap + m) * kHeadDim + r * 8;
        const float fc = (float)c;  // correctly rounded division: exact for power-of-two chunks
        if constexpr (kBf16Out) {
            uint4 o;
            o.x = f32_to_bf16(acc[0] / fc) | (f32_to_bf16(acc[1] / fc) << 16);
            o.y = f32_to_bf16(acc[2] / fc) | (f32_to_bf16(acc[3] / fc) << 16);
            o.z = f32_to_bf16(acc[4] / fc) | (f32_to_bf16(acc[5] / fc) << 16);
            o.w = f32_to_bf16(acc[6] / fc) | (f32_to_bf16(acc[7] / fc) << 16);
            st16(static_cast<uint16_t *>(p.Kmean) + off, o);
        } else {
            float *dst = static_cast<float *>(p.Kmean) + off;
            *reinterpret_cast<float4 *>(dst) = make_float4(acc[0] / fc, acc[1] / fc, acc[2] / fc, acc[3] / fc);
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(acc[4] / fc, acc[5] / fc, acc[6] / fc, acc[7] / fc);
        }
    }
}

int summarize_launch(const void *K, const tf_kv_desc *kd, int32_t chunk, int64_t first_chunk, int64_t n_chunks,
                     void *Kmean, int64_t M_cap, void *stream, bool mean_bf16) {
    if (!K || !Kmean) return TF_ERR_INVALID_ARG;
    int rc = check_desc(kd);
    if (rc != TF_OK) return rc;
    if (chunk < 1 || first_chunk < 0 || n_chunks < 0 || M_cap < 1) return TF_ERR_INVALID_ARG;
    if (chunk > 64) return TF_ERR_UNSUPPORTED;
    if (first_chunk + n_chunks > M_cap) return TF_ERR_INVALID_ARG;
    if ((first_chunk + n_chunks) * chunk > kd->capacity) return TF_ERR_INVALID_ARG;
    if (!aligned(K, 16) || !aligned(Kmean, 16)) return TF_ERR_INVALID_ARG;
    if (n_chunks == 0) return TF_OK;
    const int64_t BH = (int64_t)kd->batch * kd->heads;
    SumParams p;
    p.K = static_cast<const uint16_t *>(K);
    p.sb = kd->stride_b;
    p.sh = kd->stride_h;
    p.st = kd->stride_t;
    p.H = kd->heads;
    p.chunk = chunk;
    p.first_chunk = first_chunk;
    p.n_chunks = n_chunks;
    p.blocks_per_bh = (n_chunks + kSumChunksPerWg - 1) / kSumChunksPerWg;
    p.Kmean = Kmean;
    p.M_cap = M_cap;
    if (p.blocks_per_bh * BH >= (int64_t)1 << 31) return TF_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)(p.blocks_per_bh * BH));
    if (mean_bf16)
        hipLaunchKernelGGL(chunk_summarize_kernel<true>, grid, dim3(kSumWaves * 64), 0, static_cast<hipStream_t>(stream), p);
    else
        hipLaunchKernelGGL(chunk_summarize_kernel<false>, grid, dim3(kSumWaves * 64), 0, static_cast<hipStream_t>(stream), p);
    return hip_status(hipGetLastError());
}

}  // namespace tf
