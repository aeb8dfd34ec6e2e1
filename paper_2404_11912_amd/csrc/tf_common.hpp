// Shared host/device helpers of the gfx950 library (wave64, MFMA, LDS).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "triforce.h"

namespace tf {

constexpr int kHeadDim = TF_HEAD_DIM;  // 128 bf16 = 256 B per K/V row
constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (finite inputs)
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// 16-byte global load / store (rows are 16-byte aligned by contract)
__device__ __forceinline__ uint4 ld16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }
__device__ __forceinline__ void st16(void *p, uint4 v) { *reinterpret_cast<uint4 *>(p) = v; }

// Streaming variants (the `nt` bit): data that is touched once per pass -- the KV cache, the
// average-key table -- should not displace anything in L2 / the last-level cache. Measured on
// MI355X: +15% bandwidth on the 2 GiB-per-layer verification stream.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4v_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld16_stream(const void *p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 ld8_stream(const void *p) {
    typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
    const u32x2_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t *>(p));
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ float4 ldf4_stream(const float *p) {
    const f32x4v_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4v_t *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st16_stream(void *p, uint4 v) {
    u32x4_t w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t *>(p));
}
__device__ __forceinline__ void stf4_stream(float *p, float4 v) {
    f32x4v_t w = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(w, reinterpret_cast<f32x4v_t *>(p));
}

__device__ __forceinline__ float wave_max_xor(float v, int mask) {
    return fmaxf(v, __shfl_xor(v, mask, kWave));
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? TF_OK : TF_ERR_HIP; }

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// validates the parts of a descriptor every call relies on. The retrieval calls (summaries,
// scoring, gather) exist for head_dim 128 only; the attention calls and the cache append also
// take head_dim 64 (`allow_64`), the shape of the small draft model's cache.
inline int check_desc(const tf_kv_desc *d, bool allow_64 = false) {
    if (!d) return TF_ERR_INVALID_ARG;
    if (d->batch <= 0 || d->heads <= 0 || d->capacity <= 0) return TF_ERR_INVALID_ARG;
    if (d->head_dim != kHeadDim && !(allow_64 && d->head_dim == 64)) return TF_ERR_UNSUPPORTED;
    if (d->stride_t < d->head_dim || d->stride_b < 0 || d->stride_h < 0) return TF_ERR_INVALID_ARG;
    if ((d->stride_t % 8) || (d->stride_h % 8) || (d->stride_b % 8)) return TF_ERR_INVALID_ARG;
    return TF_OK;
}

// indexed attention: the virtual sequence is chunks idx[0..k_chunks) of the cache followed by
// the cache rows [recent_begin, len)
struct IndexedArgs {
    const int32_t *idx;
    int32_t k_chunks, chunk;
    const int32_t *recent_begin;
    int64_t recent_begin_all;
};

}  // namespace tf
