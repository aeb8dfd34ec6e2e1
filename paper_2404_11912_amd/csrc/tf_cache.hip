// tf_kv_append: write the K/V rows of newly decoded tokens into a cache (Sec. 4.3: in the
// retrieval cache they replace the least important entries; plain append for the full cache).
// A strided row copy: one wave moves 4 rows of K and of V with 16-byte accesses (16 lanes per row;
// rows of head_dim 64 use the first 8 of them).
#include "tf_common.hpp"

namespace tf {

struct AppendParams {
    const uint16_t *Kn, *Vn;
    uint16_t *K, *V;
    int64_t sb, sh, st, capacity;
    const int32_t *pos;
    int32_t pos_all, H, n, row_blocks, head_dim;
};

__global__ __launch_bounds__(256) void kv_append_kernel(const AppendParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t bh = blockIdx.x / p.row_blocks;
    const int i = (blockIdx.x % p.row_blocks) * 16 + wave * 4 + (lane >> 4);  // source row
    if (i >= p.n) return;
    const int b = (int)(bh / p.H), h = (int)(bh - (int64_t)b * p.H);
    const int64_t dst_row = (int64_t)(p.pos ? p.pos[b] : p.pos_all) + i;
    if (dst_row < 0 || dst_row >= p.capacity) return;  // rows outside the cache are dropped
    if ((lane & 15) * 8 >= p.head_dim) return;
    const int64_t src = (bh * p.n + i) * p.head_dim + (lane & 15) * 8;
    const int64_t dst = (int64_t)b * p.sb + (int64_t)h * p.sh + dst_row * p.st + (lane & 15) * 8;
    st16(p.K + dst, ld16(p.Kn + src));
    st16(p.V + dst, ld16(p.Vn + src));
}

int kv_append_launch(const void *Knew, const void *Vnew, int32_t n, void *K, void *V, const tf_kv_desc *kd,
                     const int32_t *pos, int64_t pos_all, void *stream) {
    if (!K || !V) return TF_ERR_INVALID_ARG;
    int rc = check_desc(kd, true);
    if (rc != TF_OK) return rc;
    if (n < 0 || pos_all < 0) return TF_ERR_INVALID_ARG;
    if (n > 0 && (!Knew || !Vnew)) return TF_ERR_INVALID_ARG;  // nothing is read when n == 0
    if (!pos && pos_all + n > kd->capacity) return TF_ERR_INVALID_ARG;
    if (pos_all > (int64_t)1 << 30 || n > (1 << 20)) return TF_ERR_UNSUPPORTED;
    if (!aligned(Knew, 16) || !aligned(Vnew, 16) || !aligned(K, 16) || !aligned(V, 16)) return TF_ERR_INVALID_ARG;
    if (n == 0) return TF_OK;
    const int64_t BH = (int64_t)kd->batch * kd->heads;
    AppendParams p;
    p.Kn = static_cast<const uint16_t *>(Knew);
    p.Vn = static_cast<const uint16_t *>(Vnew);
    p.K = static_cast<uint16_t *>(K);
    p.V = static_cast<uint16_t *>(V);
    p.sb = kd->stride_b;
    p.sh = kd->stride_h;
    p.st = kd->stride_t;
    p.capacity = kd->capacity;
    p.pos = pos;
    p.pos_all = (int32_t)pos_all;
    p.H = kd->heads;
    p.n = n;
    p.head_dim = kd->head_dim;
    p.row_blocks = (n + 15) / 16;
    if (BH * p.row_blocks >= (int64_t)1 << 31) return TF_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)(BH * p.row_blocks)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), p);
    return hip_status(hipGetLastError());
}

}  // namespace tf
