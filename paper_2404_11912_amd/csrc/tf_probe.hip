// tf_stream_read_probe: a plain streaming read of a device buffer, the measured ceiling the
// bandwidth-bound kernels of this library are compared with (next to the published HBM peak). Same
// ingredients as the attention kernel's stream -- one 256-thread workgroup per compute unit, each
// walking one contiguous range front to back with 16-byte nt loads -- and nothing else: the loaded
// words are XOR-ed and one word per thread is stored at the end so the loads cannot be dropped.
#include "tf_common.hpp"

namespace tf {

constexpr int kProbeDepth = 8;  // 16-byte loads in flight per lane

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *__restrict__ buf, int64_t vec_per_wg,
                                                          uint32_t *__restrict__ sink) {
    const uint4 *p = buf + (int64_t)blockIdx.x * vec_per_wg + threadIdx.x;
    const int64_t groups = vec_per_wg / (256 * kProbeDepth);  // whole groups only: never past the range
    uint32_t acc = 0;
    // two groups in flight: group g+1 is requested before group g is consumed
    uint4 va[kProbeDepth], vb[kProbeDepth];
    auto load = [&](int64_t gidx, uint4(&v)[kProbeDepth]) {
#pragma unroll
        for (int j = 0; j < kProbeDepth; ++j) v[j] = ld16_stream(p + (gidx * kProbeDepth + j) * 256);
    };
    auto eat = [&](const uint4(&v)[kProbeDepth]) {
#pragma unroll
        for (int j = 0; j < kProbeDepth; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
    };
    if (groups > 0) load(0, va);
    int64_t gidx = 0;
    for (; gidx + 2 < groups; gidx += 2) {
        load(gidx + 1, vb);
        eat(va);
        load(gidx + 2, va);
        eat(vb);
    }
    if (gidx + 1 < groups) {   // two groups left: va holds the first
        load(gidx + 1, vb);
        eat(va);
        eat(vb);
    } else if (gidx < groups) {
        eat(va);
    }
    sink[blockIdx.x * 256 + threadIdx.x] = acc;
}

int stream_read_probe_launch(const void *buf, size_t bytes, void *sink, size_t sink_bytes, size_t *bytes_read,
                             void *stream) {
    if (!buf || !sink || !bytes_read) return TF_ERR_INVALID_ARG;
    if (!aligned(buf, 16) || !aligned(sink, 4)) return TF_ERR_INVALID_ARG;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return TF_ERR_HIP;
    const int64_t group_vec = 256 * kProbeDepth;                              // vectors one workgroup reads per round
    const int wgs = cus;   // one workgroup per CU, 2 x 8 loads in flight per lane: the fastest of 1..8 per CU x 2..16 loads (7.2 TB/s)
    const int64_t vec_per_wg = (int64_t)(bytes / 16 / (size_t)wgs) / group_vec * group_vec;
    if (vec_per_wg <= 0) return TF_ERR_INVALID_ARG;                           // buffer too small to give every workgroup a round
    if (sink_bytes < (size_t)wgs * 256 * sizeof(uint32_t)) return TF_ERR_WORKSPACE;
    *bytes_read = (size_t)wgs * (size_t)vec_per_wg * 16;                      // <= bytes by construction
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)wgs), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(buf), vec_per_wg, static_cast<uint32_t *>(sink));
    return hip_status(hipGetLastError());
}

}  // namespace tf
