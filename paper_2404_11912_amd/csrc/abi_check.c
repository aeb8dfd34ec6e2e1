/* A plain C99 client of the library's C ABI (no Python, no PyTorch): allocates device memory
 * with the HIP runtime, runs tf_chunk_summarize and tf_decode_attn_full on a small cache and checks
 * two closed forms -- with scale = 0 every key is equally likely, so O is the mean of the V rows
 * and LSE = log(len); the average key of a chunk of identical rows is that row. Exit code 0 = ok.
 * Built by build.py as `abi_check`; run by the GPU tests. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "triforce.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)

static uint16_t f2bf(float f) /* exact for the small integers and halves used here */
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

int main(void)
{
    enum { B = 1, H = 2, N = 1000, D = TF_HEAD_DIM, G = 3, C = 8 };
    const size_t kv_elems = (size_t)B * H * N * D;
    uint16_t *hK = (uint16_t *)malloc(kv_elems * 2), *hV = (uint16_t *)malloc(kv_elems * 2);
    uint16_t *hQ = (uint16_t *)malloc((size_t)B * H * G * D * 2);
    double meanV[H][D];
    memset(meanV, 0, sizeof meanV);
    for (int h = 0; h < H; ++h)
        for (int t = 0; t < N; ++t)
            for (int j = 0; j < D; ++j) {
                const float k = (float)((t / C) % 7) - 3.0f;            /* constant inside a chunk */
                const float v = (float)((t * 3 + j + h) % 9) * 0.5f - 2.0f;
                hK[((size_t)h * N + t) * D + j] = f2bf(k);
                hV[((size_t)h * N + t) * D + j] = f2bf(v);
                meanV[h][j] += v / N;
            }
    for (int i = 0; i < B * H * G * D; ++i) hQ[i] = f2bf((float)(i % 5) - 2.0f);

    void *dK, *dV, *dQ, *dO, *dL, *dM, *ws;
    CK(hipMalloc(&dK, kv_elems * 2));
    CK(hipMalloc(&dV, kv_elems * 2));
    CK(hipMalloc(&dQ, (size_t)B * H * G * D * 2));
    CK(hipMalloc(&dO, (size_t)B * H * G * D * 4));
    CK(hipMalloc(&dL, (size_t)B * H * G * 4));
    CK(hipMalloc(&dM, (size_t)B * H * (N / C) * D * 4));
    const size_t ws_bytes = tf_decode_attn_full_workspace_bytes(B, H, N, G);
    CK(hipMalloc(&ws, ws_bytes));
    CK(hipMemcpy(dK, hK, kv_elems * 2, hipMemcpyHostToDevice));
    CK(hipMemcpy(dV, hV, kv_elems * 2, hipMemcpyHostToDevice));
    CK(hipMemcpy(dQ, hQ, (size_t)B * H * G * D * 2, hipMemcpyHostToDevice));

    tf_kv_desc kd;
    memset(&kd, 0, sizeof kd);
    kd.batch = B; kd.heads = H; kd.head_dim = D; kd.capacity = N;
    kd.stride_t = D; kd.stride_h = (int64_t)N * D; kd.stride_b = (int64_t)H * N * D;

    int rc = tf_decode_attn_full(dQ, dK, dV, &kd, NULL, N, G, 0.0f, 0, (float *)dO, (float *)dL, ws, ws_bytes, NULL);
    if (rc != TF_OK) { printf("tf_decode_attn_full: %s\n", tf_status_string(rc)); return 3; }
    rc = tf_chunk_summarize(dK, &kd, C, 0, N / C, (float *)dM, N / C, NULL);
    if (rc != TF_OK) { printf("tf_chunk_summarize: %s\n", tf_status_string(rc)); return 3; }
    CK(hipDeviceSynchronize());

    float *hO = (float *)malloc((size_t)B * H * G * D * 4), hL[B * H * G];
    float *hM = (float *)malloc((size_t)B * H * (N / C) * D * 4);
    CK(hipMemcpy(hO, dO, (size_t)B * H * G * D * 4, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hL, dL, sizeof hL, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hM, dM, (size_t)B * H * (N / C) * D * 4, hipMemcpyDeviceToHost));
    double err = 0.0, lerr = 0.0, merr = 0.0;
    for (int h = 0; h < H; ++h)
        for (int g = 0; g < G; ++g) {
            for (int j = 0; j < D; ++j)
                err = fmax(err, fabs((double)hO[((size_t)h * G + g) * D + j] - meanV[h][j]));
            lerr = fmax(lerr, fabs((double)hL[h * G + g] - log((double)N)));
        }
    for (int h = 0; h < H; ++h)
        for (int m = 0; m < N / C; ++m)
            for (int j = 0; j < D; ++j)
                merr = fmax(merr, fabs((double)hM[((size_t)h * (N / C) + m) * D + j] - ((double)(m % 7) - 3.0)));
    printf("abi_check: version %d, max|dO| %.2e, max|dLSE| %.2e, max|dKmean| %.2e\n", tf_version(), err, lerr, merr);
    /* error path: a bad argument is reported, nothing is launched */
    if (tf_decode_attn_full(NULL, dK, dV, &kd, NULL, N, G, 0.0f, 0, (float *)dO, NULL, ws, ws_bytes, NULL) != TF_ERR_INVALID_ARG) return 4;
    return (err < 1e-5 && lerr < 1e-5 && merr == 0.0) ? 0 : 1;
}
