/* A plain C99 client of the library's C ABI (no Python, no PyTorch): allocates device memory with
 * the HIP runtime, runs all five calls of the decode-step path on a small cache and checks closed
 * forms that need no reference implementation:
 *   tf_chunk_summarize        a chunk of identical rows averages to that row (exactly);
 *   tf_decode_attn_full       with scale = 0 every key is equally likely: O = mean of the V rows,
 *                             LSE = log(len);
 *   tf_chunk_topk_gather      keys are a(m) * q per chunk with a = 4 on planted chunks and a in
 *                             {-1, 0, 1} elsewhere: the selection is the planted chunks in ascending
 *                             index (equal scores), then the first a = 1 chunks; scores are the exact
 *                             integers a * |q|^2; gathered rows are byte-equal to the rows named;
 *   tf_decode_attn_retrieval  over that gathered cache, scale = 0, causal: query g averages the first
 *                             R-G+1+g gathered V rows, LSE = log of that count;
 *   tf_spec_accept            T = 0: the arg-max walk; T = 1 with draft == target logits: everything
 *                             is accepted whatever the uniforms, the bonus token is the one entry that
 *                             holds all but 1e-20 of the last row's mass;
 * plus one error path per call (nothing is launched, a negative status comes back).
 * Exit code 0 = ok. Built by build.py as `abi_check`; run by the GPU tests. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "triforce.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)e_, __LINE__); return 2; } } while (0)
#define TF(x) do { int rc_ = (x); if (rc_ != TF_OK) { printf("line %d: %s\n", __LINE__, tf_status_string(rc_)); return 3; } } while (0)
#define EXPECT(cond) do { if (!(cond)) { printf("abi_check: check failed at line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

enum { B = 1, H = 2, N = 1000, D = TF_HEAD_DIM, G = 3, C = 8, M = N / C, KSEL = 8, R = KSEL * C, NPLANT = 5 };
enum { AB = 2, AG = 4, AV = 1000 };   /* accept: sequences, G, vocabulary */

static uint16_t f2bf(float f) /* exact for the small integers and halves used here */
{
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

static float q_of(int h, int j) { return (float)((j + h) % 5) - 2.0f; }

static const int planted[NPLANT] = {100, 7, 64, 3, 19};

static float a_of(int h, int m) /* the factor of chunk m: its keys are a * q */
{
    for (int i = 0; i < NPLANT; ++i)
        if (planted[i] + h == m) return 4.0f;   /* head h plants chunks shifted by h */
    return (float)((m + h) % 3) - 1.0f;
}

static int upload(void **dst, const void *src, size_t bytes)
{
    CK(hipMalloc(dst, bytes));
    CK(hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice));
    return 0;
}

static int accept_checks(int *failures_out);

int main(void)
{
    int failures = 0;
    const size_t kv_elems = (size_t)B * H * N * D;
    uint16_t *hK = (uint16_t *)malloc(kv_elems * 2), *hV = (uint16_t *)malloc(kv_elems * 2);
    uint16_t *hQ = (uint16_t *)malloc((size_t)B * H * G * D * 2), hq[B * H * D];
    double meanV[H][D], qq[H];
    memset(meanV, 0, sizeof meanV);
    for (int h = 0; h < H; ++h) {
        qq[h] = 0.0;
        for (int j = 0; j < D; ++j) {
            hq[h * D + j] = f2bf(q_of(h, j));
            qq[h] += (double)q_of(h, j) * q_of(h, j);
        }
        for (int t = 0; t < N; ++t)
            for (int j = 0; j < D; ++j) {
                const float k = a_of(h, t / C) * q_of(h, j);              /* constant inside a chunk */
                const float v = (float)((t * 3 + j + h) % 9) * 0.5f - 2.0f;
                hK[((size_t)h * N + t) * D + j] = f2bf(k);
                hV[((size_t)h * N + t) * D + j] = f2bf(v);
                meanV[h][j] += v / N;
            }
    }
    for (int i = 0; i < B * H * G * D; ++i) hQ[i] = f2bf((float)(i % 5) - 2.0f);

    void *dK, *dV, *dQ, *dq, *dO, *dL, *dM, *dIdx, *dSc, *dKr, *dVr, *ws;
    if (upload(&dK, hK, kv_elems * 2) || upload(&dV, hV, kv_elems * 2) ||
        upload(&dQ, hQ, (size_t)B * H * G * D * 2) || upload(&dq, hq, sizeof hq))
        return 2;
    CK(hipMalloc(&dO, (size_t)B * H * G * D * 4));
    CK(hipMalloc(&dL, (size_t)B * H * G * 4));
    CK(hipMalloc(&dM, (size_t)B * H * M * D * 4));
    CK(hipMalloc(&dIdx, (size_t)B * H * KSEL * 4));
    CK(hipMalloc(&dSc, (size_t)B * H * KSEL * 4));
    CK(hipMalloc(&dKr, (size_t)B * H * R * D * 2));
    CK(hipMalloc(&dVr, (size_t)B * H * R * D * 2));
    size_t ws_bytes = tf_decode_attn_full_workspace_bytes(B, H, N, G);
    const size_t ws_topk = tf_chunk_topk_gather_workspace_bytes(B, H, M, KSEL);
    const size_t ws_retr = tf_decode_attn_retrieval_workspace_bytes(B, H, R, G);
    EXPECT(ws_bytes > 0 && ws_topk > 0 && ws_retr > 0);
    if (ws_topk > ws_bytes) ws_bytes = ws_topk;
    if (ws_retr > ws_bytes) ws_bytes = ws_retr;
    CK(hipMalloc(&ws, ws_bytes));

    tf_kv_desc kd, rd;
    memset(&kd, 0, sizeof kd);
    kd.batch = B; kd.heads = H; kd.head_dim = D; kd.capacity = N;
    kd.stride_t = D; kd.stride_h = (int64_t)N * D; kd.stride_b = (int64_t)H * N * D;
    rd = kd;
    rd.capacity = R; rd.stride_h = (int64_t)R * D; rd.stride_b = (int64_t)H * R * D;

    /* ---- verification attention and chunk summaries ---------------------------------------- */
    TF(tf_decode_attn_full(dQ, dK, dV, &kd, NULL, N, G, 0.0f, 0, (float *)dO, (float *)dL, ws, ws_bytes, NULL));
    TF(tf_chunk_summarize(dK, &kd, C, 0, M, (float *)dM, M, NULL));
    CK(hipDeviceSynchronize());
    float *hO = (float *)malloc((size_t)B * H * G * D * 4), hL[B * H * G];
    float *hM = (float *)malloc((size_t)B * H * M * D * 4);
    CK(hipMemcpy(hO, dO, (size_t)B * H * G * D * 4, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hL, dL, sizeof hL, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hM, dM, (size_t)B * H * M * D * 4, hipMemcpyDeviceToHost));
    double err = 0.0, lerr = 0.0, merr = 0.0;
    for (int h = 0; h < H; ++h)
        for (int g = 0; g < G; ++g) {
            for (int j = 0; j < D; ++j)
                err = fmax(err, fabs((double)hO[((size_t)h * G + g) * D + j] - meanV[h][j]));
            lerr = fmax(lerr, fabs((double)hL[h * G + g] - log((double)N)));
        }
    for (int h = 0; h < H; ++h)
        for (int m = 0; m < M; ++m)
            for (int j = 0; j < D; ++j)
                merr = fmax(merr, fabs((double)hM[((size_t)h * M + m) * D + j] - (double)(a_of(h, m) * q_of(h, j))));
    EXPECT(err < 1e-5 && lerr < 1e-5 && merr == 0.0);

    /* ---- retrieval-cache construction ------------------------------------------------------- */
    CK(hipMemset(dKr, 0xff, (size_t)B * H * R * D * 2));
    CK(hipMemset(dVr, 0xff, (size_t)B * H * R * D * 2));
    TF(tf_chunk_topk_gather(dq, (const float *)dM, M, dK, dV, &kd, C, NULL, M, KSEL, (int32_t *)dIdx, (float *)dSc,
                            dKr, dVr, &rd, ws, ws_bytes, NULL));
    /* ---- draft attention over the gathered cache --------------------------------------------- */
    TF(tf_decode_attn_retrieval(dQ, dKr, dVr, &rd, NULL, R, G, 0.0f, 1, (float *)dO, (float *)dL, ws, ws_bytes, NULL));
    CK(hipDeviceSynchronize());
    int32_t hIdx[B * H * KSEL], want[H][KSEL];
    float hSc[B * H * KSEL];
    uint16_t *hKr = (uint16_t *)malloc((size_t)B * H * R * D * 2), *hVr = (uint16_t *)malloc((size_t)B * H * R * D * 2);
    CK(hipMemcpy(hIdx, dIdx, sizeof hIdx, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hSc, dSc, sizeof hSc, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hKr, dKr, (size_t)B * H * R * D * 2, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hVr, dVr, (size_t)B * H * R * D * 2, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hO, dO, (size_t)B * H * G * D * 4, hipMemcpyDeviceToHost));
    CK(hipMemcpy(hL, dL, sizeof hL, hipMemcpyDeviceToHost));
    int idx_bad = 0, sc_bad = 0, row_bad = 0;
    double derr = 0.0, dlerr = 0.0;
    for (int h = 0; h < H; ++h) {
        int n = 0;
        for (int m = 0; m < M; ++m)                      /* a = 4 first, ascending chunk index ...   */
            if (a_of(h, m) == 4.0f) want[h][n++] = m;
        for (int m = 0; m < M && n < KSEL; ++m)          /* ... then a = 1, ascending chunk index    */
            if (a_of(h, m) == 1.0f) want[h][n++] = m;
        for (int j = 0; j < KSEL; ++j) {
            idx_bad += hIdx[h * KSEL + j] != want[h][j];
            sc_bad += (double)hSc[h * KSEL + j] != (double)a_of(h, want[h][j]) * qq[h];
            for (int i = 0; i < C; ++i) {
                const size_t src = ((size_t)h * N + (size_t)want[h][j] * C + i) * D;
                const size_t dst = ((size_t)h * R + (size_t)j * C + i) * D;
                row_bad += memcmp(hKr + dst, hK + src, D * 2) != 0;
                row_bad += memcmp(hVr + dst, hV + src, D * 2) != 0;
            }
        }
        for (int g = 0; g < G; ++g) {                    /* causal, scale 0: prefix means of the gathered V rows */
            const int n_g = R - G + 1 + g;
            for (int j = 0; j < D; ++j) {
                double mean = 0.0;
                for (int t = 0; t < n_g; ++t) {
                    uint32_t u = (uint32_t)hV[((size_t)h * N + (size_t)want[h][t / C] * C + t % C) * D + j] << 16;
                    float f;
                    memcpy(&f, &u, 4);
                    mean += f;
                }
                derr = fmax(derr, fabs((double)hO[((size_t)h * G + g) * D + j] - mean / n_g));
            }
            dlerr = fmax(dlerr, fabs((double)hL[h * G + g] - log((double)n_g)));
        }
    }
    EXPECT(idx_bad == 0 && sc_bad == 0 && row_bad == 0);
    EXPECT(derr < 1e-5 && dlerr < 1e-5);

    /* ---- error paths: a bad argument is reported, nothing is launched -------------------------- */
    EXPECT(tf_decode_attn_full(NULL, dK, dV, &kd, NULL, N, G, 0.0f, 0, (float *)dO, NULL, ws, ws_bytes, NULL) ==
           TF_ERR_INVALID_ARG);
    EXPECT(tf_chunk_summarize(dK, &kd, C, 0, M + 1, (float *)dM, M, NULL) == TF_ERR_INVALID_ARG);
    EXPECT(tf_chunk_topk_gather(dq, (const float *)dM, M, dK, dV, &kd, C, NULL, M, TF_MAX_K_CHUNKS + 1, (int32_t *)dIdx,
                                NULL, NULL, NULL, NULL, ws, ws_bytes, NULL) == TF_ERR_UNSUPPORTED);
    EXPECT(tf_chunk_topk_gather(dq, (const float *)dM, M, dK, dV, &kd, C, NULL, M, KSEL + 1, (int32_t *)dIdx,
                                NULL, dKr, dVr, &rd, ws, ws_bytes, NULL) == TF_ERR_INVALID_ARG);   /* cache too small */
    EXPECT(tf_decode_attn_retrieval(dQ, dKr, dVr, &rd, NULL, R, G, 0.0f, 1, (float *)dO, (float *)dL, ws, 16, NULL) ==
           TF_ERR_WORKSPACE);

    const int arc = accept_checks(&failures);
    if (arc) return arc;
    printf("abi_check: version %d, full max|dO| %.2e max|dLSE| %.2e, max|dKmean| %.2e, top-k idx/score/row mismatches "
           "%d/%d/%d, draft max|dO| %.2e max|dLSE| %.2e, failures %d\n",
           tf_version(), err, lerr, merr, idx_bad, sc_bad, row_bad, derr, dlerr, failures);
    return failures ? 1 : 0;
}

/* logits with a known arg-max: a low, bounded pattern and one entry at +peak */
static void fill_row(float *row, int hot, float peak, int salt)
{
    for (int v = 0; v < AV; ++v) row[v] = (float)((v * 7 + salt) % 11) * 0.1f;
    row[hot] = peak;
}

static int accept_checks(int *failures_out)
{
    int failures = 0;
    const int gamma = AG - 1;
    static float tl[AB][AG][AV], dl[AB][AG - 1][AV];
    int32_t tok[AB][AG - 1], hot[AB][AG];
    float ua[AB][AG - 1], us[AB] = {0.5f, 0.25f};
    for (int b = 0; b < AB; ++b)
        for (int i = 0; i < AG; ++i) {
            hot[b][i] = (37 * i + 411 * b + 5) % AV;
            fill_row(tl[b][i], hot[b][i], 5.0f, i + b);
            if (i < gamma) {
                fill_row(dl[b][i], (hot[b][i] + 1) % AV, 3.0f, 2 * i + b);   /* the draft model prefers another token */
                tok[b][i] = hot[b][i];
                ua[b][i] = 0.999f;
            }
        }
    tok[0][2] = (hot[0][2] + 9) % AV;   /* sequence 0: the third drafted token is not the target's arg-max */

    void *dtl, *ddl, *dtok, *dua, *dus, *dn, *dout, *ws;
    if (upload(&dtl, tl, sizeof tl) || upload(&ddl, dl, sizeof dl) || upload(&dtok, tok, sizeof tok) ||
        upload(&dua, ua, sizeof ua) || upload(&dus, us, sizeof us))
        return 2;
    CK(hipMalloc(&dn, AB * 4));
    CK(hipMalloc(&dout, AB * AG * 4));
    const size_t ws_bytes = tf_spec_accept_workspace_bytes(AB, AG, AV);
    EXPECT(ws_bytes > 0);
    CK(hipMalloc(&ws, ws_bytes));
    int32_t n[AB], out[AB][AG];

    /* T = 0: accept while the drafted token is the target's arg-max; then that arg-max */
    TF(tf_spec_accept((const float *)dtl, (const float *)ddl, (const int32_t *)dtok, AB, AG, AV, 0.0f,
                      (const float *)dua, (const float *)dus, (int32_t *)dn, (int32_t *)dout, ws, ws_bytes, NULL));
    CK(hipDeviceSynchronize());
    CK(hipMemcpy(n, dn, sizeof n, hipMemcpyDeviceToHost));
    CK(hipMemcpy(out, dout, sizeof out, hipMemcpyDeviceToHost));
    EXPECT(n[0] == 2 && out[0][0] == hot[0][0] && out[0][1] == hot[0][1] && out[0][2] == hot[0][2] && out[0][3] == -1);
    EXPECT(n[1] == 3 && out[1][0] == hot[1][0] && out[1][1] == hot[1][1] && out[1][2] == hot[1][2] &&
           out[1][3] == hot[1][3]);

    /* T = 1, draft logits == target logits (p = q): every token is accepted for any u < 1; the last
     * target row holds all but ~1e-20 of its mass on one entry, which is then the bonus token */
    for (int b = 0; b < AB; ++b) {
        fill_row(tl[b][gamma], hot[b][gamma], 60.0f, b);
        for (int i = 0; i < gamma; ++i) tok[b][i] = (hot[b][i] + 3 * i + 1) % AV;   /* any token with q > 0 */
    }
    CK(hipMemcpy(dtl, tl, sizeof tl, hipMemcpyHostToDevice));
    CK(hipMemcpy(dtok, tok, sizeof tok, hipMemcpyHostToDevice));
    TF(tf_spec_accept((const float *)dtl, (const float *)dtl /* rows i < gamma of the same [B,G,V] array */, (const int32_t *)dtok,
                      1, AG, AV, 1.0f, (const float *)dua, (const float *)dus, (int32_t *)dn, (int32_t *)dout, ws,
                      ws_bytes, NULL));
    CK(hipDeviceSynchronize());
    CK(hipMemcpy(n, dn, sizeof n, hipMemcpyDeviceToHost));
    CK(hipMemcpy(out, dout, sizeof out, hipMemcpyDeviceToHost));
    EXPECT(n[0] == gamma && out[0][0] == tok[0][0] && out[0][1] == tok[0][1] && out[0][2] == tok[0][2] &&
           out[0][3] == hot[0][gamma]);

    EXPECT(tf_spec_accept((const float *)dtl, (const float *)ddl, (const int32_t *)dtok, AB, TF_MAX_SPEC + 1, AV, 0.0f,
                          (const float *)dua, (const float *)dus, (int32_t *)dn, (int32_t *)dout, ws, ws_bytes, NULL) ==
           TF_ERR_UNSUPPORTED);
    EXPECT(tf_spec_accept((const float *)dtl, (const float *)ddl, (const int32_t *)dtok, AB, AG, AV, -1.0f,
                          (const float *)dua, (const float *)dus, (int32_t *)dn, (int32_t *)dout, ws, ws_bytes, NULL) ==
           TF_ERR_INVALID_ARG);
    *failures_out += failures;
    return 0;
}
