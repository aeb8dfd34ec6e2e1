/*
 * tf_oracle.c -- plain fp64 CPU oracle for the decode-step attention path of
 * hierarchical speculative decoding with a retrieval cache.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT. Only tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it. It shares no code with the HIP
 * library and is deliberately slow and plain: straight loops, two-pass softmax,
 * a full sort for the top-k, no blocking, no fusion, no online softmax.
 * bf16 inputs (raw uint16 bit patterns) and fp32 inputs are widened exactly to
 * fp64; all arithmetic is fp64. OpenMP only spreads independent (batch, head)
 * or sequence units over host cores; it never changes a summation order.
 *
 * What each function follows:
 *   orc_attention   model forward over a KV cache (Algorithm 1, the M_p(C_p, ...) and
 *                   M_p(C_r, ...) steps): standard scaled-dot-product attention, the
 *                   plain definition written out.
 *   orc_chunk_mean  the mean of the keys of every chunk (Sec. 4.1).
 *   orc_retrieve    score = query . average chunk key, keep the highest-scoring
 *                   chunks under a fixed budget, in descending importance
 *                   (Sec. 4.1, Sec. 4.3).
 *   orc_gather      gather the selected chunks' K/V into the retrieval cache (Sec. 4.1).
 *   orc_accept      Verify / Correct / bonus token of Algorithm 1, i.e. the standard
 *                   lossless speculative-sampling rule the paper refers to (Sec. 4.2,
 *                   "Correctness").
 *
 * Readings taken where the paper is silent are listed in the repository's design notes;
 * the ones that shape this file: raw dot-product chunk scores; ties broken toward the
 * lower chunk index; causal mask bottom-right aligned (query g of G sees keys
 * [0, kv_len-G+g]); accept iff u*q(x) < p(x); tokens drawn by inverse CDF in index order.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py against closed
 * forms, invariants, brute force and Monte-Carlo laws (none is "parity unpinned").
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_to_f64(uint16_t h)
{
    uint32_t u = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------------------
 * Attention of G queries over a KV cache, per (b, h).
 *   Q [B,H,G,d] bf16, K,V [B,H,N,d] bf16 (contiguous), kv_len[b] <= N valid tokens.
 *   causal != 0: query g sees tokens t < kv_len - G + 1 + g (the G queries are the last
 *   G tokens of the cache); causal == 0: every query sees all kv_len tokens.
 *   z_t = scale * <Q_g, K_t>;  w_t = exp(z_t - max z) ;  O_g = sum w_t V_t / sum w_t ;
 *   LSE_g = max z + log sum w_t.   wsum_g = sum_t (w_t / sum w) (should be 1).
 * Returns 0, or -1 on a bad argument / allocation failure.
 * ---------------------------------------------------------------------------------- */
int orc_attention(const uint16_t *Q, const uint16_t *K, const uint16_t *V,
                  int B, int H, int G, int64_t N, int d,
                  const int32_t *kv_len, double scale, int causal,
                  double *O, double *LSE, double *wsum)
{
    if (B <= 0 || H <= 0 || G <= 0 || N <= 0 || d <= 0) return -1;
    for (int b = 0; b < B; ++b) {
        if (kv_len[b] < 0 || kv_len[b] > N) return -1;
    }
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
        int b = bh / H;
        int64_t n_all = kv_len[b];
        const uint16_t *Kbh = K + (int64_t)bh * N * d;
        const uint16_t *Vbh = V + (int64_t)bh * N * d;
        double *z = (double *)malloc(sizeof(double) * (size_t)(n_all > 0 ? n_all : 1));
        if (!z) { failed = 1; continue; }
        for (int g = 0; g < G; ++g) {
            const uint16_t *q = Q + ((int64_t)bh * G + g) * d;
            int64_t n_g = causal ? (n_all - G + 1 + g) : n_all;
            if (n_g <= 0) { /* a query that sees no key: O = 0, LSE = -inf by convention */
                double *o0 = O + ((int64_t)bh * G + g) * d;
                for (int j = 0; j < d; ++j) o0[j] = 0.0;
                LSE[(int64_t)bh * G + g] = -INFINITY;
                if (wsum) wsum[(int64_t)bh * G + g] = 0.0;
                continue;
            }
            double m = -INFINITY;
            for (int64_t t = 0; t < n_g; ++t) {
                double acc = 0.0;
                for (int j = 0; j < d; ++j)
                    acc += bf16_to_f64(q[j]) * bf16_to_f64(Kbh[t * d + j]);
                z[t] = scale * acc;
                if (z[t] > m) m = z[t];
            }
            double denom = 0.0;
            for (int64_t t = 0; t < n_g; ++t) {
                z[t] = exp(z[t] - m);
                denom += z[t];
            }
            double *o = O + ((int64_t)bh * G + g) * d;
            for (int j = 0; j < d; ++j) o[j] = 0.0;
            double ws = 0.0;
            for (int64_t t = 0; t < n_g; ++t) {
                double w = z[t] / denom;
                ws += w;
                for (int j = 0; j < d; ++j)
                    o[j] += w * bf16_to_f64(Vbh[t * d + j]);
            }
            LSE[(int64_t)bh * G + g] = m + log(denom);
            if (wsum) wsum[(int64_t)bh * G + g] = ws;
        }
        free(z);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------------------
 * Chunk summaries: Kmean[b,h,m,:] = (1/c) * sum_{i<c} K[b,h,m*c+i,:], m < M = floor(N/c).
 * A ragged tail (N mod c tokens) has no summary. Kmean is [B,H,M,d] fp64.
 * ---------------------------------------------------------------------------------- */
int orc_chunk_mean(const uint16_t *K, int B, int H, int64_t N, int d, int c, double *Kmean)
{
    if (B <= 0 || H <= 0 || N <= 0 || d <= 0 || c <= 0) return -1;
    int64_t M = N / c;
#pragma omp parallel for schedule(static)
    for (int bh = 0; bh < B * H; ++bh) {
        const uint16_t *Kbh = K + (int64_t)bh * N * d;
        double *out = Kmean + (int64_t)bh * M * d;
        for (int64_t m = 0; m < M; ++m)
            for (int j = 0; j < d; ++j) {
                double s = 0.0;
                for (int i = 0; i < c; ++i)
                    s += bf16_to_f64(Kbh[(m * c + i) * d + j]);
                out[m * d + j] = s / (double)c;
            }
    }
    return 0;
}

typedef struct {
    double s;
    int32_t i;
} scored_t;

/* descending score, ties toward the lower index: a total order, so any sort gives the
 * result a stable sort of (-s) would give */
static int cmp_scored(const void *a, const void *b)
{
    const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->i > y->i) - (x->i < y->i);
}

/* ------------------------------------------------------------------------------------
 * Retrieval: scores[b,h,m] = <q_r[b,h,:], Kmean[b,h,m,:]> for m < n_chunks[b]; sort all
 * chunks by (score descending, index ascending); idx[b,h,0..k) = the first k.
 *   q_r [B,H,d] bf16; Kmean [B,H,M,d] fp64; scores [B,H,M] (entries >= n_chunks[b] set to
 *   -inf); idx [B,H,k] int32.  Requires 1 <= k <= n_chunks[b] <= M.
 * ---------------------------------------------------------------------------------- */
int orc_retrieve(const uint16_t *q_r, const double *Kmean, int B, int H, int64_t M, int d,
                 const int32_t *n_chunks, int k, double *scores, int32_t *idx)
{
    if (B <= 0 || H <= 0 || M <= 0 || d <= 0 || k <= 0) return -1;
    for (int b = 0; b < B; ++b)
        if (n_chunks[b] < k || n_chunks[b] > M) return -1;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * H; ++bh) {
        int b = bh / H;
        int64_t Mb = n_chunks[b];
        const double *km = Kmean + (int64_t)bh * M * d;
        const uint16_t *q = q_r + (int64_t)bh * d;
        double *sc = scores + (int64_t)bh * M;
        scored_t *tab = (scored_t *)malloc(sizeof(scored_t) * (size_t)Mb);
        if (!tab) { failed = 1; continue; }
        for (int64_t m = 0; m < M; ++m) sc[m] = -INFINITY;
        for (int64_t m = 0; m < Mb; ++m) {
            double acc = 0.0;
            for (int j = 0; j < d; ++j)
                acc += bf16_to_f64(q[j]) * km[m * d + j];
            sc[m] = acc;
            tab[m].s = acc;
            tab[m].i = (int32_t)m;
        }
        qsort(tab, (size_t)Mb, sizeof(scored_t), cmp_scored);
        for (int j = 0; j < k; ++j) idx[(int64_t)bh * k + j] = tab[j].i;
        free(tab);
    }
    return failed ? -1 : 0;
}

/* ------------------------------------------------------------------------------------
 * Gather: Kr[b,h,j*c+i,:] = K[b,h,idx[b,h,j]*c+i,:] (same for V), j < k, i < c.
 * K,V [B,H,N,d]; Kr,Vr [B,H,R_cap,d] with R_cap >= k*c; rows >= k*c are left untouched.
 * ---------------------------------------------------------------------------------- */
int orc_gather(const uint16_t *K, const uint16_t *V, int B, int H, int64_t N, int d, int c,
               const int32_t *idx, int k, int64_t R_cap, uint16_t *Kr, uint16_t *Vr)
{
    if ((int64_t)k * c > R_cap) return -1;
    for (int bh = 0; bh < B * H; ++bh)
        for (int j = 0; j < k; ++j) {
            int64_t m = idx[(int64_t)bh * k + j];
            if (m < 0 || (m + 1) * c > N) return -1;
            for (int i = 0; i < c; ++i) {
                int64_t src = ((int64_t)bh * N + m * c + i) * d;
                int64_t dst = ((int64_t)bh * R_cap + (int64_t)j * c + i) * d;
                memcpy(Kr + dst, K + src, sizeof(uint16_t) * (size_t)d);
                memcpy(Vr + dst, V + src, sizeof(uint16_t) * (size_t)d);
            }
        }
    return 0;
}

/* softmax(logits / T) in fp64 */
static void softmax_T(const float *logits, int V, double T, double *p)
{
    double m = -INFINITY;
    for (int v = 0; v < V; ++v) {
        double z = (double)logits[v] / T;
        if (z > m) m = z;
    }
    double s = 0.0;
    for (int v = 0; v < V; ++v) {
        p[v] = exp((double)logits[v] / T - m);
        s += p[v];
    }
    for (int v = 0; v < V; ++v) p[v] /= s;
}

static int argmax_first(const float *x, int V)
{
    int a = 0;
    for (int v = 1; v < V; ++v)
        if (x[v] > x[a]) a = v;
    return a;
}

/* smallest v with sum_{w<=v} r_w > target; if rounding leaves none, the last v with r_v > 0.
 * *margin = distance of target to the nearest edge of the chosen cell, relative to total. */
static int inverse_cdf(const double *r, int V, double target, double total, double *margin)
{
    double cum = 0.0;
    int last_pos = 0;
    for (int v = 0; v < V; ++v) {
        double lo = cum;
        cum += r[v];
        if (r[v] > 0.0) last_pos = v;
        if (cum > target) {
            double a = target - lo, bb = cum - target;
            *margin = (a < bb ? a : bb) / total;
            return v;
        }
    }
    *margin = 0.0;
    return last_pos;
}

/* ------------------------------------------------------------------------------------
 * Speculative accept / resample, one sequence per b.  gamma = G-1 drafted tokens.
 *   target_logits [B,G,V] fp32, draft_logits [B,gamma,V] fp32, draft_tokens [B,gamma],
 *   u_accept [B,gamma], u_sample [B] in [0,1).
 *   T > 0: p_i = softmax(target_i/T), q_i = softmax(draft_i/T). Walk i = 0..gamma-1 with
 *   x = draft_tokens[i]: accept iff u_accept[i]*q_i[x] < p_i[x]. First reject at i: draw
 *   from norm(max(p_i - q_i, 0)) (from p_i if that residual is all zero) by inverse CDF at
 *   u_sample; n_accepted = i. All accepted: draw from p_gamma; n_accepted = gamma.
 *   T == 0: p, q one-hot at the first arg-max: accept iff x == argmax target_i;
 *   correction / bonus = argmax of the target row.
 *   out_tokens [B,G]: the n accepted tokens, then the drawn token, then -1.
 *   margin_accept[b] (optional): min over evaluated tests of |u*q(x)-p(x)| / max(p(x),u*q(x));
 *   margin_sample[b] (optional): relative distance of u_sample*Z to the nearest CDF edge.
 *   (1.0 where no floating-point decision was taken, i.e. T == 0.)
 * ---------------------------------------------------------------------------------- */
int orc_accept(const float *target_logits, const float *draft_logits, const int32_t *draft_tokens,
               int B, int G, int V, double T, const float *u_accept, const float *u_sample,
               int32_t *n_accepted, int32_t *out_tokens, double *margin_accept,
               double *margin_sample)
{
    if (B <= 0 || G <= 0 || V <= 0 || T < 0.0) return -1;
    int gamma = G - 1;
    for (int64_t i = 0; i < (int64_t)B * gamma; ++i)
        if (draft_tokens[i] < 0 || draft_tokens[i] >= V) return -1;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 16)
    for (int b = 0; b < B; ++b) {
        const float *tl = target_logits + (int64_t)b * G * V;
        const float *dl = draft_logits + (int64_t)b * gamma * V;
        const int32_t *x = draft_tokens + (int64_t)b * gamma;
        int32_t *out = out_tokens + (int64_t)b * G;
        for (int i = 0; i < G; ++i) out[i] = -1;
        double ma = 1.0, ms = 1.0;
        int n = 0, tok = -1;
        if (T == 0.0) {
            for (n = 0; n < gamma; ++n)
                if (x[n] != argmax_first(tl + (int64_t)n * V, V)) break;
            tok = argmax_first(tl + (int64_t)n * V, V);
        } else {
            double *p = (double *)malloc(sizeof(double) * (size_t)V * 3);
            if (!p) { failed = 1; continue; }
            double *q = p + V, *r = q + V;
            int rejected = 0;
            for (n = 0; n < gamma; ++n) {
                softmax_T(tl + (int64_t)n * V, V, T, p);
                softmax_T(dl + (int64_t)n * V, V, T, q);
                double lhs = (double)u_accept[(int64_t)b * gamma + n] * q[x[n]];
                double rhs = p[x[n]];
                double big = lhs > rhs ? lhs : rhs;
                double mg = big > 0.0 ? fabs(lhs - rhs) / big : 0.0;
                if (mg < ma) ma = mg;
                if (!(lhs < rhs)) { rejected = 1; break; }
            }
            double us = (double)u_sample[b];
            if (rejected) {
                double Z = 0.0;
                for (int v = 0; v < V; ++v) {
                    r[v] = p[v] - q[v] > 0.0 ? p[v] - q[v] : 0.0;
                    Z += r[v];
                }
                if (Z > 0.0) {
                    tok = inverse_cdf(r, V, us * Z, Z, &ms);
                } else {
                    double S = 0.0;
                    for (int v = 0; v < V; ++v) S += p[v];
                    tok = inverse_cdf(p, V, us * S, S, &ms);
                }
            } else {
                softmax_T(tl + (int64_t)gamma * V, V, T, p);
                double S = 0.0;
                for (int v = 0; v < V; ++v) S += p[v];
                tok = inverse_cdf(p, V, us * S, S, &ms);
            }
            free(p);
        }
        for (int i = 0; i < n; ++i) out[i] = x[i];
        out[n] = tok;
        n_accepted[b] = n;
        if (margin_accept) margin_accept[b] = ma;
        if (margin_sample) margin_sample[b] = ms;
    }
    return failed ? -1 : 0;
}
