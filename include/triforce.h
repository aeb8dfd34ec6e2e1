/*
 * triforce.h -- C ABI of the MI355X (gfx950) decode-step attention library for
 * hierarchical speculative decoding with a retrieval cache (TriForce, arxiv 2404.11912).
 *
 * One call handles ONE transformer layer for all batch x head units; a decode step is L
 * such calls. The five operations are the data-parallel hot path of Algorithm 1:
 *
 *   tf_chunk_summarize        average key of every KV chunk            (Sec. 4.1)
 *   tf_chunk_topk_gather      score chunks by query . average key, keep the best k under a
 *                             fixed budget, gather their K/V           (Sec. 4.1, Sec. 4.3)
 *   tf_decode_attn_full       target model attention over the full cache C_p: verification of
 *                             the speculated tokens                    (Algorithm 1, M_p(C_p,..))
 *   tf_decode_attn_retrieval  the same attention over the retrieval cache C_r: self-drafting
 *                                                                      (Algorithm 1, M_p(C_r,..))
 *   tf_spec_accept            Verify / Correct / bonus token: lossless speculative sampling
 *                                                                      (Algorithm 1, Sec. 4.2)
 * and, beyond those five, the cache-update pieces of Sec. 4.3:
 *   tf_decode_attn_indexed    drafting through the chunk indices, no gathered copy
 *   tf_kv_append              write new tokens' K/V rows into a cache
 * and the verification pass for a token tree instead of a chain (Sec. 5.3.3, compatibility with
 * tree-based speculative decoding):
 *   tf_decode_attn_tree       tf_decode_attn_full with a per-query mask over the speculated tokens
 * and a half-size variant of the average-key table:
 *   tf_chunk_summarize_bf16, tf_chunk_topk_gather_bf16
 * and the accept step for batches with different draft lengths per sequence:
 *   tf_spec_accept_ragged
 * and, for callers and measurement rather than for the method:
 *   tf_decode_attn_retrieval_noalloc  the draft attention without a workspace argument
 *   tf_set_option, tf_set_thread_option, tf_decode_attn_plan, tf_stream_read_probe
 *
 * Conventions (all calls)
 *   - Every data pointer is a DEVICE pointer owned by the caller (the only host pointers are
 *     the tf_kv_desc structs and strings). The library keeps no reference after return.
 *   - Nothing is allocated, freed or synchronised: work is enqueued on the caller's HIP
 *     stream, passed as `void* stream` (a hipStream_t; NULL = the default stream). Scratch
 *     memory comes from a caller-provided workspace `ws` of at least the size the matching
 *     *_workspace_bytes() query returns (256-byte aligned); calls sharing one workspace must
 *     be ordered on one stream. The attention queries are monotone in the length: a workspace
 *     queried for kv_len_all = X (same batch, heads, G and knobs) serves every call with
 *     kv_len_all <= X.
 *   - bf16 tensors are raw 16-bit patterns (upper half of an IEEE fp32), fp32 is IEEE float.
 *   - Strides are in ELEMENTS. head_dim must be contiguous (stride 1) and 128; the attention
 *     calls (full, retrieval, indexed, tree) and tf_kv_append also accept 64, the head size of
 *     the small draft model whose StreamingLLM cache (sinks + recent window) the indexed call
 *     reads. Q, O then have 64 columns; workspace queries return the (larger) 128 figure.
 *   - Every call returns a status: TF_OK, or a negative TF_ERR_* after which nothing was
 *     enqueued. Errors are detected on the host before launch; the library never aborts.
 *   - Shapes are fixed per call and no call reads device memory on the host, so a sequence
 *     of calls can be captured into a HIP graph.
 */
#ifndef TRIFORCE_H
#define TRIFORCE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TF_OK 0
#define TF_ERR_INVALID_ARG (-1) /* null pointer, non-positive size, inconsistent shapes      */
#define TF_ERR_UNSUPPORTED (-2) /* head_dim not supported, G > 16, k_chunks > 2048, ...       */
#define TF_ERR_WORKSPACE (-3)   /* workspace missing, misaligned or too small                */
#define TF_ERR_HIP (-4)         /* a HIP runtime call (kernel launch) reported an error      */
#define TF_ERR_SCRATCH_LIMIT (-5) /* tf_decode_attn_retrieval_noalloc: the problem needs more
                                     scratch than the library's built-in buffer holds          */

#define TF_HEAD_DIM 128
#define TF_MAX_QUERIES 16    /* G = gamma + 1 queries (or tree nodes) per attention call      */
#define TF_MAX_K_CHUNKS 2048 /* chunks kept by one tf_chunk_topk_gather call                 */
#define TF_MAX_SPEC 16       /* G of tf_spec_accept                                          */

/* A K or V cache tensor of one layer, bf16, indexed [b][h][t][0..head_dim).
 * Element (b,h,t,j) lives at base + b*stride_b + h*stride_h + t*stride_t + j.
 * The native layout [B,H,capacity,128] has stride_t = 128, stride_h = capacity*128,
 * stride_b = heads*capacity*128. Base pointer and all strides must keep rows 16-byte
 * aligned (strides multiples of 8 elements). K and V of one call share one descriptor.
 * Grouped-query attention: with q_group > 1 the attention calls take Q, O of
 * [batch, heads*q_group, G, head_dim] and LSE of [batch, heads*q_group, G]; query head q uses KV
 * head q / q_group. G * q_group <= TF_MAX_QUERIES (the group's query rows share one pass over its K/V);
 * workspace queries then take G * q_group as their G. Other calls ignore q_group. */
typedef struct tf_kv_desc {
    int32_t batch;
    int32_t heads;    /* KV heads */
    int32_t head_dim; /* TF_HEAD_DIM, or 64 for the attention calls and tf_kv_append */
    int32_t q_group;  /* query heads per KV head for the attention calls; 0 or 1 = MHA */
    int64_t capacity; /* allocated tokens per (b,h) */
    int64_t stride_b, stride_h, stride_t;
} tf_kv_desc;

int tf_version(void);                   /* major*10000 + minor*100 + patch */
const char *tf_status_string(int code); /* static string, never NULL */

/* Tuning knobs. Known names:
 *   "attn_full_tokens_per_split", "attn_retr_tokens_per_split"  (multiples of 64; 0 = auto),
 *   "score_steps_per_wave" (16-chunk steps a wave of the scoring kernel takes; 0 = auto),
 *   "rebuild_fused" (tf_chunk_topk_gather: 0 = auto, 1 = score and select in one kernel whenever a
 *   unit has at most 16384 chunks, 2 = never; the results do not depend on it).
 * tf_set_option sets the process-wide default (an atomic: safe to call while other threads run
 * calls, which pick up either the old or the new value). tf_set_thread_option sets an override that
 * only the CALLING host thread's later workspace queries and calls see (value -1 removes it), so
 * threads that drive different streams can tune independently. Every call reads its knobs once and
 * plans, checks the workspace and launches from that one reading. Workspace queries reflect the
 * knobs the calling thread sees when they are made; change a knob between query and call and the
 * call may answer TF_ERR_WORKSPACE (never overrun the workspace).
 * Returns TF_ERR_INVALID_ARG for an unknown name or bad value. */
int tf_set_option(const char *name, int64_t value);
int tf_set_thread_option(const char *name, int64_t value);

/* ---------------------------------------------------------------------------------------
 * tf_chunk_summarize -- Sec. 4.1: every chunk of the KV cache is summarised by the mean of its keys.
 *   Kmean[b,h,m,:] = (1/chunk) * sum_{i<chunk} K[b,h,m*chunk+i,:]   for
 *   m in [first_chunk, first_chunk+n_chunks), every (b,h). Arithmetic, fixed so that the result
 *   is reproducible bit for bit: the chunk's keys are widened to fp32 and added in token order
 *   to a sum starting at +0 (each addition rounded to fp32), then one IEEE fp32 division by chunk.
 *   K      in   bf16, described by kd; (first_chunk+n_chunks)*chunk <= kd->capacity
 *   Kmean  out  fp32 [batch, heads, M_cap, 128] contiguous; other rows untouched
 *   The range arguments allow summarising only newly completed chunks. n_chunks == 0 is a
 *   no-op. chunk in [1, 64].
 * ------------------------------------------------------------------------------------- */
int tf_chunk_summarize(const void *K, const tf_kv_desc *kd, int32_t chunk, int64_t first_chunk,
                       int64_t n_chunks, float *Kmean, int64_t M_cap, void *stream);

/* ---------------------------------------------------------------------------------------
 * tf_chunk_topk_gather -- Sec. 4.1 / Sec. 4.3: retrieval-cache construction.
 *   score[b,h,m] = sum_j q_r[b,h,j] * Kmean[b,h,m,j] (raw dot product, fp32), for
 *   m < n[b], n[b] = n_chunks ? n_chunks[b] : n_chunks_all (n_chunks_all is always an upper
 *   bound of n[b] and <= M_cap). The k_chunks highest-scoring chunks are kept in descending
 *   score order, equal scores toward the lower chunk index. Then, for j < k_chunks, i < chunk:
 *     Kr[b,h,j*chunk+i,:] = K[b,h,out_idx[b,h,j]*chunk+i,:]   (same for V), bit-exact copies.
 *   q_r       in   bf16 [batch, heads, 128]
 *   Kmean     in   fp32 [batch, heads, M_cap, 128] (from tf_chunk_summarize)
 *   K, V      in   bf16, described by kd
 *   n_chunks  in   int32 [batch] device array, or NULL
 *   out_idx   out  int32 [batch, heads, k_chunks]
 *   out_score out  fp32  [batch, heads, k_chunks] or NULL
 *   Kr, Vr    out  bf16, described by rd (same batch/heads as kd, capacity >= k_chunks*chunk);
 *                  rows >= k_chunks*chunk untouched. Kr == NULL && Vr == NULL skips the gather.
 *   If n[b] < k_chunks on the device, only n[b] chunks are kept: the remaining out_idx slots
 *   are -1 (scores -inf) and the corresponding cache rows are left untouched.
 *   1 <= k_chunks <= min(n_chunks_all, TF_MAX_K_CHUNKS); chunk in [1, 64].
 * ------------------------------------------------------------------------------------- */
size_t tf_chunk_topk_gather_workspace_bytes(int32_t batch, int32_t heads, int64_t n_chunks_all,
                                            int32_t k_chunks);
int tf_chunk_topk_gather(const void *q_r, const float *Kmean, int64_t M_cap, const void *K,
                         const void *V, const tf_kv_desc *kd, int32_t chunk,
                         const int32_t *n_chunks, int64_t n_chunks_all, int32_t k_chunks,
                         int32_t *out_idx, float *out_score, void *Kr, void *Vr,
                         const tf_kv_desc *rd, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * tf_chunk_summarize_bf16 / tf_chunk_topk_gather_bf16 -- the same two operations (Sec. 4.1) with
 * the average-key table held in bf16: half the table's memory and half the scoring traffic.
 *   Kmean_bf16[b,h,m,:] = the fp32 mean exactly as tf_chunk_summarize computes it (sequential fp32
 *   sum in token order, one fp32 division), then rounded to bf16, nearest even: two roundings, so
 *   about one entry in 10^5..10^6 is one bf16 ulp away from the exact mean rounded once;
 *   scores are fp32 dot products of q_r with the widened bf16 entries; everything else
 *   (selection order, ties, gather, arguments, workspace size, errors) as in the fp32 calls.
 * A table written by tf_chunk_summarize_bf16 must be read by tf_chunk_topk_gather_bf16.
 * Rounding the averages moves scores by up to ~4e-4 at these magnitudes, so the chunks chosen
 * near the k-th score can differ from those the fp32 table selects.
 * ------------------------------------------------------------------------------------- */
int tf_chunk_summarize_bf16(const void *K, const tf_kv_desc *kd, int32_t chunk, int64_t first_chunk,
                            int64_t n_chunks, void *Kmean, int64_t M_cap, void *stream);
int tf_chunk_topk_gather_bf16(const void *q_r, const void *Kmean, int64_t M_cap, const void *K,
                              const void *V, const tf_kv_desc *kd, int32_t chunk,
                              const int32_t *n_chunks, int64_t n_chunks_all, int32_t k_chunks,
                              int32_t *out_idx, float *out_score, void *Kr, void *Vr,
                              const tf_kv_desc *rd, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * tf_decode_attn_full -- Algorithm 1, the pass of M_p over the full cache C_p: attention of the
 * G = gamma+1 speculated query tokens of one layer over the whole KV cache.
 *   len[b] = kv_len ? kv_len[b] : kv_len_all (kv_len_all is always an upper bound of len[b]
 *   and <= kd->capacity). For every (b,h,g), with n_g = causal ? len[b]-G+1+g : len[b]
 *   (the G queries are the last G tokens already appended to the cache):
 *     z_t = scale * <Q[b,h,g,:], K[b,h,t,:]>, t < n_g ;  O[b,h,g,:] = softmax_t(z) . V ;
 *     LSE[b,h,g] = log sum_t exp(z_t)   (natural log).
 *   Q       in   bf16 [batch, heads, G, 128] contiguous
 *   K, V    in   bf16, described by kd
 *   kv_len  in   int32 [batch] device array, or NULL
 *   O       out  fp32 [batch, heads, G, 128];  LSE out fp32 [batch, heads, G] or NULL
 *   bf16 inputs, fp32 accumulation. A query with no visible key (n_g <= 0) gets O = 0,
 *   LSE = -inf. 1 <= G <= TF_MAX_QUERIES; causal requires kv_len_all >= G.
 * ------------------------------------------------------------------------------------- */
size_t tf_decode_attn_full_workspace_bytes(int32_t batch, int32_t heads, int64_t kv_len_all,
                                           int32_t G);
int tf_decode_attn_full(const void *Q, const void *K, const void *V, const tf_kv_desc *kd,
                        const int32_t *kv_len, int64_t kv_len_all, int32_t G, float scale,
                        int32_t causal, float *O, float *LSE, void *ws, size_t ws_bytes,
                        void *stream);

/* Measurement aid (not a step of the method): a plain streaming read of `bytes` of device memory
 * at `buf` -- one workgroup per compute unit, each walking a contiguous range with 16-byte
 * streaming loads, nothing else -- enqueued on `stream`. Timing it gives the read bandwidth this GPU really
 * sustains, the ceiling the KV-streaming kernels (Algorithm 1's two attention passes) are compared
 * with, next to the published peak. Reads whole rounds only: *bytes_read (a HOST integer, written
 * before return) is the number of bytes the kernel reads, <= bytes. `sink` is device scratch of at
 * least 4 * 256 * (compute units) bytes (one word per thread is stored). buf must be 16-byte
 * aligned; TF_ERR_INVALID_ARG if the buffer is too small to give every workgroup 32 KiB. */
int tf_stream_read_probe(const void *buf, size_t bytes, void *sink, size_t sink_bytes, size_t *bytes_read,
                         void *stream);

/* The launch shape an attention call would take now (split-K over the KV sequence, Algorithm 1's
 * two attention passes): kind 0 = tf_decode_attn_full / tf_decode_attn_tree, 1 =
 * tf_decode_attn_retrieval, 2 = tf_decode_attn_indexed (len_all = k_chunks*chunk + recent rows).
 * Writes the number of splits per (batch, head) unit and the tokens per split to the two HOST
 * integers. Informational (profiling, tests); depends on the knobs the calling thread sees and on
 * the current device's compute-unit count. */
#define TF_PLAN_FULL 0
#define TF_PLAN_RETRIEVAL 1
#define TF_PLAN_INDEXED 2
int tf_decode_attn_plan(int32_t kind, int32_t batch, int32_t heads, int64_t len_all, int32_t *nsplit,
                        int32_t *tokens_per_split);

/* ---------------------------------------------------------------------------------------
 * tf_decode_attn_tree -- verification of a speculated token TREE (Sec. 5.3.3, the combination with
 * tree-based speculative decoding): tf_decode_attn_full with the causal triangle replaced by an
 * ancestor mask. The G speculated tokens are the last G rows of the cache, in any order that
 * puts parents before children; query g sees every row t < len[b]-G (the context) and, of the
 * speculated rows, row len[b]-G+j iff bit j of tail_mask[g] is set (normally its ancestors and
 * itself). tail_mask[g] = (2 << g) - 1 reproduces causal != 0, 0xffff reproduces causal == 0.
 *   tail_mask  in  HOST array of G 16-bit rows, read during the call (the only host-side
 *                  input); bits >= G are ignored.
 * Other arguments, outputs, limits, workspace size and errors as tf_decode_attn_full
 * (tf_decode_attn_full_workspace_bytes); requires kv_len_all >= G. A query that sees nothing
 * gets O = 0, LSE = -inf.
 * ------------------------------------------------------------------------------------- */
int tf_decode_attn_tree(const void *Q, const void *K, const void *V, const tf_kv_desc *kd,
                        const int32_t *kv_len, int64_t kv_len_all, int32_t G, float scale,
                        const uint16_t *tail_mask, float *O, float *LSE, void *ws, size_t ws_bytes,
                        void *stream);

/* ---------------------------------------------------------------------------------------
 * tf_decode_attn_retrieval -- Algorithm 1, the pass of M_p over the retrieval cache C_r: the same
 * attention over the gathered retrieval cache (K, V are Kr, Vr; kv_len is the number of valid
 * cache rows, budget plus any tokens the caller appended). Same arguments and semantics as
 * tf_decode_attn_full; tuned for short caches (launch-latency regime).
 * ------------------------------------------------------------------------------------- */
size_t tf_decode_attn_retrieval_workspace_bytes(int32_t batch, int32_t heads, int64_t kv_len_all,
                                                int32_t G);
int tf_decode_attn_retrieval(const void *Q, const void *K, const void *V, const tf_kv_desc *kd,
                             const int32_t *kv_len, int64_t kv_len_all, int32_t G, float scale,
                             int32_t causal, float *O, float *LSE, void *ws, size_t ws_bytes,
                             void *stream);

/* ---------------------------------------------------------------------------------------
 * tf_decode_attn_retrieval_noalloc -- for callers that cannot allocate or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. The same operation,
 * kernels, launch shape and results (bit for bit) as tf_decode_attn_retrieval, but the split partials
 * live in a buffer built into the library (a file-scope device array of tf_noalloc_scratch_bytes() =
 * 16 MiB that every GPU the library runs on holds until the process ends) instead of a workspace
 * argument. Neither this call nor tf_noalloc_init allocates or frees memory.
 *   - Limit: the partials of the launch shape the call plans must fit the buffer:
 *     batch * heads * nsplit * 4 * rows * 130 * 4 bytes, nsplit as tf_decode_attn_plan(TF_PLAN_RETRIEVAL,
 *     ...) reports, rows = 8 (16 when G * q_group > 8). Beyond tf_noalloc_scratch_bytes() the call
 *     returns TF_ERR_SCRATCH_LIMIT and enqueues nothing. (16 MiB hold e.g. 32 heads x 30 splits, while
 *     a 4K..16K budget plans 8.)
 *   - All calls on one GPU share that GPU's buffer: calls that may overlap on one GPU (different
 *     streams, or two captured graphs replayed concurrently) race on it and must be ordered by the
 *     caller. Nothing in the buffer has to be cleared between calls: every partial a call's merge
 *     step reads was written by that call's split step.
 *   - The buffer's device address is looked up on the first call on each device (with that device
 *     current); tf_noalloc_init() does the same lookup ahead of time for the current device, e.g.
 *     before a graph capture begins. Returns TF_ERR_HIP if the lookup fails.
 * ------------------------------------------------------------------------------------- */
int tf_noalloc_init(void);
size_t tf_noalloc_scratch_bytes(void);
int tf_decode_attn_retrieval_noalloc(const void *Q, const void *K, const void *V, const tf_kv_desc *kd,
                                     const int32_t *kv_len, int64_t kv_len_all, int32_t G, float scale,
                                     int32_t causal, float *O, float *LSE, void *stream);

/* ---------------------------------------------------------------------------------------
 * tf_decode_attn_indexed -- gather-free drafting (Algorithm 1, the pass of M_p over the retrieval
 * cache C_r; Sec. 4.1 chunk selection): the same attention, over a draft cache that is never
 * materialised. For every (b,h) the draft cache is the concatenation of
 *   (1) the chunks idx[b,h,0..k_chunks) of the cache (K,V,kd): chunk j contributes the rows
 *       idx[b,h,j]*chunk .. idx[b,h,j]*chunk+chunk-1; negative entries (and chunks reaching
 *       beyond kv_len_all) are skipped; and
 *   (2) the recent rows [rb[b], len[b]) of the same cache, rb[b] = recent_begin ?
 *       recent_begin[b] : recent_begin_all (recent_begin_all is always a lower bound of
 *       rb[b]); these are the tokens appended since idx was built, the G queries' own
 *       tokens last.
 * Causal masking is bottom-right aligned on that virtual sequence: its last G tokens are the
 * queries, so causal != 0 requires at least G recent rows (len[b] - rb[b] >= G). With idx from tf_chunk_topk_gather this equals tf_decode_attn_retrieval over the
 * gathered cache followed by the same recent rows, without the copy. idx is int32
 * [batch, heads, k_chunks]; the caller keeps selected chunks and the recent range disjoint.
 * Other arguments as in tf_decode_attn_full. k_chunks >= 0; chunk in [1, 64];
 * workspace: pass an upper bound of kv_len_all - recent_begin_all as recent_len_all.
 * ------------------------------------------------------------------------------------- */
size_t tf_decode_attn_indexed_workspace_bytes(int32_t batch, int32_t heads, int32_t k_chunks,
                                              int32_t chunk, int64_t recent_len_all, int32_t G);
int tf_decode_attn_indexed(const void *Q, const void *K, const void *V, const tf_kv_desc *kd,
                           const int32_t *idx, int32_t k_chunks, int32_t chunk,
                           const int32_t *kv_len, int64_t kv_len_all, const int32_t *recent_begin,
                           int64_t recent_begin_all, int32_t G, float scale, int32_t causal, float *O,
                           float *LSE, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * tf_kv_append -- cache update of Algorithm 1 (its last step, the update of C_r and C_q with the
 * accepted tokens; Sec. 4.3: new tokens overwrite the least important entries of the retrieval cache).
 *   K[b,h,p[b]+i,:] = Knew[b,h,i,:] (same for V) for i < n, p[b] = pos ? pos[b] : pos_all.
 *   Knew, Vnew in  bf16 [batch, heads, n, 128] contiguous
 *   K, V       out bf16, described by kd; bit-exact row copies; other rows untouched
 *   pos        in  int32 [batch] device array, or NULL
 * Destination rows outside [0, capacity) are dropped (only possible with a device `pos`).
 * n == 0 is a valid no-op (Knew and Vnew may then be NULL).
 * Appending to the full cache uses p = current length; committing accepted tokens to a
 * retrieval cache of budget R that already holds m committed tokens uses p = R - m - n (the
 * tail of the descending-importance order).
 * ------------------------------------------------------------------------------------- */
int tf_kv_append(const void *Knew, const void *Vnew, int32_t n, void *K, void *V,
                 const tf_kv_desc *kd, const int32_t *pos, int64_t pos_all, void *stream);

/* ---------------------------------------------------------------------------------------
 * tf_spec_accept -- Algorithm 1, the Verify, Correct and next-token sampling steps, i.e. the
 * standard lossless speculative-sampling rule (Sec. 4.2 "Correctness"). One sequence per b,
 * gamma = G-1 drafted tokens. With p_i = softmax(target_logits[b,i]/T),
 * q_i = softmax(draft_logits[b,i]/T) (computed in fp64):
 *   walk i = 0..gamma-1, x = draft_tokens[b,i]: accept iff u_accept[b,i]*q_i[x] < p_i[x];
 *   at the first reject draw from norm(max(p_i-q_i,0)) (from p_i if that is all zero);
 *   if none is rejected draw from p_gamma. Draws are inverse-CDF in index order at
 *   u_sample[b]: the smallest v whose cumulative mass exceeds u_sample*total.
 *   T == 0: p, q are one-hot at the first arg-max: accept iff x == argmax target row;
 *   correction / bonus = that arg-max.
 *   target_logits in fp32 [B, G, V];  draft_logits in fp32 [B, G-1, V]
 *   draft_tokens  in int32 [B, G-1] in [0,V) (out-of-range tokens are rejected)
 *   u_accept      in fp32 [B, G-1] in [0,1);  u_sample in fp32 [B] in [0,1)
 *   n_accepted    out int32 [B];  out_tokens out int32 [B, G]: the accepted tokens, then the
 *                 drawn token, then -1.
 *   1 <= G <= TF_MAX_SPEC (G == 1: no drafted token, pointers to empty arrays may be NULL),
 *   V >= 1, temperature >= 0.
 *   Logits of -inf (masked vocabulary entries) have probability 0; every row needs one finite
 *   logit; +inf and NaN are not supported.
 * ------------------------------------------------------------------------------------- */
size_t tf_spec_accept_workspace_bytes(int32_t B, int32_t G, int32_t V);
int tf_spec_accept(const float *target_logits, const float *draft_logits,
                   const int32_t *draft_tokens, int32_t B, int32_t G, int32_t V,
                   float temperature, const float *u_accept, const float *u_sample,
                   int32_t *n_accepted, int32_t *out_tokens, void *ws, size_t ws_bytes,
                   void *stream);

/* ---------------------------------------------------------------------------------------
 * tf_spec_accept_ragged -- tf_spec_accept for a batch whose sequences drafted different numbers
 * of tokens (in Algorithm 1 the first level hands the verification between gamma2 and
 * gamma1+gamma2 tokens, so the sequences of a batch differ).
 *   n_draft  in  int32 [B] device array: sequence b drafted min(max(n_draft[b],0), G-1) tokens;
 *                only its first n_draft[b] tokens / draft rows / uniforms and its first
 *                n_draft[b]+1 target rows are used (arrays keep the strides of the G-wide call).
 *   If all are accepted the bonus token is drawn from target row n_draft[b].
 * Everything else as tf_spec_accept (same workspace size).
 * ------------------------------------------------------------------------------------- */
int tf_spec_accept_ragged(const float *target_logits, const float *draft_logits,
                          const int32_t *draft_tokens, const int32_t *n_draft, int32_t B, int32_t G,
                          int32_t V, float temperature, const float *u_accept,
                          const float *u_sample, int32_t *n_accepted, int32_t *out_tokens, void *ws,
                          size_t ws_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TRIFORCE_H */
