// extern "C" entry points declared in include/triforce.h. Argument checks and kernel launches
// live next to each kernel; this file only forwards.
#include <string.h>

#include "tf_common.hpp"

namespace tf {
int summarize_launch(const void *, const tf_kv_desc *, int32_t, int64_t, int64_t, void *, int64_t, void *, bool);
size_t topk_workspace_bytes(int32_t, int32_t, int64_t, int32_t);
int topk_gather_launch(const void *, const void *, int64_t, const void *, const void *, const tf_kv_desc *, int32_t,
                       const int32_t *, int64_t, int32_t, int32_t *, float *, void *, void *, const tf_kv_desc *,
                       void *, size_t, void *, bool);
size_t attn_workspace_bytes(int32_t, int32_t, int64_t, int32_t, bool);
size_t attn_indexed_workspace_bytes(int32_t, int32_t, int32_t, int32_t, int64_t, int32_t);
int attn_launch(const void *, const void *, const void *, const tf_kv_desc *, const int32_t *, int64_t, int32_t,
                float, int32_t, float *, float *, void *, size_t, void *, bool, const IndexedArgs *, const uint16_t *);
int kv_append_launch(const void *, const void *, int32_t, void *, void *, const tf_kv_desc *, const int32_t *,
                     int64_t, void *);
int stream_read_probe_launch(const void *, size_t, void *, size_t, size_t *, void *);
int attn_noalloc_init();
size_t attn_noalloc_max_bytes();
int attn_retrieval_noalloc_launch(const void *, const void *, const void *, const tf_kv_desc *, const int32_t *, int64_t,
                                  int32_t, float, int32_t, float *, float *, void *);
int attn_plan(int32_t, int32_t, int32_t, int64_t, int32_t *, int32_t *);
int set_attn_option(bool retrieval, int64_t v, bool this_thread);
int set_score_option(int64_t v, bool this_thread);
int set_fused_option(int64_t v, bool this_thread);
size_t accept_workspace_bytes(int32_t, int32_t, int32_t);
int accept_launch(const float *, const float *, const int32_t *, int32_t, int32_t, int32_t, float, const float *,
                  const float *, int32_t *, int32_t *, void *, size_t, void *, const int32_t *);
}  // namespace tf

extern "C" {

int tf_version(void) { return 300; /* 0.3.0 */ }

const char *tf_status_string(int code) {
    switch (code) {
        case TF_OK: return "ok";
        case TF_ERR_INVALID_ARG: return "invalid argument";
        case TF_ERR_UNSUPPORTED: return "unsupported shape or size";
        case TF_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case TF_ERR_HIP: return "HIP runtime error";
        case TF_ERR_SCRATCH_LIMIT: return "problem needs more than the library's built-in scratch buffer";
        default: return "unknown status";
    }
}

static int set_option(const char *name, int64_t value, bool this_thread) {
    if (!name) return TF_ERR_INVALID_ARG;
    if (!strcmp(name, "attn_full_tokens_per_split")) return tf::set_attn_option(false, value, this_thread);
    if (!strcmp(name, "attn_retr_tokens_per_split")) return tf::set_attn_option(true, value, this_thread);
    if (!strcmp(name, "score_steps_per_wave")) return tf::set_score_option(value, this_thread);
    if (!strcmp(name, "rebuild_fused")) return tf::set_fused_option(value, this_thread);
    return TF_ERR_INVALID_ARG;
}

int tf_set_option(const char *name, int64_t value) { return set_option(name, value, false); }

int tf_set_thread_option(const char *name, int64_t value) { return set_option(name, value, true); }

int tf_chunk_summarize(const void *K, const tf_kv_desc *kd, int32_t chunk, int64_t first_chunk, int64_t n_chunks,
                       float *Kmean, int64_t M_cap, void *stream) {
    return tf::summarize_launch(K, kd, chunk, first_chunk, n_chunks, Kmean, M_cap, stream, false);
}

int tf_chunk_summarize_bf16(const void *K, const tf_kv_desc *kd, int32_t chunk, int64_t first_chunk,
                            int64_t n_chunks, void *Kmean, int64_t M_cap, void *stream) {
    return tf::summarize_launch(K, kd, chunk, first_chunk, n_chunks, Kmean, M_cap, stream, true);
}

size_t tf_chunk_topk_gather_workspace_bytes(int32_t batch, int32_t heads, int64_t n_chunks_all, int32_t k_chunks) {
    return tf::topk_workspace_bytes(batch, heads, n_chunks_all, k_chunks);
}

int tf_chunk_topk_gather(const void *q_r, const float *Kmean, int64_t M_cap, const void *K, const void *V,
                         const tf_kv_desc *kd, int32_t chunk, const int32_t *n_chunks, int64_t n_chunks_all,
                         int32_t k_chunks, int32_t *out_idx, float *out_score, void *Kr, void *Vr,
                         const tf_kv_desc *rd, void *ws, size_t ws_bytes, void *stream) {
    return tf::topk_gather_launch(q_r, Kmean, M_cap, K, V, kd, chunk, n_chunks, n_chunks_all, k_chunks, out_idx,
                                  out_score, Kr, Vr, rd, ws, ws_bytes, stream, false);
}

int tf_chunk_topk_gather_bf16(const void *q_r, const void *Kmean, int64_t M_cap, const void *K, const void *V,
                              const tf_kv_desc *kd, int32_t chunk, const int32_t *n_chunks, int64_t n_chunks_all,
                              int32_t k_chunks, int32_t *out_idx, float *out_score, void *Kr, void *Vr,
                              const tf_kv_desc *rd, void *ws, size_t ws_bytes, void *stream) {
    return tf::topk_gather_launch(q_r, Kmean, M_cap, K, V, kd, chunk, n_chunks, n_chunks_all, k_chunks, out_idx,
                                  out_score, Kr, Vr, rd, ws, ws_bytes, stream, true);
}

int tf_decode_attn_plan(int32_t kind, int32_t batch, int32_t heads, int64_t len_all, int32_t *nsplit,
                        int32_t *tokens_per_split) {
    return tf::attn_plan(kind, batch, heads, len_all, nsplit, tokens_per_split);
}

size_t tf_decode_attn_full_workspace_bytes(int32_t batch, int32_t heads, int64_t kv_len_all, int32_t G) {
    return tf::attn_workspace_bytes(batch, heads, kv_len_all, G, false);
}

int tf_decode_attn_full(const void *Q, const void *K, const void *V, const tf_kv_desc *kd, const int32_t *kv_len,
                        int64_t kv_len_all, int32_t G, float scale, int32_t causal, float *O, float *LSE, void *ws,
                        size_t ws_bytes, void *stream) {
    return tf::attn_launch(Q, K, V, kd, kv_len, kv_len_all, G, scale, causal, O, LSE, ws, ws_bytes, stream, false, nullptr, nullptr);
}

int tf_decode_attn_tree(const void *Q, const void *K, const void *V, const tf_kv_desc *kd, const int32_t *kv_len,
                        int64_t kv_len_all, int32_t G, float scale, const uint16_t *tail_mask, float *O, float *LSE,
                        void *ws, size_t ws_bytes, void *stream) {
    if (!tail_mask) return TF_ERR_INVALID_ARG;
    return tf::attn_launch(Q, K, V, kd, kv_len, kv_len_all, G, scale, 0, O, LSE, ws, ws_bytes, stream, false, nullptr,
                           tail_mask);
}

size_t tf_decode_attn_retrieval_workspace_bytes(int32_t batch, int32_t heads, int64_t kv_len_all, int32_t G) {
    return tf::attn_workspace_bytes(batch, heads, kv_len_all, G, true);
}

int tf_decode_attn_retrieval(const void *Q, const void *K, const void *V, const tf_kv_desc *kd,
                             const int32_t *kv_len, int64_t kv_len_all, int32_t G, float scale, int32_t causal,
                             float *O, float *LSE, void *ws, size_t ws_bytes, void *stream) {
    return tf::attn_launch(Q, K, V, kd, kv_len, kv_len_all, G, scale, causal, O, LSE, ws, ws_bytes, stream, true, nullptr, nullptr);
}

int tf_stream_read_probe(const void *buf, size_t bytes, void *sink, size_t sink_bytes, size_t *bytes_read,
                         void *stream) {
    return tf::stream_read_probe_launch(buf, bytes, sink, sink_bytes, bytes_read, stream);
}

int tf_noalloc_init(void) { return tf::attn_noalloc_init(); }

size_t tf_noalloc_scratch_bytes(void) { return tf::attn_noalloc_max_bytes(); }

int tf_decode_attn_retrieval_noalloc(const void *Q, const void *K, const void *V, const tf_kv_desc *kd,
                                     const int32_t *kv_len, int64_t kv_len_all, int32_t G, float scale,
                                     int32_t causal, float *O, float *LSE, void *stream) {
    return tf::attn_retrieval_noalloc_launch(Q, K, V, kd, kv_len, kv_len_all, G, scale, causal, O, LSE, stream);
}

size_t tf_decode_attn_indexed_workspace_bytes(int32_t batch, int32_t heads, int32_t k_chunks, int32_t chunk,
                                              int64_t recent_len_all, int32_t G) {
    return tf::attn_indexed_workspace_bytes(batch, heads, k_chunks, chunk, recent_len_all, G);
}

int tf_decode_attn_indexed(const void *Q, const void *K, const void *V, const tf_kv_desc *kd, const int32_t *idx,
                           int32_t k_chunks, int32_t chunk, const int32_t *kv_len, int64_t kv_len_all,
                           const int32_t *recent_begin, int64_t recent_begin_all, int32_t G, float scale,
                           int32_t causal, float *O, float *LSE, void *ws, size_t ws_bytes, void *stream) {
    const tf::IndexedArgs ix{idx, k_chunks, chunk, recent_begin, recent_begin_all};
    return tf::attn_launch(Q, K, V, kd, kv_len, kv_len_all, G, scale, causal, O, LSE, ws, ws_bytes, stream, true,
                           &ix, nullptr);
}

int tf_kv_append(const void *Knew, const void *Vnew, int32_t n, void *K, void *V, const tf_kv_desc *kd,
                 const int32_t *pos, int64_t pos_all, void *stream) {
    return tf::kv_append_launch(Knew, Vnew, n, K, V, kd, pos, pos_all, stream);
}

size_t tf_spec_accept_workspace_bytes(int32_t B, int32_t G, int32_t V) {
    return tf::accept_workspace_bytes(B, G, V);
}

int tf_spec_accept(const float *target_logits, const float *draft_logits, const int32_t *draft_tokens, int32_t B,
                   int32_t G, int32_t V, float temperature, const float *u_accept, const float *u_sample,
                   int32_t *n_accepted, int32_t *out_tokens, void *ws, size_t ws_bytes, void *stream) {
    return tf::accept_launch(target_logits, draft_logits, draft_tokens, B, G, V, temperature, u_accept, u_sample,
                             n_accepted, out_tokens, ws, ws_bytes, stream, nullptr);
}

int tf_spec_accept_ragged(const float *target_logits, const float *draft_logits, const int32_t *draft_tokens,
                          const int32_t *n_draft, int32_t B, int32_t G, int32_t V, float temperature,
                          const float *u_accept, const float *u_sample, int32_t *n_accepted, int32_t *out_tokens,
                          void *ws, size_t ws_bytes, void *stream) {
    if (!n_draft) return TF_ERR_INVALID_ARG;
    return tf::accept_launch(target_logits, draft_logits, draft_tokens, B, G, V, temperature, u_accept, u_sample,
                             n_accepted, out_tokens, ws, ws_bytes, stream, n_draft);
}

}  // extern "C"
