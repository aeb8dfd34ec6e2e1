"""MI355X-native decode-step attention path of hierarchical speculative decoding with a
retrieval cache (TriForce, arxiv 2404.11912): a C-ABI HIP library plus this thin binding.

    from paper_2404_11912_amd import tf_decode_attn_full, ...

`synth` holds the seeded synthetic input generators (no method arithmetic).
The shared library is loaded on first use; there is no CPU fallback.
"""
from . import synth  # noqa: F401
from .binding import (  # noqa: F401
    EXPORTS,
    LIB_PATH,
    TfError,
    kv_desc,
    load_library,
    tf_chunk_summarize,
    tf_chunk_topk_gather,
    tf_chunk_topk_gather_workspace_bytes,
    tf_decode_attn_full,
    tf_decode_attn_indexed,
    tf_decode_attn_indexed_workspace_bytes,
    tf_decode_attn_plan,
    tf_kv_append,
    tf_decode_attn_tree,
    tf_chunk_summarize_bf16,
    tf_chunk_topk_gather_bf16,
    tf_spec_accept_ragged,
    tf_decode_attn_full_workspace_bytes,
    tf_decode_attn_retrieval,
    tf_decode_attn_retrieval_workspace_bytes,
    tf_decode_attn_retrieval_noalloc,
    tf_noalloc_init,
    tf_noalloc_scratch_bytes,
    tf_set_option,
    tf_set_thread_option,
    tf_spec_accept,
    tf_stream_read_probe,
    tf_spec_accept_workspace_bytes,
    tf_version,
    workspace,
)
