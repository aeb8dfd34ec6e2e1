"""fp64 CPU oracle (test infrastructure, not the product).

Only tests, `__graft_entry__.smoke()` and `bench.py`'s cpu_baseline leg may import
this package. It never imports the HIP package and shares no code with it.
"""
from .tf_oracle import (  # noqa: F401
    accept,
    accept_ragged,
    attention,
    attention_gqa,
    attention_indexed,
    attention_tree,
    build_oracle,
    chunk_mean,
    chunk_mean_bf16,
    chunk_mean_bf16_once,
    chunk_mean_fp32,
    gather,
    kv_append,
    num_threads,
    retrieve,
    round_to_bf16,
)
