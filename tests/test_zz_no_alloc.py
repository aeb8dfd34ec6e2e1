"""The entry point that allocates nothing (tf_decode_attn_retrieval_noalloc): same results, bit for
bit, as tf_decode_attn_retrieval with a caller workspace, on two calls in a row that share the
library's built-in scratch buffer, the second with a smaller input (so stale partials of the first
call lie behind the second call's); sizes beyond the buffer are refused; and neither call changes
the amount of device memory in use."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_11912_amd as tf
from paper_2404_11912_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _inputs(B, H, N, G, seed):
    x = synth.make_layer(B=B, H=H, N=N, G=G, c=8, P=2, seed=seed, device="cpu")
    return x, x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)


def _run_both(Q, K, V, kv_len=None, causal=True):
    B, H, G, d = Q.shape
    N = K.shape[2]
    ws = tf.workspace(tf.tf_decode_attn_retrieval_workspace_bytes(B, H, N, G), DEV)
    want_O = torch.empty((B, H, G, d), dtype=torch.float32, device=DEV)
    want_L = torch.empty((B, H, G), dtype=torch.float32, device=DEV)
    O = torch.full_like(want_O, float("nan"))
    L = torch.full_like(want_L, float("nan"))
    kv = None if kv_len is None else torch.tensor(kv_len, dtype=torch.int32, device=DEV)
    tf.tf_decode_attn_retrieval(Q, K, V, want_O, want_L, kv_len=kv, causal=causal, ws=ws)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    tf.tf_decode_attn_retrieval_noalloc(Q, K, V, O, L, kv_len=kv, causal=causal)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before          # nothing was allocated on the device
    return O, L, want_O, want_L


def test_noalloc_entry_point_two_calls_in_a_row():
    print("case noalloc first call: B=2 H=8 N=4099 G=3 seed=19001", flush=True)
    tf.tf_noalloc_init()
    assert tf.tf_noalloc_scratch_bytes() == 16 << 20
    x1, Q1, K1, V1 = _inputs(2, 8, 4099, 3, 19001)
    O, L, want_O, want_L = _run_both(Q1, K1, V1, kv_len=[4099, 3000])
    assert torch.equal(O, want_O) and torch.equal(L, want_L)
    # the first call against the oracle as well (the existing entry point's own bar)
    Oo, Lo, _ = oracle.attention(synth.as_u16(x1["Q"]), synth.as_u16(x1["K"]), synth.as_u16(x1["V"]),
                                 kv_len=[4099, 3000], scale=1.0, causal=True)
    assert np.max(np.abs(O.cpu().numpy() - Oo)) <= 2e-3 and np.max(np.abs(L.cpu().numpy() - Lo)) <= 1e-3

    print("case noalloc second call, smaller: B=1 H=3 N=333 G=5 seed=19002", flush=True)
    x2, Q2, K2, V2 = _inputs(1, 3, 333, 5, 19002)
    O, L, want_O, want_L = _run_both(Q2, K2, V2, causal=False)
    assert torch.equal(O, want_O) and torch.equal(L, want_L)
    Oo, Lo, _ = oracle.attention(synth.as_u16(x2["Q"]), synth.as_u16(x2["K"]), synth.as_u16(x2["V"]), scale=1.0,
                                 causal=False)
    assert np.max(np.abs(O.cpu().numpy() - Oo)) <= 2e-3 and np.max(np.abs(L.cpu().numpy() - Lo)) <= 1e-3

    print("case noalloc third call, the first input again", flush=True)
    O, L, want_O, want_L = _run_both(Q1, K1, V1, kv_len=[4099, 3000])
    assert torch.equal(O, want_O) and torch.equal(L, want_L)


def test_noalloc_entry_point_refuses_sizes_beyond_its_buffer():
    """A problem whose partials exceed the built-in buffer is refused on the host (nothing is enqueued,
    no device memory is touched): 1024 heads x 16K tokens need more than 16 MiB of partials."""
    print("case noalloc size limit", flush=True)
    B, H, N, G = 1, 1024, 16384, 3
    nsplit = tf.tf_decode_attn_plan(1, B, H, N)[0]
    assert B * H * nsplit * 4 * 8 * 130 * 4 > tf.tf_noalloc_scratch_bytes()
    K = torch.empty((B, H, N, 128), dtype=torch.bfloat16, device=DEV)      # 4 GiB, never read
    Q = torch.zeros((B, H, G, 128), dtype=torch.bfloat16, device=DEV)
    O = torch.zeros((B, H, G, 128), dtype=torch.float32, device=DEV)
    with pytest.raises(tf.TfError) as e:
        tf.tf_decode_attn_retrieval_noalloc(Q, K, K, O)
    assert e.value.code == -5


def test_noalloc_entry_point_under_hip_graph_capture():
    """What the entry point is for: captured into a HIP graph (nothing in it allocates or needs a
    workspace argument), replayed several times with eager work in between; every replay must equal
    the eager result of the workspace entry point."""
    print("case noalloc graph capture: B=1 H=8 N=2051 G=3 seed=19003", flush=True)
    tf.tf_noalloc_init()                                   # address lookup before the capture begins
    x, Q, K, V = _inputs(1, 8, 2051, 3, 19003)
    want_O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    want_L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_retrieval(Q, K, V, want_O, want_L, causal=True)
    O = torch.zeros_like(want_O)
    L = torch.zeros_like(want_L)
    tf.tf_decode_attn_retrieval_noalloc(Q, K, V, O, L, causal=True)     # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        tf.tf_decode_attn_retrieval_noalloc(Q, K, V, O, L, causal=True)
    torch.cuda.synchronize()
    for rep in range(3):
        O.zero_()
        L.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(O, want_O) and torch.equal(L, want_L), f"replay {rep}"
