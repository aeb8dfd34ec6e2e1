"""The calls allocate nothing, never synchronise and read no device memory on the host, so a
decode step can be captured into a HIP graph. Replays are checked against the eager result
several times, with eager work and synchronisations in between."""
import pytest
import torch

import paper_2404_11912_amd as tf
from paper_2404_11912_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_step_captured_in_a_hip_graph_replays_bit_exactly():
    print("case graph_capture seed=140", flush=True)
    B, H, N, G, c, k = 2, 4, 3000, 5, 8, 64
    x = synth.make_layer(B, H, N, G, c, 6, seed=140)
    K, V, Q, q_r = (x[n].to(DEV) for n in ("K", "V", "Q", "q_r"))
    M = N // c
    Kmean = torch.empty((B, H, M, 128), dtype=torch.float32, device=DEV)
    idx = torch.empty((B, H, k), dtype=torch.int32, device=DEV)
    Kr = torch.zeros((B, H, k * c, 128), dtype=torch.bfloat16, device=DEV)
    Vr = torch.zeros_like(Kr)
    O = torch.empty((B, H, G, 128), dtype=torch.float32, device=DEV)
    L = torch.empty((B, H, G), dtype=torch.float32, device=DEV)
    O_d = torch.empty_like(O)
    a = synth.make_accept_inputs(B, G - 1, 1000, 0.6, 141, correlated=True, device=DEV)
    n_acc = torch.empty((B,), dtype=torch.int32, device=DEV)
    out = torch.empty((B, G), dtype=torch.int32, device=DEV)
    ws = tf.workspace(max(tf.tf_decode_attn_full_workspace_bytes(B, H, N, G),
                          tf.tf_decode_attn_retrieval_workspace_bytes(B, H, k * c, G),
                          tf.tf_chunk_topk_gather_workspace_bytes(B, H, M, k),
                          tf.tf_spec_accept_workspace_bytes(B, G, 1000)), DEV)

    def step():
        tf.tf_chunk_summarize(K, c, Kmean, 0, M)
        tf.tf_chunk_topk_gather(q_r, Kmean, K, V, c, k, idx, Kr, Vr, ws=ws)
        tf.tf_decode_attn_retrieval(Q, Kr, Vr, O_d, causal=False, ws=ws)
        tf.tf_decode_attn_full(Q, K, V, O, L, ws=ws)
        tf.tf_spec_accept(a["target_logits"], a["draft_logits"], a["draft_tokens"], 0.6, a["u_accept"],
                          a["u_sample"], n_acc, out, ws=ws)

    outs = (Kmean, idx, Kr, Vr, O_d, O, L, n_acc, out)
    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in outs]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in outs:
            t.zero_()                      # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for t, wnt in zip(outs, want):
            assert torch.equal(t, wnt), f"replay {rep} differs from the eager result"
