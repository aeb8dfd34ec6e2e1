"""GPU parity of tf_decode_attn_tree (verification attention for a speculated token tree,
Sec. 5.3.3) against the fp64 oracle, through the C ABI. Bar: max-abs-error 2e-3 on O, 1e-3 on LSE."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_11912_amd as tf
from paper_2404_11912_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda"
ATTN_TOL, LSE_TOL = 2e-3, 1e-3


def say(msg):
    print(msg, flush=True)


def ancestor_masks(parent):
    masks = []
    for g in range(len(parent)):
        m, a = 0, g
        while a >= 0:
            m |= 1 << a
            a = parent[a]
        masks.append(m)
    return masks


TREES = {
    "chain5": [-1, 0, 1, 2, 3],
    "star8": [-1, 0, 0, 0, 0, 0, 0, 0],
    "binary7": [-1, 0, 0, 1, 1, 2, 2],
    "two_chains6": [-1, 0, 1, -1, 3, 4],          # independent sequences sharing only the context
    "single": [-1],
    "binary16": [-1, 0, 0, 1, 1, 2, 2, 3, 3, 4, 4, 5, 5, 6, 6, 7],
}


def run(x, masks, kv_len=None, scale=1.0, tag=""):
    Q, K, V = x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    G = len(masks)
    Q = Q[:, :, :G].contiguous()
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    kv = None if kv_len is None else torch.tensor(kv_len, dtype=torch.int32, device=DEV)
    tf.tf_decode_attn_tree(Q, K, V, masks, O, L, kv_len=kv, scale=scale)
    torch.cuda.synchronize()
    Oo, Lo = oracle.attention_tree(synth.as_u16(Q), synth.as_u16(x["K"]), synth.as_u16(x["V"]), masks,
                                   kv_len=kv_len, scale=scale)
    O, L = O.cpu().numpy().astype(np.float64), L.cpu().numpy().astype(np.float64)
    both_inf = np.isinf(Lo) & np.isinf(L) & (L < 0)
    err = float(np.max(np.abs(O - Oo)))
    lerr = float(np.max(np.abs(np.where(both_inf, 0.0, L) - np.where(both_inf, 0.0, Lo))))
    say(f"[tree {tag}] max|dO|={err:.3e} max|dLSE|={lerr:.3e}")
    assert np.array_equal(np.isinf(Lo), np.isinf(L))
    assert err <= ATTN_TOL and lerr <= LSE_TOL
    return O, L


@pytest.mark.parametrize("name", list(TREES))
@pytest.mark.parametrize("N", [1000, 4099])
def test_tree_attention_vs_oracle(name, N):
    parent = TREES[name]
    say(f"case tree {name} N={N}")
    x = synth.make_layer(B=2, H=3, N=N, G=16, c=8, P=4, seed=5300 + N + len(parent), device="cpu")
    run(x, ancestor_masks(parent), tag=f"{name} N={N}")


def test_tree_with_per_sequence_lengths_and_arbitrary_masks():
    """Ragged batch, masks that are not ancestor-closed (any bit pattern is legal), a query that
    sees no speculated token, and a sequence whose context is empty."""
    say("case tree ragged/arbitrary masks")
    x = synth.make_layer(B=3, H=2, N=777, G=8, c=8, P=2, seed=5311, device="cpu")
    masks = [0b000001, 0b000000, 0b101010, 0b111111, 0b010001, 0b100000]
    run(x, masks, kv_len=[777, 130, 6], scale=0.5, tag="ragged arbitrary")


def test_chain_mask_equals_the_causal_call_bit_for_bit():
    say("case tree chain == causal")
    x = synth.make_layer(B=1, H=4, N=3000, G=6, c=8, P=4, seed=5312, device="cpu")
    Q, K, V = x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    O1 = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    O2 = torch.empty_like(O1)
    L1 = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    L2 = torch.empty_like(L1)
    tf.tf_decode_attn_full(Q, K, V, O1, L1, causal=True)
    tf.tf_decode_attn_tree(Q, K, V, [(2 << g) - 1 for g in range(6)], O2, L2)
    torch.cuda.synchronize()
    assert torch.equal(O1, O2) and torch.equal(L1, L2)


def test_tree_at_the_128k_layer_shape_on_sampled_heads():
    """The launch configuration bench.py times (one layer of the 128K workload, default split
    planning), a 7-node binary tree; the oracle computes 3 sampled heads."""
    w = synth.WORKLOADS["step128k"]
    say("case tree full-size step128k layer 5")
    x = synth.make_workload_layer(w, 5, DEV)
    masks = ancestor_masks(TREES["binary7"])
    G = len(masks)
    g = torch.Generator(device="cpu"); g.manual_seed(5313)
    Q = (torch.randn((w.B, w.H, G, w.d), generator=g) / w.d ** 0.5).to(torch.bfloat16).to(DEV)
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_tree(Q, x["K"], x["V"], masks, O, L)
    torch.cuda.synchronize()
    assert torch.isfinite(O).all()
    for h in (0, 13, 31):
        Oo, Lo = oracle.attention_tree(synth.as_u16(Q[:, h:h + 1]), synth.as_u16(x["K"][:, h:h + 1]),
                                       synth.as_u16(x["V"][:, h:h + 1]), masks)
        e = float(np.max(np.abs(O[:, h:h + 1].cpu().numpy() - Oo)))
        el = float(np.max(np.abs(L[:, h:h + 1].cpu().numpy() - Lo)))
        say(f"[tree 128K head {h}] max|dO|={e:.2e} max|dLSE|={el:.2e}")
        assert e <= ATTN_TOL and el <= LSE_TOL
