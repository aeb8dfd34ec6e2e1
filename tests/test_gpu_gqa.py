"""GPU parity of the attention calls with grouped-query heads (q_group query heads per KV head,
G * q_group <= 16 query rows share one pass over the KV head's cache). Not a shape of the paper's
models (Llama2 is multi-head); it is the variant newer long-context models need. Same bars."""
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


def make(B, Hkv, qg, N, G, seed, d=128):
    x = synth.make_layer(B=B, H=Hkv, N=N, G=G, c=8, P=2, seed=seed, device="cpu", d=d)
    g = torch.Generator().manual_seed(seed + 1)
    x["Qg"] = (torch.randn((B, Hkv * qg, G, d), generator=g) / d ** 0.5).to(torch.bfloat16)
    return x


def compare(O, L, Oo, Lo, tag):
    e = float(np.max(np.abs(O.cpu().numpy() - Oo)))
    el = float(np.max(np.abs(L.cpu().numpy() - Lo)))
    say(f"[gqa {tag}] max|dO|={e:.2e} max|dLSE|={el:.2e}")
    assert e <= ATTN_TOL and el <= LSE_TOL


@pytest.mark.parametrize("qg,G", [(4, 4), (2, 8), (8, 2), (16, 1), (4, 3), (2, 5), (3, 5), (1, 6)])
@pytest.mark.parametrize("causal", [True, False])
def test_gqa_full_attention(qg, G, causal):
    say(f"case gqa full q_group={qg} G={G} causal={causal}")
    B, Hkv, N = 2, 2, 3001
    x = make(B, Hkv, qg, N, G, 7100 + 16 * qg + G)
    Q, K, V = x["Qg"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    kv = [N, 700]
    tf.tf_decode_attn_full(Q, K, V, O, L, kv_len=torch.tensor(kv, dtype=torch.int32, device=DEV), kv_len_all=N,
                           scale=1.0, causal=causal)
    torch.cuda.synchronize()
    Oo, Lo = oracle.attention_gqa(synth.as_u16(x["Qg"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]), kv_len=kv,
                                  scale=1.0, causal=causal)
    compare(O, L, Oo, Lo, f"q_group={qg} G={G}")


def test_gqa_retrieval_head_dim_64_and_tree():
    say("case gqa d64 + tree")
    B, Hkv, qg, N, G = 1, 3, 4, 1500, 4
    x = make(B, Hkv, qg, N, G, 7201, d=64)
    Q, K, V = x["Qg"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_retrieval(Q, K, V, O, L, causal=True)
    torch.cuda.synchronize()
    Oo, Lo = oracle.attention_gqa(synth.as_u16(x["Qg"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]), causal=True)
    compare(O, L, Oo, Lo, "retrieval d64")
    # tree mask with grouped heads: every query head of a group uses the same mask rows
    masks = [0b0001, 0b0011, 0b0101, 0b1101]
    tf.tf_decode_attn_tree(Q, K, V, masks, O, L)
    torch.cuda.synchronize()
    Kr = np.ascontiguousarray(np.repeat(synth.as_u16(x["K"]), qg, axis=1))
    Vr = np.ascontiguousarray(np.repeat(synth.as_u16(x["V"]), qg, axis=1))
    Oo, Lo = oracle.attention_tree(synth.as_u16(x["Qg"]), Kr, Vr, masks)
    compare(O, L, Oo, Lo, "tree d64")


def test_gqa_indexed():
    say("case gqa indexed")
    B, Hkv, qg, N, G, c, k = 2, 2, 4, 4096, 3, 8, 32
    x = make(B, Hkv, qg, N, G, 7301)
    Q, K, V = x["Qg"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    g = torch.Generator().manual_seed(7302)
    idx = torch.stack([torch.stack([torch.randperm(N // c - 8, generator=g)[:k] for _ in range(Hkv)])
                       for _ in range(B)]).to(torch.int32)
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_indexed(Q, K, V, idx.to(DEV), c, O, L, kv_len_all=N, recent_begin_all=N - G, causal=True)
    torch.cuda.synchronize()
    # oracle: per query head, the indexed definition with its KV head's indices
    Ku, Vu, Qu = synth.as_u16(x["K"]), synth.as_u16(x["V"]), synth.as_u16(x["Qg"])
    Kr, Vr = np.repeat(Ku, qg, axis=1), np.repeat(Vu, qg, axis=1)
    idx_r = np.repeat(idx.numpy(), qg, axis=1)
    Oo, Lo = oracle.attention_indexed(Qu, np.ascontiguousarray(Kr), np.ascontiguousarray(Vr), idx_r, c,
                                      recent_begin=N - G, causal=True)[:2]
    compare(O, L, Oo, Lo, "indexed")


def test_gqa_limits():
    K = torch.zeros((1, 2, 64, 128), dtype=torch.bfloat16, device=DEV)
    Q = torch.zeros((1, 2 * 4, 5, 128), dtype=torch.bfloat16, device=DEV)      # 4 x 5 = 20 rows > 16
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    with pytest.raises(tf.TfError):
        tf.tf_decode_attn_full(Q, K, K, O)


def test_gqa_group_of_four_costs_one_pass():
    """One layer of a 128K cache with 8 KV heads x 4 query heads, G = 4: 16 query rows per KV head
    ride on one pass over its K/V. Sampled heads against the oracle, and the time is reported."""
    say("case gqa 128K 8 kv heads x 4")
    B, Hkv, qg, N, G = 1, 8, 4, 131072, 4
    g = torch.Generator(device=DEV).manual_seed(7401)
    K = torch.randn((B, Hkv, N, 128), generator=g, device=DEV).to(torch.bfloat16)
    V = torch.randn((B, Hkv, N, 128), generator=g, device=DEV).to(torch.bfloat16)
    Q = (torch.randn((B, Hkv * qg, G, 128), generator=g, device=DEV) / 128 ** 0.5).to(torch.bfloat16)
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    ws = tf.workspace(tf.tf_decode_attn_full_workspace_bytes(B, Hkv, N, G * qg), DEV)
    for _ in range(3):
        tf.tf_decode_attn_full(Q, K, V, O, L, causal=True, ws=ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        tf.tf_decode_attn_full(Q, K, V, O, L, causal=True, ws=ws)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 100
    say(f"[gqa 128K] {us:.1f} us per call, {2 * Hkv * N * 256 / us / 1e6:.2f} TB/s of K/V")
    for h in (0, 5):
        Oo, Lo = oracle.attention_gqa(synth.as_u16(Q[:, h * qg:(h + 1) * qg]), synth.as_u16(K[:, h:h + 1]),
                                      synth.as_u16(V[:, h:h + 1]), causal=True)
        compare(O[:, h * qg:(h + 1) * qg], L[:, h * qg:(h + 1) * qg], Oo, Lo, f"128K kv head {h}")
