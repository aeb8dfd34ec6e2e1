"""GPU parity of the attention calls and the cache append at head_dim 64: the shape of the small
draft model's cache (Sec. 5.1: a 68M Llama with a StreamingLLM cache -- attention sinks plus a
recent window, Sec. 2.2 -- 12 heads of 64 dims). Same bars as head_dim 128."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_11912_amd as tf
from paper_2404_11912_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda"
ATTN_TOL, LSE_TOL = 2e-3, 1e-3
D = 64


def say(msg):
    print(msg, flush=True)


def make(B, H, N, G, seed):
    return synth.make_layer(B=B, H=H, N=N, G=G, c=8, P=2, seed=seed, device="cpu", d=D)


def compare(O, L, Oo, Lo, tag):
    e = float(np.max(np.abs(O.cpu().numpy() - Oo)))
    el = float(np.max(np.abs(L.cpu().numpy() - Lo)))
    say(f"[d64 {tag}] max|dO|={e:.2e} max|dLSE|={el:.2e}")
    assert e <= ATTN_TOL and el <= LSE_TOL


@pytest.mark.parametrize("fn_name", ["tf_decode_attn_full", "tf_decode_attn_retrieval"])
@pytest.mark.parametrize("N,G,causal", [(1024, 1, True), (1027, 4, True), (5000, 8, False), (37, 3, True)])
def test_attention_head_dim_64(fn_name, N, G, causal):
    say(f"case d64 {fn_name} N={N} G={G} causal={causal}")
    x = make(2, 12, N, G, 6400 + N + G)
    Q, K, V = x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    kv = [N, max(N // 3, G)]
    getattr(tf, fn_name)(Q, K, V, O, L, kv_len=torch.tensor(kv, dtype=torch.int32, device=DEV), kv_len_all=N,
                         scale=D ** -0.5 * 8.0, causal=causal)
    torch.cuda.synchronize()
    Oo, Lo, _ = oracle.attention(synth.as_u16(x["Q"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]), kv_len=kv,
                                 scale=D ** -0.5 * 8.0, causal=causal)
    compare(O, L, Oo, Lo, f"{fn_name} N={N} G={G}")


def test_streaming_cache_of_the_draft_model():
    """Sinks + recent window through the indexed call: 4 sink tokens (chunk 0 of size 4), a window
    of 252 recent tokens, one new query -- the draft model's StreamingLLM cache at a 256 budget."""
    say("case d64 streaming cache")
    B, H, N, G, c = 2, 12, 3000, 1, 4
    x = make(B, H, N, G, 6411)
    Q, K, V = x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    idx = torch.zeros((B, H, 1), dtype=torch.int32, device=DEV)            # chunk 0 = the sinks
    lens = np.array([3000, 1777], dtype=np.int32)
    kv = torch.tensor(lens, device=DEV)
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_indexed(Q, K, V, idx, c, O, L, kv_len=kv, kv_len_all=N, recent_begin=kv - 252,
                              recent_begin_all=int(lens.min()) - 252, causal=True)
    torch.cuda.synchronize()
    Oo, Lo = oracle.attention_indexed(synth.as_u16(x["Q"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]),
                                      idx.cpu().numpy(), c, kv_len=lens, recent_begin=lens - 252, causal=True)[:2]
    compare(O, L, Oo, Lo, "sinks+window")
    # the same rows, gathered by hand, through the plain call
    rows = [np.concatenate([np.arange(4), np.arange(n - 252, n)]) for n in lens]
    for b in range(B):
        Kb = K[b:b + 1, :, torch.as_tensor(rows[b], device=DEV)].contiguous()
        Vb = V[b:b + 1, :, torch.as_tensor(rows[b], device=DEV)].contiguous()
        O2 = torch.empty((1, H, G, D), dtype=torch.float32, device=DEV)
        tf.tf_decode_attn_retrieval(Q[b:b + 1].contiguous(), Kb, Vb, O2, causal=True)
        torch.cuda.synchronize()
        assert float((O2 - O[b:b + 1]).abs().max()) < 1e-5


def test_tree_mask_head_dim_64():
    say("case d64 tree")
    x = make(1, 12, 2050, 7, 6412)
    masks = [0b0000001, 0b0000011, 0b0000101, 0b0001011, 0b0010011, 0b0100101, 0b1000101]
    Q, K, V = x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_tree(Q, K, V, masks, O, L)
    torch.cuda.synchronize()
    Oo, Lo = oracle.attention_tree(synth.as_u16(x["Q"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]), masks)
    compare(O, L, Oo, Lo, "tree")


@pytest.mark.parametrize("n", [1, 5, 33])
def test_kv_append_head_dim_64(n):
    say(f"case d64 kv_append n={n}")
    B, H, N = 3, 12, 200
    g = torch.Generator().manual_seed(6420 + n)
    K = torch.randn((B, H, N, D), generator=g).to(torch.bfloat16)
    V = torch.randn((B, H, N, D), generator=g).to(torch.bfloat16)
    Kn = torch.randn((B, H, n, D), generator=g).to(torch.bfloat16)
    Vn = torch.randn((B, H, n, D), generator=g).to(torch.bfloat16)
    pos = np.array([0, 57, N - n], dtype=np.int32)
    Kd, Vd = K.to(DEV), V.to(DEV)
    tf.tf_kv_append(Kn.to(DEV), Vn.to(DEV), Kd, Vd, pos=torch.tensor(pos, device=DEV))
    torch.cuda.synchronize()
    Ko, Vo = oracle.kv_append(synth.as_u16(Kn), synth.as_u16(Vn), synth.as_u16(K), synth.as_u16(V), pos)
    assert np.array_equal(synth.as_u16(Kd.cpu()), Ko) and np.array_equal(synth.as_u16(Vd.cpu()), Vo)


def test_retrieval_calls_refuse_head_dim_64():
    K = torch.zeros((1, 2, 64, D), dtype=torch.bfloat16, device=DEV)
    Kmean = torch.zeros((1, 2, 8, D), dtype=torch.float32, device=DEV)
    with pytest.raises(tf.TfError):
        tf.tf_chunk_summarize(K, 8, Kmean, 0, 8)
