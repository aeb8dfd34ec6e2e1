"""GPU parity of the cache-update pieces (Sec. 4.3): gather-free draft attention through the
chunk indices (tf_decode_attn_indexed) and the row append / commit (tf_kv_append)."""
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


def _run_indexed(Q, K, V, idx, c, kv_len=None, recent_begin=None, kv_len_all=None, recent_begin_all=None,
                 causal=True, scale=1.0):
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    kv = None if kv_len is None else torch.tensor(kv_len, dtype=torch.int32, device=DEV)
    rb = None if recent_begin is None else torch.tensor(recent_begin, dtype=torch.int32, device=DEV)
    tf.tf_decode_attn_indexed(Q, K, V, idx, c, O, L, kv_len=kv, kv_len_all=kv_len_all, recent_begin=rb,
                              recent_begin_all=recent_begin_all, scale=scale, causal=causal)
    torch.cuda.synchronize()
    return O.cpu().numpy().astype(np.float64), L.cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("c,k,G", [(8, 40, 3), (4, 100, 5), (16, 9, 8), (12, 7, 1), (1, 33, 2)])
def test_indexed_attention_vs_oracle(c, k, G):
    say(f"case indexed_attention c={c} k={k} G={G} seed=150")
    B, H, N = 2, 3, 1500
    x = synth.make_layer(B, H, N, G, c, 0, seed=150 + c)
    rng = np.random.default_rng(150 + c)
    M_sel = (N - 200) // c                                  # chunks strictly before every recent range
    idx = np.stack([np.stack([rng.permutation(M_sel)[:k] for _ in range(H)]) for _ in range(B)]).astype(np.int32)
    idx[0, 1, k // 2] = -1                                  # skipped slots
    idx[1, 2, 0] = -1
    kv_len, recent_begin = [1500, 1431], [1390, 1400]
    Qd, Kd, Vd = x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    idx_d = torch.from_numpy(idx).to(DEV)
    O, L = _run_indexed(Qd, Kd, Vd, idx_d, c, kv_len=kv_len, recent_begin=recent_begin, kv_len_all=1500,
                        recent_begin_all=1390)
    Oo, Lo = oracle.attention_indexed(synth.as_u16(x["Q"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]), idx, c,
                                      kv_len=kv_len, recent_begin=recent_begin, kv_len_all=1500)
    e, el = float(np.max(np.abs(O - Oo))), float(np.max(np.abs(L - Lo)))
    say(f"[indexed c={c}] max|dO|={e:.2e} max|dLSE|={el:.2e}")
    assert e <= ATTN_TOL and el <= LSE_TOL


def test_indexed_attention_split_with_more_chunks_than_the_kernel_stages():
    """One split that walks 1500 single-token chunks: the kernel keeps the first 1024 chunk indices
    of a split on chip and reads the rest from memory."""
    say("case indexed_long_split seed=158")
    B, H, N, c, k, G = 1, 2, 4000, 1, 1500, 2
    x = synth.make_layer(B, H, N, G, c, 0, seed=158)
    rng = np.random.default_rng(158)
    idx = np.stack([np.stack([rng.permutation(N - 100)[:k] for _ in range(H)]) for _ in range(B)]).astype(np.int32)
    idx[0, 0, 1400] = -1
    tf.tf_set_option("attn_retr_tokens_per_split", 2048)
    try:
        O, L = _run_indexed(x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV), torch.from_numpy(idx).to(DEV), c,
                            kv_len_all=N, recent_begin_all=N - 10)
    finally:
        tf.tf_set_option("attn_retr_tokens_per_split", 0)
    Oo, Lo = oracle.attention_indexed(synth.as_u16(x["Q"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]), idx, c,
                                      kv_len=[N], recent_begin=[N - 10], kv_len_all=N)
    assert float(np.max(np.abs(O - Oo))) <= ATTN_TOL and float(np.max(np.abs(L - Lo))) <= LSE_TOL


def test_indexed_matches_retrieval_attention_over_the_gathered_cache():
    """The same draft attention two ways on the GPU: through the indices, and over the gathered
    retrieval cache with the recent rows appended behind it."""
    say("case indexed_vs_gathered seed=151")
    w = synth.WORKLOADS["tiny"]
    x = synth.make_workload_layer(w, 2)
    Qd, Kd, Vd = x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    B, H, N, d = Kd.shape
    n_recent = 24
    n_old = (N - n_recent) // w.c                           # chunks that may be selected
    Kmean = torch.empty((B, H, w.M, d), dtype=torch.float32, device=DEV)
    tf.tf_chunk_summarize(Kd, w.c, Kmean, 0, n_old)
    idx = torch.empty((B, H, w.k), dtype=torch.int32, device=DEV)
    Kr = torch.zeros((B, H, w.R + n_recent, d), dtype=torch.bfloat16, device=DEV)
    Vr = torch.zeros_like(Kr)
    tf.tf_chunk_topk_gather(x["q_r"].to(DEV), Kmean, Kd, Vd, w.c, w.k, idx, Kr, Vr, n_chunks_all=n_old)
    tf.tf_kv_append(Kd[:, :, N - n_recent:].contiguous(), Vd[:, :, N - n_recent:].contiguous(), Kr, Vr, pos_all=w.R)
    O_g = torch.empty(Qd.shape, dtype=torch.float32, device=DEV)
    L_g = torch.empty(Qd.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_retrieval(Qd, Kr, Vr, O_g, L_g, causal=True)
    O_i, L_i = _run_indexed(Qd, Kd, Vd, idx, w.c, kv_len_all=N, recent_begin_all=N - n_recent)
    torch.cuda.synchronize()
    assert np.max(np.abs(O_i - O_g.cpu().numpy())) < 1e-6 and np.max(np.abs(L_i - L_g.cpu().numpy())) < 1e-6
    Oo, Lo = oracle.attention_indexed(synth.as_u16(x["Q"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]),
                                      idx.cpu().numpy(), w.c, recent_begin=[N - n_recent])
    assert np.max(np.abs(O_i - Oo)) <= ATTN_TOL and np.max(np.abs(L_i - Lo)) <= LSE_TOL


def test_indexed_without_chunks_is_window_attention():
    """k = 0: only the recent rows remain, i.e. attention over a sliding window of the cache."""
    say("case indexed_window seed=152")
    x = synth.make_layer(1, 2, 700, 4, 8, 0, seed=152)
    idx = torch.empty((1, 2, 0), dtype=torch.int32, device=DEV)
    O, L = _run_indexed(x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV), idx, 8, kv_len_all=700, recent_begin_all=500)
    Ku, Vu = synth.as_u16(x["K"])[:, :, 500:], synth.as_u16(x["V"])[:, :, 500:]
    Oo, Lo, _ = oracle.attention(synth.as_u16(x["Q"]), Ku, Vu, causal=True)
    assert np.max(np.abs(O - Oo)) <= ATTN_TOL and np.max(np.abs(L - Lo)) <= LSE_TOL


@pytest.mark.parametrize("n", [1, 5, 16, 37])
def test_kv_append_bit_exact(n):
    say(f"case kv_append n={n} seed=153")
    B, H, cap = 3, 4, 120
    x = synth.make_layer(B, H, cap, 1, 1, 0, seed=153)
    new = synth.make_layer(B, H, n, 1, 1, 0, seed=154)
    pos = [0, cap - n, cap - n // 2 - 1]                    # the last one drops rows beyond the capacity
    Kd, Vd = x["K"].to(DEV), x["V"].to(DEV)
    tf.tf_kv_append(new["K"].to(DEV), new["V"].to(DEV), Kd, Vd, pos=torch.tensor(pos, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    Ko, Vo = oracle.kv_append(synth.as_u16(new["K"]), synth.as_u16(new["V"]), synth.as_u16(x["K"]),
                              synth.as_u16(x["V"]), pos)
    assert np.array_equal(synth.as_u16(Kd), Ko) and np.array_equal(synth.as_u16(Vd), Vo)


def test_kv_append_into_a_strided_cache_with_a_scalar_position():
    say("case kv_append_strided seed=155")
    B, H, cap, n = 2, 3, 50, 4
    x = synth.make_layer(B, H, cap, 1, 1, 0, seed=155)
    new = synth.make_layer(B, H, n, 1, 1, 0, seed=156)
    Kd = x["K"].to(DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)      # token-major storage
    Vd = x["V"].to(DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    tf.tf_kv_append(new["K"].to(DEV), new["V"].to(DEV), Kd, Vd, pos_all=46)
    torch.cuda.synchronize()
    Ko, Vo = oracle.kv_append(synth.as_u16(new["K"]), synth.as_u16(new["V"]), synth.as_u16(x["K"]),
                              synth.as_u16(x["V"]), 46)
    assert np.array_equal(synth.as_u16(Kd.contiguous()), Ko) and np.array_equal(synth.as_u16(Vd.contiguous()), Vo)
    with pytest.raises(tf.TfError):
        tf.tf_kv_append(new["K"].to(DEV), new["V"].to(DEV), Kd, Vd, pos_all=47)     # would run off the end
    empty = torch.empty((B, H, 0, 128), dtype=torch.bfloat16, device=DEV)         # nothing accepted: a no-op
    tf.tf_kv_append(empty, empty, Kd, Vd, pos_all=50)
    torch.cuda.synchronize()
    assert np.array_equal(synth.as_u16(Kd.contiguous()), Ko) and np.array_equal(synth.as_u16(Vd.contiguous()), Vo)


def test_retrieval_cache_maintenance_scenario():
    """Sec. 4.3 in miniature: build C_r, then for three steps append the new tokens to the full
    cache, stage the step's query tokens behind the budget, draft over C_r + staging, and commit
    the accepted tokens over the least important slots. Checked against the oracle run on the
    same sequence of operations."""
    say("case maintenance_scenario seed=157")
    B, H, N0, c, k, G = 1, 4, 512, 8, 16, 3
    R = k * c
    cap = N0 + 64
    x = synth.make_layer(B, H, cap, G, c, 4, seed=157)
    Kd, Vd = x["K"].to(DEV), x["V"].to(DEV)
    Ku, Vu = synth.as_u16(x["K"]), synth.as_u16(x["V"])
    Kmean = torch.empty((B, H, cap // c, 128), dtype=torch.float32, device=DEV)
    tf.tf_chunk_summarize(Kd, c, Kmean, 0, N0 // c)
    idx = torch.empty((B, H, k), dtype=torch.int32, device=DEV)
    Kr = torch.zeros((B, H, R + G, 128), dtype=torch.bfloat16, device=DEV)
    Vr = torch.zeros_like(Kr)
    tf.tf_chunk_topk_gather(x["q_r"].to(DEV), Kmean, Kd, Vd, c, k, idx, Kr, Vr, n_chunks_all=N0 // c)
    km = oracle.chunk_mean(Ku[:, :, :N0], c)
    _, o_idx = oracle.retrieve(synth.as_u16(x["q_r"]), km, k)
    oKr, oVr = oracle.gather(Ku, Vu, o_idx, c, R_cap=R + G)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), o_idx)
    committed, length = 0, N0
    for step in range(3):
        new = synth.make_layer(B, H, G, G, 1, 0, seed=158 + step)
        nK, nV, Q = new["K"].to(DEV), new["V"].to(DEV), new["Q"].to(DEV)
        tf.tf_kv_append(nK, nV, Kd, Vd, pos_all=length)                 # full cache grows by the G speculated tokens
        tf.tf_kv_append(nK, nV, Kr, Vr, pos_all=R)                      # staging rows behind the budget
        oKr, oVr = oracle.kv_append(synth.as_u16(new["K"]), synth.as_u16(new["V"]), oKr, oVr, R)
        O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
        tf.tf_decode_attn_retrieval(Q, Kr, Vr, O, kv_len_all=R + G, causal=True)
        torch.cuda.synchronize()
        Oo, _, _ = oracle.attention(synth.as_u16(new["Q"]), oKr, oVr, causal=True)
        assert np.max(np.abs(O.cpu().numpy() - Oo)) <= ATTN_TOL
        n_acc = 2                                                       # pretend two of the tokens were accepted
        committed += n_acc
        tf.tf_kv_append(nK[:, :, :n_acc].contiguous(), nV[:, :, :n_acc].contiguous(), Kr, Vr, pos_all=R - committed)
        oKr, oVr = oracle.kv_append(synth.as_u16(new["K"])[:, :, :n_acc], synth.as_u16(new["V"])[:, :, :n_acc],
                                    oKr, oVr, R - committed)
        length += n_acc
        torch.cuda.synchronize()
        assert np.array_equal(synth.as_u16(Kr), oKr) and np.array_equal(synth.as_u16(Vr), oVr)


def test_sinks_plus_recent_window_is_a_streaming_cache():
    """The StreamingLLM cache shape (Sec. 2.2: attention sinks + recent tokens) is the indexed
    call with the sink chunk(s) as indices and the window as the recent range."""
    say("case streaming_cache seed=159")
    B, H, N, G, c = 2, 4, 5000, 4, 4
    x = synth.make_layer(B, H, N, G, c, 0, seed=159)
    kv_len, window = [5000, 3777], 1020
    rb = [n - window for n in kv_len]
    idx = torch.zeros((B, H, 1), dtype=torch.int32, device=DEV)        # chunk 0 = the 4 sink tokens
    O, L = _run_indexed(x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV), idx, c, kv_len=kv_len, recent_begin=rb,
                        kv_len_all=N, recent_begin_all=min(rb))
    Ku, Vu, Qu = synth.as_u16(x["K"]), synth.as_u16(x["V"]), synth.as_u16(x["Q"])
    for b in range(B):
        Kc = np.concatenate([Ku[b:b + 1, :, :c], Ku[b:b + 1, :, rb[b]:kv_len[b]]], axis=2)
        Vc = np.concatenate([Vu[b:b + 1, :, :c], Vu[b:b + 1, :, rb[b]:kv_len[b]]], axis=2)
        Oo, Lo, _ = oracle.attention(Qu[b:b + 1], Kc, Vc, causal=True)
        assert np.max(np.abs(O[b] - Oo[0])) <= ATTN_TOL and np.max(np.abs(L[b] - Lo[0])) <= LSE_TOL
