"""GPU parity at the full per-layer sizes of the specified workloads, in the launch configuration
bench.py times (default split planning, one layer = all batch x head units). Inputs are drawn by
the seeded device generator and copied to the host one layer at a time; the oracle then computes
every (batch, head) unit of the layer. Properties that hold at any size are checked as well.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_11912_amd as tf
from paper_2404_11912_amd import synth

pytestmark = pytest.mark.gpu

DEV = "cuda"
ATTN_TOL, LSE_TOL, TIE_BAND = 2e-3, 1e-3, 1e-4


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("name,layer", [
    ("step128k", 0), ("step128k", 31),                             # first and last layer of each of the
    ("batch4x64k", 0), ("batch4x64k", 1), ("batch4x64k", 31),      # three big workloads, every unit
    ("extreme1m", 0), ("extreme1m", 1), ("extreme1m", 7),
    ("batch2x56k", 0), ("batch6x19k", 3), ("batch10x12k", 31),     # batch shapes of Table 4
])
def test_one_layer_at_full_size(name, layer):
    w = synth.WORKLOADS[name]
    say(f"case fullsize {name} layer={layer} seed={synth.seed_for(w, layer)}")
    x = synth.make_workload_layer(w, layer, DEV)
    K, V, Q, q_r = x["K"], x["V"], x["Q"], x["q_r"]
    B, H, N, d = K.shape

    # whole path on the device, default launch configuration
    Kmean = torch.empty((B, H, w.M, d), dtype=torch.float32, device=DEV)
    tf.tf_chunk_summarize(K, w.c, Kmean, 0, w.M)
    idx = torch.empty((B, H, w.k), dtype=torch.int32, device=DEV)
    score = torch.empty((B, H, w.k), dtype=torch.float32, device=DEV)
    Kr = torch.zeros((B, H, w.R, d), dtype=torch.bfloat16, device=DEV)
    Vr = torch.zeros_like(Kr)
    tf.tf_chunk_topk_gather(q_r, Kmean, K, V, w.c, w.k, idx, Kr, Vr, out_score=score)
    Qd = Q[:, :, -w.G_d:, :].contiguous()
    O_d = torch.empty(Qd.shape, dtype=torch.float32, device=DEV)
    L_d = torch.empty(Qd.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_retrieval(Qd, Kr, Vr, O_d, L_d, causal=False)
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_full(Q, K, V, O, L, causal=True)
    # the draft pass as the benchmark step runs it: the G_d tokens in flight staged behind the budget
    # (rows [R, R+G_d) of a second cache), kv_len = R + G_d, bottom-right causal mask
    Ks = torch.zeros((B, H, w.R + w.G_d, d), dtype=torch.bfloat16, device=DEV)
    Vs = torch.zeros_like(Ks)
    Ks[:, :, :w.R], Vs[:, :, :w.R] = Kr, Vr
    tf.tf_kv_append(K[:, :, N - w.G_d:].contiguous(), V[:, :, N - w.G_d:].contiguous(), Ks, Vs, pos_all=w.R)
    O_s = torch.empty(Qd.shape, dtype=torch.float32, device=DEV)
    L_s = torch.empty(Qd.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_retrieval(Qd, Ks, Vs, O_s, L_s, kv_len_all=w.R + w.G_d, causal=True)
    torch.cuda.synchronize()
    say(f"[{name}] device path done")

    # properties on every unit ------------------------------------------------------------
    idx_h = idx.cpu().numpy()
    assert idx_h.min() >= 0 and idx_h.max() < w.M
    srt = np.sort(idx_h, axis=-1)
    assert np.all(srt[..., 1:] > srt[..., :-1])                       # distinct
    sc_h = score.cpu().numpy().astype(np.float64)
    assert np.all(sc_h[..., 1:] <= sc_h[..., :-1])                    # descending importance
    planted = x["planted"].cpu().numpy()
    for b in range(B):
        for h in range(H):
            assert set(planted[b, h].tolist()) <= set(idx_h[b, h].tolist())
    if w.P == w.k:                                                     # budget == planted chunks
        assert np.array_equal(srt, np.sort(planted, axis=-1))
    # gathered rows are bit-exact copies of the rows the indices name (checked on the device)
    rows = (idx.long()[..., None] * w.c + torch.arange(w.c, device=DEV)).reshape(B, H, w.k * w.c)
    gi = rows[..., None].expand(B, H, w.k * w.c, d)
    assert torch.equal(Kr.view(torch.int16), torch.gather(K, 2, gi).view(torch.int16))
    assert torch.equal(Vr.view(torch.int16), torch.gather(V, 2, gi).view(torch.int16))
    assert torch.isfinite(O).all() and torch.isfinite(L).all() and torch.isfinite(O_d).all()
    del gi, rows

    # every unit against the oracle -------------------------------------------------------
    Ku, Vu, Qu = synth.as_u16(K), synth.as_u16(V), synth.as_u16(Q)
    del K, V, x
    torch.cuda.empty_cache()
    km = oracle.chunk_mean(Ku, w.c)
    got_km = Kmean.cpu().numpy()
    e_km = float(np.max(np.abs(got_km - km)))
    assert e_km < 2e-7 * max(1.0, float(np.abs(km).max()))
    del got_km
    o_scores, o_idx = oracle.retrieve(synth.as_u16(q_r), km, w.k)
    del km
    exact = unique = 0
    for b in range(B):
        for h in range(H):
            s, got = o_scores[b, h], idx_h[b, h]
            tau = s[o_idx[b, h, -1]]
            assert set(np.where(s > tau + TIE_BAND)[0].tolist()) <= set(got.tolist())
            assert not (set(got.tolist()) & set(np.where(s < tau - TIE_BAND)[0].tolist()))
            along = s[got]
            assert np.all(along[1:] <= along[:-1] + TIE_BAND)
            assert np.max(np.abs(sc_h[b, h] - along)) < 2e-5 * max(1.0, np.abs(along).max())
            exact += int(np.array_equal(got, o_idx[b, h]))
            unique += int(set(got.tolist()) == set(o_idx[b, h].tolist()))
    say(f"[{name}] chunk means max err {e_km:.1e}; top-k: {exact}/{B * H} units identical in order, "
        f"{unique}/{B * H} identical as sets")
    # verification attention over the full cache, every unit
    Oo, Lo, _ = oracle.attention(Qu, Ku, Vu, scale=1.0, causal=True)
    e = float(np.max(np.abs(O.cpu().numpy() - Oo)))
    el = float(np.max(np.abs(L.cpu().numpy() - Lo)))
    say(f"[{name}] verify attention, all {B * H} units: max|dO|={e:.2e} max|dLSE|={el:.2e}")
    assert e <= ATTN_TOL and el <= LSE_TOL
    # draft attention over the retrieval cache: comparable on units whose selected set is unique
    oKr, oVr = oracle.gather(Ku, Vu, o_idx, w.c)
    Od, Ld, _ = oracle.attention(np.ascontiguousarray(Qu[:, :, -w.G_d:, :]), oKr, oVr, scale=1.0, causal=False)
    same = np.array([[set(idx_h[b, h].tolist()) == set(o_idx[b, h].tolist()) for h in range(H)] for b in range(B)])
    ed = float(np.max(np.abs(O_d.cpu().numpy() - Od)[same]))
    eld = float(np.max(np.abs(L_d.cpu().numpy() - Ld)[same]))
    say(f"[{name}] draft attention on {int(same.sum())} units: max|dO|={ed:.2e} max|dLSE|={eld:.2e}")
    assert same.sum() >= 0.9 * B * H and ed <= ATTN_TOL and eld <= LSE_TOL
    # the staged, causal draft pass, every unit: the draft cache written out from the device's own (valid)
    # selection -- chunks in that order, then the newest G_d rows -- and plain attention over it
    Os, Ls = oracle.attention_indexed(np.ascontiguousarray(Qu[:, :, -w.G_d:, :]), Ku, Vu, idx_h, w.c,
                                      recent_begin=N - w.G_d, scale=1.0, causal=True)[:2]
    es = float(np.max(np.abs(O_s.cpu().numpy() - Os)))
    els = float(np.max(np.abs(L_s.cpu().numpy() - Ls)))
    say(f"[{name}] staged causal draft attention, all units: max|dO|={es:.2e} max|dLSE|={els:.2e}")
    assert es <= ATTN_TOL and els <= LSE_TOL


@pytest.mark.parametrize("gamma", [2, 4, 6])
def test_accept_batch4_vocab_32000(gamma):
    """Batched accept of the batch-4 workload: per-sequence seeds, gamma in {2,4,6}, T = 0.6."""
    w = synth.WORKLOADS["batch4x64k"]
    say(f"case fullsize accept gamma={gamma}")
    parts = [synth.make_accept_inputs(1, gamma, w.V, 0.6, synth.seed_for(w, 0, b) + 7, correlated=(b % 2 == 0))
             for b in range(w.B)]
    a = {k: torch.cat([p[k] for p in parts], 0) for k in parts[0] if torch.is_tensor(parts[0][k])}
    Tf = float(np.float32(0.6))
    n_o, out_o, ma, ms = oracle.accept(a["target_logits"].numpy(), a["draft_logits"].numpy(),
                                       a["draft_tokens"].numpy(), Tf, a["u_accept"].numpy(), a["u_sample"].numpy())
    n = torch.empty((w.B,), dtype=torch.int32, device=DEV)
    out = torch.empty((w.B, gamma + 1), dtype=torch.int32, device=DEV)
    tf.tf_spec_accept(a["target_logits"].to(DEV), a["draft_logits"].to(DEV), a["draft_tokens"].to(DEV), 0.6,
                      a["u_accept"].to(DEV), a["u_sample"].to(DEV), n, out)
    torch.cuda.synchronize()
    safe = (ma > 1e-9) & (ms > 1e-9)
    assert safe.all()
    assert np.array_equal(n.cpu().numpy(), n_o) and np.array_equal(out.cpu().numpy(), out_o)


@pytest.mark.parametrize("gamma", [2, 6])
def test_batch4x64k_attention_with_other_draft_lengths(gamma):
    """The batch-4 workload speculates gamma in {2, 4, 6} tokens (4 is the workload's default and is
    covered above): verification attention with G = 3 and 7 queries on the full 4 x 64K layer shape,
    every unit, and the draft attention of the same G over the gathered retrieval cache with the
    queries' own tokens staged behind the budget (kv_len = R + G, bottom-right causal mask)."""
    import dataclasses
    G = gamma + 1
    w = dataclasses.replace(synth.WORKLOADS["batch4x64k"], G=G)
    say(f"case fullsize batch4x64k layer=5 G={G} seed={synth.seed_for(w, 5)}")
    x = synth.make_workload_layer(w, 5, DEV)
    K, V, Q, q_r = x["K"], x["V"], x["Q"], x["q_r"]
    B, H, N, d = K.shape
    assert Q.shape[2] == G
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_full(Q, K, V, O, L, causal=True)
    Kmean = torch.empty((B, H, w.M, d), dtype=torch.float32, device=DEV)
    tf.tf_chunk_summarize(K, w.c, Kmean, 0, w.M)
    idx = torch.empty((B, H, w.k), dtype=torch.int32, device=DEV)
    Kr = torch.zeros((B, H, w.R + G, d), dtype=torch.bfloat16, device=DEV)
    Vr = torch.zeros_like(Kr)
    tf.tf_chunk_topk_gather(q_r, Kmean, K, V, w.c, w.k, idx, Kr, Vr)
    tf.tf_kv_append(K[:, :, N - G:].contiguous(), V[:, :, N - G:].contiguous(), Kr, Vr, pos_all=w.R)
    O_d = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L_d = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_retrieval(Q, Kr, Vr, O_d, L_d, kv_len_all=w.R + G, causal=True)
    torch.cuda.synchronize()
    Ku, Vu, Qu = synth.as_u16(K), synth.as_u16(V), synth.as_u16(Q)
    idx_h = idx.cpu().numpy()
    del K, V, x, Kmean
    torch.cuda.empty_cache()
    Oo, Lo, _ = oracle.attention(Qu, Ku, Vu, scale=1.0, causal=True)
    e = float(np.max(np.abs(O.cpu().numpy() - Oo)))
    el = float(np.max(np.abs(L.cpu().numpy() - Lo)))
    say(f"[batch4x64k G={G}] verify attention, all {B * H} units: max|dO|={e:.2e} max|dLSE|={el:.2e}")
    assert e <= ATTN_TOL and el <= LSE_TOL
    # draft cache by its definition, from the device's (valid) selection: chunks in that order, then
    # the G newest rows; the selection itself is judged in the tests above
    assert idx_h.min() >= 0 and idx_h.max() < w.M
    Od, Ld = oracle.attention_indexed(Qu, Ku, Vu, idx_h, w.c, recent_begin=N - G, scale=1.0, causal=True)[:2]
    ed = float(np.max(np.abs(O_d.cpu().numpy() - Od)))
    eld = float(np.max(np.abs(L_d.cpu().numpy() - Ld)))
    say(f"[batch4x64k G={G}] draft attention over the gathered cache + staged tokens: max|dO|={ed:.2e} "
        f"max|dLSE|={eld:.2e}")
    assert ed <= ATTN_TOL and eld <= LSE_TOL


def test_batch_with_per_sequence_lengths_at_a_batching_shape():
    """The 6 x 19K batch shape of Table 4 with six different context lengths (a ragged batch, one
    of them not a multiple of the chunk or tile size): summaries, retrieval with per-sequence
    chunk counts, draft and verification attention with per-sequence lengths, every unit."""
    w = synth.WORKLOADS["batch6x19k"]
    say("case fullsize ragged batch6x19k layer=1")
    x = synth.make_workload_layer(w, 1, DEV)
    K, V, Q, q_r = x["K"], x["V"], x["Q"], x["q_r"]
    B, H, N, d = K.shape
    lens = np.array([N, N - 8, 12345, 9000, 4099, 1024], dtype=np.int32)
    ncs = (lens // w.c).astype(np.int32)
    kv = torch.tensor(lens, device=DEV)
    nc = torch.tensor(ncs, device=DEV)
    Kmean = torch.empty((B, H, w.M, d), dtype=torch.float32, device=DEV)
    tf.tf_chunk_summarize(K, w.c, Kmean, 0, w.M)
    idx = torch.empty((B, H, w.k), dtype=torch.int32, device=DEV)
    Kr = torch.zeros((B, H, w.R, d), dtype=torch.bfloat16, device=DEV)
    Vr = torch.zeros_like(Kr)
    tf.tf_chunk_topk_gather(q_r, Kmean, K, V, w.c, w.k, idx, Kr, Vr, n_chunks=nc, n_chunks_all=w.M)
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_full(Q, K, V, O, L, kv_len=kv, kv_len_all=N, causal=True)
    Qd = Q[:, :, -w.G_d:, :].contiguous()
    O_d = torch.empty(Qd.shape, dtype=torch.float32, device=DEV)
    L_d = torch.empty(Qd.shape[:3], dtype=torch.float32, device=DEV)
    tf.tf_decode_attn_indexed(Qd, K, V, idx, w.c, O_d, L_d, kv_len=kv, kv_len_all=N,
                              recent_begin=kv - w.G_d, recent_begin_all=int(lens.min()) - w.G_d, causal=True)
    torch.cuda.synchronize()
    Ku, Vu, Qu = synth.as_u16(K), synth.as_u16(V), synth.as_u16(Q)
    km = oracle.chunk_mean(Ku, w.c)
    o_scores, o_idx = oracle.retrieve(synth.as_u16(q_r), km, w.k, n_chunks=ncs)
    idx_h = idx.cpu().numpy()
    same = np.zeros((B, H), dtype=bool)
    for b in range(B):
        for h in range(H):
            s, got = o_scores[b, h][:ncs[b]], idx_h[b, h]
            assert got.min() >= 0 and got.max() < ncs[b] and len(set(got.tolist())) == w.k
            tau = s[o_idx[b, h, -1]]
            assert set(np.where(s > tau + TIE_BAND)[0].tolist()) <= set(got.tolist())
            assert not (set(got.tolist()) & set(np.where(s < tau - TIE_BAND)[0].tolist()))
            assert np.all(s[got][1:] <= s[got][:-1] + TIE_BAND)
            same[b, h] = np.array_equal(got, o_idx[b, h])
    Oo, Lo, _ = oracle.attention(Qu, Ku, Vu, kv_len=lens, scale=1.0, causal=True)
    e = float(np.max(np.abs(O.cpu().numpy() - Oo)))
    el = float(np.max(np.abs(L.cpu().numpy() - Lo)))
    say(f"[ragged 6x19k] verify attention: max|dO|={e:.2e} max|dLSE|={el:.2e}")
    assert e <= ATTN_TOL and el <= LSE_TOL
    # draft attention through the device's own indices (any valid selection defines a cache)
    Od, Ld = oracle.attention_indexed(np.ascontiguousarray(Qu[:, :, -w.G_d:, :]), Ku, Vu, idx_h, w.c, kv_len=lens,
                                      recent_begin=lens - w.G_d, scale=1.0, causal=True)[:2]
    ed = float(np.max(np.abs(O_d.cpu().numpy() - Od)))
    eld = float(np.max(np.abs(L_d.cpu().numpy() - Ld)))
    say(f"[ragged 6x19k] indexed draft attention: max|dO|={ed:.2e} max|dLSE|={eld:.2e}; "
        f"top-k order identical on {int(same.sum())}/{B * H} units")
    assert ed <= ATTN_TOL and eld <= LSE_TOL


@pytest.mark.parametrize("name,n_pairs", [("step128k", 64), ("batch4x64k", 64), ("extreme1m", 64)])
def test_random_layer_head_pairs(name, n_pairs):
    """Seeded random (layer, batch, head) units spread over all layers of a workload: the whole
    layer runs on the device in the benchmark's launch configuration, the oracle checks the
    sampled units (chunk means, selection per the tie-band rule, verification and draft attention)."""
    w = synth.WORKLOADS[name]
    rng = np.random.default_rng(4242 + w.index)
    flat = rng.choice(w.L * w.B * w.H, size=n_pairs, replace=False)
    by_layer = {}
    for f in sorted(flat.tolist()):
        l, rem = divmod(f, w.B * w.H)
        by_layer.setdefault(l, []).append(divmod(rem, w.H))
    say(f"case fullsize random pairs {name}: {n_pairs} units over layers {sorted(by_layer)}")
    worst = dict(o=0.0, l=0.0, od=0.0, km=0.0)
    for l, units in by_layer.items():
        x = synth.make_workload_layer(w, l, DEV)
        K, V, Q, q_r = x["K"], x["V"], x["Q"], x["q_r"]
        B, H, N, d = K.shape
        Kmean = torch.empty((B, H, w.M, d), dtype=torch.float32, device=DEV)
        tf.tf_chunk_summarize(K, w.c, Kmean, 0, w.M)
        idx = torch.empty((B, H, w.k), dtype=torch.int32, device=DEV)
        tf.tf_chunk_topk_gather(q_r, Kmean, K, V, w.c, w.k, idx)
        O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
        L = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
        tf.tf_decode_attn_full(Q, K, V, O, L, causal=True)
        Qd = Q[:, :, -w.G_d:, :].contiguous()
        O_d = torch.empty(Qd.shape, dtype=torch.float32, device=DEV)
        L_d = torch.empty(Qd.shape[:3], dtype=torch.float32, device=DEV)
        tf.tf_decode_attn_indexed(Qd, K, V, idx, w.c, O_d, L_d, kv_len_all=N, recent_begin_all=N - w.G_d, causal=True)
        torch.cuda.synchronize()
        for (b, h) in units:
            Ku, Vu = synth.as_u16(K[b:b + 1, h:h + 1]), synth.as_u16(V[b:b + 1, h:h + 1])
            Qu, qu = synth.as_u16(Q[b:b + 1, h:h + 1]), synth.as_u16(q_r[b:b + 1, h:h + 1])
            km = oracle.chunk_mean(Ku, w.c)
            worst["km"] = max(worst["km"], float(np.max(np.abs(Kmean[b, h].cpu().numpy() - km[0, 0]))))
            s, o_idx = oracle.retrieve(qu, km, w.k)
            s, got = s[0, 0], idx[b, h].cpu().numpy()
            tau = s[o_idx[0, 0, -1]]
            assert len(set(got.tolist())) == w.k and got.min() >= 0 and got.max() < w.M
            assert set(np.where(s > tau + TIE_BAND)[0].tolist()) <= set(got.tolist())
            assert not (set(got.tolist()) & set(np.where(s < tau - TIE_BAND)[0].tolist()))
            assert np.all(s[got][1:] <= s[got][:-1] + TIE_BAND)
            Oo, Lo, _ = oracle.attention(Qu, Ku, Vu, scale=1.0, causal=True)
            worst["o"] = max(worst["o"], float(np.max(np.abs(O[b, h].cpu().numpy() - Oo[0, 0]))))
            worst["l"] = max(worst["l"], float(np.max(np.abs(L[b, h].cpu().numpy() - Lo[0, 0]))))
            Od, _ = oracle.attention_indexed(np.ascontiguousarray(Qu[:, :, -w.G_d:, :]), Ku, Vu, got[None, None], w.c,
                                             recent_begin=N - w.G_d, causal=True)[:2]
            worst["od"] = max(worst["od"], float(np.max(np.abs(O_d[b, h].cpu().numpy() - Od[0, 0]))))
        del x, K, V, Kmean
        torch.cuda.empty_cache()
    say(f"[{name} random pairs] max|dO| verify {worst['o']:.2e}, draft {worst['od']:.2e}; max|dLSE| {worst['l']:.2e}; "
        f"chunk means {worst['km']:.1e}")
    assert worst["o"] <= ATTN_TOL and worst["od"] <= ATTN_TOL and worst["l"] <= LSE_TOL and worst["km"] < 2e-6
