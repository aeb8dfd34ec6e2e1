"""GPU parity: every C-ABI call against the fp64 CPU oracle on the same seeded inputs.

Bars: indices / counts / copied bytes bit-exact (top-k: within the 1e-4 tie band either choice
is valid); attention outputs within max-abs-error 2e-3 (bf16 inputs, fp32 accumulation).
No oracle input ever comes from the GPU: both sides start from the seeded generators.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2404_11912_amd as tf
from paper_2404_11912_amd import synth
from tests.util import bf16_u16, u16_torch

pytestmark = pytest.mark.gpu

ATTN_TOL = 2e-3          # max-abs-error on attention outputs
LSE_TOL = 1e-3
TIE_BAND = 1e-4          # chunk scores closer than this may be ordered either way
DEV = "cuda"


def say(msg):
    print(msg, flush=True)


def run_attn(fn, Q, K, V, kv_len=None, kv_len_all=None, scale=1.0, causal=True):
    O = torch.empty(Q.shape, dtype=torch.float32, device=DEV)
    LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=DEV)
    kv = None if kv_len is None else torch.tensor(kv_len, dtype=torch.int32, device=DEV)
    fn(Q, K, V, O, LSE, kv_len=kv, kv_len_all=kv_len_all, scale=scale, causal=causal)
    torch.cuda.synchronize()
    return O.cpu().numpy().astype(np.float64), LSE.cpu().numpy().astype(np.float64)


def check_attn(x, fn, kv_len=None, scale=1.0, causal=True, kv_len_all=None, tag=""):
    Qd, Kd, Vd = x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    O, LSE = run_attn(fn, Qd, Kd, Vd, kv_len, kv_len_all, scale, causal)
    N = x["K"].shape[2]
    kv = kv_len if kv_len is not None else (kv_len_all if kv_len_all is not None else N)
    Oo, Lo, _ = oracle.attention(synth.as_u16(x["Q"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]),
                                 kv_len=kv, scale=scale, causal=causal)
    err = float(np.max(np.abs(O - Oo)))
    lerr = float(np.max(np.abs(LSE - Lo)))
    say(f"[attn {tag}] max|dO|={err:.3e} max|dLSE|={lerr:.3e}")
    assert np.isfinite(O).all()
    assert err <= ATTN_TOL and lerr <= LSE_TOL
    return err


# ----------------------------------------------------------------------------- attention
@pytest.mark.parametrize("G", [1, 5, 8])
@pytest.mark.parametrize("causal", [True, False])
def test_attn_full_small_ragged(G, causal):
    """Several tiles, several splits and a ragged tail (N = 1000 is not a multiple of 16)."""
    say(f"case attn_full_small_ragged G={G} causal={causal} seed=101")
    x = synth.make_layer(2, 3, 1000, G, 8, 4, seed=101)
    tf.tf_set_option("attn_full_tokens_per_split", 192)
    try:
        check_attn(x, tf.tf_decode_attn_full, causal=causal, tag=f"ragged G={G} causal={causal}")
    finally:
        tf.tf_set_option("attn_full_tokens_per_split", 0)


@pytest.mark.parametrize("scale", [1.0 / math.sqrt(128.0), 4.0, 0.0])
def test_attn_full_scales(scale):
    """Near-uniform softmax (1/sqrt(d)), peaked softmax (scale 4: a few tokens dominate), scale 0."""
    say(f"case attn_full_scales scale={scale} seed=102")
    x = synth.make_layer(1, 4, 2048 + 37, 5, 8, 8, seed=102)
    check_attn(x, tf.tf_decode_attn_full, scale=scale, tag=f"scale={scale:.3f}")


def test_attn_full_per_sequence_lengths_and_default_splits():
    say("case attn_full_per_sequence_lengths seed=103")
    x = synth.make_layer(3, 2, 3000, 4, 8, 0, seed=103)
    check_attn(x, tf.tf_decode_attn_full, kv_len=[3000, 517, 4], kv_len_all=3000, tag="kv_len=[3000,517,4]")


@pytest.mark.parametrize("N,G", [(1, 1), (5, 5), (16, 3), (17, 8), (63, 2), (64, 8), (65, 1)])
def test_attn_tiny_contexts(N, G):
    say(f"case attn_tiny_contexts N={N} G={G} seed=104")
    x = synth.make_layer(1, 2, N, G, 1, 0, seed=104 + N)
    check_attn(x, tf.tf_decode_attn_full, tag=f"N={N} G={G} full")
    check_attn(x, tf.tf_decode_attn_retrieval, tag=f"N={N} G={G} retr")


def test_attn_strided_token_major_layout():
    """Cache stored [B,N,H,d] (token-major) and viewed as [B,H,N,d]: stride_t = H*d."""
    say("case attn_strided_layout seed=105")
    x = synth.make_layer(2, 4, 777, 5, 8, 0, seed=105)
    Kd = x["K"].to(DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    Vd = x["V"].to(DEV).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    assert Kd.stride(2) == 4 * 128
    O, LSE = run_attn(tf.tf_decode_attn_full, x["Q"].to(DEV), Kd, Vd)
    Oo, Lo, _ = oracle.attention(synth.as_u16(x["Q"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]))
    assert np.max(np.abs(O - Oo)) <= ATTN_TOL and np.max(np.abs(LSE - Lo)) <= LSE_TOL


def test_attn_capacity_larger_than_length():
    say("case attn_capacity seed=106")
    x = synth.make_layer(1, 2, 900, 3, 8, 0, seed=106)
    check_attn(x, tf.tf_decode_attn_full, kv_len_all=555, tag="capacity 900, len 555")
    check_attn(x, tf.tf_decode_attn_retrieval, kv_len_all=555, tag="capacity 900, len 555 (retr)")


def test_attn_closed_form_one_hot_keys():
    """A hand-built case with an exact answer, independent of the oracle: key t is e_t * 8, the
    query is e_7 * 8 and scale is 1, so token 7 has logit 64 and all others 0."""
    say("case attn_closed_form")
    N = 100
    Q = np.zeros((1, 1, 1, 128)); Q[0, 0, 0, 7] = 8.0
    K = np.zeros((1, 1, N, 128))
    for t in range(N):
        K[0, 0, t, t % 128] = 8.0
    rng = np.random.default_rng(5)
    Vu = bf16_u16(rng.standard_normal((1, 1, N, 128)))
    O, LSE = run_attn(tf.tf_decode_attn_full, u16_torch(bf16_u16(Q), DEV), u16_torch(bf16_u16(K), DEV),
                      u16_torch(Vu, DEV), causal=False)
    want = (Vu[0, 0, 7].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.max(np.abs(O[0, 0, 0] - want)) < 1e-5
    assert abs(LSE[0, 0, 0] - 64.0) < 1e-4


def test_attn_is_deterministic():
    say("case attn_deterministic seed=107")
    x = synth.make_layer(1, 4, 5000, 5, 8, 0, seed=107)
    Qd, Kd, Vd = x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    outs = []
    for _ in range(2):
        O = torch.empty(Qd.shape, dtype=torch.float32, device=DEV)
        L = torch.empty(Qd.shape[:3], dtype=torch.float32, device=DEV)
        tf.tf_decode_attn_full(Qd, Kd, Vd, O, L)
        torch.cuda.synchronize()
        outs.append((O.cpu(), L.cpu()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


# ----------------------------------------------------------------------------- chunk summaries
@pytest.mark.parametrize("c", [1, 4, 8, 16, 32, 12])
def test_chunk_summarize(c):
    say(f"case chunk_summarize c={c} seed=110")
    x = synth.make_layer(2, 3, 1000 + 5, 1, 1, 0, seed=110)
    Kd = x["K"].to(DEV)
    M = Kd.shape[2] // c
    Kmean = torch.full((2, 3, M + 3, 128), float("nan"), dtype=torch.float32, device=DEV)
    tf.tf_chunk_summarize(Kd, c, Kmean, 0, M)
    torch.cuda.synchronize()
    want = oracle.chunk_mean(synth.as_u16(x["K"]), c)
    got = Kmean.cpu().numpy().astype(np.float64)
    # fp32 sums of c bf16 values, then one correctly rounded division
    tol = 2.0 ** -23 * (c + 1) * np.maximum(1.0, np.abs(want))
    assert np.all(np.abs(got[:, :, :M] - want) <= tol)
    assert np.isnan(got[:, :, M:]).all()                  # rows outside the range untouched
    if c in (1, 4, 8, 16):
        assert float(np.max(np.abs(got[:, :, :M] - want))) < 2e-7
    # the call fixes its arithmetic (sequential fp32 sum in token order, one fp32 division): bit-equal
    # to the oracle's fp32 transcription of that definition
    assert np.array_equal(Kmean.cpu().numpy()[:, :, :M], oracle.chunk_mean_fp32(synth.as_u16(x["K"]), c))


def test_chunk_summarize_incremental_range():
    say("case chunk_summarize_incremental seed=111")
    x = synth.make_layer(1, 2, 512, 1, 1, 0, seed=111)
    Kd = x["K"].to(DEV)
    full = torch.zeros((1, 2, 64, 128), dtype=torch.float32, device=DEV)
    part = torch.zeros_like(full)
    tf.tf_chunk_summarize(Kd, 8, full, 0, 64)
    tf.tf_chunk_summarize(Kd, 8, part, 0, 40)
    tf.tf_chunk_summarize(Kd, 8, part, 40, 24)            # newly completed chunks only
    torch.cuda.synchronize()
    assert torch.equal(full, part)


# ----------------------------------------------------------------------------- retrieval
def gpu_retrieve(x, c, k, n_chunks=None, R_cap=None, Kmean_override=None):
    Kd, Vd = x["K"].to(DEV), x["V"].to(DEV)
    B, H, N, d = Kd.shape
    M = N // c
    if Kmean_override is None:
        Kmean = torch.empty((B, H, M, d), dtype=torch.float32, device=DEV)
        tf.tf_chunk_summarize(Kd, c, Kmean, 0, M)
    else:
        Kmean = Kmean_override
    idx = torch.full((B, H, k), -7, dtype=torch.int32, device=DEV)
    score = torch.empty((B, H, k), dtype=torch.float32, device=DEV)
    R_cap = k * c if R_cap is None else R_cap
    Kr = torch.zeros((B, H, R_cap, d), dtype=torch.bfloat16, device=DEV)
    Vr = torch.zeros_like(Kr)
    nc = None if n_chunks is None else torch.tensor(n_chunks, dtype=torch.int32, device=DEV)
    tf.tf_chunk_topk_gather(x["q_r"].to(DEV), Kmean, Kd, Vd, c, k, idx, Kr, Vr, out_score=score, n_chunks=nc)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), score.cpu().numpy().astype(np.float64), Kr.cpu(), Vr.cpu()


def check_topk(idx, score, o_scores, o_idx, n_valid, k, tag=""):
    """Set / order rule for ties: every chunk above tau+band must be selected, none below
    tau-band may be, entries are distinct and valid, oracle scores along the GPU order are
    non-increasing within the band. Returns how many (b,h) matched the oracle exactly."""
    B, H, _ = idx.shape
    exact = 0
    for b in range(B):
        nb = int(n_valid[b])
        for h in range(H):
            s = o_scores[b, h, :nb]
            got = idx[b, h]
            assert len(set(got.tolist())) == k and got.min() >= 0 and got.max() < nb, (tag, b, h)
            tau = s[o_idx[b, h, k - 1]]
            must = set(np.where(s > tau + TIE_BAND)[0].tolist())
            may_not = set(np.where(s < tau - TIE_BAND)[0].tolist())
            gs = set(got.tolist())
            assert must <= gs and not (gs & may_not), (tag, b, h)
            along = s[got]
            assert np.all(along[1:] <= along[:-1] + TIE_BAND), (tag, b, h)
            assert np.max(np.abs(score[b, h] - along)) < 2e-5 * max(1.0, np.abs(along).max()), (tag, b, h)
            srt = np.sort(s)[::-1][:k + 1]
            if np.array_equal(got, o_idx[b, h]):
                exact += 1
            elif len(srt) > 1 and np.min(-np.diff(srt)) > TIE_BAND:
                raise AssertionError(f"{tag}: no tie within the band, yet indices differ at b={b} h={h}")
    return exact


def check_gather(x, c, idx, Kr, Vr):
    """Copied rows are bit-exact copies of the rows the returned indices name."""
    Ku, Vu = synth.as_u16(x["K"]), synth.as_u16(x["V"])
    Kru, Vru = synth.as_u16(Kr), synth.as_u16(Vr)
    B, H, k = idx.shape
    rows = (idx[..., None].astype(np.int64) * c + np.arange(c)[None, None, None, :]).reshape(B, H, k * c)
    wantK = np.take_along_axis(Ku, rows[..., None], axis=2)
    wantV = np.take_along_axis(Vu, rows[..., None], axis=2)
    assert np.array_equal(Kru[:, :, :k * c], wantK) and np.array_equal(Vru[:, :, :k * c], wantV)
    assert not Kru[:, :, k * c:].any() and not Vru[:, :, k * c:].any()      # rows beyond the budget untouched


@pytest.mark.parametrize("N,c,k,P", [(4096, 8, 64, 8), (1000, 4, 250, 3), (37 * 16, 16, 5, 2), (2048, 1, 100, 0),
                                     (8, 8, 1, 0), (4100, 8, 512, 16)])
def test_topk_gather_vs_oracle(N, c, k, P):
    say(f"case topk_gather N={N} c={c} k={k} P={P} seed=120")
    x = synth.make_layer(2, 3, N, 2, c, P, seed=120 + N)
    idx, score, Kr, Vr = gpu_retrieve(x, c, k, R_cap=k * c + 8)
    km = oracle.chunk_mean(synth.as_u16(x["K"]), c)
    o_scores, o_idx = oracle.retrieve(synth.as_u16(x["q_r"]), km, k)
    M = N // c
    exact = check_topk(idx, score, o_scores, o_idx, [M, M], k, tag=f"N={N}")
    say(f"[topk N={N} c={c} k={k}] exact index match on {exact}/6 heads")
    check_gather(x, c, idx, Kr, Vr)
    if P:
        planted = x["planted"].numpy()
        for b in range(2):
            for h in range(3):
                assert set(idx[b, h, :P].tolist()) == set(planted[b, h].tolist())


def test_topk_exact_ties_go_to_lower_index():
    """Duplicated summary rows score identically on both sides: the order is then fully
    determined (lower index first) and must match bit-exactly."""
    say("case topk_exact_ties seed=121")
    rng = np.random.default_rng(121)
    B, H, M, k = 1, 2, 300, 40
    base = rng.standard_normal((B, H, 20, 128)).astype(np.float32)
    km = np.ascontiguousarray(base[:, :, rng.integers(0, 20, M), :])      # 300 rows drawn from 20 distinct ones
    q = bf16_u16(rng.standard_normal((B, H, 128)) * 0.3)
    x = {"K": torch.zeros(B, H, M, 128, dtype=torch.bfloat16), "V": torch.zeros(B, H, M, 128, dtype=torch.bfloat16),
         "q_r": u16_torch(q)}
    idx, score, _, _ = gpu_retrieve(x, 1, k, Kmean_override=torch.from_numpy(km).to(DEV))
    o_scores, o_idx = oracle.retrieve(q, km.astype(np.float64), k)
    # the 20 distinct rows are random, so distinct scores differ by far more than the band
    assert np.array_equal(idx, o_idx)


def _retrieve_on_table(q_u16, km32, k, bf16_table):
    """Run the selection on a given average-key table (values exact in bf16 when bf16_table)."""
    B, H, M, _ = km32.shape
    table = torch.from_numpy(km32).to(DEV)
    if bf16_table:
        assert torch.equal(table.to(torch.bfloat16).float(), table)
        table = table.to(torch.bfloat16)
    Kz = torch.zeros(B, H, M, 128, dtype=torch.bfloat16, device=DEV)
    idx = torch.full((B, H, k), -7, dtype=torch.int32, device=DEV)
    score = torch.empty((B, H, k), dtype=torch.float32, device=DEV)
    fn = tf.tf_chunk_topk_gather_bf16 if bf16_table else tf.tf_chunk_topk_gather
    fn(u16_torch(q_u16, DEV), table, Kz, Kz, 1, k, idx, out_score=score)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), score.cpu().numpy()


@pytest.mark.parametrize("bf16_table", [False, True])
def test_topk_zero_query_every_score_ties(bf16_table):
    """q_r = 0: every score is zero whatever the signs of the averages (a product 0 * negative is
    -0; the sum must still be +0 so that all scores compare equal): indices 0..k-1 in order."""
    say(f"case topk_zero_query bf16_table={bf16_table}")
    rng = np.random.default_rng(123)
    B, H, M, k = 1, 3, 500, 37
    km = (rng.integers(-8, 9, (B, H, M, 128)) / 4.0).astype(np.float32)
    km[:, 1] = -np.abs(km[:, 1]) - 0.25                           # a head whose averages are all negative
    km[:, 2, ::3] = -np.abs(km[:, 2, ::3]) - 0.25                 # and one where every third row is
    q = np.zeros((B, H, 128), dtype=np.uint16)
    q[:, 2, ::2] = 0x8000                                         # -0 entries in the query as well
    idx, score = _retrieve_on_table(q, km, k, bf16_table)
    _, o_idx = oracle.retrieve(q, km.astype(np.float64), k)
    assert np.array_equal(o_idx, np.broadcast_to(np.arange(k), (B, H, k)))
    assert np.array_equal(idx, o_idx)
    assert np.all(score == 0.0) and not np.signbit(score).any()


@pytest.mark.parametrize("bf16_table", [False, True])
def test_topk_one_exactly_zero_score_among_others(bf16_table):
    """Scores that are small exact integers (one query component is 1, the rest 0), among them
    exactly one zero and rows whose other entries are negative: the order is fully determined and
    must equal the oracle's."""
    say(f"case topk_single_zero_score bf16_table={bf16_table}")
    rng = np.random.default_rng(124)
    B, H, M, k = 1, 2, 64, 40
    km = -np.abs(rng.integers(1, 9, (B, H, M, 128)) / 2.0).astype(np.float32)
    for h in range(H):
        km[0, h, :, 5] = rng.permutation(M) - 30                  # scores -30 .. 33, each once, one of them 0
    q = np.zeros((B, H, 128), dtype=np.uint16)
    q[:, :, 5] = 0x3f80                                           # 1.0
    idx, score = _retrieve_on_table(q, km, k, bf16_table)
    o_scores, o_idx = oracle.retrieve(q, km.astype(np.float64), k)
    assert np.array_equal(idx, o_idx)
    assert np.array_equal(score.astype(np.float64), np.take_along_axis(o_scores, o_idx.astype(np.int64), axis=2))


def test_topk_per_sequence_chunk_counts_and_full_budget():
    say("case topk_n_chunks seed=122")
    x = synth.make_layer(2, 2, 1024, 2, 8, 4, seed=122)
    n_chunks = [128, 50]
    idx, score, Kr, Vr = gpu_retrieve(x, 8, 50, n_chunks=n_chunks)
    km = oracle.chunk_mean(synth.as_u16(x["K"]), 8)
    o_scores, o_idx = oracle.retrieve(synth.as_u16(x["q_r"]), km, 50, n_chunks=n_chunks)
    check_topk(idx, score, o_scores, o_idx, n_chunks, 50, tag="n_chunks")
    assert np.array_equal(np.sort(idx[1], axis=-1), np.broadcast_to(np.arange(50), (2, 50)))   # k = n: permutation
    check_gather(x, 8, idx, Kr, Vr)


def test_full_budget_retrieval_attention_matches_full_attention_on_gpu():
    """k = M: the retrieval cache is a permutation of the full cache, so (non-causal)
    attention over it must agree with full attention (both on the GPU) and with the oracle."""
    say("case full_budget_identity seed=123")
    x = synth.make_layer(1, 4, 2048, 4, 8, 8, seed=123)
    idx, _, Kr, Vr = gpu_retrieve(x, 8, 256)
    Qd = x["Q"].to(DEV)
    O_r, L_r = run_attn(tf.tf_decode_attn_retrieval, Qd, Kr.to(DEV), Vr.to(DEV), causal=False)
    O_f, L_f = run_attn(tf.tf_decode_attn_full, Qd, x["K"].to(DEV), x["V"].to(DEV), causal=False)
    Oo, Lo, _ = oracle.attention(synth.as_u16(x["Q"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]), causal=False)
    assert np.max(np.abs(O_r - Oo)) <= ATTN_TOL and np.max(np.abs(O_f - Oo)) <= ATTN_TOL
    assert np.max(np.abs(L_r - Lo)) <= LSE_TOL and np.max(np.abs(L_f - Lo)) <= LSE_TOL


def _oracle_chain(x, c, k, G_d, scale=1.0):
    Ku, Vu = synth.as_u16(x["K"]), synth.as_u16(x["V"])
    km = oracle.chunk_mean(Ku, c)
    o_scores, o_idx = oracle.retrieve(synth.as_u16(x["q_r"]), km, k)
    Kr, Vr = oracle.gather(Ku, Vu, o_idx, c)
    Qd = synth.as_u16(x["Q"])[:, :, -G_d:, :]
    O, L, _ = oracle.attention(Qd, Kr, Vr, scale=scale, causal=False)
    return o_scores, o_idx, O, L


def _boundary_gap(o_scores, k):
    s = np.sort(o_scores, axis=-1)[..., ::-1]
    return float(np.min(s[..., k - 1] - s[..., k])) if s.shape[-1] > k else float("inf")


@pytest.mark.parametrize("name", ["tiny", "layer32k"])
def test_whole_path_on_workload(name):
    """summarize -> score/top-k/gather -> draft attention over the retrieval cache, and
    verification attention over the full cache, on the seeded workload shapes. The seed is
    advanced (and reported) until the oracle's k-th / (k+1)-th scores are more than the tie
    band apart, so the selected set is unique and the chained draft attention comparable."""
    w = synth.WORKLOADS[name]
    layer = 0
    while True:
        x = synth.make_workload_layer(w, layer)
        o_scores, o_idx, O_d, L_d = _oracle_chain(x, w.c, w.k, w.G_d)
        gap = _boundary_gap(o_scores, w.k)
        if gap > TIE_BAND:
            break
        say(f"[{name}] layer/seed {layer}: boundary gap {gap:.2e} inside the tie band, advancing")
        layer += 1
        assert layer < 8
    say(f"case whole_path {name} layer={layer} seed={synth.seed_for(w, layer)}")
    idx, score, Kr, Vr = gpu_retrieve(x, w.c, w.k)
    exact = check_topk(idx, score, o_scores, o_idx, [w.M] * w.B, w.k, tag=name)
    say(f"[{name}] exact index match on {exact}/{w.B * w.H} heads")
    check_gather(x, w.c, idx, Kr, Vr)
    assert np.array_equal(np.sort(idx, axis=-1), np.sort(o_idx, axis=-1))      # unique set
    planted = x["planted"].numpy()
    for h in range(w.H):
        assert set(planted[0, h].tolist()) <= set(idx[0, h].tolist())
    Qd = x["Q"].to(DEV)
    O, L = run_attn(tf.tf_decode_attn_retrieval, Qd[:, :, -w.G_d:, :].contiguous(), Kr.to(DEV), Vr.to(DEV),
                    causal=False)
    err = float(np.max(np.abs(O - O_d)))
    say(f"[{name}] draft attention over the retrieval cache: max|dO|={err:.3e}")
    assert err <= ATTN_TOL and np.max(np.abs(L - L_d)) <= LSE_TOL
    check_attn(x, tf.tf_decode_attn_full, tag=f"{name} verify")


# ----------------------------------------------------------------------------- accept
def check_accept(B, gamma, V, T, seed, correlated, mask=None):
    a = synth.make_accept_inputs(B, gamma, V, T, seed, correlated=correlated)
    if mask is not None:                              # vocabulary entries masked out with -inf logits
        a["target_logits"][..., mask] = -float("inf")
        a["draft_logits"][..., mask] = -float("inf")
        keep = torch.nonzero(~torch.as_tensor(mask)).flatten()
        a["draft_tokens"] = keep[a["draft_tokens"].long() % keep.numel()].to(torch.int32)
    Tf = float(np.float32(T))                         # the C ABI takes the temperature as fp32
    n_o, out_o, ma, ms = oracle.accept(a["target_logits"].numpy(), a["draft_logits"].numpy(),
                                       a["draft_tokens"].numpy(), Tf, a["u_accept"].numpy(),
                                       a["u_sample"].numpy())
    dev = {k: (v.to(DEV) if torch.is_tensor(v) else v) for k, v in a.items()}
    n = torch.full((B,), -9, dtype=torch.int32, device=DEV)
    out = torch.full((B, gamma + 1), -9, dtype=torch.int32, device=DEV)
    tf.tf_spec_accept(dev["target_logits"], dev["draft_logits"], dev["draft_tokens"], T, dev["u_accept"],
                      dev["u_sample"], n, out)
    torch.cuda.synchronize()
    n, out = n.cpu().numpy(), out.cpu().numpy()
    # decisions are taken in fp64 on both sides; only cases within 1e-9 (relative) of a tie are
    # excluded from the bit-exact comparison
    safe = (ma > 1e-9) & (ms > 1e-9)
    assert safe.mean() > 0.99
    assert np.array_equal(n[safe], n_o[safe]) and np.array_equal(out[safe], out_o[safe])
    return n_o


@pytest.mark.parametrize("T", [0.0, 0.6, 1.0])
@pytest.mark.parametrize("correlated", [False, True])
def test_spec_accept_vocab_32000(T, correlated):
    say(f"case spec_accept V=32000 T={T} correlated={correlated} seed=11919")
    n = check_accept(16, 4, 32000, T, 11912 + 7, correlated)
    say(f"[accept T={T} corr={correlated}] accepted counts: {np.bincount(n, minlength=5).tolist()}")


@pytest.mark.parametrize("gamma", [0, 1, 2, 6, 15])
def test_spec_accept_gammas_small_vocab(gamma):
    say(f"case spec_accept gamma={gamma} V=1000 seed=130")
    check_accept(64, gamma, 1000, 0.6, 130 + gamma, correlated=True)


def test_spec_accept_branches_are_exercised():
    """Tiny vocabulary, correlated drafts: all-accepted, early and late rejects all occur."""
    say("case spec_accept_branches seed=131")
    n = check_accept(512, 4, 17, 1.0, 131, correlated=True)
    assert len(set(n.tolist())) == 5


def test_spec_accept_closed_form_identical_distributions():
    """draft == target: everything is accepted whatever the uniforms (no oracle involved)."""
    say("case spec_accept_identical seed=132")
    a = synth.make_accept_inputs(8, 3, 500, 0.7, 132)
    tl = a["target_logits"].to(DEV)
    dl = tl[:, :3, :].contiguous()
    n = torch.empty(8, dtype=torch.int32, device=DEV)
    out = torch.empty((8, 4), dtype=torch.int32, device=DEV)
    tf.tf_spec_accept(tl, dl, a["draft_tokens"].to(DEV), 0.7, a["u_accept"].to(DEV), a["u_sample"].to(DEV), n, out)
    torch.cuda.synchronize()
    assert n.cpu().tolist() == [3] * 8
    assert torch.equal(out[:, :3].cpu(), a["draft_tokens"])


# ----------------------------------------------------------------------------- maximum sizes
def test_spec_accept_large_vocabulary_generic_path():
    """A vocabulary beyond 32768 (and not a multiple of 4) takes the kernels' looping path."""
    say("case spec_accept V=150001 seed=133")
    check_accept(3, 3, 150001, 0.8, 133, correlated=True)
    check_accept(2, 2, 150001, 0.0, 134, correlated=False)


def test_topk_maximum_k_and_many_chunks():
    """k = 2048 (the documented maximum) out of 65536 chunks, c = 1, no gather."""
    say("case topk_max seed=124")
    rng = np.random.default_rng(124)
    B, H, M, k = 1, 2, 65536, tf.binding.TF_MAX_K_CHUNKS
    km = rng.standard_normal((B, H, M, 128)).astype(np.float32)
    q = bf16_u16(rng.standard_normal((B, H, 128)) * 0.3)
    idx = torch.empty((B, H, k), dtype=torch.int32, device=DEV)
    score = torch.empty((B, H, k), dtype=torch.float32, device=DEV)
    K = torch.zeros((B, H, M, 128), dtype=torch.bfloat16, device=DEV)
    tf.tf_chunk_topk_gather(u16_torch(q, DEV), torch.from_numpy(km).to(DEV), K, K, 1, k, idx, out_score=score)
    torch.cuda.synchronize()
    o_scores, o_idx = oracle.retrieve(q, km.astype(np.float64), k)
    check_topk(idx.cpu().numpy(), score.cpu().numpy().astype(np.float64), o_scores, o_idx, [M], k, tag="max k")
    with pytest.raises(tf.TfError):
        tf.tf_chunk_topk_gather(u16_torch(q, DEV), torch.from_numpy(km).to(DEV), K, K, 1, k + 1,
                                torch.empty((B, H, k + 1), dtype=torch.int32, device=DEV))


@pytest.mark.parametrize("M", [16384, 16385, 32768, 32769])
def test_topk_select_register_tiers(M):
    """Chunk counts on both sides of the limits where the select kernel keeps 16 keys per thread in
    registers, 32, or streams the scores on every pass; the second sequence is shorter."""
    say(f"case topk_tiers M={M} seed=125")
    rng = np.random.default_rng(125 + M)
    B, H, k = 2, 2, 300
    km = rng.standard_normal((B, H, M, 128)).astype(np.float32)
    q = bf16_u16(rng.standard_normal((B, H, 128)) * 0.3)
    nc = [M, M - 4097]
    idx = torch.empty((B, H, k), dtype=torch.int32, device=DEV)
    score = torch.empty((B, H, k), dtype=torch.float32, device=DEV)
    K = torch.zeros((B, H, M, 128), dtype=torch.bfloat16, device=DEV)
    tf.tf_chunk_topk_gather(u16_torch(q, DEV), torch.from_numpy(km).to(DEV), K, K, 1, k, idx, out_score=score,
                            n_chunks=torch.tensor(nc, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    got, gs = idx.cpu().numpy(), score.cpu().numpy().astype(np.float64)
    for b in range(B):
        o_scores, o_idx = oracle.retrieve(q[b:b + 1], km[b:b + 1, :, :nc[b]].astype(np.float64), k)
        check_topk(got[b:b + 1], gs[b:b + 1], o_scores, o_idx, [nc[b]], k, tag=f"tiers M={M} b={b}")


def test_attn_eight_queries_many_splits():
    say("case attn_G8_many_splits seed=108")
    x = synth.make_layer(1, 2, 20000 + 9, 8, 8, 4, seed=108)
    tf.tf_set_option("attn_full_tokens_per_split", 64)       # 313 splits per head
    try:
        check_attn(x, tf.tf_decode_attn_full, tag="G=8, 313 splits")
    finally:
        tf.tf_set_option("attn_full_tokens_per_split", 0)


@pytest.mark.parametrize("G", [9, 12, 16])
@pytest.mark.parametrize("causal", [True, False])
def test_attn_more_than_eight_queries(G, causal):
    """Algorithm 1 verifies up to gamma1 + gamma2 + 1 tokens in one pass (9 at gamma1 = 2, gamma2 = 6);
    up to 16 query rows fit the kernel's 16 MFMA columns."""
    say(f"case attn G={G} causal={causal}")
    x = synth.make_layer(B=2, H=3, N=2500, G=G, c=8, P=2, seed=9500 + G, device="cpu")
    check_attn(x, tf.tf_decode_attn_full, kv_len=[2500, 333], kv_len_all=2500, causal=causal, tag=f"G={G}")
    check_attn(x, tf.tf_decode_attn_retrieval, causal=causal, tag=f"G={G} retr")


@pytest.mark.parametrize("T", [0.0, 0.7])
def test_spec_accept_with_masked_vocabulary(T):
    """-inf logits (masked or padded vocabulary entries), including a whole 4096-entry segment and
    the tail of the vocabulary: such entries have probability 0 on both sides."""
    say(f"case spec_accept masked vocabulary T={T}")
    V = 14000
    mask = np.zeros(V, dtype=bool)
    mask[4096:8192] = True                            # one whole segment of the kernel
    mask[13000:] = True                               # a padded tail
    mask[np.random.default_rng(5).integers(0, 4096, 300)] = True
    check_accept(16, 4, V, T, 9700, correlated=True, mask=mask)
    check_accept(8, 3, V, T, 9701, correlated=False, mask=mask)


@pytest.mark.parametrize("causal", [True, False])
def test_attn_empty_and_shorter_than_G_sequences(causal):
    """Per-sequence lengths 0 and 2 < G in a batch: queries without a visible key return O = 0,
    LSE = -inf; the others match the oracle."""
    say(f"case attn short sequences causal={causal}")
    x = synth.make_layer(B=4, H=2, N=700, G=5, c=8, P=2, seed=9800, device="cpu")
    kv = [700, 0, 2, 5]
    Qd, Kd, Vd = x["Q"].to(DEV), x["K"].to(DEV), x["V"].to(DEV)
    for fn in (tf.tf_decode_attn_full, tf.tf_decode_attn_retrieval):
        O, L = run_attn(fn, Qd, Kd, Vd, kv, 700, 1.0, causal)
        Oo, Lo, _ = oracle.attention(synth.as_u16(x["Q"]), synth.as_u16(x["K"]), synth.as_u16(x["V"]), kv_len=kv,
                                     scale=1.0, causal=causal)
        assert np.array_equal(np.isneginf(L), np.isneginf(Lo))
        fin = np.isfinite(Lo)
        assert np.max(np.abs(O - Oo)) <= ATTN_TOL and np.max(np.abs(L[fin] - Lo[fin])) <= LSE_TOL
        assert np.all(O[np.isneginf(Lo)] == 0.0)


@pytest.mark.parametrize("T", [0.0, 0.6])
def test_spec_accept_ragged(T):
    """Per-sequence numbers of drafted tokens (as after the first level of Algorithm 1), vocabulary
    32000, against the oracle's per-sequence reduction."""
    say(f"case spec_accept ragged T={T}")
    B, gamma, V = 12, 8, 32000
    a = synth.make_accept_inputs(B, gamma, V, T, 9900, correlated=True)
    nd = np.array([8, 0, 3, 8, 6, 1, 7, 2, 8, 5, 4, 0], dtype=np.int32)
    Tf = float(np.float32(T))
    n_o, out_o, ma, ms = oracle.accept_ragged(a["target_logits"].numpy(), a["draft_logits"].numpy(),
                                              a["draft_tokens"].numpy(), nd, Tf, a["u_accept"].numpy(),
                                              a["u_sample"].numpy())
    n = torch.full((B,), -9, dtype=torch.int32, device=DEV)
    out = torch.full((B, gamma + 1), -9, dtype=torch.int32, device=DEV)
    tf.tf_spec_accept_ragged(a["target_logits"].to(DEV), a["draft_logits"].to(DEV), a["draft_tokens"].to(DEV),
                             torch.tensor(nd, device=DEV), T, a["u_accept"].to(DEV), a["u_sample"].to(DEV), n, out)
    torch.cuda.synchronize()
    safe = (ma > 1e-9) & (ms > 1e-9)
    assert safe.all()
    assert np.array_equal(n.cpu().numpy(), n_o) and np.array_equal(out.cpu().numpy(), out_o)
    assert np.all(n_o <= nd)


def test_spec_accept_zero_residual_falls_back_to_the_target_distribution():
    """p = q (identical logits) and the drafted token on a masked (-inf) entry at some position:
    there p(x) = q(x) = 0, so the test u q(x) < p(x) fails and the token is rejected, while the
    residual max(p - q, 0) is zero everywhere: the correction is then drawn from p itself (the
    kernel's whole-row path). u_sample runs from 0 to the largest fp32 below 1."""
    say("case spec_accept zero residual seed=9950")
    B, gamma, V, T = 12, 3, 9000, 0.8
    a = synth.make_accept_inputs(B, gamma, V, T, 9950, correlated=True)
    mask = np.zeros(V, dtype=bool)
    mask[100:300] = True
    mask[4096:8192] = True                       # one whole segment of the kernel
    mask[8900:] = True                           # the tail: the last positive entry is not the last entry
    a["target_logits"][..., mask] = -float("inf")
    a["draft_logits"] = a["target_logits"][:, :gamma, :].clone()
    keep = torch.nonzero(~torch.as_tensor(mask)).flatten()
    toks = keep[a["draft_tokens"].long() % keep.numel()].to(torch.int32)
    want_n = []
    for b in range(B):
        pos = b % (gamma + 1)                    # gamma: nothing rejected (bonus token from p_gamma)
        if pos < gamma:
            toks[b, pos] = 150 + b               # a masked entry
        want_n.append(pos)
    a["draft_tokens"] = toks
    a["u_sample"] = torch.tensor([0.0, 0.5, 1.0 - 2.0 ** -24, 0.999, 1e-7, 0.25, 1.0 - 2.0 ** -24, 0.75, 0.1,
                                  1.0 - 2.0 ** -23, 0.9, 0.3], dtype=torch.float32)
    Tf = float(np.float32(T))
    n_o, out_o, ma, ms = oracle.accept(a["target_logits"].numpy(), a["draft_logits"].numpy(), toks.numpy(), Tf,
                                       a["u_accept"].numpy(), a["u_sample"].numpy())
    assert n_o.tolist() == want_n                # p = q accepts every unmasked token, whatever u_accept
    n = torch.full((B,), -9, dtype=torch.int32, device=DEV)
    out = torch.full((B, gamma + 1), -9, dtype=torch.int32, device=DEV)
    tf.tf_spec_accept(a["target_logits"].to(DEV), a["draft_logits"].to(DEV), toks.to(DEV), T, a["u_accept"].to(DEV),
                      a["u_sample"].to(DEV), n, out)
    torch.cuda.synchronize()
    n, out = n.cpu().numpy(), out.cpu().numpy()
    assert np.array_equal(n, n_o)
    # the accept decisions here are exact on both sides (0 < 0 is false; u q < q is true for u < 1);
    # only the draw's distance to a cell edge can make the two summation orders disagree
    safe = ms > 1e-9
    assert safe.sum() >= B - 2
    assert np.array_equal(out[safe], out_o[safe])
    drawn = out[np.arange(B), n]
    assert not mask[drawn].any()                 # never a zero-probability token, also at u -> 1
