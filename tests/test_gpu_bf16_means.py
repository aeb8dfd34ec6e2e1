"""GPU parity of the bf16 average-key variant (tf_chunk_summarize_bf16, tf_chunk_topk_gather_bf16).
One definition on both sides: a table entry is the fp32 chunk mean (sequential fp32 sum in token
order, one fp32 division) rounded to bf16, nearest even. The device's table must equal the oracle's
BIT FOR BIT; the device's selection is judged against the oracle's selection on the ORACLE's table
(no device value ever enters the oracle), with the 1e-4 tie band of the fp32 path: the tables being
equal, the scores differ only by the fp32 rounding of a 128-term dot product."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_11912_amd as tf
from paper_2404_11912_amd import synth
from tests.util import u16_f64

pytestmark = pytest.mark.gpu

DEV = "cuda"
TIE_BAND = 1e-4


def say(msg):
    print(msg, flush=True)


def device_table(Kmean_bf16):
    """The device's table widened exactly to float64 (compared with the oracle's, never fed to it)."""
    return u16_f64(synth.as_u16(Kmean_bf16.cpu()))


@pytest.mark.parametrize("c", [1, 8, 12, 16, 32])
def test_summarize_bf16(c):
    say(f"case bf16 means summarize c={c}")
    x = synth.make_layer(B=2, H=3, N=2048 + 5, G=4, c=c, P=2, seed=8100 + c, device="cpu")
    K = x["K"].to(DEV)
    M = K.shape[2] // c
    Kmean = torch.zeros((2, 3, M, 128), dtype=torch.bfloat16, device=DEV)
    tf.tf_chunk_summarize_bf16(K, c, Kmean)
    torch.cuda.synchronize()
    want = oracle.chunk_mean_bf16(synth.as_u16(x["K"]), c)
    assert np.array_equal(device_table(Kmean), want)          # bit-equal: same two roundings on both sides


def test_summarize_bf16_on_the_double_rounding_example():
    """A chunk on which rounding the fp32 mean differs from rounding the exact mean once (keys 4,
    12/256, -2^-30, 0: fp32 mean exactly halfway -> even -> 1 + 2^-6; exact mean rounds to
    1 + 2^-7), and one whose fp32 sum depends on the order of the additions."""
    say("case bf16 means double rounding by hand")
    K = torch.zeros((1, 1, 16, 128), dtype=torch.float64)
    K[0, 0, 0:4] = torch.tensor([4.0, 12.0 / 256.0, -2.0 ** -30, 0.0], dtype=torch.float64)[:, None]
    K[0, 0, 4:8] = torch.tensor([2.0 ** 24, 1.0, 1.0, 1.0], dtype=torch.float64)[:, None]
    K[0, 0, 8:12] = torch.tensor([1.0, 1.0, 1.0, 2.0 ** 24], dtype=torch.float64)[:, None]
    Kb = K.to(torch.bfloat16)
    assert torch.equal(Kb.double(), K)
    Kmean = torch.zeros((1, 1, 4, 128), dtype=torch.bfloat16, device=DEV)
    tf.tf_chunk_summarize_bf16(Kb.to(DEV), 4, Kmean)
    torch.cuda.synchronize()
    got = device_table(Kmean)
    assert np.all(got[0, 0, 0] == 1 + 2.0 ** -6)
    assert np.all(got[0, 0, 1] == 2.0 ** 22) and np.all(got[0, 0, 2] == 2.0 ** 22)   # 2^22 + 1 is no bf16 value
    assert np.array_equal(got, oracle.chunk_mean_bf16(synth.as_u16(Kb), 4))


@pytest.mark.parametrize("N,c,k,P", [(4096, 8, 64, 8), (32768, 8, 512, 64), (8192, 16, 100, 16), (3000, 4, 37, 4)])
def test_topk_gather_bf16_vs_oracle(N, c, k, P):
    say(f"case bf16 means topk N={N} c={c} k={k}")
    B, H = 2, 4
    x = synth.make_layer(B=B, H=H, N=N, G=5, c=c, P=P, seed=8200 + N + c, device="cpu")
    K, V, q_r = x["K"].to(DEV), x["V"].to(DEV), x["q_r"].to(DEV)
    M = N // c
    Kmean = torch.empty((B, H, M, 128), dtype=torch.bfloat16, device=DEV)
    tf.tf_chunk_summarize_bf16(K, c, Kmean)
    idx = torch.empty((B, H, k), dtype=torch.int32, device=DEV)
    score = torch.empty((B, H, k), dtype=torch.float32, device=DEV)
    Kr = torch.zeros((B, H, k * c, 128), dtype=torch.bfloat16, device=DEV)
    Vr = torch.zeros_like(Kr)
    tf.tf_chunk_topk_gather_bf16(q_r, Kmean, K, V, c, k, idx, Kr, Vr, out_score=score)
    torch.cuda.synchronize()
    o_table = oracle.chunk_mean_bf16(synth.as_u16(x["K"]), c)
    assert np.array_equal(device_table(Kmean), o_table)
    o_scores, o_idx = oracle.retrieve(synth.as_u16(x["q_r"]), o_table, k)
    idx_h, sc_h = idx.cpu().numpy(), score.cpu().numpy().astype(np.float64)
    same = 0
    for b in range(B):
        for h in range(H):
            s, got = o_scores[b, h], idx_h[b, h]
            assert got.min() >= 0 and got.max() < M and len(set(got.tolist())) == k
            tau = s[o_idx[b, h, -1]]
            assert set(np.where(s > tau + TIE_BAND)[0].tolist()) <= set(got.tolist())
            assert not (set(got.tolist()) & set(np.where(s < tau - TIE_BAND)[0].tolist()))
            assert np.all(s[got][1:] <= s[got][:-1] + TIE_BAND)
            assert np.max(np.abs(sc_h[b, h] - s[got])) < 2e-5 * max(1.0, np.abs(s[got]).max())
            assert set(x["planted"][b, h].tolist()) <= set(got.tolist())
            same += int(np.array_equal(got, o_idx[b, h]))
    say(f"[bf16 means topk] identical order on {same}/{B * H} units")
    rows = (idx.long()[..., None] * c + torch.arange(c, device=DEV)).reshape(B, H, k * c)
    gi = rows[..., None].expand(B, H, k * c, 128)
    assert torch.equal(Kr.view(torch.int16), torch.gather(K, 2, gi).view(torch.int16))
    assert torch.equal(Vr.view(torch.int16), torch.gather(V, 2, gi).view(torch.int16))


def test_bf16_table_per_sequence_counts_and_ties():
    """Per-sequence chunk counts, and exact ties (duplicated chunks) resolved toward the lower index."""
    say("case bf16 means ragged + ties")
    B, H, N, c, k = 2, 2, 1024, 8, 16
    x = synth.make_layer(B=B, H=H, N=N, G=3, c=c, P=4, seed=8301, device="cpu")
    K = x["K"].clone()
    K[:, :, 40 * c:41 * c] = K[:, :, 3 * c:4 * c]           # chunk 40 duplicates chunk 3
    pl = x["planted"][0, 0, 0].item()
    K[:, :, 90 * c:91 * c] = K[:, :, pl * c:(pl + 1) * c]   # and chunk 90 a planted one (b = 0, h = 0)
    Kd, Vd, q_r = K.to(DEV), x["V"].to(DEV), x["q_r"].to(DEV)
    M = N // c
    Kmean = torch.empty((B, H, M, 128), dtype=torch.bfloat16, device=DEV)
    tf.tf_chunk_summarize_bf16(Kd, c, Kmean)
    nc = np.array([M, 100], dtype=np.int32)
    idx = torch.empty((B, H, k), dtype=torch.int32, device=DEV)
    tf.tf_chunk_topk_gather_bf16(q_r, Kmean, Kd, Vd, c, k, idx, n_chunks=torch.tensor(nc, device=DEV),
                                 n_chunks_all=M)
    torch.cuda.synchronize()
    o_table = oracle.chunk_mean_bf16(synth.as_u16(K), c)
    assert np.array_equal(device_table(Kmean), o_table)
    o_scores, o_idx = oracle.retrieve(synth.as_u16(x["q_r"]), o_table, k, n_chunks=nc)
    got = idx.cpu().numpy()
    assert got[1].max() < 100
    g00 = got[0, 0].tolist()
    if pl in g00 and 90 in g00 and pl < 90:
        assert g00.index(pl) + 1 == g00.index(90)            # equal scores: lower index first, adjacent
    for b in range(B):
        for h in range(H):
            s = o_scores[b, h][:nc[b]]
            tau = s[o_idx[b, h, -1]]
            assert set(np.where(s > tau + TIE_BAND)[0].tolist()) <= set(got[b, h].tolist())


def test_bf16_table_at_the_128k_layer_shape():
    """One layer of the 128K workload through the bf16 table, all heads; reports how many of the
    fp32 table's selections survive the rounding."""
    w = synth.WORKLOADS["step128k"]
    say("case bf16 means full-size step128k layer 2")
    x = synth.make_workload_layer(w, 2, DEV)
    K, V, q_r = x["K"], x["V"], x["q_r"]
    B, H, N, d = K.shape
    Kb = torch.empty((B, H, w.M, d), dtype=torch.bfloat16, device=DEV)
    Kf = torch.empty((B, H, w.M, d), dtype=torch.float32, device=DEV)
    tf.tf_chunk_summarize_bf16(K, w.c, Kb)
    tf.tf_chunk_summarize(K, w.c, Kf)
    idx_b = torch.empty((B, H, w.k), dtype=torch.int32, device=DEV)
    idx_f = torch.empty_like(idx_b)
    tf.tf_chunk_topk_gather_bf16(q_r, Kb, K, V, w.c, w.k, idx_b)
    tf.tf_chunk_topk_gather(q_r, Kf, K, V, w.c, w.k, idx_f)
    torch.cuda.synchronize()
    assert torch.equal(Kb, Kf.to(torch.bfloat16))             # the bf16 table is the fp32 table rounded (nearest even)
    o_table = oracle.chunk_mean_bf16(synth.as_u16(K.cpu()), w.c)   # 1 GiB of keys through the oracle: seconds
    assert np.array_equal(device_table(Kb), o_table)
    o_scores, o_idx = oracle.retrieve(synth.as_u16(q_r.cpu()), o_table, w.k)
    got = idx_b.cpu().numpy()
    planted = x["planted"].cpu().numpy()
    overlap = []
    for h in range(H):
        s = o_scores[0, h]
        tau = s[o_idx[0, h, -1]]
        assert set(np.where(s > tau + TIE_BAND)[0].tolist()) <= set(got[0, h].tolist())
        assert not (set(got[0, h].tolist()) & set(np.where(s < tau - TIE_BAND)[0].tolist()))
        assert set(planted[0, h].tolist()) <= set(got[0, h].tolist())
        overlap.append(len(set(got[0, h].tolist()) & set(idx_f[0, h].cpu().tolist())))
    say(f"[bf16 means 128K] chunks shared with the fp32 table's selection: min {min(overlap)} / {w.k}, "
        f"mean {np.mean(overlap):.1f}")
    assert min(overlap) >= 0.9 * w.k
