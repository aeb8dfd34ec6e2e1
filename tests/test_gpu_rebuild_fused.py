"""tf_chunk_topk_gather has two launch shapes: scoring, selection and gather as three kernels, or
scoring and selection fused in one kernel per (batch, head) unit whose scores never leave the chip
(taken automatically when there are at least two units per compute unit, as when all layers of a
decode step are rebuilt in one call). Both compute the same fp32 scores in the same order, so every
output must be bit-equal between them; the fused shape is also checked against the oracle directly."""
import numpy as np
import pytest
import torch

import oracle
import paper_2404_11912_amd as tf
from paper_2404_11912_amd import synth
from tests.test_gpu_parity import check_gather, check_topk
from tests.util import bf16_u16, u16_torch

pytestmark = pytest.mark.gpu
DEV = "cuda"


def say(msg):
    print(msg, flush=True)


def run(x, c, k, fused, bf16_table=False, n_chunks=None, Kmean=None, gather=True):
    """The retrieval call with the launch shape forced (1 = fused, 2 = three kernels)."""
    Kd, Vd = x["K"].to(DEV), x["V"].to(DEV)
    B, H, N, d = Kd.shape
    M = N // c
    if Kmean is None:
        Kmean = torch.empty((B, H, M, d), dtype=torch.bfloat16 if bf16_table else torch.float32, device=DEV)
        (tf.tf_chunk_summarize_bf16 if bf16_table else tf.tf_chunk_summarize)(Kd, c, Kmean, 0, M)
    idx = torch.full((B, H, k), -7, dtype=torch.int32, device=DEV)
    score = torch.full((B, H, k), float("nan"), dtype=torch.float32, device=DEV)
    Kr = torch.zeros((B, H, k * c + 8, d), dtype=torch.bfloat16, device=DEV) if gather else None
    Vr = torch.zeros_like(Kr) if gather else None
    nc = None if n_chunks is None else torch.tensor(n_chunks, dtype=torch.int32, device=DEV)
    fn = tf.tf_chunk_topk_gather_bf16 if bf16_table else tf.tf_chunk_topk_gather
    tf.tf_set_thread_option("rebuild_fused", fused)
    try:
        fn(x["q_r"].to(DEV), Kmean, Kd, Vd, c, k, idx, Kr, Vr, out_score=score, n_chunks=nc)
    finally:
        tf.tf_set_thread_option("rebuild_fused", -1)
    torch.cuda.synchronize()
    return idx, score, Kr, Vr


def same(a, b):
    for t, u in zip(a, b):
        if t is None:
            assert u is None
        elif t.dtype.is_floating_point and t.dtype == torch.float32:
            assert torch.equal(t.view(torch.int32), u.view(torch.int32))          # bit for bit, NaN and -0 included
        else:
            assert torch.equal(t.view(torch.int16) if t.dtype == torch.bfloat16 else t,
                               u.view(torch.int16) if u.dtype == torch.bfloat16 else u)


@pytest.mark.parametrize("bf16_table", [False, True])
@pytest.mark.parametrize("N,c,k,P", [(4096, 8, 64, 8), (1000, 4, 250, 3), (37 * 16, 16, 5, 2), (2048, 1, 100, 0),
                                     (8, 8, 1, 0), (4100, 8, 512, 16), (16384 * 2, 2, 2048, 32), (16383, 1, 777, 5)])
def test_fused_equals_three_kernels_and_the_oracle(N, c, k, P, bf16_table):
    say(f"case fused rebuild N={N} c={c} k={k} P={P} bf16_table={bf16_table} seed={300 + N}")
    x = synth.make_layer(2, 3, N, 2, c, P, seed=300 + N)
    a = run(x, c, k, 1, bf16_table)
    b = run(x, c, k, 2, bf16_table)
    same(a, b)
    Ku = synth.as_u16(x["K"])
    km = oracle.chunk_mean_bf16(Ku, c) if bf16_table else oracle.chunk_mean(Ku, c)
    o_scores, o_idx = oracle.retrieve(synth.as_u16(x["q_r"]), km, k)
    M = N // c
    idx, score, Kr, Vr = a
    check_topk(idx.cpu().numpy(), score.cpu().numpy().astype(np.float64), o_scores, o_idx, [M, M], k, tag=f"fused N={N}")
    check_gather(x, c, idx.cpu().numpy(), Kr.cpu()[:, :, :k * c + 8], Vr.cpu()[:, :, :k * c + 8])


@pytest.mark.parametrize("bf16_table", [False, True])
def test_fused_per_sequence_counts_short_and_empty_sequences(bf16_table):
    """Per-sequence chunk counts, among them fewer chunks than k and none at all: unused slots are
    -1 / -inf and their cache rows untouched, on both launch shapes."""
    say(f"case fused rebuild n_chunks bf16_table={bf16_table} seed=310")
    x = synth.make_layer(4, 2, 2048, 2, 8, 4, seed=310)
    nc = [256, 50, 7, 0]
    k = 40
    a = run(x, 8, k, 1, bf16_table, n_chunks=nc)
    b = run(x, 8, k, 2, bf16_table, n_chunks=nc)
    same(a, b)
    idx = a[0].cpu().numpy()
    Ku = synth.as_u16(x["K"])
    km = oracle.chunk_mean_bf16(Ku, 8) if bf16_table else oracle.chunk_mean(Ku, 8)
    for bi, n in enumerate(nc):
        keff = min(k, n)
        assert np.all(idx[bi, :, keff:] == -1)
        assert np.all(np.isneginf(a[1].cpu().numpy()[bi, :, keff:]))
        assert not a[2][bi, :, keff * 8:].cpu().view(torch.int16).numpy().any()      # rows beyond stay zero
        if keff:
            s, o_idx = oracle.retrieve(synth.as_u16(x["q_r"])[bi:bi + 1], km[bi:bi + 1, :, :n], keff)
            check_topk(idx[bi:bi + 1, :, :keff], a[1].cpu().numpy()[bi:bi + 1, :, :keff].astype(np.float64), s, o_idx,
                       [n], keff, tag=f"fused n={n}")


@pytest.mark.parametrize("bf16_table", [False, True])
def test_fused_exact_ties_and_zero_scores(bf16_table):
    """Duplicated table rows (bit-equal scores: lower index first) and an all-zero query (every score
    +0: indices 0..k-1), fused launch shape, against the oracle's order."""
    say(f"case fused rebuild ties bf16_table={bf16_table} seed=320")
    rng = np.random.default_rng(320)
    B, H, M, k = 1, 3, 1500, 200
    base = (rng.integers(-16, 17, (B, H, 25, 128)) / 8.0).astype(np.float32)          # exact in bf16
    km = np.ascontiguousarray(np.take_along_axis(base, rng.integers(0, 25, (B, H, M, 1)), axis=2))
    q = bf16_u16(rng.standard_normal((B, H, 128)) * 0.3)
    q[:, 2] = 0                                                                       # head 2: every score ties at +0
    x = {"K": torch.zeros(B, H, M, 128, dtype=torch.bfloat16), "V": torch.zeros(B, H, M, 128, dtype=torch.bfloat16),
         "q_r": u16_torch(q)}
    table = torch.from_numpy(km).to(DEV)
    if bf16_table:
        table = table.to(torch.bfloat16)
    idx, score, _, _ = run(x, 1, k, 1, bf16_table, Kmean=table, gather=False)
    _, o_idx = oracle.retrieve(q, km.astype(np.float64), k)
    assert np.array_equal(idx.cpu().numpy(), o_idx)
    assert np.array_equal(idx.cpu().numpy()[0, 2], np.arange(k))
    assert not np.signbit(score.cpu().numpy()[0, 2]).any()


def test_all_layers_in_one_call_take_the_fused_shape():
    """The rebuild as a decode step issues it: every layer's units in one call (1024 units of 16384
    chunks, a synthetic fp32 table of 8 GiB). The automatic choice must agree bit for bit with the
    three-kernel shape on every unit, and with the oracle on sampled units."""
    say("case fused rebuild 1024 units x 16384 chunks seed=330")
    LB, H, M, k = 32, 32, 16384, 512
    g = torch.Generator(device=DEV)
    g.manual_seed(330)
    table = torch.randn((LB, H, M, 128), generator=g, device=DEV, dtype=torch.float32) * 0.35
    q = (torch.randn((LB, H, 128), generator=g, device=DEV, dtype=torch.float32) / 128 ** 0.5).to(torch.bfloat16)
    planted = torch.randint(0, M, (LB, H, 64), generator=g, device=DEV)
    rows = table.gather(2, planted[..., None].expand(-1, -1, -1, 128)) * 0.5 + 3.0 * torch.nn.functional.normalize(
        q.float(), dim=-1)[:, :, None, :]
    table.scatter_(2, planted[..., None].expand(-1, -1, -1, 128), rows)
    Kz = torch.empty((LB, H, M, 128), dtype=torch.bfloat16, device=DEV)            # 4 GiB, never read: no gather
    outs = []
    for mode in (-1, 2):                                                            # automatic, then three kernels
        idx = torch.empty((LB, H, k), dtype=torch.int32, device=DEV)
        score = torch.empty((LB, H, k), dtype=torch.float32, device=DEV)
        tf.tf_set_thread_option("rebuild_fused", mode)
        try:
            tf.tf_chunk_topk_gather(q, table, Kz, Kz, 1, k, idx, out_score=score, n_chunks_all=M)
        finally:
            tf.tf_set_thread_option("rebuild_fused", -1)
        torch.cuda.synchronize()
        outs.append((idx, score))
    same(outs[0], outs[1])
    rng = np.random.default_rng(331)
    for f in rng.choice(LB * H, 24, replace=False).tolist():
        l, h = divmod(f, H)
        km = table[l, h].cpu().numpy().astype(np.float64)[None, None]
        s, o_idx = oracle.retrieve(synth.as_u16(q[l:l + 1, h:h + 1]), km, k)
        check_topk(outs[0][0][l:l + 1, h:h + 1].cpu().numpy(), outs[0][1][l:l + 1, h:h + 1].cpu().numpy().astype(np.float64),
                   s, o_idx, [M], k, tag=f"unit {l},{h}")
