"""Pins for the oracle's chunk summaries, retrieval (score / top-k) and gather (CPU only)."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2404_11912_amd import synth
from tests.util import bf16_u16, u16_f64

D = 128


def _rand_u16(rng, shape, std=1.0):
    return bf16_u16(rng.standard_normal(shape) * std)


# ------------------------------------------------------------------ chunk means
def test_chunk_mean_hand_example():
    """Rows t = 0..7 hold the constant t in every dim; chunks of 4 average to 1.5 and 5.5."""
    K = np.broadcast_to(np.arange(8, dtype=np.float64)[None, None, :, None], (1, 1, 8, D))
    km = oracle.chunk_mean(bf16_u16(K), 4)
    assert km.shape == (1, 1, 2, D)
    assert np.array_equal(km[0, 0, 0], np.full(D, 1.5)) and np.array_equal(km[0, 0, 1], np.full(D, 5.5))


def test_chunk_mean_identities():
    rng = np.random.default_rng(10)
    K = _rand_u16(rng, (2, 3, 64, D))
    Kf = u16_f64(K)
    # c = 1: the summary is the key itself
    assert np.array_equal(oracle.chunk_mean(K, 1), Kf)
    # mean of equal-sized chunk means = global mean
    for c in (4, 8, 16, 32):
        km = oracle.chunk_mean(K, c)
        assert np.max(np.abs(km.mean(axis=2) - Kf.mean(axis=2))) < 1e-13
    # a chunk of identical keys averages to that key; dims stay separate
    K2 = K.copy()
    K2[:, :, 8:16, :] = K[:, :, 8:9, :]
    assert np.array_equal(oracle.chunk_mean(K2, 8)[:, :, 1, :], Kf[:, :, 8, :])


def test_chunk_mean_ragged_tail_dropped():
    rng = np.random.default_rng(11)
    K = _rand_u16(rng, (1, 1, 21, D))
    km = oracle.chunk_mean(K, 8)
    assert km.shape[2] == 2
    assert np.max(np.abs(km[0, 0, 1] - u16_f64(K)[0, 0, 8:16].mean(axis=0))) < 1e-14


# ------------------------------------------------------------------ scoring + top-k
def test_scores_and_topk_match_brute_force():
    rng = np.random.default_rng(12)
    B, H, M, k = 2, 3, 50, 7
    q = _rand_u16(rng, (B, H, D), 0.3)
    km = rng.standard_normal((B, H, M, D))
    scores, idx = oracle.retrieve(q, km, k)
    want_s = np.einsum("bhd,bhmd->bhm", u16_f64(q), km)
    assert np.max(np.abs(scores - want_s)) < 1e-12
    want_idx = np.argsort(-scores, axis=-1, kind="stable")[..., :k]
    assert np.array_equal(idx, want_idx)


def test_topk_maximises_total_score_over_all_subsets():
    rng = np.random.default_rng(13)
    M, k = 9, 4
    q = _rand_u16(rng, (1, 1, D))
    km = rng.standard_normal((1, 1, M, D))
    scores, idx = oracle.retrieve(q, km, k)
    s = scores[0, 0]
    best = max(itertools.combinations(range(M), k), key=lambda c: sum(s[i] for i in c))
    assert set(idx[0, 0].tolist()) == set(best)
    assert np.all(np.diff(s[idx[0, 0]]) <= 0)          # descending importance


def test_ties_go_to_lower_index():
    rng = np.random.default_rng(14)
    q = _rand_u16(rng, (1, 1, D))
    row = rng.standard_normal(D)
    km = np.tile(row, (1, 1, 6, 1))                     # six identical chunks: all scores tie
    km[0, 0, 4] = row + 4.0 * u16_f64(q)[0, 0]          # one clearly better
    _, idx = oracle.retrieve(q, km, 3)
    assert idx[0, 0].tolist() == [4, 0, 1]


def test_n_chunks_limits_the_candidates():
    rng = np.random.default_rng(15)
    q = _rand_u16(rng, (2, 1, D))
    km = rng.standard_normal((2, 1, 20, D))
    km[:, :, 15:] += 10.0 * u16_f64(q)[:, :, None, :]   # very attractive, but beyond n_chunks of b=1
    scores, idx = oracle.retrieve(q, km, 4, n_chunks=[20, 12])
    assert set(idx[0, 0].tolist()) <= set(range(15, 20))
    assert idx[1, 0].max() < 12 and np.all(np.isneginf(scores[1, 0, 12:]))


def test_single_chunk_context():
    rng = np.random.default_rng(16)
    q = _rand_u16(rng, (1, 2, D))
    K = _rand_u16(rng, (1, 2, 8, D))
    V = _rand_u16(rng, (1, 2, 8, D))
    km = oracle.chunk_mean(K, 8)
    _, idx = oracle.retrieve(q, km, 1)
    assert idx.tolist() == [[[0], [0]]]
    Kr, Vr = oracle.gather(K, V, idx, 8)
    assert np.array_equal(Kr, K) and np.array_equal(Vr, V)


def test_chunk_size_one_is_token_topk():
    rng = np.random.default_rng(17)
    q = _rand_u16(rng, (1, 2, D))
    K = _rand_u16(rng, (1, 2, 40, D))
    scores, idx = oracle.retrieve(q, oracle.chunk_mean(K, 1), 5)
    s = np.einsum("bhd,bhtd->bht", u16_f64(q), u16_f64(K))
    assert np.array_equal(idx, np.argsort(-s, axis=-1, kind="stable")[..., :5])


def test_gather_copies_the_selected_chunks_in_order():
    rng = np.random.default_rng(18)
    B, H, N, c = 2, 2, 48, 4
    K = _rand_u16(rng, (B, H, N, D)); V = _rand_u16(rng, (B, H, N, D))
    idx = np.stack([np.stack([rng.permutation(N // c)[:5] for _ in range(H)]) for _ in range(B)]).astype(np.int32)
    Kr, Vr = oracle.gather(K, V, idx, c, R_cap=32)
    for b in range(B):
        for h in range(H):
            for j in range(5):
                src = slice(idx[b, h, j] * c, idx[b, h, j] * c + c)
                assert np.array_equal(Kr[b, h, j * c:(j + 1) * c], K[b, h, src])
                assert np.array_equal(Vr[b, h, j * c:(j + 1) * c], V[b, h, src])
    assert not Kr[:, :, 20:].any() and not Vr[:, :, 20:].any()


# ------------------------------------------------------------------ whole retrieval path
def test_planted_chunks_are_retrieved_first():
    """Needle-style structure: the planted chunks (keys aligned with the query) must all be
    selected and must occupy the first P ranks."""
    w = synth.WORKLOADS["tiny"]
    x = synth.make_workload_layer(w, 0)
    K = synth.as_u16(x["K"])
    km = oracle.chunk_mean(K, w.c)
    scores, idx = oracle.retrieve(synth.as_u16(x["q_r"]), km, w.k)
    planted = x["planted"].numpy()
    for h in range(w.H):
        assert set(idx[0, h, :w.P].tolist()) == set(planted[0, h].tolist())
        rest = np.delete(scores[0, h], planted[0, h])
        assert scores[0, h, planted[0, h]].min() > rest.max() + 1.0


@pytest.mark.parametrize("c", [4, 8, 16])
def test_full_budget_retrieval_attention_equals_full_attention(c):
    """With k = M the selected chunks are a permutation of all chunks and (non-causal)
    attention over the retrieval cache equals attention over the full cache."""
    rng = np.random.default_rng(19)
    B, H, G, N = 1, 2, 3, 96
    Q = _rand_u16(rng, (B, H, G, D), 0.3)
    K = _rand_u16(rng, (B, H, N, D)); V = _rand_u16(rng, (B, H, N, D))
    M = N // c
    _, idx = oracle.retrieve(Q[:, :, -1, :], oracle.chunk_mean(K, c), M)
    assert np.array_equal(np.sort(idx, axis=-1), np.broadcast_to(np.arange(M), (B, H, M)))
    Kr, Vr = oracle.gather(K, V, idx, c)
    O_full, L_full, _ = oracle.attention(Q, K, V, scale=1.0, causal=False)
    O_r, L_r, _ = oracle.attention(Q, Kr, Vr, scale=1.0, causal=False)
    assert np.max(np.abs(O_full - O_r)) < 1e-12
    assert np.max(np.abs(L_full - L_r)) < 1e-12


def test_round_to_bf16_matches_a_library_conversion():
    """The bf16 average-key variant rounds the fp32 chunk mean to bf16. The rounding helper is
    pinned against torch's float32 -> bfloat16 conversion (round to nearest even) on values that
    are exact in float32, and on hand-made ties."""
    import torch
    rng = np.random.default_rng(5)
    x32 = (rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))).astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.round_to_bf16(x32.astype(np.float64))
    assert np.array_equal(got, want)
    # ties: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7 -> even (1); 1 + 3*2^-8 -> 1 + 2^-6
    assert oracle.round_to_bf16(np.array([1 + 2.0 ** -8]))[0] == 1.0
    assert oracle.round_to_bf16(np.array([1 + 3 * 2.0 ** -8]))[0] == 1 + 2.0 ** -6
    assert oracle.round_to_bf16(np.array([-(1 + 2.0 ** -8 + 2.0 ** -30)]))[0] == -(1 + 2.0 ** -7)
    assert oracle.round_to_bf16(np.array([0.0]))[0] == 0.0
    # the table itself: a chunk of identical keys keeps that key; c = 1 reproduces K
    K = bf16_u16(rng.standard_normal((1, 2, 16, 128)))
    assert np.array_equal(oracle.chunk_mean_bf16(K, 1), u16_f64(K))


def test_bf16_table_definition_two_roundings_by_hand():
    """The bf16 table is defined as: fp32 sequential sum in token order, one fp32 division, then
    round-to-nearest-even to bf16. Hand-worked chunk (c = 4) on which this differs from the exact
    mean rounded once: keys 4, 12/256, -2^-30, 0. fp32: 4 + 0.046875 = 4.046875 (exact);
    adding -2^-30 rounds back to 4.046875 (fp32 spacing at 4 is 2^-21); / 4 = 1 + 3*2^-8, exactly
    halfway between the bf16 neighbours 1 + 2^-7 and 1 + 2^-6 -> even -> 1 + 2^-6. The exact mean
    is 1 + 3*2^-8 - 2^-32, just below the halfway point -> 1 + 2^-7 when rounded once."""
    vals = [4.0, 12.0 / 256.0, -2.0 ** -30, 0.0]
    K = np.zeros((1, 1, 8, D), dtype=np.float64)
    K[0, 0, :4, :] = np.array(vals)[:, None]
    K[0, 0, 4:, 0] = [1.0, 2.0, 3.0, 4.0]               # a second, ordinary chunk: mean 2.5
    Ku = bf16_u16(K)
    assert np.array_equal(u16_f64(Ku), K)               # every value is a bf16 value
    f32 = oracle.chunk_mean_fp32(Ku, 4)
    assert f32.dtype == np.float32 and f32[0, 0, 0, 5] == np.float32(1 + 3 * 2.0 ** -8)
    tab = oracle.chunk_mean_bf16(Ku, 4)
    assert tab[0, 0, 0, 7] == 1 + 2.0 ** -6
    assert oracle.chunk_mean_bf16_once(Ku, 4)[0, 0, 0, 7] == 1 + 2.0 ** -7
    assert tab[0, 0, 1, 0] == 2.5 and tab[0, 0, 1, 1] == 0.0


def test_bf16_table_order_of_the_fp32_additions():
    """Token order matters in fp32: 2^24 + 1 + 1 + ... added front to back loses every 1, added
    back to front it does not. Keys (c = 4): 2^24, 1, 1, 1 -> sequential fp32 sum 2^24 (each +1 is
    a tie that rounds to the even neighbour 2^24), mean 2^22; the reverse order adds 1 + 1 + 1 = 3
    first, and 3 + 2^24 rounds to 2^24 + 4: mean 2^22 + 1."""
    K = np.zeros((1, 1, 8, D))
    K[0, 0, :4, :] = np.array([2.0 ** 24, 1.0, 1.0, 1.0])[:, None]
    K[0, 0, 4:, :] = np.array([1.0, 1.0, 1.0, 2.0 ** 24])[:, None]
    f32 = oracle.chunk_mean_fp32(bf16_u16(K), 4)
    assert f32[0, 0, 0, 3] == np.float32(2.0 ** 22)
    assert f32[0, 0, 1, 3] == np.float32(2.0 ** 22 + 1)


def test_bf16_table_against_the_exact_mean():
    """Away from rounding boundaries the definition agrees with the exact mean: the fp32 mean is
    within (c+1) 2^-24 relative of the fp64 mean (c-1 additions and one division, half an ulp
    each), the table is the fp64 mean rounded once except for rare boundary cases, which differ by
    exactly one bf16 ulp; power-of-two chunks of identical keys return that key."""
    rng = np.random.default_rng(77)
    for c in (1, 3, 8, 12, 16):
        K = _rand_u16(rng, (2, 3, 50 * c + c // 2, D))   # ragged tail never summarised
        exact = oracle.chunk_mean(K, c)
        f32 = oracle.chunk_mean_fp32(K, c).astype(np.float64)
        amax = np.abs(u16_f64(K)[:, :, :50 * c].reshape(2, 3, 50, c, D)).max(axis=3)
        assert np.all(np.abs(f32 - exact) <= (c + 1) * 2.0 ** -24 * np.maximum(amax, np.abs(exact)))
        two, once = oracle.chunk_mean_bf16(K, c), oracle.chunk_mean_bf16_once(K, c)
        diff = two != once
        assert diff.mean() < 1e-3
        if diff.any():
            ulp = 2.0 ** (np.floor(np.log2(np.abs(once[diff]))) - 7)
            assert np.all(np.abs(two[diff] - once[diff]) <= ulp * 1.0000001)
    K = np.repeat(_rand_u16(rng, (1, 2, 5, 1, D)), 8, axis=3).reshape(1, 2, 40, D)
    assert np.array_equal(oracle.chunk_mean_bf16(K, 8), u16_f64(K[:, :, ::8]))
