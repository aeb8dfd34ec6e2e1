"""Pins for the oracle's attention (CPU only).

The paper prints no worked numeric example, so the oracle is pinned by closed forms,
invariants, special cases and a library softmax on tiny inputs. Each pin is chosen so that
one plausible mistake (dropped scale, wrong causal offset, transposed operand, swapped
query/key index, un-normalised weights) fails it.
"""
import math

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

import oracle
from tests.util import bf16_u16, u16_f64

D = 128


def _rand_u16(rng, shape, std=1.0):
    return bf16_u16(rng.standard_normal(shape) * std)


def test_rows_sum_to_one():
    rng = np.random.default_rng(0)
    Q = _rand_u16(rng, (2, 3, 4, D), 0.3)
    K = _rand_u16(rng, (2, 3, 70, D))
    V = _rand_u16(rng, (2, 3, 70, D))
    _, _, ws = oracle.attention(Q, K, V, scale=1.0, causal=True)
    assert np.max(np.abs(ws - 1.0)) < 1e-12


@pytest.mark.parametrize("causal", [True, False])
def test_scale_zero_is_prefix_mean(causal):
    """scale = 0 makes every visible key equally likely: O_g = mean(V[0:n_g]), LSE_g = log n_g.
    This pins the bottom-right causal alignment n_g = kv_len - G + 1 + g exactly."""
    rng = np.random.default_rng(1)
    B, H, G, N = 2, 2, 5, 37
    kv = np.array([37, 21], dtype=np.int32)
    Q = _rand_u16(rng, (B, H, G, D))
    K = _rand_u16(rng, (B, H, N, D))
    V = _rand_u16(rng, (B, H, N, D))
    O, LSE, _ = oracle.attention(Q, K, V, kv_len=kv, scale=0.0, causal=causal)
    Vf = u16_f64(V)
    for b in range(B):
        for g in range(G):
            n_g = kv[b] - G + 1 + g if causal else kv[b]
            want = Vf[b, :, :n_g, :].mean(axis=1)
            assert np.max(np.abs(O[b, :, g, :] - want)) < 1e-13
            assert np.max(np.abs(LSE[b, :, g] - math.log(n_g))) < 1e-13


def test_two_key_closed_form():
    """q = e_0, k_0 = 2 e_0, k_1 = 0, scale = ln(3)/2: weights are exactly 3/4 and 1/4,
    LSE = ln 4. Pins the use of `scale`, the exponential and the V weighting."""
    rng = np.random.default_rng(2)
    q = np.zeros((1, 1, 1, D)); q[..., 0] = 1.0
    K = np.zeros((1, 1, 2, D)); K[0, 0, 0, 0] = 2.0
    V = _rand_u16(rng, (1, 1, 2, D))
    O, LSE, _ = oracle.attention(bf16_u16(q), bf16_u16(K), V, scale=math.log(3.0) / 2.0, causal=False)
    Vf = u16_f64(V)
    want = 0.75 * Vf[0, 0, 0] + 0.25 * Vf[0, 0, 1]
    assert np.max(np.abs(O[0, 0, 0] - want)) < 1e-14
    assert abs(LSE[0, 0, 0] - math.log(4.0)) < 1e-14


def test_one_hot_routing():
    """Q_g = 64 e_g and K_t = e_{pi(t)}: query g puts all its weight on the key with
    pi(t) = g, so O_g = V[pi^-1(g)]. Fails if query/key/dim indices are mixed up."""
    rng = np.random.default_rng(3)
    G, N = 4, 8
    pi = rng.permutation(N)
    Q = np.zeros((1, 1, G, D)); K = np.zeros((1, 1, N, D))
    for g in range(G):
        Q[0, 0, g, g] = 64.0
    for t in range(N):
        K[0, 0, t, pi[t]] = 1.0
    V = _rand_u16(rng, (1, 1, N, D))
    O, LSE, _ = oracle.attention(bf16_u16(Q), bf16_u16(K), V, scale=1.0, causal=False)
    Vf = u16_f64(V)
    for g in range(G):
        t = int(np.where(pi == g)[0][0])
        assert np.max(np.abs(O[0, 0, g] - Vf[0, 0, t])) < 1e-20 + 8 * math.exp(-64.0) * 10
        assert abs(LSE[0, 0, g] - 64.0) < 1e-12


def test_identical_keys_and_single_token():
    rng = np.random.default_rng(4)
    Q = _rand_u16(rng, (1, 2, 3, D))
    krow = _rand_u16(rng, (1, 2, 1, D))
    K = np.repeat(krow, 16, axis=2)
    V = _rand_u16(rng, (1, 2, 16, D))
    O, _, _ = oracle.attention(Q, K, V, scale=0.7, causal=False)
    want = u16_f64(V).mean(axis=2)
    for g in range(3):
        assert np.max(np.abs(O[:, :, g, :] - want)) < 1e-13
    # N = 1, G = 1: the output is V[0] and LSE is the single logit
    O1, L1, _ = oracle.attention(Q[:, :, :1], K[:, :, :1], V[:, :, :1], scale=0.7, causal=True)
    assert np.array_equal(O1[:, :, 0, :], u16_f64(V)[:, :, 0, :])
    z = 0.7 * np.einsum("bhd,bhd->bh", u16_f64(Q)[:, :, 0], u16_f64(K)[:, :, 0])
    assert np.max(np.abs(L1[:, :, 0] - z)) < 1e-13


def test_dominant_key_selects_its_value():
    """One key whose logit is 50 above all others takes (almost) all the weight."""
    rng = np.random.default_rng(5)
    N = 40
    q = np.zeros((1, 1, 1, D)); q[..., 3] = 1.0
    K = rng.standard_normal((1, 1, N, D)); K[..., 3] = 0.0
    K[0, 0, 17, 3] = 50.0
    V = _rand_u16(rng, (1, 1, N, D))
    O, _, _ = oracle.attention(bf16_u16(q), bf16_u16(K), V, scale=1.0, causal=False)
    assert np.max(np.abs(O[0, 0, 0] - u16_f64(V)[0, 0, 17])) < 1e-18


def test_key_shift_invariance():
    """Adding one vector to every key shifts all logits of a query equally: O is unchanged,
    LSE moves by scale * <q, shift>. Values are chosen exactly representable in bf16."""
    rng = np.random.default_rng(6)
    Q = np.round(rng.standard_normal((1, 2, 3, D)) * 4) / 8
    K = np.round(rng.standard_normal((1, 2, 33, D)) * 4) / 4
    V = _rand_u16(rng, (1, 2, 33, D))
    shift = np.round(rng.standard_normal((1, 2, 1, D)) * 4) / 4
    O0, L0, _ = oracle.attention(bf16_u16(Q), bf16_u16(K), V, scale=0.5, causal=True)
    O1, L1, _ = oracle.attention(bf16_u16(Q), bf16_u16(K + shift), V, scale=0.5, causal=True)
    assert np.max(np.abs(O0 - O1)) < 1e-12
    dz = 0.5 * np.einsum("bhgd,bhd->bhg", Q, shift[:, :, 0])
    assert np.max(np.abs((L1 - L0) - dz)) < 1e-11


def test_split_halves_merge_by_lse():
    """Attention over [0,N) equals the LSE-weighted merge of attention over two halves."""
    rng = np.random.default_rng(7)
    Q = _rand_u16(rng, (1, 2, 4, D), 0.2)
    K = _rand_u16(rng, (1, 2, 64, D))
    V = _rand_u16(rng, (1, 2, 64, D))
    O, L, _ = oracle.attention(Q, K, V, scale=1.0, causal=False)
    Oa, La, _ = oracle.attention(Q, K[:, :, :24], V[:, :, :24], scale=1.0, causal=False)
    Ob, Lb, _ = oracle.attention(Q, K[:, :, 24:], V[:, :, 24:], scale=1.0, causal=False)
    Lm = np.logaddexp(La, Lb)
    Om = np.exp(La - Lm)[..., None] * Oa + np.exp(Lb - Lm)[..., None] * Ob
    assert np.max(np.abs(Om - O)) < 1e-12
    assert np.max(np.abs(Lm - L)) < 1e-12


@pytest.mark.parametrize("causal", [True, False])
def test_matches_library_softmax_on_tiny_inputs(causal):
    """numpy einsum + scipy.special.softmax / logsumexp on a tiny case, with ragged kv_len."""
    rng = np.random.default_rng(8)
    B, H, G, N = 2, 3, 4, 19
    kv = np.array([19, 11], dtype=np.int32)
    Q = _rand_u16(rng, (B, H, G, D), 0.4)
    K = _rand_u16(rng, (B, H, N, D))
    V = _rand_u16(rng, (B, H, N, D))
    scale = 0.37
    O, L, _ = oracle.attention(Q, K, V, kv_len=kv, scale=scale, causal=causal)
    Qf, Kf, Vf = u16_f64(Q), u16_f64(K), u16_f64(V)
    for b in range(B):
        z = scale * np.einsum("hgd,htd->hgt", Qf[b], Kf[b])
        t = np.arange(N)[None, None, :]
        g = np.arange(G)[None, :, None]
        vis = (t < kv[b] - G + 1 + g) if causal else (t < kv[b] + 0 * g)
        z = np.where(vis, z, -np.inf)
        want = np.einsum("hgt,htd->hgd", softmax(z, axis=-1), Vf[b])
        assert np.max(np.abs(O[b] - want)) < 1e-12
        assert np.max(np.abs(L[b] - logsumexp(z, axis=-1))) < 1e-12


def test_bad_arguments_raise():
    Q = np.zeros((1, 1, 4, D), np.uint16)
    K = np.zeros((1, 1, 8, D), np.uint16)
    with pytest.raises(ValueError):
        oracle.attention(Q, K, K, kv_len=[-1], causal=True)  # negative length
    with pytest.raises(ValueError):
        oracle.attention(Q, K, K, kv_len=[9], causal=False)  # beyond capacity


def test_grouped_query_oracle_reduces_to_per_head_attention():
    """Grouped-query attention: query head q uses KV head q // q_group. Pinned head by head against
    the plain attention on the sliced arrays, and for q_group = 1 against the plain call itself."""
    rng = np.random.default_rng(77)
    B, Hkv, qg, G, N = 2, 3, 4, 3, 50
    Q = _rand_u16(rng, (B, Hkv * qg, G, D), 0.3)
    K = _rand_u16(rng, (B, Hkv, N, D))
    V = _rand_u16(rng, (B, Hkv, N, D))
    kv = np.array([50, 17], dtype=np.int32)
    O, L = oracle.attention_gqa(Q, K, V, kv_len=kv, scale=0.8, causal=True)
    for q in range(Hkv * qg):
        h = q // qg
        o, l, _ = oracle.attention(np.ascontiguousarray(Q[:, q:q + 1]), np.ascontiguousarray(K[:, h:h + 1]),
                                   np.ascontiguousarray(V[:, h:h + 1]), kv_len=kv, scale=0.8, causal=True)
        assert np.array_equal(O[:, q:q + 1], o) and np.array_equal(L[:, q:q + 1], l)
    # a wrong grouping (q % Hkv instead of q // q_group) would differ
    o_wrong, _, _ = oracle.attention(np.ascontiguousarray(Q[:, 1:2]), np.ascontiguousarray(K[:, 1:2]),
                                     np.ascontiguousarray(V[:, 1:2]), kv_len=kv, scale=0.8, causal=True)
    assert np.max(np.abs(O[:, 1:2] - o_wrong)) > 1e-6
    Q1 = np.ascontiguousarray(Q[:, :Hkv])
    O1, L1 = oracle.attention_gqa(Q1, K, V, kv_len=kv, scale=0.8, causal=False)
    O2, L2, _ = oracle.attention(Q1, K, V, kv_len=kv, scale=0.8, causal=False)
    assert np.array_equal(O1, O2) and np.array_equal(L1, L2)


def test_sequences_shorter_than_the_query_block_and_empty_sequences():
    """kv_len < G with the causal mask, and kv_len = 0: query g sees max(0, kv_len - G + 1 + g) keys;
    a query that sees none gets O = 0 and LSE = -inf (the library's documented convention). Pinned by
    the scale-0 closed form and by the independently coded tree-mask path with the chain mask."""
    rng = np.random.default_rng(91)
    B, H, G, N = 4, 2, 5, 12
    kv = np.array([12, 0, 2, 5], dtype=np.int32)
    Q = _rand_u16(rng, (B, H, G, D), 0.3)
    K = _rand_u16(rng, (B, H, N, D))
    V = _rand_u16(rng, (B, H, N, D))
    O, LSE, ws = oracle.attention(Q, K, V, kv_len=kv, scale=0.0, causal=True)
    Vf = u16_f64(V)
    for b in range(B):
        for g in range(G):
            n_g = max(0, int(kv[b]) - G + 1 + g)
            if n_g == 0:
                assert np.all(O[b, :, g] == 0.0) and np.all(np.isneginf(LSE[b, :, g])) and np.all(ws[b, :, g] == 0.0)
            else:
                assert np.max(np.abs(O[b, :, g] - Vf[b, :, :n_g].mean(axis=1))) < 1e-13
                assert np.max(np.abs(LSE[b, :, g] - math.log(n_g))) < 1e-13
    O1, L1, _ = oracle.attention(Q, K, V, kv_len=kv, scale=0.9, causal=True)
    O2, L2 = oracle.attention_tree(Q, K, V, [(2 << g) - 1 for g in range(G)], kv_len=kv, scale=0.9)
    assert np.max(np.abs(O1 - O2)) < 1e-13
    assert np.array_equal(np.isneginf(L1), np.isneginf(L2))
    fin = np.isfinite(L1)
    assert np.max(np.abs(L1[fin] - L2[fin])) < 1e-13
    O3, L3, _ = oracle.attention(Q, K, V, kv_len=np.array([3, 0, 0, 1], dtype=np.int32), scale=1.0, causal=False)
    assert np.all(O3[1:3] == 0.0) and np.all(np.isneginf(L3[1:3])) and np.all(np.isfinite(L3[[0, 3]]))
