"""Pins for the oracle's tree-mask attention (Sec. 5.3.3: verification of a token tree), CPU only.

The tree attention of a node is, by definition, the attention of that node over the context and
its root path. The pins: the chain mask reduces to the (separately pinned) causal attention, the
full mask to the unmasked one, a brute-force softmax written with numpy on tiny inputs, the
independence of a branch from its sibling branch, and the scale-0 closed form (mean of the
visible V rows, LSE = log of their count).
"""
import math

import numpy as np
from scipy.special import logsumexp, softmax

import oracle
from tests.util import bf16_u16, u16_f64

D = 128


def _rand_u16(rng, shape, std=1.0):
    return bf16_u16(rng.standard_normal(shape) * std)


def _inputs(seed, B=2, H=2, G=5, N=40):
    rng = np.random.default_rng(seed)
    return _rand_u16(rng, (B, H, G, D), 0.3), _rand_u16(rng, (B, H, N, D)), _rand_u16(rng, (B, H, N, D))


# a tree over 6 speculated tokens: 0 root; 1, 2 children of 0; 3 child of 1; 4 child of 2; 5 child of 4
PARENT = [-1, 0, 0, 1, 2, 4]


def ancestor_masks(parent):
    masks = []
    for g in range(len(parent)):
        m, a = 0, g
        while a >= 0:
            m |= 1 << a
            a = parent[a]
        masks.append(m)
    return masks


def test_chain_mask_is_causal_attention():
    Q, K, V = _inputs(0)
    G = Q.shape[2]
    kv = np.array([40, 23], dtype=np.int32)
    Ot, Lt = oracle.attention_tree(Q, K, V, [(2 << g) - 1 for g in range(G)], kv_len=kv, scale=0.7)
    Oc, Lc, _ = oracle.attention(Q, K, V, kv_len=kv, scale=0.7, causal=True)
    assert np.max(np.abs(Ot - Oc)) < 1e-13 and np.max(np.abs(Lt - Lc)) < 1e-13


def test_full_mask_is_unmasked_attention():
    Q, K, V = _inputs(1)
    G = Q.shape[2]
    Ot, Lt = oracle.attention_tree(Q, K, V, [(1 << G) - 1] * G, scale=1.0)
    On, Ln, _ = oracle.attention(Q, K, V, scale=1.0, causal=False)
    assert np.max(np.abs(Ot - On)) < 1e-13 and np.max(np.abs(Lt - Ln)) < 1e-13


def test_tree_against_numpy_softmax():
    """Brute force: a dense [G, N] visibility matrix and a library softmax."""
    Q, K, V = _inputs(2, B=1, H=3, G=6, N=19)
    masks = ancestor_masks(PARENT)
    G, N = 6, 19
    O, L = oracle.attention_tree(Q, K, V, masks, scale=0.9)
    Qf, Kf, Vf = u16_f64(Q), u16_f64(K), u16_f64(V)
    vis = np.zeros((G, N), dtype=bool)
    vis[:, :N - G] = True
    for g in range(G):
        for j in range(G):
            vis[g, N - G + j] = bool((masks[g] >> j) & 1)
    for h in range(3):
        z = 0.9 * Qf[0, h] @ Kf[0, h].T
        z[~vis] = -np.inf
        assert np.max(np.abs(softmax(z, axis=1) @ Vf[0, h] - O[0, h])) < 1e-12
        assert np.max(np.abs(logsumexp(z, axis=1) - L[0, h])) < 1e-12


def test_a_branch_does_not_see_its_sibling():
    """Nodes 1 and 3 (one branch) must not change when the K/V rows of nodes 2, 4, 5 (the other
    branch) are replaced; nodes 4 and 5 must change."""
    Q, K, V = _inputs(3, B=1, H=2, G=6, N=30)
    masks = ancestor_masks(PARENT)
    O1, L1 = oracle.attention_tree(Q, K, V, masks)
    rng = np.random.default_rng(33)
    K2, V2 = K.copy(), V.copy()
    for j in (2, 4, 5):
        K2[:, :, 30 - 6 + j] = _rand_u16(rng, (1, 2, D))
        V2[:, :, 30 - 6 + j] = _rand_u16(rng, (1, 2, D))
    O2, L2 = oracle.attention_tree(Q, K2, V2, masks)
    for g in (0, 1, 3):
        assert np.array_equal(O1[:, :, g], O2[:, :, g]) and np.array_equal(L1[:, :, g], L2[:, :, g])
    for g in (2, 4, 5):
        assert np.max(np.abs(O1[:, :, g] - O2[:, :, g])) > 1e-6


def test_scale_zero_counts_the_visible_rows():
    Q, K, V = _inputs(4, B=2, H=1, G=6, N=25)
    kv = np.array([25, 9], dtype=np.int32)
    masks = ancestor_masks(PARENT)
    O, L = oracle.attention_tree(Q, K, V, masks, kv_len=kv, scale=0.0)
    Vf = u16_f64(V)
    for b in range(2):
        n = int(kv[b])
        for g in range(6):
            rows = list(range(n - 6)) + [n - 6 + j for j in range(6) if (masks[g] >> j) & 1]
            assert np.max(np.abs(O[b, 0, g] - Vf[b, 0, rows].mean(axis=0))) < 1e-13
            assert abs(L[b, 0, g] - math.log(len(rows))) < 1e-13


def test_query_that_sees_nothing():
    Q, K, V = _inputs(5, B=1, H=1, G=3, N=3)
    O, L = oracle.attention_tree(Q, K, V, [0b001, 0b000, 0b101])
    assert np.all(O[0, 0, 1] == 0.0) and L[0, 0, 1] == -np.inf
    assert np.isfinite(L[0, 0, 0]) and np.isfinite(L[0, 0, 2])
