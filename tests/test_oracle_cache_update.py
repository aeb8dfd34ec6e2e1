"""Pins for the oracle's gather-free (indexed) draft attention and cache append (CPU only)."""
import numpy as np

import oracle
from tests.util import bf16_u16

D = 128


def _rand_u16(rng, shape, std=1.0):
    return bf16_u16(rng.standard_normal(shape) * std)


def test_indexed_with_all_chunks_in_order_is_plain_attention():
    rng = np.random.default_rng(30)
    B, H, G, N, c = 2, 2, 3, 64, 8
    Q = _rand_u16(rng, (B, H, G, D), 0.3); K = _rand_u16(rng, (B, H, N, D)); V = _rand_u16(rng, (B, H, N, D))
    idx = np.broadcast_to(np.arange(N // c - 1), (B, H, N // c - 1))   # the last chunk is the recent range
    O, L = oracle.attention_indexed(Q, K, V, idx, c, recent_begin=N - c, causal=True)
    Op, Lp, _ = oracle.attention(Q, K, V, causal=True)
    assert np.array_equal(O, Op) and np.array_equal(L, Lp)        # same rows in the same order


def test_indexed_chunks_then_recent_rows_cover_the_cache():
    """Chunks [0, 5) in a shuffled order plus the recent rows [40, 61): every row once, the G
    queries' own tokens last, so causal attention equals plain causal attention over 61 tokens."""
    rng = np.random.default_rng(31)
    B, H, G, N, c = 1, 3, 4, 64, 8
    Q = _rand_u16(rng, (B, H, G, D), 0.3); K = _rand_u16(rng, (B, H, N, D)); V = _rand_u16(rng, (B, H, N, D))
    idx = np.stack([rng.permutation(5) for _ in range(H)])[None]
    O, L = oracle.attention_indexed(Q, K, V, idx, c, kv_len=[61], recent_begin=[40], causal=True)
    Op, Lp, _ = oracle.attention(Q, K, V, kv_len=[61], causal=True)
    assert np.max(np.abs(O - Op)) < 1e-12 and np.max(np.abs(L - Lp)) < 1e-12


def test_indexed_equals_attention_over_the_gathered_cache_plus_appended_rows():
    rng = np.random.default_rng(32)
    B, H, G, N, c, k = 2, 2, 2, 96, 4, 6
    Q = _rand_u16(rng, (B, H, G, D), 0.3); K = _rand_u16(rng, (B, H, N, D)); V = _rand_u16(rng, (B, H, N, D))
    idx = np.stack([np.stack([rng.permutation(20)[:k] for _ in range(H)]) for _ in range(B)]).astype(np.int32)
    idx[0, 1, 2] = -1                                                  # a skipped slot
    kv, rb = np.array([96, 90]), np.array([88, 85])
    O, L = oracle.attention_indexed(Q, K, V, idx, c, kv_len=kv, recent_begin=rb, causal=True)
    for b in range(B):
        for h in range(H):
            keep = [m for m in idx[b, h] if m >= 0]
            Kr, Vr = oracle.gather(K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], np.array(keep)[None, None], c)
            Kc = np.concatenate([Kr, K[b:b + 1, h:h + 1, rb[b]:kv[b]]], axis=2)
            Vc = np.concatenate([Vr, V[b:b + 1, h:h + 1, rb[b]:kv[b]]], axis=2)
            o, l, _ = oracle.attention(Q[b:b + 1, h:h + 1], Kc, Vc, causal=True)
            assert np.array_equal(O[b, h], o[0, 0]) and np.array_equal(L[b, h], l[0, 0])


def test_kv_append_hand_example():
    K = np.zeros((2, 1, 6, D), np.uint16); V = np.zeros_like(K)
    Kn = np.full((2, 1, 2, D), 7, np.uint16); Kn[:, :, 1] = 9
    Vn = Kn + 1
    K2, V2 = oracle.kv_append(Kn, Vn, K, V, [1, 5])
    assert K2[0, 0, :, 0].tolist() == [0, 7, 9, 0, 0, 0] and V2[0, 0, :, 0].tolist() == [0, 8, 10, 0, 0, 0]
    assert K2[1, 0, :, 0].tolist() == [0, 0, 0, 0, 0, 7]              # second row falls off the end: dropped
    assert not K.any()                                                # inputs untouched
