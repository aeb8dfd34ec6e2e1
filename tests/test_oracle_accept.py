"""Pins for the oracle's speculative accept / resample step (CPU only).

The rule is the standard lossless speculative-sampling rule that Sec. 4.2 ("Correctness")
refers to. Closed forms used below come from that rule's analysis: with target p and draft
q at one position, P(accept) = sum_v min(p_v, q_v) and the emitted token is distributed
exactly as p; with fixed rows p_0, p_1, ... the emitted prefix (a_0, .., a_{j-1}, b) of
length j+1 has probability prod_{i<j} min(p_i(a_i), q_i(a_i)) * p_j(b).
"""
import itertools
import json
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "spec_accept_closed_form.json")


def _softmax(x, T):
    z = np.asarray(x, dtype=np.float64) / T
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def _inv_cdf(p, u):
    return int(np.searchsorted(np.cumsum(p), u * p.sum(), side="right"))


def test_identical_distributions_accept_everything():
    rng = np.random.default_rng(20)
    B, G, V = 64, 5, 50
    tl = rng.standard_normal((B, G, V)).astype(np.float32) * 2
    dl = tl[:, :G - 1].copy()
    toks = rng.integers(0, V, (B, G - 1))
    ua = rng.random((B, G - 1)).astype(np.float32)
    ua[0, :] = np.float32(1.0) - np.float32(2.0 ** -24)      # the largest float below 1
    us = rng.random(B).astype(np.float32)
    n, out, _, _ = oracle.accept(tl, dl, toks, 0.6, ua, us)
    assert np.all(n == G - 1)
    assert np.array_equal(out[:, :G - 1], toks)
    # the bonus token is the inverse CDF of the last target row
    for b in range(B):
        assert out[b, G - 1] == _inv_cdf(_softmax(tl[b, G - 1], 0.6), float(us[b]))


def test_disjoint_supports_reject_at_once_and_draw_from_target():
    rng = np.random.default_rng(21)
    B, V = 200, 8
    tl = np.full((B, 2, V), -np.inf, dtype=np.float32)
    dl = np.full((B, 1, V), -np.inf, dtype=np.float32)
    tl[:, :, :4] = rng.standard_normal((B, 2, 4))
    dl[:, :, 4:] = rng.standard_normal((B, 1, 4))
    toks = rng.integers(4, 8, (B, 1))
    ua = rng.random((B, 1)).astype(np.float32); us = rng.random(B).astype(np.float32)
    n, out, _, _ = oracle.accept(tl, dl, toks, 1.0, ua, us)
    assert np.all(n == 0) and np.all(out[:, 1] == -1)
    for b in range(B):
        assert out[b, 0] == _inv_cdf(_softmax(tl[b, 0], 1.0), float(us[b]))


def test_temperature_zero_is_argmax_comparison():
    rng = np.random.default_rng(22)
    B, G, V = 300, 4, 11
    tl = rng.integers(-3, 4, (B, G, V)).astype(np.float32)        # many exact ties
    dl = rng.integers(-3, 4, (B, G - 1, V)).astype(np.float32)
    am = tl.argmax(axis=-1)                                        # numpy: first maximum
    toks = np.where(rng.random((B, G - 1)) < 0.7, am[:, :G - 1], rng.integers(0, V, (B, G - 1)))
    n, out, ma, ms = oracle.accept(tl, dl, toks, 0.0, np.zeros((B, G - 1)), np.zeros(B))
    for b in range(B):
        ok = (toks[b] == am[b, :G - 1])
        want_n = G - 1 if ok.all() else int(np.argmin(ok))
        assert n[b] == want_n
        assert out[b, :want_n].tolist() == toks[b, :want_n].tolist()
        assert out[b, want_n] == am[b, want_n]
        assert np.all(out[b, want_n + 1:] == -1)
    assert np.all(ma == 1.0) and np.all(ms == 1.0)


def test_accept_test_has_no_division():
    """q(x) = 0 < p(x) accepts for every u; p(x) = 0 rejects, also when q(x) = 0 too."""
    tl = np.array([[[0.0, 0.0, -np.inf], [0.0, 0.0, 0.0]]], dtype=np.float32)
    dl = np.array([[[-np.inf, 0.0, 0.0]]], dtype=np.float32)
    for u in (0.0, 0.999):
        n, _, _, _ = oracle.accept(tl, dl, [[0]], 1.0, [[u]], [0.5])
        assert n[0] == 1
        n, _, _, _ = oracle.accept(tl, dl, [[2]], 1.0, [[u]], [0.5])
        assert n[0] == 0
    dl2 = np.array([[[0.0, 0.0, -np.inf]]], dtype=np.float32)
    n, out, _, _ = oracle.accept(tl, dl2, [[2]], 1.0, [[0.0]], [0.75])
    assert n[0] == 0 and out[0, 0] == 1          # residual is all zero -> falls back to p = (1/2, 1/2, 0)


def test_golden_closed_form_fixture():
    """Hand-worked case stored under tests/golden (p, q over 4 tokens, exact rationals)."""
    with open(GOLDEN) as f:
        gold = json.load(f)
    p = np.array(gold["p"]); q = np.array(gold["q"])
    tl = np.log(p)[None, None, :].repeat(2, axis=1).astype(np.float32)
    dl = np.log(q)[None, None, :].astype(np.float32)
    for case in gold["cases"]:
        n, out, _, _ = oracle.accept(tl, dl, [[case["x"]]], 1.0, [[case["u_accept"]]], [case["u_sample"]])
        assert int(n[0]) == case["n_accepted"], case
        assert out[0].tolist() == case["out_tokens"], case


def test_monte_carlo_first_token_follows_target():
    """Vocab 8, one drafted token, 2e6 trials: the first emitted token is distributed as p
    (chi-square, 7 dof) and the acceptance frequency is sum min(p, q) = 1 - TV(p, q)."""
    rng = np.random.default_rng(23)
    V, B, T = 8, 2_000_000, 0.8
    t_row = np.array([1.2, -0.3, 0.5, 2.0, -1.5, 0.1, 0.9, -0.7], dtype=np.float32)
    d_row = np.array([0.2, 0.8, -0.5, 1.0, 0.3, -1.1, 1.6, -0.2], dtype=np.float32)
    p = _softmax(t_row, T); q = _softmax(d_row, T)
    tl = np.broadcast_to(np.stack([t_row, t_row[::-1]]), (B, 2, V))
    dl = np.broadcast_to(d_row, (B, 1, V))
    toks = rng.choice(V, size=(B, 1), p=q)
    ua = rng.random((B, 1), dtype=np.float32); us = rng.random(B, dtype=np.float32)
    n, out, _, _ = oracle.accept(tl, dl, toks, T, ua, us)
    acc = float((n == 1).mean())
    want_acc = float(np.minimum(p, q).sum())
    assert abs(acc - want_acc) < 4.0 * np.sqrt(want_acc * (1 - want_acc) / B)
    counts = np.bincount(out[:, 0], minlength=V).astype(np.float64)
    chi2 = float(((counts - B * p) ** 2 / (B * p)).sum())
    assert chi2 < 29.9                      # P(chi2_7 > 29.9) ~ 1e-4
    # a wrong residual (e.g. max(q - p, 0)) or sampling the correction from q would shift
    # the law of the first token far beyond this bound
    # bonus token after an accept follows the second target row
    p1 = _softmax(t_row[::-1], T)
    c1 = np.bincount(out[n == 1, 1], minlength=V).astype(np.float64)
    m = c1.sum()
    assert float(((c1 - m * p1) ** 2 / (m * p1)).sum()) < 29.9


def test_exhaustive_sequence_law_on_a_grid():
    """Vocab 3, gamma = 2: enumerate every draft pair and a midpoint grid of the three
    uniforms; the measure of each emitted prefix must match the closed form."""
    T = 1.0
    tl_rows = np.log(np.array([[0.5, 0.3, 0.2], [0.1, 0.6, 0.3], [0.25, 0.25, 0.5]]))
    dl_rows = np.log(np.array([[0.2, 0.5, 0.3], [0.3, 0.3, 0.4]]))
    p = _softmax(tl_rows, T); q = _softmax(dl_rows, T)
    n_u = 48
    grid = (np.arange(n_u) + 0.5) / n_u
    law = {}
    for x0, x1 in itertools.product(range(3), range(3)):
        u0, u1, us = np.meshgrid(grid, grid, grid, indexing="ij")
        B = u0.size
        tl = np.broadcast_to(tl_rows.astype(np.float32), (B, 3, 3))
        dl = np.broadcast_to(dl_rows.astype(np.float32), (B, 2, 3))
        toks = np.broadcast_to(np.array([x0, x1]), (B, 2))
        ua = np.stack([u0.ravel(), u1.ravel()], axis=1)
        n, out, _, _ = oracle.accept(tl, dl, toks, T, ua, us.ravel())
        w = q[0, x0] * q[1, x1] / B
        keys, cnt = np.unique(out, axis=0, return_counts=True)
        for kk, c in zip(keys, cnt):
            key = tuple(int(v) for v in kk if v >= 0)
            law[key] = law.get(key, 0.0) + w * c
    assert abs(sum(law.values()) - 1.0) < 1e-12
    tol = 3.0 / n_u
    first = np.zeros(3)
    for key, pr in law.items():
        first[key[0]] += pr
        # prefix probability, closed form:
        # length 1: token b emitted after rejecting x0:  p0(b) - min(p0(b), q0(b))
        # length 2: a accepted, then b emitted after rejecting x1: min(p0,q0)(a) * (p1(b) - min(p1,q1)(b))
        # length 3: a, b accepted, then bonus c: min(p0,q0)(a) * min(p1,q1)(b) * p2(c)
        m0 = np.minimum(p[0], q[0]); m1 = np.minimum(p[1], q[1])
        if len(key) == 1:
            want = p[0, key[0]] - m0[key[0]]
        elif len(key) == 2:
            want = m0[key[0]] * (p[1, key[1]] - m1[key[1]])
        else:
            want = m0[key[0]] * m1[key[1]] * p[2, key[2]]
        assert abs(pr - want) < tol, (key, pr, want)
    # marginal of the first emitted token is p_0, whatever happens later
    assert np.max(np.abs(first - p[0])) < tol


def test_margins_flag_near_boundary_decisions():
    tl = np.log(np.array([[[0.5, 0.5], [0.5, 0.5]]])).astype(np.float32)
    dl = np.log(np.array([[[0.5, 0.5]]])).astype(np.float32)
    # u * q(x) = 0.25 vs p(x) = 0.5: relative margin 0.5 ; u_sample = 0.25 sits 0.25 from an edge
    n, _, ma, ms = oracle.accept(tl, dl, [[0]], 1.0, [[0.5]], [0.25])
    assert n[0] == 1 and abs(ma[0] - 0.5) < 1e-12 and abs(ms[0] - 0.25) < 1e-12


def test_bad_token_raises():
    tl = np.zeros((1, 2, 4), np.float32); dl = np.zeros((1, 1, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.accept(tl, dl, [[4]], 1.0, [[0.1]], [0.1])


def test_masked_vocabulary_entries_equal_the_compacted_problem():
    """-inf logits have probability 0: the result must be that of the problem with those entries
    removed from the vocabulary (indices mapped back), and no masked token is ever emitted."""
    rng = np.random.default_rng(61)
    V, B, gamma = 40, 200, 3
    mask = np.zeros(V, dtype=bool)
    mask[rng.choice(V, 15, replace=False)] = True
    keep = np.nonzero(~mask)[0]
    t = (rng.standard_normal((B, gamma + 1, V)) * 2).astype(np.float32)
    d = (t[:, :gamma] + rng.standard_normal((B, gamma, V)) * 0.7).astype(np.float32)
    t[..., mask] = -np.inf
    d[..., mask] = -np.inf
    toks_c = rng.integers(0, keep.size, (B, gamma)).astype(np.int32)
    ua = rng.random((B, gamma), dtype=np.float32)
    us = rng.random(B, dtype=np.float32)
    for T in (0.0, 0.8):
        n1, o1, _, _ = oracle.accept(t, d, keep[toks_c].astype(np.int32), T, ua, us)
        n2, o2, _, _ = oracle.accept(np.ascontiguousarray(t[..., keep]), np.ascontiguousarray(d[..., keep]), toks_c, T,
                                     ua, us)
        assert np.array_equal(n1, n2)
        mapped = np.where(o2 >= 0, keep[np.maximum(o2, 0)], -1)
        assert np.array_equal(o1, mapped)
        assert not mask[o1[o1 >= 0]].any()


def test_ragged_accept_is_the_per_sequence_problem():
    """n_draft = G-1 for every sequence reproduces the fixed-length call; a sequence with fewer drafted
    tokens never looks past them: changing its unused trailing rows changes nothing, and with
    n_draft = 0 the token is the inverse-CDF draw from target row 0."""
    rng = np.random.default_rng(71)
    B, G, V = 6, 5, 23
    t = (rng.standard_normal((B, G, V)) * 2).astype(np.float32)
    d = (t[:, :-1] + rng.standard_normal((B, G - 1, V)) * 0.5).astype(np.float32)
    tok = rng.integers(0, V, (B, G - 1)).astype(np.int32)
    ua = rng.random((B, G - 1), dtype=np.float32)
    us = rng.random(B, dtype=np.float32)
    full = oracle.accept(t, d, tok, 0.9, ua, us)
    same = oracle.accept_ragged(t, d, tok, [G - 1] * B, 0.9, ua, us)
    assert np.array_equal(full[0], same[0]) and np.array_equal(full[1], same[1])
    nd = [0, 1, 2, 3, 4, 2]
    r1 = oracle.accept_ragged(t, d, tok, nd, 0.9, ua, us)
    t2, d2, tok2 = t.copy(), d.copy(), tok.copy()
    for b, g in enumerate(nd):
        t2[b, g + 1:] = 7.0
        d2[b, g:] = -3.0
        tok2[b, g:] = 0
    r2 = oracle.accept_ragged(t2, d2, tok2, nd, 0.9, ua, us)
    assert np.array_equal(r1[0], r2[0]) and np.array_equal(r1[1], r2[1])
    assert np.all(r1[0] <= np.array(nd))
    p0 = np.exp(t[0, 0].astype(np.float64) / np.float64(np.float32(0.9)))
    cdf = np.cumsum(p0 / p0.sum())
    assert r1[1][0, 0] == int(np.searchsorted(cdf, float(us[0]), side="right")) and r1[0][0] == 0
    for b, g in enumerate(nd):                       # emitted: accepted tokens, one drawn token, then -1
        n = r1[0][b]
        assert np.array_equal(r1[1][b, :n], tok[b, :n]) and r1[1][b, n] >= 0 and np.all(r1[1][b, n + 1:] == -1)
