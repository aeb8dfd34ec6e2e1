"""Pins for the oracle's transcription of Algorithm 1 and for the rebuild policy (CPU only)."""
import numpy as np

from oracle.triforce_loop import triforce_generate
from paper_2404_11912_amd.controller import RebuildPolicy


def _tables(rng, n_pos, V, corr=None, std=2.0):
    t = (rng.standard_normal((n_pos, V)) * std).astype(np.float32)
    if corr is None:
        r = (rng.standard_normal((n_pos, V)) * std).astype(np.float32)
        d = (rng.standard_normal((n_pos, V)) * std).astype(np.float32)
    else:
        r = (t + rng.standard_normal((n_pos, V)) * corr).astype(np.float32)
        d = (t + rng.standard_normal((n_pos, V)) * 3 * corr).astype(np.float32)
    return d, r, t


def _uniform(seed):
    rng = np.random.default_rng(seed)
    return lambda n: rng.random(n, dtype=np.float32)


def test_greedy_output_is_the_target_models_argmax_whatever_the_drafts():
    """Losslessness at T = 0 (Sec. 4.2 'Correctness'): both speculation levels may propose
    anything, the generated sequence is what the target model alone would produce."""
    rng = np.random.default_rng(40)
    d, r, t = _tables(rng, 80, 50)
    for g1, g2 in ((2, 6), (1, 1), (4, 3)):
        tokens, stats = triforce_generate(d, r, t, _uniform(1), 40, g1, g2, 0.0)
        assert len(tokens) >= 40
        assert tokens == t.argmax(axis=1)[:len(tokens)].tolist()
        assert stats["accepted_l2"] <= stats["drafted_l2"]


def test_identical_models_accept_every_token():
    rng = np.random.default_rng(41)
    t = (rng.standard_normal((100, 30)) * 2).astype(np.float32)
    tokens, stats = triforce_generate(t, t, t, _uniform(2), 50, 2, 6, 0.8)
    assert stats["accepted_l1"] == stats["drafted_l1"] and stats["accepted_l2"] == stats["drafted_l2"]
    # each inner iteration then yields gamma1 + 1 tokens, so n = 6 after two of them; each outer step fixes n + 1
    assert stats["inner_steps"] == 2 * stats["outer_steps"] and len(tokens) == 7 * stats["outer_steps"]


def test_monte_carlo_output_law_is_the_target_models():
    """T = 1, vocabulary 5, unrelated drafts at both levels: over many runs every one of the first
    eight generated tokens -- they span several inner iterations, corrections, bonus tokens and at
    least two verification passes -- is distributed as softmax(target row of its position)
    (chi-square, 4 dof per position). The tables are indexed by position only, so the joint law is
    the product of these marginals: this is the whole losslessness claim of Sec. 4.2 for this case."""
    rng = np.random.default_rng(42)
    V, runs, n_pos = 5, 5000, 8
    for seed, (g1, g2) in ((3, (2, 3)), (4, (2, 6))):
        d, r, t = _tables(rng, 32, V, std=1.0)
        p = np.exp(t[:n_pos].astype(np.float64)); p /= p.sum(axis=1, keepdims=True)
        uni = _uniform(seed)
        counts = np.zeros((n_pos, V))
        for _ in range(runs):
            tokens, _ = triforce_generate(d, r, t, uni, n_pos, g1, g2, 1.0)
            for i in range(n_pos):
                counts[i, tokens[i]] += 1
        chi2 = ((counts - runs * p) ** 2 / (runs * p)).sum(axis=1)
        assert chi2.max() < 27.9, (g1, g2, chi2)      # P(chi2_4 > 27.9) ~ 1.3e-5 per position


def test_acceptance_rates_follow_the_closed_form():
    """Acceptance frequency at a fixed position is sum_v min(p, q) (one minus the total variation
    distance): the first drafted token of the first inner iteration is accepted at level 1 with
    sum min(p_hat_0, q_0), whatever happens later."""
    rng = np.random.default_rng(43)
    V, runs = 6, 8000
    d, r, t = _tables(rng, 16, V, std=1.0)
    sm = lambda x: np.exp(x.astype(np.float64)) / np.exp(x.astype(np.float64)).sum()
    want = np.minimum(sm(r[0]), sm(d[0])).sum()
    uni = _uniform(5)
    first_accepted = 0
    for _ in range(runs):
        # gamma1 = 1, gamma2 = 1: one inner iteration per outer step, so accepted_l1 of a 1-step run is that event
        _, stats = triforce_generate(d, r, t, uni, 1, 1, 1, 1.0)
        first_accepted += stats["accepted_l1"] > 0
    se = np.sqrt(want * (1 - want) / runs)
    assert abs(first_accepted / runs - want) < 4.5 * se


def test_rebuild_policy_triggers():
    pol = RebuildPolicy(stride=3)
    assert [pol.update(4, 6) for _ in range(7)] == [False, False, True, False, False, True, False]
    pol = RebuildPolicy(threshold=0.5, window=4)
    fired = [pol.update(a, 6) for a in (6, 6, 6, 6, 1, 1, 1, 1, 1)]
    assert fired == [False, False, False, False, False, False, True, False, False]
