"""Algorithm 1 driven by the GPU accept kernel (controller.TriForceController) against the
oracle's transcription, on synthetic logits tables and the same stream of uniforms."""
import numpy as np
import pytest
import torch

from oracle.triforce_loop import triforce_generate
from paper_2404_11912_amd.controller import RebuildPolicy, TriForceController

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _tables(seed, n_pos, V, corr):
    rng = np.random.default_rng(seed)
    t = (rng.standard_normal((n_pos, V)) * 2).astype(np.float32)
    r = (t + rng.standard_normal((n_pos, V)) * corr).astype(np.float32)
    d = (t + rng.standard_normal((n_pos, V)) * 3 * corr).astype(np.float32)
    return d, r, t


def _uniform(seed):
    rng = np.random.default_rng(seed)
    return lambda n: rng.random(n, dtype=np.float32)


@pytest.mark.parametrize("g1,g2,T,V", [(2, 6, 0.6, 1000), (2, 6, 0.0, 1000), (1, 3, 1.0, 32000), (4, 8, 0.6, 257)])
def test_controller_matches_oracle_loop(g1, g2, T, V):
    print(f"case controller g1={g1} g2={g2} T={T} V={V} seed=160", flush=True)
    n_tokens = 48
    d, r, t = _tables(160 + g1, n_tokens + 40, V, corr=0.4)
    Tf = float(np.float32(T))
    want_tokens, want_stats = triforce_generate(d, r, t, _uniform(161), n_tokens, g1, g2, Tf)
    dd, rd, td = (torch.from_numpy(a).to(DEV) for a in (d, r, t))
    updates = []
    ctl = TriForceController(lambda pos, n: dd[pos:pos + n], lambda pos, n: rd[pos:pos + n],
                             lambda pos, n: td[pos:pos + n], _uniform(161), V, gamma1=g1, gamma2=g2,
                             temperature=T, policy=RebuildPolicy(stride=4),
                             on_update=lambda toks, rebuild: updates.append((len(toks), rebuild)), device=DEV)
    tokens = ctl.generate(n_tokens)
    assert tokens == want_tokens
    for k, v in want_stats.items():
        assert ctl.stats[k] == v, k
    assert sum(n for n, _ in updates) == len(tokens)
    assert ctl.stats["rebuilds"] == ctl.stats["outer_steps"] // 4
    if T == 0.0:
        assert tokens == t.argmax(axis=1)[:len(tokens)].tolist()      # lossless greedy decoding
    print(f"[controller] {len(tokens)} tokens in {ctl.stats['outer_steps']} verification steps, "
          f"level-1 acceptance {ctl.stats['accepted_l1'] / ctl.stats['drafted_l1']:.2f}, "
          f"level-2 acceptance {ctl.stats['accepted_l2'] / ctl.stats['drafted_l2']:.2f}", flush=True)
