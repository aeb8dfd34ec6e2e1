"""End to end: Algorithm 1 (both speculation levels, cache updates, retrieval rebuilds) driving a toy
attention language model whose every attention, cache write, chunk summary, chunk selection and
accept step runs through the C-ABI calls. The method's claim is that the output is that of the
target model (Sec. 4.2): at temperature 0 the generated tokens must equal plain autoregressive
greedy decoding of the target model, which the fp64 oracle computes on the CPU."""
import numpy as np
import pytest
import torch

import paper_2404_11912_amd as tf
from paper_2404_11912_amd.controller import RebuildPolicy, TriForceModelLoop
from tests.toy_lm import ToyLM

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


@pytest.mark.parametrize("g1,g2,stride,seed", [(2, 6, 3, 1), (1, 3, 1, 2), (3, 4, 0, 3)])
def test_hierarchical_speculation_is_lossless_at_temperature_zero(g1, g2, stride, seed):
    say(f"case end-to-end g1={g1} g2={g2} stride={stride} seed={seed}")
    vocab, heads, n_prompt, n_new = 256, 2, 1500, 48
    lm = ToyLM(vocab, heads, capacity=2048, chunk=8, k_chunks=16, window=48, seed=100 + seed)
    g = torch.Generator().manual_seed(200 + seed)
    prompt = torch.randint(0, vocab, (n_prompt,), generator=g).tolist()
    want, gaps = lm.reference_greedy(prompt, n_new)
    assert min(gaps) > 1e-4, "seed gives a near-tie in the target arg-max; pick another"
    lm.prefill(prompt)
    rng = np.random.default_rng(seed)
    loop = TriForceModelLoop(lm.draft_step, lm.retrieval_pass, lm.target_pass,
                             lambda n: rng.random(n, dtype=np.float32), vocab, gamma1=g1, gamma2=g2, temperature=0.0,
                             policy=RebuildPolicy(stride=stride), on_update=lm.commit)
    got = loop.generate(n_new)
    st = loop.stats
    say(f"[end-to-end] {len(got)} tokens in {st['outer_steps']} verification steps "
        f"({len(got) / st['outer_steps']:.2f} tokens per step), level-1 acceptance "
        f"{st['accepted_l1']}/{st['drafted_l1']}, level-2 acceptance {st['accepted_l2']}/{st['drafted_l2']}, "
        f"{st['rebuilds']} rebuilds; smallest arg-max gap of the reference {min(gaps):.2e}")
    assert got[:n_new] == want
    assert lm.committed == prompt + got
    if stride:
        assert st["rebuilds"] >= 1


def test_sampling_mode_runs_and_counts_are_consistent():
    """Temperature 0.8: no token-by-token reference exists for a stochastic run; the loop's
    bookkeeping must be consistent and every emitted token valid."""
    say("case end-to-end sampling")
    vocab = 256
    lm = ToyLM(vocab, 2, capacity=1024, chunk=8, k_chunks=8, window=32, seed=321)
    g = torch.Generator().manual_seed(322)
    prompt = torch.randint(0, vocab, (600,), generator=g).tolist()
    lm.prefill(prompt)
    rng = np.random.default_rng(9)
    loop = TriForceModelLoop(lm.draft_step, lm.retrieval_pass, lm.target_pass,
                             lambda n: rng.random(n, dtype=np.float32), vocab, gamma1=2, gamma2=4, temperature=0.8,
                             policy=RebuildPolicy(stride=2), on_update=lm.commit)
    got = loop.generate(40)
    st = loop.stats
    assert all(0 <= t < vocab for t in got)
    assert len(got) == st["accepted_l2"] + st["outer_steps"] and len(got) >= 40
    assert st["accepted_l1"] <= st["drafted_l1"] and st["accepted_l2"] <= st["drafted_l2"]
    assert lm.committed == prompt + got


def test_first_generated_token_follows_the_target_distribution():
    """Temperature 1: over many runs with fresh uniforms, the first token the hierarchy emits must be
    distributed as the target model's next-token distribution (Sec. 4.2), whatever the two draft
    tiers propose. Chi-square test on a 24-token vocabulary, 4000 runs, fixed seeds."""
    from scipy.stats import chi2
    say("case end-to-end first-token law")
    vocab, runs = 24, 4000
    lm = ToyLM(vocab, 2, capacity=512, chunk=8, k_chunks=4, window=16, seed=555)
    g = torch.Generator().manual_seed(556)
    prompt = torch.randint(0, vocab, (300,), generator=g).tolist()
    lm.prefill(prompt)
    lm.Wo *= 1.5 / float(lm.target_pass([])[0].std())       # a spread-out but not flat distribution
    p = torch.softmax(lm.target_pass([])[0].double(), dim=0).cpu().numpy()
    rng = np.random.default_rng(77)
    counts = np.zeros(vocab)
    acc1 = 0
    for _ in range(runs):
        lm.committed = list(prompt)                         # cache rows of the prompt stay valid
        loop = TriForceModelLoop(lm.draft_step, lm.retrieval_pass, lm.target_pass,
                                 lambda n: rng.random(n, dtype=np.float32), vocab, gamma1=2, gamma2=3, temperature=1.0,
                                 on_update=lm.commit)
        counts[loop.generate(1)[0]] += 1
        acc1 += loop.stats["accepted_l2"] > 0
    keep = p * runs >= 5                                     # cells with enough expected mass; the rest pooled
    obs = np.append(counts[keep], counts[~keep].sum())
    exp = np.append(p[keep], p[~keep].sum()) * runs
    stat = float(((obs - exp) ** 2 / np.maximum(exp, 1e-12)).sum())
    dof = len(obs) - 1
    pval = float(chi2.sf(stat, dof))
    say(f"[end-to-end law] chi2 = {stat:.1f} on {dof} dof, p = {pval:.3f}; first drafted token accepted in "
        f"{acc1}/{runs} runs; largest target probability {p.max():.3f}")
    assert pval > 1e-3
    assert 0.05 * runs < acc1 < 0.999 * runs                 # the drafts are neither useless nor the target itself


def test_batched_hierarchical_speculation_is_lossless_at_temperature_zero():
    """Three sequences of different prompt lengths advancing in lockstep (the batched setting of
    Table 4): per-sequence cache lengths, per-sequence chunk counts and recent ranges, a different
    number of speculated tokens per sequence at the verification (tf_spec_accept_ragged). Each
    sequence must reproduce its own plain greedy decoding."""
    from paper_2404_11912_amd.controller import TriForceBatchLoop
    from tests.toy_lm import ToyLMBatch
    say("case end-to-end batched")
    vocab, heads, n_new, B = 256, 2, 32, 3
    lm = ToyLMBatch(B, vocab, heads, capacity=1536, chunk=8, k_chunks=12, window=40, seed=777)
    g = torch.Generator().manual_seed(778)
    prompts = [torch.randint(0, vocab, (n,), generator=g).tolist() for n in (1200, 433, 900)]
    wants = []
    for p in prompts:
        want, gaps = lm.reference_greedy(p, n_new)
        assert min(gaps) > 1e-4, "seed gives a near-tie in the target arg-max; pick another"
        wants.append(want)
    lm.prefill(prompts)
    rng = np.random.default_rng(4)
    loop = TriForceBatchLoop(B, lm.draft_step, lm.retrieval_pass, lm.target_pass,
                             lambda n: rng.random(n, dtype=np.float32), vocab, gamma1=2, gamma2=4, temperature=0.0,
                             policy=RebuildPolicy(stride=3), on_update=lm.commit)
    got = loop.generate(n_new)
    st = loop.stats
    say(f"[end-to-end batched] {[len(t) for t in got]} tokens in {st['outer_steps']} verification steps, level-2 "
        f"acceptance {st['accepted_l2']}/{st['drafted_l2']}, {st['rebuilds']} rebuilds")
    for b in range(B):
        assert got[b][:n_new] == wants[b]
        assert lm.committed[b] == prompts[b] + got[b]
