"""Plain transcription of Algorithm 1 (hierarchical speculation) on top of the oracle's accept
rule. TEST INFRASTRUCTURE. The three models are logits tables indexed by generated position, so
the process is defined without any network: row `pos` of each table is the distribution that
model assigns to the token at generated position `pos`.

Uniforms are consumed in this order, which the GPU controller under test must follow:
  inner iteration: gamma1 (draft sampling), gamma1 (level-1 accept tests), 1 (level-1 draw);
  after the inner loop: n (level-2 accept tests), 1 (level-2 draw).
"""
from __future__ import annotations

import numpy as np

from .tf_oracle import accept


def _draw(logits_row, T, u):
    """One token from softmax(logits/T) by inverse CDF (arg-max at T = 0): the accept rule with
    no drafted token draws exactly that."""
    n, out, _, _ = accept(logits_row[None, None, :], np.zeros((1, 0, logits_row.shape[0]), np.float32),
                          np.zeros((1, 0), np.int32), T, np.zeros((1, 0), np.float32), np.array([u], np.float32))
    return int(out[0, 0])


def triforce_generate(draft_table, retrieval_table, target_table, uniform, n_tokens, gamma1, gamma2, T):
    """Algorithm 1. Tables are float32 [positions, V]; `uniform(n)` yields the next n uniforms.
    Returns (tokens, stats) with stats = counts of drafted / accepted tokens at both levels."""
    tokens, N = [], 0
    stats = {"outer_steps": 0, "inner_steps": 0, "drafted_l1": 0, "accepted_l1": 0, "drafted_l2": 0, "accepted_l2": 0}
    while N < n_tokens:
        n, x_hat = 0, []
        while n < gamma2:
            base = N + n
            q = draft_table[base:base + gamma1]
            u_draft = uniform(gamma1)
            x_tilde = np.array([_draw(q[i], T, u_draft[i]) for i in range(gamma1)], np.int32)
            p_hat = retrieval_table[base:base + gamma1 + 1]
            u_acc, u_smp = uniform(gamma1), uniform(1)
            n1, out, _, _ = accept(p_hat[None], q[None], x_tilde[None], T, u_acc[None], u_smp)
            n1 = int(n1[0])
            x_hat += out[0, :n1 + 1].tolist()
            n += n1 + 1
            stats["inner_steps"] += 1
            stats["drafted_l1"] += gamma1
            stats["accepted_l1"] += n1
        p = target_table[N:N + n + 1]
        p_hat_all = retrieval_table[N:N + n]
        u_acc, u_smp = uniform(n), uniform(1)
        n2, out, _, _ = accept(p[None], p_hat_all[None], np.array(x_hat, np.int32)[None], T, u_acc[None], u_smp)
        n2 = int(n2[0])
        tokens += out[0, :n2 + 1].tolist()
        N += n2 + 1
        stats["outer_steps"] += 1
        stats["drafted_l2"] += n
        stats["accepted_l2"] += n2
    return tokens, stats
