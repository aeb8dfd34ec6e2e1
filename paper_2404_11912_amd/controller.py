"""Host controller of the hierarchical speculation loop (Algorithm 1) and the retrieval-cache
rebuild policy (Sec. 4.3). Host logic only: every accept / resample decision and every draw
runs in `tf_spec_accept` on the GPU; the three "models" are callbacks returning logits, so the
controller works with real forward passes as well as with synthetic logits tables.

Notation follows Algorithm 1: M_q is the small draft model (logits q_i), M_p with the retrieval
cache gives p-hat_i, M_p with the full cache gives p_i; gamma1 / gamma2 are the two speculation
lengths; N counts generated tokens.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

from . import binding as tf


@dataclass
class RebuildPolicy:
    """When to rebuild the retrieval cache (Sec. 4.3): at a fixed stride of verification steps,
    or when the running mean of the acceptance rate at the verification level falls below a
    threshold. stride = 0 / threshold = 0 switch the respective trigger off."""
    stride: int = 0
    threshold: float = 0.0
    window: int = 16
    _steps: int = 0
    _hist: list = field(default_factory=list)

    def update(self, accepted: int, drafted: int) -> bool:
        self._steps += 1
        if drafted > 0:
            self._hist.append(accepted / drafted)
            self._hist = self._hist[-self.window:]
        by_stride = self.stride > 0 and self._steps % self.stride == 0
        by_rate = (self.threshold > 0.0 and len(self._hist) == self.window
                   and sum(self._hist) / len(self._hist) < self.threshold)
        if by_stride or by_rate:
            self._hist = []
            return True
        return False


class TriForceController:
    """Algorithm 1 for one sequence.

    draft_fn(pos, n)     -> fp32 logits [n, V] of M_q for generated positions pos .. pos+n-1
    retrieval_fn(pos, n) -> fp32 logits [n, V] of M_p over the retrieval cache (p-hat)
    target_fn(pos, n)    -> fp32 logits [n, V] of M_p over the full cache (p)
    uniform(n)           -> n fp32 uniforms in [0,1) as a numpy array (the caller's seeded source;
                            consumed in a fixed order so a reference can replay them)
    on_update(tokens, rebuild) is called after every verification with the newly fixed tokens.
    """

    def __init__(self, draft_fn, retrieval_fn, target_fn, uniform, vocab: int, gamma1: int = 2, gamma2: int = 6,
                 temperature: float = 0.6, policy: RebuildPolicy | None = None, on_update=None, device="cuda"):
        if gamma1 < 1 or gamma2 < 1 or gamma1 + gamma2 + 1 > tf.TF_MAX_SPEC:
            raise ValueError("need 1 <= gamma1, gamma2 and gamma1 + gamma2 + 1 <= TF_MAX_SPEC")
        self.draft_fn, self.retrieval_fn, self.target_fn, self.uniform = draft_fn, retrieval_fn, target_fn, uniform
        self.V, self.g1, self.g2, self.T = vocab, gamma1, gamma2, float(temperature)
        self.policy, self.on_update, self.dev = policy or RebuildPolicy(), on_update, torch.device(device)
        self.ws = tf.workspace(tf.tf_spec_accept_workspace_bytes(gamma1, tf.TF_MAX_SPEC, vocab), self.dev)
        self.stats = {"outer_steps": 0, "inner_steps": 0, "drafted_l1": 0, "accepted_l1": 0, "drafted_l2": 0,
                      "accepted_l2": 0, "rebuilds": 0}

    def _u(self, n):
        return torch.from_numpy(np.ascontiguousarray(self.uniform(n), dtype=np.float32)).to(self.dev)

    def _accept(self, target_logits, draft_logits, draft_tokens, u_accept, u_sample):
        """One tf_spec_accept call for a single sequence; returns (n_accepted, emitted tokens list)."""
        G = target_logits.shape[0]
        n = torch.empty((1,), dtype=torch.int32, device=self.dev)
        out = torch.empty((1, G), dtype=torch.int32, device=self.dev)
        tf.tf_spec_accept(target_logits[None].contiguous(),
                          None if G == 1 else draft_logits[None].contiguous(),
                          None if G == 1 else draft_tokens[None].contiguous(), self.T,
                          None if G == 1 else u_accept[None].contiguous(), u_sample, n, out, ws=self.ws)
        n_acc = int(n.item())
        return n_acc, out[0, :n_acc + 1].tolist()

    def _sample_rows(self, logits, u):
        """Draw one token from every row of `logits` (rows ride in the batch dimension, G = 1)."""
        rows = logits.shape[0]
        n = torch.empty((rows,), dtype=torch.int32, device=self.dev)
        out = torch.empty((rows, 1), dtype=torch.int32, device=self.dev)
        tf.tf_spec_accept(logits[:, None, :].contiguous(), None, None, self.T, None, u, n, out, ws=self.ws)
        return out[:, 0].contiguous()

    def generate(self, n_tokens: int):
        """Run Algorithm 1 until at least n_tokens are generated; returns the token list."""
        tokens, N = [], 0
        while N < n_tokens:
            n, x_hat = 0, []
            while n < self.g2:                                   # first level: M_q drafts for M_p(C_r)
                base = N + n
                q = self.draft_fn(base, self.g1)
                x_tilde = self._sample_rows(q, self._u(self.g1))
                p_hat = self.retrieval_fn(base, self.g1 + 1)
                n1, emitted = self._accept(p_hat, q, x_tilde, self._u(self.g1), self._u(1))
                x_hat += emitted
                n += n1 + 1
                self.stats["inner_steps"] += 1
                self.stats["drafted_l1"] += self.g1
                self.stats["accepted_l1"] += n1
            p = self.target_fn(N, n + 1)                         # second level: M_p(C_p) verifies x_hat
            p_hat_all = self.retrieval_fn(N, n)
            xs = torch.tensor(x_hat, dtype=torch.int32, device=self.dev)
            n2, emitted = self._accept(p, p_hat_all, xs, self._u(n), self._u(1))
            tokens += emitted
            N += n2 + 1
            self.stats["outer_steps"] += 1
            self.stats["drafted_l2"] += n
            self.stats["accepted_l2"] += n2
            rebuild = self.policy.update(n2, n)
            self.stats["rebuilds"] += int(rebuild)
            if self.on_update is not None:
                self.on_update(emitted, rebuild)
        return tokens


class TriForceModelLoop(TriForceController):
    """Algorithm 1 for models whose next-token distribution depends on the tokens fed so far (real
    forward passes with KV caches), where the position-indexed callbacks above do not suffice.
    `spec` always denotes the tokens speculated in the current outer iteration, after the committed
    sequence the model object keeps itself.

    draft_fn(spec)            -> fp32 logits [V]: M_q's distribution of the token after committed + spec
    retrieval_fn(spec, new)   -> fp32 logits [len(new)+1, V]: M_p over the retrieval cache, for the
                                 positions after committed + spec + new[:i], i = 0 .. len(new)
    target_fn(spec)           -> fp32 logits [len(spec)+1, V]: M_p over the full cache
    on_update(tokens, rebuild)   the verified tokens to append to the committed sequence
    """

    def generate(self, n_tokens: int):
        tokens, N = [], 0
        while N < n_tokens:
            x_hat, p_hat_rows = [], []
            while len(x_hat) < self.g2:                          # first level
                x_tilde, q_rows = [], []
                for _ in range(self.g1):                         # M_q drafts token by token
                    q = self.draft_fn(x_hat + x_tilde)
                    q_rows.append(q)
                    x_tilde.append(int(self._sample_rows(q[None], self._u(1))[0].item()))
                q = torch.stack(q_rows)
                p_hat = self.retrieval_fn(list(x_hat), list(x_tilde))
                xt = torch.tensor(x_tilde, dtype=torch.int32, device=self.dev)
                n1, emitted = self._accept(p_hat, q, xt, self._u(self.g1), self._u(1))
                x_hat += emitted
                p_hat_rows.append(p_hat[:n1 + 1])                # the rows that fixed these tokens
                self.stats["inner_steps"] += 1
                self.stats["drafted_l1"] += self.g1
                self.stats["accepted_l1"] += n1
            n = len(x_hat)
            p = self.target_fn(list(x_hat))                      # second level
            xs = torch.tensor(x_hat, dtype=torch.int32, device=self.dev)
            n2, emitted = self._accept(p, torch.cat(p_hat_rows), xs, self._u(n), self._u(1))
            tokens += emitted
            N += n2 + 1
            self.stats["outer_steps"] += 1
            self.stats["drafted_l2"] += n
            self.stats["accepted_l2"] += n2
            rebuild = self.policy.update(n2, n)
            self.stats["rebuilds"] += int(rebuild)
            if self.on_update is not None:
                self.on_update(emitted, rebuild)
        return tokens


class TriForceBatchLoop(TriForceController):
    """Algorithm 1 for a batch of sequences advancing in lockstep (the batched setting of Sec. 5.1 /
    Table 4). The first level repeats until every sequence holds at least gamma2 speculated tokens;
    a sequence that already does sits the remaining inner iterations out (its slot still rides
    through the calls, the results are ignored). The verification then sees a different number of
    tokens per sequence, which `tf_spec_accept_ragged` handles; models pad the shorter sequences
    BEHIND their real tokens, so the bottom-right causal mask keeps the padding invisible.

    draft_fn(specs)          -> fp32 logits [B, V]   (specs: per sequence, the tokens speculated so far)
    retrieval_fn(specs, new) -> fp32 logits [B, gamma1+1, V]
    target_fn(specs)         -> fp32 logits [B, max_b len(specs[b]) + 1, V], rows left-aligned
    on_update(emitted, rebuild): per-sequence lists of verified tokens, one rebuild flag for the batch
    """

    def __init__(self, batch: int, *args, **kwargs):
        super().__init__(*args, **kwargs)
        self.B = batch
        self.ws = tf.workspace(tf.tf_spec_accept_workspace_bytes(batch, tf.TF_MAX_SPEC, self.V), self.dev)

    def _accept_batch(self, target_logits, draft_logits, draft_tokens, n_draft=None):
        B, G = target_logits.shape[:2]
        n = torch.empty((B,), dtype=torch.int32, device=self.dev)
        out = torch.empty((B, G), dtype=torch.int32, device=self.dev)
        ua = self._u(B * (G - 1)).view(B, G - 1)
        us = self._u(B)
        if n_draft is None:
            tf.tf_spec_accept(target_logits, draft_logits, draft_tokens, self.T, ua, us, n, out, ws=self.ws)
        else:
            tf.tf_spec_accept_ragged(target_logits, draft_logits, draft_tokens, n_draft, self.T, ua, us, n, out,
                                     ws=self.ws)
        return n.tolist(), out.tolist()

    def generate(self, n_tokens: int):
        B = self.B
        tokens = [[] for _ in range(B)]
        while min(len(t) for t in tokens) < n_tokens:
            x_hat = [[] for _ in range(B)]
            rows = [[] for _ in range(B)]
            while min(len(x) for x in x_hat) < self.g2:          # first level
                active = [len(x) < self.g2 for x in x_hat]
                x_tilde = [[] for _ in range(B)]
                q_rows = []
                for _ in range(self.g1):
                    q = self.draft_fn([x_hat[b] + x_tilde[b] for b in range(B)])
                    q_rows.append(q)
                    drawn = self._sample_rows(q, self._u(B)).tolist()
                    for b in range(B):
                        x_tilde[b].append(drawn[b])
                q = torch.stack(q_rows, dim=1).contiguous()                  # [B, g1, V]
                p_hat = self.retrieval_fn([list(x) for x in x_hat], [list(x) for x in x_tilde]).contiguous()
                xt = torch.tensor(x_tilde, dtype=torch.int32, device=self.dev)
                n1, out = self._accept_batch(p_hat, q, xt)
                for b in range(B):
                    if active[b]:
                        x_hat[b] += out[b][:n1[b] + 1]
                        rows[b].append(p_hat[b, :n1[b] + 1])
                        self.stats["drafted_l1"] += self.g1
                        self.stats["accepted_l1"] += n1[b]
                self.stats["inner_steps"] += 1
            n_b = [len(x) for x in x_hat]
            Gm = max(n_b) + 1
            p = self.target_fn([list(x) for x in x_hat]).contiguous()        # second level
            d = torch.zeros((B, Gm - 1, self.V), dtype=torch.float32, device=self.dev)
            xs = torch.zeros((B, Gm - 1), dtype=torch.int32, device=self.dev)
            for b in range(B):
                d[b, :n_b[b]] = torch.cat(rows[b])
                xs[b, :n_b[b]] = torch.tensor(x_hat[b], dtype=torch.int32, device=self.dev)
            n2, out = self._accept_batch(p, d, xs, torch.tensor(n_b, dtype=torch.int32, device=self.dev))
            emitted = [out[b][:n2[b] + 1] for b in range(B)]
            for b in range(B):
                tokens[b] += emitted[b]
            self.stats["outer_steps"] += 1
            self.stats["drafted_l2"] += sum(n_b)
            self.stats["accepted_l2"] += sum(n2)
            rebuild = self.policy.update(sum(n2), sum(n_b))
            self.stats["rebuilds"] += int(rebuild)
            if self.on_update is not None:
                self.on_update(emitted, rebuild)
        return tokens
