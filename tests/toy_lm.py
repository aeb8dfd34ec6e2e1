"""A toy one-layer attention language model for end-to-end tests of Algorithm 1 (test harness, not
part of the library). Per-token query / key / value tables plus a position table, one multi-head
attention layer over a KV cache, a linear read-out to logits. All attention, cache writes, chunk
summaries and chunk selection run through the library's C-ABI calls on the GPU; the same model is
also evaluated step by step on the CPU with the fp64 oracle (`reference_greedy`), from the same
tables, so that the two share no arithmetic beyond elementwise table look-ups.

Three tiers as in Algorithm 1, all sharing the weights and the full KV cache:
  target     M_p over the full cache                    (tf_decode_attn_full)
  retrieval  M_p over selected chunks + recent tokens   (tf_decode_attn_indexed, chunks from
             tf_chunk_summarize + tf_chunk_topk_gather)
  draft      a StreamingLLM-style cache: the first chunk (sinks) + a recent window
             (tf_decode_attn_indexed)
Invariant: the cache rows [0, len(committed) - 1) hold the committed tokens; the last committed
token has not been fed yet. A pass feeds that token (or the last speculated one) plus new ones.
"""
import numpy as np
import torch

import paper_2404_11912_amd as tf

D = 128


class ToyLM:
    def __init__(self, vocab, heads, capacity, chunk, k_chunks, window, seed, device="cuda"):
        g = torch.Generator().manual_seed(seed)
        self.V, self.H, self.cap, self.c, self.kc, self.win = vocab, heads, capacity, chunk, k_chunks, window
        self.dev = torch.device(device)
        r = lambda *shape: torch.randn(shape, generator=g)
        self.Qtab = (r(vocab, heads, D) * 0.2).to(self.dev)
        self.Ktab = r(vocab, heads, D).to(self.dev)
        self.Vtab = r(vocab, heads, D).to(self.dev)
        self.Pq = (r(capacity, D) * 0.2).to(self.dev)                 # position tables (independent for queries
        self.Pk = (r(capacity, D) * 0.5).to(self.dev)                 # and keys), shared by the heads
        self.Wo = (r(heads * D, vocab) * 0.5).to(self.dev)
        self.K = torch.zeros((1, heads, capacity, D), dtype=torch.bfloat16, device=self.dev)
        self.V_ = torch.zeros_like(self.K)
        self.Kmean = torch.zeros((1, heads, capacity // chunk, D), dtype=torch.float32, device=self.dev)
        self.idx = torch.full((1, heads, k_chunks), -1, dtype=torch.int32, device=self.dev)
        self.sink = torch.zeros((1, heads, 1), dtype=torch.int32, device=self.dev)
        self.committed, self.rb, self.summarized = [], 0, 0

    # ---- elementwise look-ups (identical on CPU and GPU: one IEEE add, one rounding to bf16) ----
    def qkv(self, tokens, pos0, tabs=None):
        Qtab, Ktab, Vtab, Pq, Pk = tabs or (self.Qtab, self.Ktab, self.Vtab, self.Pq, self.Pk)
        t = torch.as_tensor(tokens, dtype=torch.long, device=Qtab.device)
        pq = Pq[pos0:pos0 + len(tokens)][:, None, :]
        pk = Pk[pos0:pos0 + len(tokens)][:, None, :]
        q = (Qtab[t] + pq).to(torch.bfloat16).permute(1, 0, 2)[None].contiguous()      # [1,H,n,D]
        k = (Ktab[t] + pk).to(torch.bfloat16).permute(1, 0, 2)[None].contiguous()
        v = Vtab[t].to(torch.bfloat16).permute(1, 0, 2)[None].contiguous()
        return q, k, v

    def _feed(self, tokens, pos0):
        q, k, v = self.qkv(tokens, pos0)
        tf.tf_kv_append(k, v, self.K, self.V_, pos_all=pos0)
        return q

    def _logits(self, O):                                              # [1,H,G,D] fp32 -> [G,V]
        G = O.shape[2]
        return (O[0].permute(1, 0, 2).reshape(G, self.H * D) @ self.Wo).contiguous()

    # ---- the three tiers -------------------------------------------------------------------
    def prefill(self, prompt):
        self.committed = list(prompt)
        self._feed(prompt[:-1], 0)
        self.rebuild()

    def rebuild(self):
        """Summaries of the chunks completed by committed tokens, then chunk selection by the query of
        the last committed token (Sec. 4.1); tokens behind the last complete chunk count as recent."""
        n_rows = len(self.committed) - 1
        n_chunks = n_rows // self.c
        if n_chunks > self.summarized:
            tf.tf_chunk_summarize(self.K, self.c, self.Kmean, self.summarized, n_chunks - self.summarized)
            self.summarized = n_chunks
        q, _, _ = self.qkv(self.committed[-1:], n_rows)
        k = min(self.kc, n_chunks)
        self.idx.fill_(-1)
        if k > 0:
            sel = torch.empty((1, self.H, k), dtype=torch.int32, device=self.dev)
            tf.tf_chunk_topk_gather(q[:, :, 0].contiguous(), self.Kmean, self.K, self.V_, self.c, k, sel,
                                    n_chunks_all=n_chunks)
            self.idx[:, :, :k] = sel
        self.rb = n_chunks * self.c

    def target_pass(self, spec):
        fed = [self.committed[-1]] + list(spec)
        pos0 = len(self.committed) - 1
        Q = self._feed(fed, pos0)
        O = torch.empty(Q.shape, dtype=torch.float32, device=self.dev)
        tf.tf_decode_attn_full(Q, self.K, self.V_, O, kv_len_all=pos0 + len(fed), scale=1.0, causal=True)
        return self._logits(O)

    def retrieval_pass(self, spec, new):
        prev = spec[-1] if spec else self.committed[-1]
        fed = [prev] + list(new)
        pos0 = len(self.committed) - 1 + len(spec)
        Q = self._feed(fed, pos0)
        O = torch.empty(Q.shape, dtype=torch.float32, device=self.dev)
        tf.tf_decode_attn_indexed(Q, self.K, self.V_, self.idx, self.c, O, kv_len_all=pos0 + len(fed),
                                  recent_begin_all=self.rb, scale=1.0, causal=True)
        return self._logits(O)

    def draft_step(self, spec):
        prev = spec[-1] if spec else self.committed[-1]
        pos0 = len(self.committed) - 1 + len(spec)
        Q = self._feed([prev], pos0)
        O = torch.empty(Q.shape, dtype=torch.float32, device=self.dev)
        length = pos0 + 1
        tf.tf_decode_attn_indexed(Q, self.K, self.V_, self.sink, self.c, O, kv_len_all=length,
                                  recent_begin_all=max(self.c, length - self.win), scale=1.0, causal=True)
        return self._logits(O)[0].contiguous()

    def commit(self, tokens, rebuild):
        self.committed += list(tokens)
        if rebuild:
            self.rebuild()

    # ---- plain autoregressive greedy decoding of the target model on the CPU (fp64 oracle) -----
    def reference_greedy(self, prompt, n_new):
        import oracle
        from paper_2404_11912_amd import synth
        tabs = tuple(t.cpu() for t in (self.Qtab, self.Ktab, self.Vtab, self.Pq, self.Pk))
        Wo = self.Wo.cpu().double().numpy()
        toks = list(prompt)
        _, k, v = self.qkv(toks, 0, tabs)
        Kc, Vc = [synth.as_u16(k)], [synth.as_u16(v)]
        gaps = []
        for _ in range(n_new):
            L = len(toks)
            q, _, _ = self.qkv(toks[-1:], L - 1, tabs)
            O, _, _ = oracle.attention(synth.as_u16(q), np.concatenate(Kc, axis=2), np.concatenate(Vc, axis=2),
                                       scale=1.0, causal=False)
            logits = O[0].transpose(1, 0, 2).reshape(1, self.H * D) @ Wo
            order = np.argsort(-logits[0], kind="stable")
            gaps.append(float(logits[0, order[0]] - logits[0, order[1]]))
            toks.append(int(order[0]))
            _, k, v = self.qkv(toks[-1:], L, tabs)
            Kc.append(synth.as_u16(k))
            Vc.append(synth.as_u16(v))
        return toks[len(prompt):], gaps


class ToyLMBatch(ToyLM):
    """The same toy model for a batch of sequences of different lengths advancing in lockstep.
    Rectangular calls: token lists are padded BEHIND the real tokens (token 0); the bottom-right
    causal mask hides the padding from the real queries, whose outputs stay left-aligned."""

    def __init__(self, batch, *args, **kwargs):
        super().__init__(*args, **kwargs)
        B = self.B = batch
        self.K = torch.zeros((B, self.H, self.cap, D), dtype=torch.bfloat16, device=self.dev)
        self.V_ = torch.zeros_like(self.K)
        self.Kmean = torch.zeros((B, self.H, self.cap // self.c, D), dtype=torch.float32, device=self.dev)
        self.idx = torch.full((B, self.H, self.kc), -1, dtype=torch.int32, device=self.dev)
        self.sink = torch.zeros((B, self.H, 1), dtype=torch.int32, device=self.dev)
        self.committed = [[] for _ in range(B)]
        self.rb = torch.zeros((B,), dtype=torch.int32, device=self.dev)

    def _i32(self, v):
        return torch.tensor(v, dtype=torch.int32, device=self.dev)

    def _feed_batch(self, fed, pos0):
        """fed: per-sequence token lists, pos0: per-sequence first position. Returns Q [B,H,n,D]
        (n = longest list) after writing the K/V rows of all (padded) tokens."""
        n = max(len(f) for f in fed)
        qs, ks, vs = [], [], []
        for b in range(self.B):
            q, k, v = self.qkv(list(fed[b]) + [0] * (n - len(fed[b])), pos0[b])
            qs.append(q); ks.append(k); vs.append(v)
        Q, Kn, Vn = torch.cat(qs), torch.cat(ks), torch.cat(vs)
        tf.tf_kv_append(Kn, Vn, self.K, self.V_, pos=self._i32(pos0))
        return Q, n

    def prefill(self, prompts):
        self.committed = [list(p) for p in prompts]
        for b, p in enumerate(prompts):
            _, k, v = self.qkv(p[:-1], 0)
            self.K[b:b + 1, :, :len(p) - 1] = k
            self.V_[b:b + 1, :, :len(p) - 1] = v
        self.rebuild()

    def rebuild(self):
        n_rows = [len(c) - 1 for c in self.committed]
        n_chunks = [r // self.c for r in n_rows]
        top = max(n_chunks)
        self.idx.fill_(-1)
        if top > 0:
            tf.tf_chunk_summarize(self.K, self.c, self.Kmean, 0, top)
            q = torch.cat([self.qkv(self.committed[b][-1:], n_rows[b])[0] for b in range(self.B)])
            k = min(self.kc, top)
            sel = torch.empty((self.B, self.H, k), dtype=torch.int32, device=self.dev)
            tf.tf_chunk_topk_gather(q[:, :, 0].contiguous(), self.Kmean, self.K, self.V_, self.c, k, sel,
                                    n_chunks=self._i32(n_chunks), n_chunks_all=top)
            self.idx[:, :, :k] = sel
        self.rb = self._i32([n * self.c for n in n_chunks])

    def target_pass(self, specs):
        fed = [[self.committed[b][-1]] + list(specs[b]) for b in range(self.B)]
        pos0 = [len(self.committed[b]) - 1 for b in range(self.B)]
        Q, n = self._feed_batch(fed, pos0)
        O = torch.empty(Q.shape, dtype=torch.float32, device=self.dev)
        tf.tf_decode_attn_full(Q, self.K, self.V_, O, kv_len=self._i32([p + n for p in pos0]),
                               kv_len_all=max(pos0) + n, scale=1.0, causal=True)
        return torch.stack([self._logits(O[b:b + 1]) for b in range(self.B)])

    def retrieval_pass(self, specs, news):
        fed = [[specs[b][-1] if specs[b] else self.committed[b][-1]] + list(news[b]) for b in range(self.B)]
        pos0 = [len(self.committed[b]) - 1 + len(specs[b]) for b in range(self.B)]
        Q, n = self._feed_batch(fed, pos0)
        O = torch.empty(Q.shape, dtype=torch.float32, device=self.dev)
        tf.tf_decode_attn_indexed(Q, self.K, self.V_, self.idx, self.c, O, kv_len=self._i32([p + n for p in pos0]),
                                  kv_len_all=max(pos0) + n, recent_begin=self.rb,
                                  recent_begin_all=int(self.rb.min().item()), scale=1.0, causal=True)
        return torch.stack([self._logits(O[b:b + 1]) for b in range(self.B)])

    def draft_step(self, specs):
        fed = [[specs[b][-1] if specs[b] else self.committed[b][-1]] for b in range(self.B)]
        pos0 = [len(self.committed[b]) - 1 + len(specs[b]) for b in range(self.B)]
        Q, _ = self._feed_batch(fed, pos0)
        O = torch.empty(Q.shape, dtype=torch.float32, device=self.dev)
        lens = [p + 1 for p in pos0]
        rbs = [max(self.c, L - self.win) for L in lens]
        tf.tf_decode_attn_indexed(Q, self.K, self.V_, self.sink, self.c, O, kv_len=self._i32(lens),
                                  kv_len_all=max(lens), recent_begin=self._i32(rbs), recent_begin_all=min(rbs),
                                  scale=1.0, causal=True)
        return torch.stack([self._logits(O[b:b + 1])[0] for b in range(self.B)]).contiguous()

    def commit(self, emitted, rebuild):
        for b in range(self.B):
            self.committed[b] += list(emitted[b])
        if rebuild:
            self.rebuild()
