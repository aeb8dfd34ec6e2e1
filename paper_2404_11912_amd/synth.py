"""Seeded synthetic inputs for the decode-step attention path.

This module only *draws inputs*: random K/V caches, queries, planted relevant
chunks, logits, draft tokens and uniforms. It holds none of the method's
arithmetic (no attention, no chunk means, no top-k, no accept rule), so both the
CPU oracle's tests and the HIP path's tests may import it.

The shapes stand in for a Llama2-7B-128K decode step (32 layers x 32 MHA heads,
head_dim 128, 4K retrieval budget; Sec. 5.1 "Setup" of the paper); the "few
relevant chunks among many irrelevant ones" structure stands in for the needle
retrieval workload of Sec. 4.1 / Table 1. No dataset item is reproduced.

bf16 tensors are returned as torch.bfloat16; `as_u16` gives the raw bit pattern
as a numpy uint16 array (numpy has no bf16 type) for the CPU oracle.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

HEAD_DIM = 128


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: B sequences, L layers, H heads, context N, chunk
    size c, retrieval budget R (tokens), G = gamma+1 verify queries, G_d draft
    queries, vocab V, P planted chunks per (b, layer, head)."""
    name: str
    index: int
    B: int
    L: int
    H: int
    N: int
    c: int
    R: int
    G: int
    V: int
    P: int
    G_d: int = 3
    temps: tuple = (0.6,)
    d: int = HEAD_DIM

    @property
    def M(self) -> int:
        return self.N // self.c

    @property
    def k(self) -> int:
        return self.R // self.c

    @property
    def gamma(self) -> int:
        return self.G - 1

    def kv_bytes_per_layer(self) -> int:
        return 2 * self.B * self.H * self.N * self.d * 2


# The five configurations this build is specified on (index = position in that list), then
# three more.
WORKLOADS = {
    "tiny": Workload("tiny", 0, B=1, L=1, H=4, N=4096, c=8, R=512, G=5, V=1000, P=8),
    "layer32k": Workload("layer32k", 1, B=1, L=1, H=32, N=32768, c=8, R=4096, G=6, V=32000, P=64),
    "step128k": Workload("step128k", 2, B=1, L=32, H=32, N=131072, c=8, R=4096, G=5, V=32000,
                         P=64, temps=(0.0, 0.6, 1.0)),
    "extreme1m": Workload("extreme1m", 3, B=1, L=8, H=32, N=1048576, c=16, R=8192, G=5, V=32000,
                          P=512),
    "batch4x64k": Workload("batch4x64k", 4, B=4, L=32, H=32, N=65536, c=8, R=4096, G=5, V=32000,
                           P=64),
    # beyond the five: the batch shapes of the paper's batching table (Table 4: batch x context
    # with the per-sequence retrieval budget it lists), same model shape
    "batch2x56k": Workload("batch2x56k", 5, B=2, L=32, H=32, N=57344, c=8, R=1024, G=5, V=32000,
                           P=64, temps=(0.0, 0.6)),
    "batch6x19k": Workload("batch6x19k", 6, B=6, L=32, H=32, N=19456, c=8, R=768, G=5, V=32000,
                           P=48, temps=(0.0, 0.6)),
    "batch10x12k": Workload("batch10x12k", 7, B=10, L=32, H=32, N=12288, c=8, R=768, G=5, V=32000,
                            P=48, temps=(0.0, 0.6)),
}


def seed_for(w: Workload, layer: int = 0, b: int = 0) -> int:
    return 11912 + 1000 * w.index + 17 * layer + 101 * b


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def as_u16(t: torch.Tensor) -> np.ndarray:
    """Raw bf16 bit patterns of a torch.bfloat16 tensor as a contiguous numpy uint16 array."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def make_layer(B: int, H: int, N: int, G: int, c: int, P: int, seed: int,
               device="cpu", d: int = HEAD_DIM, q_std: float | None = None,
               plant_gain: float = 3.0, plant_noise: float = 0.5):
    """One layer's inputs.

    K, V   bf16 [B,H,N,d], i.i.d. N(0,1)
    Q      bf16 [B,H,G,d], N(0,1)/sqrt(d) (softmax scale folded in; callers use scale=1)
    q_r    bf16 [B,H,d]  = Q[:, :, G-1]  (the query that scores the chunks)
    planted int64 [B,H,P]: distinct chunk ids whose keys were overwritten by
           plant_gain * q_r/|q_r| + N(0, plant_noise^2) per component.
    """
    dev = torch.device(device)
    g = _gen(seed, dev)
    q_std = (1.0 / np.sqrt(d)) if q_std is None else q_std
    Q = (torch.randn(B, H, G, d, generator=g, device=dev, dtype=torch.float32) * q_std).to(torch.bfloat16)
    K = torch.empty(B, H, N, d, device=dev, dtype=torch.bfloat16)
    V = torch.empty(B, H, N, d, device=dev, dtype=torch.bfloat16)
    # head by head so the fp32 staging buffer stays small at long contexts
    for b in range(B):
        for h in range(H):
            K[b, h] = torch.randn(N, d, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
            V[b, h] = torch.randn(N, d, generator=g, device=dev, dtype=torch.float32).to(torch.bfloat16)
    q_r = Q[:, :, G - 1, :].contiguous()
    M = N // c
    planted = torch.empty(B, H, P, dtype=torch.int64, device=dev)
    if P > 0:
        assert P <= M
        qf = q_r.to(torch.float32)
        qhat = qf / qf.norm(dim=-1, keepdim=True).clamp_min(1e-20)
        for b in range(B):
            for h in range(H):
                ids = torch.randperm(M, generator=g, device=dev)[:P]
                planted[b, h] = ids
                rows = (ids[:, None] * c + torch.arange(c, device=dev)[None, :]).reshape(-1)
                noise = torch.randn(P * c, d, generator=g, device=dev, dtype=torch.float32) * plant_noise
                K[b, h, rows] = (plant_gain * qhat[b, h][None, :] + noise).to(torch.bfloat16)
    return {"Q": Q, "K": K, "V": V, "q_r": q_r, "planted": planted}


def make_workload_layer(w: Workload, layer: int, device="cpu"):
    """Layer `layer` of workload `w`; per-sequence seeds when B > 1."""
    if w.B == 1:
        return make_layer(1, w.H, w.N, w.G, w.c, w.P, seed_for(w, layer), device, w.d)
    parts = [make_layer(1, w.H, w.N, w.G, w.c, w.P, seed_for(w, layer, b), device, w.d)
             for b in range(w.B)]
    return {k: torch.cat([p[k] for p in parts], dim=0) for k in parts[0]}


def make_accept_inputs(B: int, gamma: int, V: int, temperature: float, seed: int,
                       correlated: bool = False, logit_std: float = 2.0,
                       corr_noise: float = 0.5, device="cpu"):
    """Inputs of the accept/resample step.

    target_logits fp32 [B,gamma+1,V] ~ N(0, logit_std^2)
    draft_logits  fp32 [B,gamma,V]   independent of the target, or (correlated)
                  target + N(0, corr_noise^2) so late rejects / all-accepted occur
    draft_tokens  int32 [B,gamma]   drawn from softmax(draft_logits/T) (arg-max at T=0)
    u_accept      fp32 [B,gamma] in [0,1);  u_sample fp32 [B] in [0,1)
    Drawn on the CPU generator (small tensors), then moved to `device`.
    """
    g = _gen(seed, "cpu")
    G = gamma + 1
    tl = torch.randn(B, G, V, generator=g, dtype=torch.float32) * logit_std
    if correlated:
        dl = tl[:, :gamma, :] + torch.randn(B, gamma, V, generator=g, dtype=torch.float32) * corr_noise
    else:
        dl = torch.randn(B, gamma, V, generator=g, dtype=torch.float32) * logit_std
    dl = dl.contiguous()
    if gamma > 0:
        if temperature > 0:
            probs = torch.softmax(dl.double() / temperature, dim=-1)
            toks = torch.multinomial(probs.reshape(B * gamma, V), 1, generator=g).reshape(B, gamma)
        else:
            toks = dl.argmax(dim=-1)
    else:
        toks = torch.zeros(B, 0, dtype=torch.int64)
    ua = torch.rand(B, gamma, generator=g, dtype=torch.float32)
    us = torch.rand(B, generator=g, dtype=torch.float32)
    dev = torch.device(device)
    return {"target_logits": tl.to(dev), "draft_logits": dl.to(dev),
            "draft_tokens": toks.to(torch.int32).to(dev), "u_accept": ua.to(dev),
            "u_sample": us.to(dev), "temperature": float(temperature)}
