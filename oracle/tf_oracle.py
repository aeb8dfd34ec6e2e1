"""ctypes front end of the plain-C fp64 oracle (`tf_oracle.c`).

TEST INFRASTRUCTURE: argument marshalling only; every number comes from the C file.
Arrays are numpy: bf16 tensors travel as uint16 bit patterns, results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tf_oracle.c")
_LIB = os.path.join(_HERE, "libtf_oracle.so")
_lib = None

_i32p = ctypes.POINTER(ctypes.c_int32)
_u16p = ctypes.POINTER(ctypes.c_uint16)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)


def build_oracle(force: bool = False) -> str:
    """Compile tf_oracle.c with gcc (-O2, no fast-math, OpenMP). Returns the .so path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        # TF_ORACLE_LIB: a test that plants a mistake in a copy of tf_oracle.c points the pins at it
        _lib = ctypes.CDLL(os.environ.get("TF_ORACLE_LIB") or build_oracle())
        _lib.orc_num_threads.restype = ctypes.c_int
        for name in ("orc_attention", "orc_chunk_mean", "orc_retrieve", "orc_gather", "orc_accept"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _p(a: np.ndarray, typ):
    return a.ctypes.data_as(typ)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def num_threads() -> int:
    return int(_load().orc_num_threads())


def attention(Q, K, V, kv_len=None, scale: float = 1.0, causal: bool = True):
    """Q [B,H,G,d], K,V [B,H,N,d] uint16(bf16) -> (O f64 [B,H,G,d], LSE f64 [B,H,G], wsum f64 [B,H,G])."""
    Q, K, V = _u16(Q), _u16(K), _u16(V)
    B, H, G, d = Q.shape
    N = K.shape[2]
    assert K.shape == (B, H, N, d) and V.shape == K.shape
    if kv_len is None:
        kv = np.full(B, N, dtype=np.int32)
    else:
        kv = np.ascontiguousarray(np.broadcast_to(np.asarray(kv_len, dtype=np.int32), (B,)))
    O = np.empty((B, H, G, d), dtype=np.float64)
    LSE = np.empty((B, H, G), dtype=np.float64)
    ws = np.empty((B, H, G), dtype=np.float64)
    rc = _load().orc_attention(_p(Q, _u16p), _p(K, _u16p), _p(V, _u16p), B, H, G,
                               ctypes.c_int64(N), d, _p(kv, _i32p), ctypes.c_double(scale),
                               int(bool(causal)), _p(O, _f64p), _p(LSE, _f64p), _p(ws, _f64p))
    if rc != 0:
        raise ValueError("orc_attention: bad argument")
    return O, LSE, ws


def chunk_mean(K, c: int) -> np.ndarray:
    """K [B,H,N,d] uint16(bf16) -> Kmean f64 [B,H,N//c,d]."""
    K = _u16(K)
    B, H, N, d = K.shape
    M = N // c
    out = np.empty((B, H, M, d), dtype=np.float64)
    rc = _load().orc_chunk_mean(_p(K, _u16p), B, H, ctypes.c_int64(N), d, int(c), _p(out, _f64p))
    if rc != 0:
        raise ValueError("orc_chunk_mean: bad argument")
    return out


def round_to_bf16(x) -> np.ndarray:
    """Round float64 values to the nearest bf16 value (8 significant bits, ties to even), returned
    as float64. Written from the format's definition: x = m * 2^e with 0.5 <= |m| < 1, m is
    rounded to a multiple of 2^-8. (Finite, normal-range values only.)"""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)
    return np.ldexp(np.rint(m * 256.0), e - 8)


def chunk_mean_fp32(K, c: int) -> np.ndarray:
    """The average key of every chunk (Sec. 4.1) as an IEEE fp32 computation with a fixed order:
    the chunk's c keys are widened to fp32 and added one after the other in token order to a sum
    that starts at +0, every addition rounded to fp32; then one fp32 division by c. This is the
    value the bf16 table is defined from (see chunk_mean_bf16): a table entry is a quantised code,
    so the precision in which it is decided has to be fixed, and it is fixed to this.
    K [B,H,N,d] uint16(bf16) -> float32 [B,H,N//c,d]."""
    K = _u16(K)
    B, H, N, d = K.shape
    M = N // c
    rows = (K[:, :, :M * c].astype(np.uint32) << 16).view(np.float32).reshape(B, H, M, c, d)
    acc = np.zeros((B, H, M, d), dtype=np.float32)
    for i in range(c):                          # one rounded fp32 addition per key
        acc = (acc + rows[:, :, :, i]).astype(np.float32)
    return (acc / np.float32(c)).astype(np.float32)


def chunk_mean_bf16(K, c: int) -> np.ndarray:
    """Average keys held in bf16 (variant of Sec. 4.1's average-key table). Definition, the same
    on both sides of the parity tests: the fp32 chunk mean of chunk_mean_fp32 (sequential fp32 sum
    in token order, one fp32 division), rounded to bf16 by round-to-nearest-even. Two roundings:
    in rare cases (about one entry in 10^5..10^6) the result differs by one bf16 ulp from the
    exact mean rounded once. Returned as float64 [B,H,M,d] holding bf16-representable values."""
    return round_to_bf16(chunk_mean_fp32(K, c).astype(np.float64))


def chunk_mean_bf16_once(K, c: int) -> np.ndarray:
    """The exact (fp64) chunk mean rounded once to bf16: not the table's definition, kept to state
    how far the two-rounding definition is from it (tests bound the difference)."""
    return round_to_bf16(chunk_mean(K, c))


def retrieve(q_r, Kmean, k: int, n_chunks=None):
    """q_r [B,H,d] uint16(bf16), Kmean f64 [B,H,M,d] -> (scores f64 [B,H,M], idx int32 [B,H,k])."""
    q_r = _u16(q_r)
    Kmean = np.ascontiguousarray(Kmean, dtype=np.float64)
    B, H, M, d = Kmean.shape
    assert q_r.shape == (B, H, d)
    if n_chunks is None:
        nc = np.full(B, M, dtype=np.int32)
    else:
        nc = np.ascontiguousarray(np.broadcast_to(np.asarray(n_chunks, dtype=np.int32), (B,)))
    scores = np.empty((B, H, M), dtype=np.float64)
    idx = np.empty((B, H, k), dtype=np.int32)
    rc = _load().orc_retrieve(_p(q_r, _u16p), _p(Kmean, _f64p), B, H, ctypes.c_int64(M), d,
                              _p(nc, _i32p), int(k), _p(scores, _f64p), _p(idx, _i32p))
    if rc != 0:
        raise ValueError("orc_retrieve: bad argument")
    return scores, idx


def gather(K, V, idx, c: int, R_cap: int | None = None):
    """K,V [B,H,N,d] uint16, idx int32 [B,H,k] -> (Kr, Vr) uint16 [B,H,R_cap,d]; rows >= k*c are zero."""
    K, V = _u16(K), _u16(V)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    B, H, N, d = K.shape
    k = idx.shape[2]
    R_cap = k * c if R_cap is None else int(R_cap)
    Kr = np.zeros((B, H, R_cap, d), dtype=np.uint16)
    Vr = np.zeros((B, H, R_cap, d), dtype=np.uint16)
    rc = _load().orc_gather(_p(K, _u16p), _p(V, _u16p), B, H, ctypes.c_int64(N), d, int(c),
                            _p(idx, _i32p), k, ctypes.c_int64(R_cap), _p(Kr, _u16p), _p(Vr, _u16p))
    if rc != 0:
        raise ValueError("orc_gather: bad argument")
    return Kr, Vr


def accept(target_logits, draft_logits, draft_tokens, temperature: float, u_accept, u_sample):
    """-> (n_accepted int32 [B], out_tokens int32 [B,G], margin_accept f64 [B], margin_sample f64 [B])."""
    tl = np.ascontiguousarray(target_logits, dtype=np.float32)
    B, G, V = tl.shape
    gamma = G - 1
    dl = np.ascontiguousarray(draft_logits, dtype=np.float32).reshape(B, gamma, V)
    dt = np.ascontiguousarray(draft_tokens, dtype=np.int32).reshape(B, gamma)
    ua = np.ascontiguousarray(u_accept, dtype=np.float32).reshape(B, gamma)
    us = np.ascontiguousarray(u_sample, dtype=np.float32).reshape(B)
    n_acc = np.empty(B, dtype=np.int32)
    out = np.empty((B, G), dtype=np.int32)
    ma = np.empty(B, dtype=np.float64)
    ms = np.empty(B, dtype=np.float64)
    rc = _load().orc_accept(_p(tl, _f32p), _p(dl, _f32p), _p(dt, _i32p), B, G, V,
                            ctypes.c_double(temperature), _p(ua, _f32p), _p(us, _f32p),
                            _p(n_acc, _i32p), _p(out, _i32p), _p(ma, _f64p), _p(ms, _f64p))
    if rc != 0:
        raise ValueError("orc_accept: bad argument")
    return n_acc, out, ma, ms


def accept_ragged(target_logits, draft_logits, draft_tokens, n_draft, temperature: float, u_accept, u_sample):
    """Accept step for a batch whose sequences drafted different numbers of tokens: sequence b is
    the fixed-length problem with gamma = n_draft[b] on its leading rows (Algorithm 1 applied per
    sequence). Same outputs as `accept`, out_tokens padded with -1 to the batch's G."""
    tl = np.ascontiguousarray(target_logits, dtype=np.float32)
    B, G, V = tl.shape
    dl = np.asarray(draft_logits, dtype=np.float32).reshape(B, G - 1, V)
    dt = np.asarray(draft_tokens, dtype=np.int32).reshape(B, G - 1)
    ua = np.asarray(u_accept, dtype=np.float32).reshape(B, G - 1)
    us = np.asarray(u_sample, dtype=np.float32).reshape(B)
    n_acc = np.empty(B, dtype=np.int32)
    out = np.full((B, G), -1, dtype=np.int32)
    ma, ms = np.empty(B), np.empty(B)
    for b in range(B):
        g = int(min(max(int(n_draft[b]), 0), G - 1))
        n, o, a, s = accept(tl[b:b + 1, :g + 1], dl[b:b + 1, :g], dt[b:b + 1, :g], temperature, ua[b:b + 1, :g],
                            us[b:b + 1])
        n_acc[b], ma[b], ms[b] = n[0], a[0], s[0]
        out[b, :g + 1] = o[0]
    return n_acc, out, ma, ms


def attention_indexed(Q, K, V, idx, c: int, kv_len=None, recent_begin=None, scale: float = 1.0,
                      causal: bool = True, kv_len_all: int | None = None):
    """Gather-free drafting, written as its definition (Algorithm 1, M_p(C_r, ...); Sec. 4.1): for
    every (b,h) build the draft cache explicitly -- the rows of chunks idx[b,h,:] in that order
    (chunk m = rows m*c .. m*c+c-1; negative entries and chunks reaching beyond kv_len_all are
    skipped), then the recent rows [recent_begin[b], kv_len[b]) -- and run the plain attention
    over it (causal mask bottom-right aligned on the concatenation; the G queries' own rows are
    the last recent rows, so causal needs at least G recent rows).
    Q [B,H,G,d], K,V [B,H,N,d] uint16(bf16), idx int [B,H,k] -> (O, LSE) float64."""
    Q, K, V = _u16(Q), _u16(K), _u16(V)
    idx = np.asarray(idx)
    B, H, G, d = Q.shape
    N = K.shape[2]
    kv_len_all = N if kv_len_all is None else int(kv_len_all)
    kv = np.broadcast_to(np.asarray(kv_len_all if kv_len is None else kv_len, dtype=np.int64), (B,))
    rb = np.broadcast_to(np.asarray(kv if recent_begin is None else recent_begin, dtype=np.int64), (B,))
    O = np.zeros((B, H, G, d), dtype=np.float64)
    LSE = np.full((B, H, G), -np.inf, dtype=np.float64)
    for b in range(B):
        for h in range(H):
            rows = [np.arange(m * c, m * c + c) for m in idx[b, h].tolist() if m >= 0 and (m + 1) * c <= kv_len_all]
            rows.append(np.arange(min(int(rb[b]), int(kv[b])), int(kv[b])))
            rows = np.concatenate(rows).astype(np.int64)
            if causal and int(kv[b]) - min(int(rb[b]), int(kv[b])) < G:
                raise ValueError("causal indexed attention needs at least G recent rows")
            if rows.size == 0:
                continue
            Kv = np.ascontiguousarray(K[b, h][rows])[None, None]
            Vv = np.ascontiguousarray(V[b, h][rows])[None, None]
            o, l, _ = attention(Q[b:b + 1, h:h + 1], Kv, Vv, scale=scale, causal=causal)
            O[b, h], LSE[b, h] = o[0, 0], l[0, 0]
    return O, LSE


def attention_gqa(Q, K, V, kv_len=None, scale: float = 1.0, causal: bool = True):
    """Grouped-query attention written as its definition: query head q attends with the K/V of KV
    head q // q_group (q_group = query heads / KV heads); each KV head is repeated for its group
    and the plain attention is called. Q [B,Hq,G,d], K,V [B,Hkv,N,d] -> (O, LSE) float64."""
    Q, K, V = _u16(Q), _u16(K), _u16(V)
    q_group = Q.shape[1] // K.shape[1]
    assert q_group * K.shape[1] == Q.shape[1]
    Kr = np.ascontiguousarray(np.repeat(K, q_group, axis=1))
    Vr = np.ascontiguousarray(np.repeat(V, q_group, axis=1))
    O, LSE, _ = attention(Q, Kr, Vr, kv_len=kv_len, scale=scale, causal=causal)
    return O, LSE


def attention_tree(Q, K, V, tail_mask, kv_len=None, scale: float = 1.0):
    """Verification attention for a speculated token tree (Sec. 5.3.3), written as its definition:
    the G speculated tokens are the last G rows of each sequence; query g attends to the context
    rows [0, len-G) and to speculated row len-G+j iff bit j of tail_mask[g] is set. For every
    (b, g) the visible rows are collected explicitly and the plain (unmasked) attention of that one
    query over them is computed by the C routine.
    Q [B,H,G,d], K,V [B,H,N,d] uint16(bf16), tail_mask G ints -> (O, LSE) float64."""
    Q, K, V = _u16(Q), _u16(K), _u16(V)
    B, H, G, d = Q.shape
    N = K.shape[2]
    kv = np.broadcast_to(np.asarray(N if kv_len is None else kv_len, dtype=np.int64), (B,))
    mask = [int(m) for m in tail_mask]
    assert len(mask) == G
    O = np.zeros((B, H, G, d), dtype=np.float64)
    LSE = np.full((B, H, G), -np.inf, dtype=np.float64)
    for b in range(B):
        n = int(kv[b])
        ctx = np.arange(max(n - G, 0))
        for g in range(G):
            tail = [n - G + j for j in range(G) if (mask[g] >> j) & 1 and n - G + j >= 0]
            rows = np.concatenate([ctx, np.asarray(tail, dtype=np.int64)]).astype(np.int64)
            if rows.size == 0:
                continue
            Kv = np.ascontiguousarray(K[b][:, rows])[None]
            Vv = np.ascontiguousarray(V[b][:, rows])[None]
            o, l, _ = attention(np.ascontiguousarray(Q[b:b + 1, :, g:g + 1]), Kv, Vv, scale=scale, causal=False)
            O[b, :, g], LSE[b, :, g] = o[0, :, 0], l[0, :, 0]
    return O, LSE


def kv_append(Knew, Vnew, K, V, pos):
    """Cache update (last step of Algorithm 1; Sec. 4.3): returns copies of K, V with
    K[b,h,pos[b]+i] = Knew[b,h,i] (same for V); destination rows outside the cache are dropped."""
    Knew, Vnew, K, V = _u16(Knew), _u16(Vnew), _u16(K).copy(), _u16(V).copy()
    B, H, n, d = Knew.shape
    pos = np.broadcast_to(np.asarray(pos, dtype=np.int64), (B,))
    for b in range(B):
        for i in range(n):
            t = int(pos[b]) + i
            if 0 <= t < K.shape[2]:
                K[b, :, t] = Knew[b, :, i]
                V[b, :, t] = Vnew[b, :, i]
    return K, V
