"""ctypes binding of libtriforce_hip.so: same names as the C ABI, argument marshalling only.

Every step runs in the HIP kernels; PyTorch is used for device memory and the current
stream. There is no CPU fallback: if the library is missing or a call fails, an exception
is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtriforce_hip.so")

TF_OK = 0
TF_MAX_QUERIES = 16
TF_MAX_K_CHUNKS = 2048
TF_MAX_SPEC = 16

EXPORTS = (
    "tf_version", "tf_status_string", "tf_set_option", "tf_set_thread_option", "tf_decode_attn_plan",
    "tf_noalloc_init", "tf_noalloc_scratch_bytes", "tf_decode_attn_retrieval_noalloc", "tf_stream_read_probe",
    "tf_chunk_summarize",
    "tf_chunk_topk_gather_workspace_bytes", "tf_chunk_topk_gather",
    "tf_decode_attn_full_workspace_bytes", "tf_decode_attn_full",
    "tf_decode_attn_retrieval_workspace_bytes", "tf_decode_attn_retrieval",
    "tf_spec_accept_workspace_bytes", "tf_spec_accept",
    "tf_decode_attn_indexed_workspace_bytes", "tf_decode_attn_indexed", "tf_kv_append",
    "tf_decode_attn_tree",
    "tf_chunk_summarize_bf16", "tf_chunk_topk_gather_bf16",
    "tf_spec_accept_ragged",
)


class TfError(RuntimeError):
    def __init__(self, call: str, code: int, text: str):
        super().__init__(f"{call} failed: {text} ({code})")
        self.code = code


class tf_kv_desc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("q_group", ctypes.c_int32), ("capacity", ctypes.c_int64),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_t", ctypes.c_int64)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the built shared library (fails loudly when it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                           "`python -m paper_2404_11912_amd.build` (there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    dp = ctypes.POINTER(tf_kv_desc)
    lib.tf_version.restype = ctypes.c_int
    lib.tf_version.argtypes = []
    lib.tf_status_string.restype = ctypes.c_char_p
    lib.tf_status_string.argtypes = [ctypes.c_int]
    lib.tf_set_option.restype = ctypes.c_int
    lib.tf_set_option.argtypes = [ctypes.c_char_p, i64]
    lib.tf_set_thread_option.restype = ctypes.c_int
    lib.tf_set_thread_option.argtypes = [ctypes.c_char_p, i64]
    lib.tf_chunk_summarize.restype = ctypes.c_int
    lib.tf_chunk_summarize.argtypes = [vp, dp, i32, i64, i64, vp, i64, vp]
    lib.tf_chunk_summarize_bf16.restype = ctypes.c_int
    lib.tf_chunk_summarize_bf16.argtypes = lib.tf_chunk_summarize.argtypes
    lib.tf_chunk_topk_gather_workspace_bytes.restype = sz
    lib.tf_chunk_topk_gather_workspace_bytes.argtypes = [i32, i32, i64, i32]
    lib.tf_chunk_topk_gather.restype = ctypes.c_int
    lib.tf_chunk_topk_gather.argtypes = [vp, vp, i64, vp, vp, dp, i32, vp, i64, i32, vp, vp, vp, vp, dp,
                                         vp, sz, vp]
    lib.tf_chunk_topk_gather_bf16.restype = ctypes.c_int
    lib.tf_chunk_topk_gather_bf16.argtypes = lib.tf_chunk_topk_gather.argtypes
    for name in ("tf_decode_attn_full", "tf_decode_attn_retrieval"):
        getattr(lib, name + "_workspace_bytes").restype = sz
        getattr(lib, name + "_workspace_bytes").argtypes = [i32, i32, i64, i32]
        getattr(lib, name).restype = ctypes.c_int
        getattr(lib, name).argtypes = [vp, vp, vp, dp, vp, i64, i32, f32, i32, vp, vp, vp, sz, vp]
    lib.tf_stream_read_probe.restype = ctypes.c_int
    lib.tf_stream_read_probe.argtypes = [vp, sz, vp, sz, ctypes.POINTER(sz), vp]
    lib.tf_noalloc_init.restype = ctypes.c_int
    lib.tf_noalloc_init.argtypes = []
    lib.tf_noalloc_scratch_bytes.restype = sz
    lib.tf_noalloc_scratch_bytes.argtypes = []
    lib.tf_decode_attn_retrieval_noalloc.restype = ctypes.c_int
    lib.tf_decode_attn_retrieval_noalloc.argtypes = [vp, vp, vp, dp, vp, i64, i32, f32, i32, vp, vp, vp]
    lib.tf_decode_attn_plan.restype = ctypes.c_int
    lib.tf_decode_attn_plan.argtypes = [i32, i32, i32, i64, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.tf_decode_attn_indexed_workspace_bytes.restype = sz
    lib.tf_decode_attn_indexed_workspace_bytes.argtypes = [i32, i32, i32, i32, i64, i32]
    lib.tf_decode_attn_indexed.restype = ctypes.c_int
    lib.tf_decode_attn_indexed.argtypes = [vp, vp, vp, dp, vp, i32, i32, vp, i64, vp, i64, i32, f32, i32, vp, vp,
                                           vp, sz, vp]
    lib.tf_decode_attn_tree.restype = ctypes.c_int
    lib.tf_decode_attn_tree.argtypes = [vp, vp, vp, dp, vp, i64, i32, f32, ctypes.POINTER(ctypes.c_uint16), vp, vp, vp,
                                        sz, vp]
    lib.tf_kv_append.restype = ctypes.c_int
    lib.tf_kv_append.argtypes = [vp, vp, i32, vp, vp, dp, vp, i64, vp]
    lib.tf_spec_accept_workspace_bytes.restype = sz
    lib.tf_spec_accept_workspace_bytes.argtypes = [i32, i32, i32]
    lib.tf_spec_accept.restype = ctypes.c_int
    lib.tf_spec_accept.argtypes = [vp, vp, vp, i32, i32, i32, f32, vp, vp, vp, vp, vp, sz, vp]
    lib.tf_spec_accept_ragged.restype = ctypes.c_int
    lib.tf_spec_accept_ragged.argtypes = [vp, vp, vp, vp, i32, i32, i32, f32, vp, vp, vp, vp, vp, sz, vp]
    _lib = lib
    return lib


def _check(call: str, code: int):
    if code != TF_OK:
        raise TfError(call, code, load_library().tf_status_string(code).decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


_raw_current_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)
_raw_current_device = getattr(torch._C, "_cuda_getDevice", None)


def _stream(stream=None):
    """The HIP stream handle to launch on: `stream`, else the current device's current stream (looked
    up through torch's C accessors where this build has them: a third of the Python cost of a call)."""
    if stream is not None:
        return ctypes.c_void_p(stream.cuda_stream)
    if _raw_current_stream is not None and _raw_current_device is not None:
        return ctypes.c_void_p(_raw_current_stream(_raw_current_device()))
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _need(t: torch.Tensor, dtype, name: str, contiguous=True):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA/HIP tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if contiguous and not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


def kv_desc(t: torch.Tensor) -> tf_kv_desc:
    """Descriptor of a bf16 cache tensor indexed [b][h][t][d] (any strides with d contiguous)."""
    _need(t, torch.bfloat16, "cache", contiguous=False)
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("cache must be 4-D [B,H,N,d] with a contiguous last dim")
    B, H, N, d = t.shape
    return tf_kv_desc(B, H, d, 0, N, t.stride(0), t.stride(1), t.stride(2))


def workspace(nbytes: int, device) -> torch.Tensor:
    """A 256-byte aligned scratch buffer (torch's caching allocator aligns to >= 512 B)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _temp_workspace(nbytes: int, device, stream) -> torch.Tensor:
    """Scratch for one call when the caller passed none. The tensor is dropped as soon as the call
    has enqueued its kernels, so the block must belong to the stream the kernels run on: the caching
    allocator hands a freed block back only to later work of the stream it was allocated on, which
    is then ordered behind those kernels. (Allocated on another stream, the block could be given to
    that stream's next allocation while the kernels still use it.)"""
    if stream is None:
        return workspace(nbytes, device)
    with torch.cuda.stream(stream):
        return workspace(nbytes, device)


def tf_version() -> int:
    return int(load_library().tf_version())


def tf_set_option(name: str, value: int) -> None:
    _check("tf_set_option", load_library().tf_set_option(name.encode(), int(value)))


def tf_set_thread_option(name: str, value: int) -> None:
    """Override a knob for the calling host thread only (-1 removes the override)."""
    _check("tf_set_thread_option", load_library().tf_set_thread_option(name.encode(), int(value)))


def tf_chunk_summarize_bf16(K, chunk: int, Kmean, first_chunk: int = 0, n_chunks: int | None = None, stream=None):
    """tf_chunk_summarize with a bf16 table: the fp32 mean rounded to bf16."""
    return tf_chunk_summarize(K, chunk, Kmean, first_chunk, n_chunks, stream, _name="tf_chunk_summarize_bf16")


def tf_chunk_topk_gather_bf16(q_r, Kmean, K, V, chunk: int, k_chunks: int, out_idx, Kr=None, Vr=None,
                              out_score=None, n_chunks=None, n_chunks_all: int | None = None, ws=None, stream=None):
    """tf_chunk_topk_gather over a bf16 average-key table."""
    return tf_chunk_topk_gather(q_r, Kmean, K, V, chunk, k_chunks, out_idx, Kr, Vr, out_score, n_chunks,
                                n_chunks_all, ws, stream, _name="tf_chunk_topk_gather_bf16")


def tf_chunk_summarize(K, chunk: int, Kmean, first_chunk: int = 0, n_chunks: int | None = None, stream=None,
                       _name: str = "tf_chunk_summarize"):
    """Kmean[b,h,m,:] = mean of K[b,h,m*chunk:(m+1)*chunk,:] for m in [first_chunk, first_chunk+n_chunks)."""
    lib = load_library()
    _need(Kmean, torch.bfloat16 if _name.endswith("_bf16") else torch.float32, "Kmean")
    d = kv_desc(K)
    if Kmean.dim() != 4 or Kmean.shape[0] != d.batch or Kmean.shape[1] != d.heads or Kmean.shape[3] != d.head_dim:
        raise ValueError("Kmean must be [B,H,M_cap,d]")
    M_cap = Kmean.shape[2]
    if n_chunks is None:
        n_chunks = min(M_cap, K.shape[2] // chunk) - first_chunk
    _check(_name,
           getattr(lib, _name)(_ptr(K), ctypes.byref(d), int(chunk), int(first_chunk), int(n_chunks),
                               _ptr(Kmean), int(M_cap), _stream(stream)))
    return Kmean


def tf_chunk_topk_gather_workspace_bytes(batch: int, heads: int, n_chunks_all: int, k_chunks: int) -> int:
    return int(load_library().tf_chunk_topk_gather_workspace_bytes(batch, heads, n_chunks_all, k_chunks))


def tf_chunk_topk_gather(q_r, Kmean, K, V, chunk: int, k_chunks: int, out_idx, Kr=None, Vr=None,
                         out_score=None, n_chunks=None, n_chunks_all: int | None = None, ws=None, stream=None,
                         _name: str = "tf_chunk_topk_gather"):
    """Score chunks by q_r . Kmean, keep the k_chunks best (descending), gather their K/V into Kr/Vr."""
    lib = load_library()
    _need(q_r, torch.bfloat16, "q_r")
    _need(Kmean, torch.bfloat16 if _name.endswith("_bf16") else torch.float32, "Kmean")
    _need(out_idx, torch.int32, "out_idx")
    d = kv_desc(K)
    kv_desc(V)
    if V.stride() != K.stride() or V.shape != K.shape:
        raise ValueError("K and V must share shape and strides")
    if Kmean.dim() != 4 or tuple(Kmean.shape[:2]) != (d.batch, d.heads) or Kmean.shape[3] != d.head_dim:
        raise ValueError("Kmean must be [B,H,M_cap,d]")
    if tuple(q_r.shape) != (d.batch, d.heads, d.head_dim):
        raise ValueError("q_r must be [B,H,d]")
    if tuple(out_idx.shape) != (d.batch, d.heads, int(k_chunks)):
        raise ValueError("out_idx must be [B,H,k_chunks]")
    M_cap = Kmean.shape[2]
    if n_chunks_all is None:
        n_chunks_all = min(M_cap, K.shape[2] // chunk)
    if n_chunks is not None:
        _need(n_chunks, torch.int32, "n_chunks")
        if tuple(n_chunks.shape) != (d.batch,):
            raise ValueError("n_chunks must be [B]")
    if out_score is not None:
        _need(out_score, torch.float32, "out_score")
        if tuple(out_score.shape) != (d.batch, d.heads, int(k_chunks)):
            raise ValueError("out_score must be [B,H,k_chunks]")
    rd = None
    if Kr is not None or Vr is not None:
        rd = kv_desc(Kr)
        kv_desc(Vr)
        if Vr.stride() != Kr.stride() or Vr.shape != Kr.shape:
            raise ValueError("Kr and Vr must share shape and strides")
        if (rd.batch, rd.heads, rd.head_dim) != (d.batch, d.heads, d.head_dim):
            raise ValueError("Kr, Vr must be [B,H,R_cap,d] with the cache's B, H, d")
    if ws is None:
        ws = _temp_workspace(tf_chunk_topk_gather_workspace_bytes(d.batch, d.heads, n_chunks_all, k_chunks),
                             K.device, stream)
    _check(_name,
           getattr(lib, _name)(_ptr(q_r), _ptr(Kmean), int(M_cap), _ptr(K), _ptr(V), ctypes.byref(d),
                               int(chunk), _ptr(n_chunks), int(n_chunks_all), int(k_chunks),
                               _ptr(out_idx), _ptr(out_score), _ptr(Kr), _ptr(Vr),
                               ctypes.byref(rd) if rd is not None else None,
                               _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))
    return out_idx


def _attn(name, Q, K, V, O, LSE, kv_len, kv_len_all, scale, causal, ws, stream, tail_mask=None):
    lib = load_library()
    _need(Q, torch.bfloat16, "Q")
    _need(O, torch.float32, "O")
    d = kv_desc(K)
    kv_desc(V)
    if V.stride() != K.stride() or V.shape != K.shape:
        raise ValueError("K and V must share shape and strides")
    if Q.dim() != 4 or Q.shape[0] != d.batch or Q.shape[1] % d.heads or Q.shape[3] != d.head_dim:
        raise ValueError("Q must be [B,H*q_group,G,d]")
    d.q_group = Q.shape[1] // d.heads                     # grouped-query heads share their KV head's pass
    G = Q.shape[2]
    if tuple(O.shape) != tuple(Q.shape):
        raise ValueError("O must be [B,H*q_group,G,d]")
    if LSE is not None:
        _need(LSE, torch.float32, "LSE")
        if tuple(LSE.shape) != tuple(Q.shape[:3]):
            raise ValueError("LSE must be [B,H,G]")
    if kv_len is not None:
        _need(kv_len, torch.int32, "kv_len")
        if tuple(kv_len.shape) != (d.batch,):
            raise ValueError("kv_len must be [B]")
    if kv_len_all is None:
        kv_len_all = K.shape[2]
    if name == "tf_decode_attn_retrieval_noalloc":        # no workspace argument: the library's own buffer
        _check(name, getattr(lib, name)(_ptr(Q), _ptr(K), _ptr(V), ctypes.byref(d), _ptr(kv_len), int(kv_len_all),
                                        int(G), float(scale), int(bool(causal)), _ptr(O), _ptr(LSE),
                                        _stream(stream)))
        return O
    if ws is None:
        ws_name = "tf_decode_attn_full" if tail_mask is not None else name
        nbytes = getattr(lib, ws_name + "_workspace_bytes")(d.batch, d.heads, int(kv_len_all), int(G) * d.q_group)
        ws = _temp_workspace(nbytes, K.device, stream)
    if tail_mask is not None:
        rows = [int(m) for m in tail_mask]
        if len(rows) != G or any(m < 0 or m > 0xffff for m in rows):
            raise ValueError("tail_mask must hold G values in [0, 65535]")
        mask_arg = (ctypes.c_uint16 * G)(*rows)            # host array, read during the call
    else:
        mask_arg = int(bool(causal))
    _check(name, getattr(lib, name)(_ptr(Q), _ptr(K), _ptr(V), ctypes.byref(d), _ptr(kv_len), int(kv_len_all),
                                    int(G), float(scale), mask_arg, _ptr(O), _ptr(LSE), _ptr(ws),
                                    ws.numel() * ws.element_size(), _stream(stream)))
    return O


def tf_decode_attn_plan(kind: int, batch: int, heads: int, len_all: int):
    """(splits per (b,h) unit, tokens per split) an attention call would take now; kind 0 = full /
    tree, 1 = retrieval, 2 = indexed."""
    ns, tps = ctypes.c_int32(0), ctypes.c_int32(0)
    _check("tf_decode_attn_plan", load_library().tf_decode_attn_plan(int(kind), int(batch), int(heads), int(len_all),
                                                                    ctypes.byref(ns), ctypes.byref(tps)))
    return ns.value, tps.value


def tf_decode_attn_full_workspace_bytes(batch: int, heads: int, kv_len_all: int, G: int) -> int:
    return int(load_library().tf_decode_attn_full_workspace_bytes(batch, heads, kv_len_all, G))


def tf_decode_attn_retrieval_workspace_bytes(batch: int, heads: int, kv_len_all: int, G: int) -> int:
    return int(load_library().tf_decode_attn_retrieval_workspace_bytes(batch, heads, kv_len_all, G))


def tf_decode_attn_full(Q, K, V, O, LSE=None, kv_len=None, kv_len_all=None, scale: float = 1.0,
                        causal: bool = True, ws=None, stream=None):
    """Verification attention: G queries [B,H,G,d] over the full cache K,V [B,H,N,d] -> O fp32, LSE fp32."""
    return _attn("tf_decode_attn_full", Q, K, V, O, LSE, kv_len, kv_len_all, scale, causal, ws, stream)


def tf_decode_attn_tree(Q, K, V, tail_mask, O, LSE=None, kv_len=None, kv_len_all=None, scale: float = 1.0,
                        ws=None, stream=None):
    """Verification attention for a token tree: tail_mask[g] bit j = query g sees speculated token j
    (the last G cache rows); every query sees the rows before them."""
    return _attn("tf_decode_attn_tree", Q, K, V, O, LSE, kv_len, kv_len_all, scale, False, ws, stream,
                 tail_mask=tail_mask)


def tf_decode_attn_retrieval(Q, K, V, O, LSE=None, kv_len=None, kv_len_all=None, scale: float = 1.0,
                             causal: bool = True, ws=None, stream=None):
    """Draft attention: the same operation over the retrieval cache (K, V = Kr, Vr)."""
    return _attn("tf_decode_attn_retrieval", Q, K, V, O, LSE, kv_len, kv_len_all, scale, causal, ws, stream)


def tf_stream_read_probe(buf: torch.Tensor, sink: torch.Tensor, stream=None) -> int:
    """Enqueue a plain streaming read of the whole tensor `buf` (contiguous); returns the bytes the
    kernel reads. `sink`: device scratch of at least 4 * 256 * (compute units) bytes."""
    if not (buf.is_cuda and sink.is_cuda and buf.is_contiguous() and sink.is_contiguous()):
        raise ValueError("buf and sink must be contiguous device tensors")
    n = ctypes.c_size_t(0)
    _check("tf_stream_read_probe",
           load_library().tf_stream_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink),
                                               sink.numel() * sink.element_size(), ctypes.byref(n), _stream(stream)))
    return int(n.value)


def tf_noalloc_init() -> None:
    """Look up the built-in scratch buffer of the current device (no allocation)."""
    _check("tf_noalloc_init", load_library().tf_noalloc_init())


def tf_noalloc_scratch_bytes() -> int:
    return int(load_library().tf_noalloc_scratch_bytes())


def tf_decode_attn_retrieval_noalloc(Q, K, V, O, LSE=None, kv_len=None, kv_len_all=None, scale: float = 1.0,
                                     causal: bool = True, stream=None):
    """tf_decode_attn_retrieval with the library's built-in scratch buffer: no workspace argument and
    no allocation anywhere on the way (this wrapper allocates nothing either)."""
    return _attn("tf_decode_attn_retrieval_noalloc", Q, K, V, O, LSE, kv_len, kv_len_all, scale, causal, None,
                 stream)


def tf_decode_attn_indexed_workspace_bytes(batch: int, heads: int, k_chunks: int, chunk: int,
                                           recent_len_all: int, G: int) -> int:
    return int(load_library().tf_decode_attn_indexed_workspace_bytes(batch, heads, k_chunks, chunk,
                                                                     recent_len_all, G))


def tf_decode_attn_indexed(Q, K, V, idx, chunk: int, O, LSE=None, kv_len=None, kv_len_all=None,
                           recent_begin=None, recent_begin_all=None, scale: float = 1.0, causal: bool = True,
                           ws=None, stream=None):
    """Draft attention through chunk indices: chunks idx[b,h,:] of the cache, then its rows
    [recent_begin, len). recent_begin_all defaults to kv_len_all (no recent rows)."""
    lib = load_library()
    _need(Q, torch.bfloat16, "Q")
    _need(O, torch.float32, "O")
    _need(idx, torch.int32, "idx")
    d = kv_desc(K)
    kv_desc(V)
    if V.stride() != K.stride() or V.shape != K.shape:
        raise ValueError("K and V must share shape and strides")
    if Q.dim() != 4 or Q.shape[0] != d.batch or Q.shape[1] % d.heads or Q.shape[3] != d.head_dim:
        raise ValueError("Q must be [B,H*q_group,G,d]")
    d.q_group = Q.shape[1] // d.heads
    if idx.dim() != 3 or idx.shape[0] != d.batch or idx.shape[1] != d.heads:
        raise ValueError("idx must be [B,H,k]")
    G, k = Q.shape[2], idx.shape[2]
    if tuple(O.shape) != tuple(Q.shape):
        raise ValueError("O must be [B,H,G,d]")
    if LSE is not None:
        _need(LSE, torch.float32, "LSE")
        if tuple(LSE.shape) != tuple(Q.shape[:3]):
            raise ValueError("LSE must be [B,H*q_group,G]")
    if kv_len is not None:
        _need(kv_len, torch.int32, "kv_len")
        if tuple(kv_len.shape) != (d.batch,):
            raise ValueError("kv_len must be [B]")
    if recent_begin is not None:
        _need(recent_begin, torch.int32, "recent_begin")
        if tuple(recent_begin.shape) != (d.batch,):
            raise ValueError("recent_begin must be [B]")
    if kv_len_all is None:
        kv_len_all = K.shape[2]
    if recent_begin_all is None:
        recent_begin_all = kv_len_all
    if ws is None:
        nbytes = lib.tf_decode_attn_indexed_workspace_bytes(d.batch, d.heads, int(k), int(chunk),
                                                            int(kv_len_all - recent_begin_all), int(G) * d.q_group)
        ws = _temp_workspace(nbytes, K.device, stream)
    _check("tf_decode_attn_indexed",
           lib.tf_decode_attn_indexed(_ptr(Q), _ptr(K), _ptr(V), ctypes.byref(d), _ptr(idx), int(k), int(chunk),
                                      _ptr(kv_len), int(kv_len_all), _ptr(recent_begin), int(recent_begin_all),
                                      int(G), float(scale), int(bool(causal)), _ptr(O), _ptr(LSE), _ptr(ws),
                                      ws.numel() * ws.element_size(), _stream(stream)))
    return O


def tf_kv_append(Knew, Vnew, K, V, pos=None, pos_all: int = 0, stream=None):
    """K[b,h,p+i] = Knew[b,h,i] (and V) for i < n, p = pos[b] (device int32) or pos_all."""
    lib = load_library()
    _need(Knew, torch.bfloat16, "Knew")
    _need(Vnew, torch.bfloat16, "Vnew")
    d = kv_desc(K)
    kv_desc(V)
    if V.stride() != K.stride() or V.shape != K.shape:
        raise ValueError("K and V must share shape and strides")
    if Knew.dim() != 4 or tuple(Knew.shape[:2]) != (d.batch, d.heads) or Knew.shape[3] != d.head_dim \
            or tuple(Vnew.shape) != tuple(Knew.shape):
        raise ValueError("Knew, Vnew must be [B,H,n,d]")
    if pos is not None:
        _need(pos, torch.int32, "pos")
    _check("tf_kv_append", lib.tf_kv_append(_ptr(Knew), _ptr(Vnew), int(Knew.shape[2]), _ptr(K), _ptr(V),
                                            ctypes.byref(d), _ptr(pos), int(pos_all), _stream(stream)))


def tf_spec_accept_workspace_bytes(B: int, G: int, V: int) -> int:
    return int(load_library().tf_spec_accept_workspace_bytes(B, G, V))


def tf_spec_accept_ragged(target_logits, draft_logits, draft_tokens, n_draft, temperature: float, u_accept,
                          u_sample, n_accepted, out_tokens, ws=None, stream=None):
    """tf_spec_accept with a per-sequence number of drafted tokens n_draft [B] (device int32)."""
    return tf_spec_accept(target_logits, draft_logits, draft_tokens, temperature, u_accept, u_sample, n_accepted,
                          out_tokens, ws, stream, n_draft=n_draft)


def tf_spec_accept(target_logits, draft_logits, draft_tokens, temperature: float, u_accept, u_sample,
                   n_accepted, out_tokens, ws=None, stream=None, n_draft=None):
    """Verify / Correct / bonus token for B sequences: fills n_accepted [B] and out_tokens [B,G]."""
    lib = load_library()
    _need(target_logits, torch.float32, "target_logits")
    B, G, V = target_logits.shape
    if G > 1:
        _need(draft_logits, torch.float32, "draft_logits")
        _need(draft_tokens, torch.int32, "draft_tokens")
        _need(u_accept, torch.float32, "u_accept")
        if tuple(draft_logits.shape) != (B, G - 1, V) or tuple(draft_tokens.shape) != (B, G - 1) \
                or tuple(u_accept.shape) != (B, G - 1):
            raise ValueError("draft tensors must be [B,G-1,V] / [B,G-1]")
    _need(u_sample, torch.float32, "u_sample")
    _need(n_accepted, torch.int32, "n_accepted")
    _need(out_tokens, torch.int32, "out_tokens")
    if tuple(u_sample.shape) != (B,) or tuple(n_accepted.shape) != (B,) or tuple(out_tokens.shape) != (B, G):
        raise ValueError("u_sample / n_accepted must be [B], out_tokens [B,G]")
    if ws is None:
        ws = _temp_workspace(tf_spec_accept_workspace_bytes(B, G, V), target_logits.device, stream)
    if n_draft is not None:
        _need(n_draft, torch.int32, "n_draft")
        if tuple(n_draft.shape) != (B,):
            raise ValueError("n_draft must be [B]")
        _check("tf_spec_accept_ragged",
               lib.tf_spec_accept_ragged(_ptr(target_logits), _ptr(draft_logits) if G > 1 else None,
                                         _ptr(draft_tokens) if G > 1 else None, _ptr(n_draft), B, G, V,
                                         float(temperature), _ptr(u_accept) if G > 1 else None, _ptr(u_sample),
                                         _ptr(n_accepted), _ptr(out_tokens), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream(stream)))
        return n_accepted, out_tokens
    _check("tf_spec_accept",
           lib.tf_spec_accept(_ptr(target_logits), _ptr(draft_logits) if G > 1 else None,
                              _ptr(draft_tokens) if G > 1 else None, B, G, V, float(temperature),
                              _ptr(u_accept) if G > 1 else None, _ptr(u_sample), _ptr(n_accepted),
                              _ptr(out_tokens), _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))
    return n_accepted, out_tokens
