"""Thin ctypes binding over the C-ABI library libsl.so (argument marshalling only).

Every step of the hot path runs in the library's HIP kernels; PyTorch is used for device
memory and the current stream.  Importing this module needs only the built library; calling an
operation needs a GPU.  There is no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import math
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsl.so")

SL_OK = 0
SL_F32, SL_BF16 = 0, 1
OP_SEARCH_PREFILL, OP_SEARCH_DECODE, OP_ATTENTION_PREFILL, OP_ATTENTION_DECODE = 0, 1, 2, 3
SL_MAX_TOPK = 32

EXPORTS = ("sl_workspace_bytes", "sl_span_keys", "sl_span_search_prefill", "sl_span_search_decode",
           "sl_span_attention_prefill", "sl_span_attention_decode", "sl_noalloc_scratch_bytes",
           "sl_span_attention_decode_noalloc", "sl_span_attention_combined_prefill",
           "sl_span_attention_combined_decode", "sl_anchor_workspace_bytes", "sl_anchor_search_decode",
           "sl_anchor_attention_decode", "sl_anchor_search_prefill", "sl_anchor_prefill_workspace_bytes",
           "sl_anchor_attention_prefill",
           "sl_decode_batched_workspace_bytes", "sl_span_search_decode_batched",
           "sl_span_attention_decode_batched", "sl_span_attention_combined_decode_batched",
           "sl_anchor_batched_workspace_bytes", "sl_anchor_search_decode_batched",
           "sl_anchor_attention_decode_batched", "sl_set_profile_events", "sl_status_string", "sl_version")


class SlAnchorGeometry(ctypes.Structure):
    _fields_ = [("window", ctypes.c_int64), ("backward_factor", ctypes.c_int32),
                ("forward_factor", ctypes.c_int32), ("search_root", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class SlDecodeSeq(ctypes.Structure):
    _fields_ = [("Qs", ctypes.c_void_p), ("Q", ctypes.c_void_p), ("K", ctypes.c_void_p),
                ("V", ctypes.c_void_p), ("Ks", ctypes.c_void_p), ("idx", ctypes.c_void_p),
                ("scores", ctypes.c_void_p), ("O", ctypes.c_void_p), ("LSE", ctypes.c_void_p),
                ("L", ctypes.c_int64)]


class SlParams(ctypes.Structure):
    _fields_ = [
        ("L", ctypes.c_int64), ("Lq", ctypes.c_int64), ("q_pos0", ctypes.c_int64),
        ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
        ("S", ctypes.c_int32), ("topk", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_float), ("span_stride", ctypes.c_int32),
        ("q_stride_h", ctypes.c_int64), ("q_stride_t", ctypes.c_int64),
        ("kv_stride_h", ctypes.c_int64), ("kv_stride_t", ctypes.c_int64),
    ]

WORKSPACE_INVALID = ctypes.c_size_t(-1).value


class SlError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


_lib = None


def load():
    """Load libsl.so (built in-tree by paper_2601_18401_amd.build). Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} not found: build it first (python -m paper_2601_18401_amd.build, or "
            "__graft_entry__.build()). There is no fallback path.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32p, f32p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    pp = ctypes.POINTER(SlParams)
    lib.sl_workspace_bytes.restype = ctypes.c_size_t
    lib.sl_workspace_bytes.argtypes = [pp, ctypes.c_int]
    lib.sl_span_keys.restype = ctypes.c_int
    lib.sl_span_keys.argtypes = [pp, vp, vp, vp]
    for name in ("sl_span_search_prefill", "sl_span_search_decode"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [pp, vp, vp, vp, i32p, f32p, vp, ctypes.c_size_t, vp]
    for name in ("sl_span_attention_prefill", "sl_span_attention_decode"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [pp, vp, vp, vp, i32p, vp, f32p, vp, ctypes.c_size_t, vp]
    lib.sl_noalloc_scratch_bytes.restype = ctypes.c_size_t
    lib.sl_noalloc_scratch_bytes.argtypes = []
    lib.sl_span_attention_decode_noalloc.restype = ctypes.c_int
    lib.sl_span_attention_decode_noalloc.argtypes = [pp, vp, vp, vp, i32p, vp, f32p, vp]
    for name in ("sl_span_attention_combined_prefill", "sl_span_attention_combined_decode"):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [pp, vp, vp, vp, i32p, f32p, vp, vp, ctypes.c_size_t, vp]
    gp = ctypes.POINTER(SlAnchorGeometry)
    lib.sl_anchor_workspace_bytes.restype = ctypes.c_size_t
    lib.sl_anchor_workspace_bytes.argtypes = [pp, gp]
    lib.sl_anchor_search_decode.restype = ctypes.c_int
    lib.sl_anchor_search_decode.argtypes = [pp, gp, vp, vp, i32p, f32p, vp]
    lib.sl_anchor_attention_decode.restype = ctypes.c_int
    lib.sl_anchor_attention_decode.argtypes = [pp, gp, vp, vp, vp, i32p, f32p, vp, vp, ctypes.c_size_t, vp]
    lib.sl_anchor_search_prefill.restype = ctypes.c_int
    lib.sl_anchor_search_prefill.argtypes = [pp, gp, vp, vp, i32p, f32p, vp]
    lib.sl_anchor_attention_prefill.restype = ctypes.c_int
    lib.sl_anchor_attention_prefill.argtypes = [pp, gp, vp, vp, vp, i32p, f32p, vp, vp, ctypes.c_size_t, vp]
    lib.sl_anchor_prefill_workspace_bytes.restype = ctypes.c_size_t
    lib.sl_anchor_prefill_workspace_bytes.argtypes = [pp, gp]
    lib.sl_decode_batched_workspace_bytes.restype = ctypes.c_size_t
    lib.sl_decode_batched_workspace_bytes.argtypes = [pp, ctypes.c_int32]
    lib.sl_span_search_decode_batched.restype = ctypes.c_int
    lib.sl_span_search_decode_batched.argtypes = [pp, vp, ctypes.c_int32, vp]
    lib.sl_span_attention_decode_batched.restype = ctypes.c_int
    lib.sl_span_attention_decode_batched.argtypes = [pp, vp, ctypes.c_int32, vp, ctypes.c_size_t, vp]
    lib.sl_span_attention_combined_decode_batched.restype = ctypes.c_int
    lib.sl_span_attention_combined_decode_batched.argtypes = [pp, vp, ctypes.c_int32, vp, ctypes.c_size_t, vp]
    lib.sl_anchor_batched_workspace_bytes.restype = ctypes.c_size_t
    lib.sl_anchor_batched_workspace_bytes.argtypes = [pp, gp, ctypes.c_int32]
    lib.sl_anchor_search_decode_batched.restype = ctypes.c_int
    lib.sl_anchor_search_decode_batched.argtypes = [pp, gp, vp, ctypes.c_int32, vp]
    lib.sl_anchor_attention_decode_batched.restype = ctypes.c_int
    lib.sl_anchor_attention_decode_batched.argtypes = [pp, gp, vp, ctypes.c_int32, vp, ctypes.c_size_t, vp]
    lib.sl_set_profile_events.restype = None
    lib.sl_set_profile_events.argtypes = [vp, vp]
    lib.sl_status_string.restype = ctypes.c_char_p
    lib.sl_status_string.argtypes = [ctypes.c_int]
    lib.sl_version.restype = ctypes.c_int
    lib.sl_version.argtypes = []
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().sl_status_string(int(status)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SL_F32
    if t.dtype == torch.bfloat16:
        return SL_BF16
    raise TypeError(f"unsupported dtype {t.dtype}: fp32 or bf16 only")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _arm(prof):
    """prof = (start, stop) hipEvent_t handles for the next call's dominant kernel, or None."""
    if prof is not None:
        load().sl_set_profile_events(ctypes.c_void_p(prof[0]), ctypes.c_void_p(prof[1]))


def make_params(Q, K, S, topk, q_pos0=0, scale=0.0, span_stride=0) -> SlParams:
    """Q: [Hq, Lq, D] (innermost contiguous), K: [Hkv, L, D]."""
    if Q.dim() != 3 or K.dim() != 3 or Q.stride(2) != 1 or K.stride(2) != 1:
        raise ValueError("expect Q [Hq, Lq, D] and K [Hkv, L, D] with contiguous innermost dimension")
    p = SlParams()
    p.L, p.Lq, p.q_pos0 = K.shape[1], Q.shape[1], int(q_pos0)
    p.Hq, p.Hkv, p.D = Q.shape[0], K.shape[0], Q.shape[2]
    p.S, p.topk, p.dtype = int(S), int(topk), _dtype_code(Q)
    p.scale = float(scale)
    p.span_stride = int(span_stride)
    p.q_stride_h, p.q_stride_t = Q.stride(0), Q.stride(1)
    p.kv_stride_h, p.kv_stride_t = K.stride(0), K.stride(1)
    return p


def workspace_bytes(p: SlParams, op: int) -> int:
    """Scratch bytes of the operation; 0 for parameters the entry point will reject (it reports why)."""
    need = int(load().sl_workspace_bytes(ctypes.byref(p), op))
    return 0 if need == WORKSPACE_INVALID else need


class Workspace:
    """Caller-owned scratch: one growing uint8 device tensor per instance."""

    def __init__(self, device="cuda"):
        self.device = device
        self.buf = None

    def get(self, nbytes: int):
        if nbytes == 0:
            return None, 0
        if self.buf is None or self.buf.numel() < nbytes:
            self.buf = torch.empty(int(nbytes) + 256, dtype=torch.uint8, device=self.device)
        off = (-self.buf.data_ptr()) % 256
        return ctypes.c_void_p(self.buf.data_ptr() + off), self.buf.numel() - off


_default_ws = None


def _ws(ws):
    global _default_ws
    if ws is not None:
        return ws
    if _default_ws is None:
        _default_ws = Workspace()
    return _default_ws


def _need(nbytes) -> int:
    """A *_workspace_bytes result as a size to allocate: invalid parameters need nothing (the entry
    point rejects them and says why)."""
    nbytes = int(nbytes)
    return 0 if nbytes == WORKSPACE_INVALID else nbytes


def _check(status, where):
    if status != SL_OK:
        raise SlError(status, where)


def sl_span_keys(K, S, out=None):
    """Ks[kv, j] = K[kv, (j+1)S - 1] for every complete span j; returns Ks [Hkv, ceil(L/S), D]."""
    Hkv, L, D = K.shape
    n = -(-L // S)
    if out is None:
        out = torch.zeros((Hkv, n, D), dtype=K.dtype, device=K.device)
    p = make_params(K[:, :1], K, S, 0)
    p.Hq = Hkv
    _check(load().sl_span_keys(ctypes.byref(p), _ptr(K), _ptr(out), _stream()), "sl_span_keys")
    return out


def _search(fn_name, op, Qs, K, Ks, S, topk, q_pos0, want_scores, ws, prof):
    lib = load()
    p = make_params(Qs, K, S, topk, q_pos0)
    Hq, Lq, _ = Qs.shape
    idx = torch.empty((Hq, Lq, topk), dtype=torch.int32, device=Qs.device)
    scores = torch.empty((Hq, Lq, topk), dtype=torch.float32, device=Qs.device) if want_scores else None
    wptr, wbytes = _ws(ws).get(workspace_bytes(p, op))
    _arm(prof)
    st = getattr(lib, fn_name)(ctypes.byref(p), _ptr(Qs), _ptr(K), _ptr(Ks), _ptr(idx), _ptr(scores),
                               wptr, wbytes, _stream())
    _check(st, fn_name)
    return (idx, scores) if want_scores else idx


def sl_span_search_prefill(Qs, K, Ks, S, topk, q_pos0=0, want_scores=False, ws=None, prof=None):
    return _search("sl_span_search_prefill", OP_SEARCH_PREFILL, Qs, K, Ks, S, topk, q_pos0,
                   want_scores, ws, prof)


def sl_span_search_decode(Qs, K, Ks, S, topk, q_pos0=None, want_scores=False, ws=None, prof=None):
    q_pos0 = K.shape[1] - 1 if q_pos0 is None else q_pos0
    return _search("sl_span_search_decode", OP_SEARCH_DECODE, Qs, K, Ks, S, topk, q_pos0,
                   want_scores, ws, prof)


def _attention(fn_name, op, Q, K, V, idx, S, q_pos0, scale, ws, prof, out, span_stride=0):
    lib = load()
    topk = 0 if idx is None else idx.shape[2]
    p = make_params(Q, K, S, topk, q_pos0, scale, span_stride)
    if V.shape != K.shape or V.stride() != K.stride():
        raise ValueError("V must have the shape and strides of K")
    Hq, Lq, D = Q.shape
    if out is None:
        O = torch.empty((Hq, Lq, D), dtype=Q.dtype, device=Q.device)
        LSE = torch.empty((Hq, Lq), dtype=torch.float32, device=Q.device)
    else:
        O, LSE = out
    wptr, wbytes = _ws(ws).get(workspace_bytes(p, op))
    _arm(prof)
    st = getattr(lib, fn_name)(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), _ptr(O), _ptr(LSE),
                               wptr, wbytes, _stream())
    _check(st, fn_name)
    return O, LSE


def sl_noalloc_scratch_bytes() -> int:
    return int(load().sl_noalloc_scratch_bytes())


def sl_span_attention_decode_noalloc(Q, K, V, idx, S, out, q_pos0=None, scale=0.0):
    """sl_span_attention_decode without a workspace: the library's own device array holds the partial
    records.  `out` = (O, LSE) must be given: this wrapper allocates nothing either."""
    topk = 0 if idx is None else idx.shape[2]
    q_pos0 = K.shape[1] - 1 if q_pos0 is None else q_pos0
    p = make_params(Q, K, S, topk, q_pos0, scale)
    if V.shape != K.shape or V.stride() != K.stride():
        raise ValueError("V must have the shape and strides of K")
    O, LSE = out
    st = load().sl_span_attention_decode_noalloc(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(idx),
                                                 _ptr(O), _ptr(LSE), _stream())
    _check(st, "sl_span_attention_decode_noalloc")
    return O, LSE


def _combined(fn_name, op, Q, K, V, idx, scores, S, q_pos0, scale, ws, out, span_stride=0):
    lib = load()
    topk = 0 if idx is None else idx.shape[2]
    p = make_params(Q, K, S, topk, q_pos0, scale, span_stride)
    if V.shape != K.shape or V.stride() != K.stride():
        raise ValueError("V must have the shape and strides of K")
    if topk > 0 and (scores is None or scores.shape != idx.shape or scores.dtype != torch.float32
                     or not scores.is_contiguous()):
        raise ValueError("scores must be a contiguous float32 tensor of the shape of idx")
    Hq, Lq, D = Q.shape
    O = torch.empty((Hq, Lq, D), dtype=Q.dtype, device=Q.device) if out is None else out
    wptr, wbytes = _ws(ws).get(workspace_bytes(p, op))
    st = getattr(lib, fn_name)(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), _ptr(scores), _ptr(O),
                               wptr, wbytes, _stream())
    _check(st, fn_name)
    return O


def sl_span_attention_combined_prefill(Q, K, V, idx, scores, S, q_pos0=0, scale=0.0, ws=None, out=None,
                                       span_stride=0):
    return _combined("sl_span_attention_combined_prefill", OP_ATTENTION_PREFILL, Q, K, V, idx, scores, S,
                     q_pos0, scale, ws, out, span_stride)


def sl_span_attention_combined_decode(Q, K, V, idx, scores, S, q_pos0=None, scale=0.0, ws=None, out=None,
                                      span_stride=0):
    q_pos0 = K.shape[1] - 1 if q_pos0 is None else q_pos0
    return _combined("sl_span_attention_combined_decode", OP_ATTENTION_DECODE, Q, K, V, idx, scores, S,
                     q_pos0, scale, ws, out, span_stride)


def sl_anchor_search_decode(Qs, K, topk, window, want_scores=False, prof=None, search_root=2):
    """Top-k anchors of the query at the end of the cache on the paper's stride pattern."""
    lib = load()
    p = make_params(Qs, K, 1, topk, K.shape[1] - 1)
    g = SlAnchorGeometry(window, 0, 0, search_root, 0)
    Hq = Qs.shape[0]
    anchors = torch.empty((Hq, 1, topk), dtype=torch.int32, device=Qs.device)
    scores = torch.empty((Hq, 1, topk), dtype=torch.float32, device=Qs.device) if want_scores else None
    _arm(prof)
    st = lib.sl_anchor_search_decode(ctypes.byref(p), ctypes.byref(g), _ptr(Qs), _ptr(K), _ptr(anchors),
                                     _ptr(scores), _stream())
    _check(st, "sl_anchor_search_decode")
    return (anchors, scores) if want_scores else anchors


def sl_anchor_attention_decode(Q, K, V, anchors, scores, window, backward_factor, forward_factor,
                               scale=0.0, ws=None, prof=None, out=None, search_root=2):
    """Algorithm 1's span-attention + combination for the query at the end of the cache."""
    lib = load()
    topk = 0 if anchors is None else anchors.shape[2]
    p = make_params(Q, K, 1, topk, K.shape[1] - 1, scale)
    g = SlAnchorGeometry(window, backward_factor, forward_factor, search_root, 0)
    if V.shape != K.shape or V.stride() != K.stride():
        raise ValueError("V must have the shape and strides of K")
    Hq, Lq, D = Q.shape
    O = torch.empty((Hq, Lq, D), dtype=Q.dtype, device=Q.device) if out is None else out
    need = _need(lib.sl_anchor_workspace_bytes(ctypes.byref(p), ctypes.byref(g)))
    wptr, wbytes = _ws(ws).get(need)
    _arm(prof)
    st = lib.sl_anchor_attention_decode(ctypes.byref(p), ctypes.byref(g), _ptr(Q), _ptr(K), _ptr(V),
                                        _ptr(anchors), _ptr(scores), _ptr(O), wptr, wbytes, _stream())
    _check(st, "sl_anchor_attention_decode")
    return O


def sl_anchor_search_prefill(Qs, K, topk, window, q_pos0=0, want_scores=False, prof=None, search_root=2):
    """Top-k anchors of every query row on the paper's stride pattern (row r sits at q_pos0 + r)."""
    lib = load()
    p = make_params(Qs, K, 1, topk, q_pos0)
    g = SlAnchorGeometry(window, 0, 0, search_root, 0)
    Hq, Lq, _ = Qs.shape
    anchors = torch.empty((Hq, Lq, topk), dtype=torch.int32, device=Qs.device)
    scores = torch.empty((Hq, Lq, topk), dtype=torch.float32, device=Qs.device) if want_scores else None
    _arm(prof)
    st = lib.sl_anchor_search_prefill(ctypes.byref(p), ctypes.byref(g), _ptr(Qs), _ptr(K), _ptr(anchors),
                                      _ptr(scores), _stream())
    _check(st, "sl_anchor_search_prefill")
    return (anchors, scores) if want_scores else anchors


def sl_anchor_attention_prefill(Q, K, V, anchors, scores, window, backward_factor, forward_factor,
                                q_pos0=0, scale=0.0, prof=None, out=None, search_root=2, ws=None,
                                row_stationary=False):
    """Algorithm 1's span-attention + combination for every query row.  The matrix-core form runs
    where it applies (bf16, D = 128, window >= 1) unless row_stationary is set."""
    lib = load()
    topk = 0 if anchors is None else anchors.shape[2]
    p = make_params(Q, K, 1, topk, q_pos0, scale)
    g = SlAnchorGeometry(window, backward_factor, forward_factor, search_root, 0)
    if V.shape != K.shape or V.stride() != K.stride():
        raise ValueError("V must have the shape and strides of K")
    Hq, Lq, D = Q.shape
    O = torch.empty((Hq, Lq, D), dtype=Q.dtype, device=Q.device) if out is None else out
    need = 0 if row_stationary else _need(lib.sl_anchor_prefill_workspace_bytes(ctypes.byref(p), ctypes.byref(g)))
    wptr, wbytes = _ws(ws).get(need)
    _arm(prof)
    st = lib.sl_anchor_attention_prefill(ctypes.byref(p), ctypes.byref(g), _ptr(Q), _ptr(K), _ptr(V),
                                         _ptr(anchors), _ptr(scores), _ptr(O), wptr, wbytes, _stream())
    _check(st, "sl_anchor_attention_prefill")
    return O


def sl_span_attention_prefill(Q, K, V, idx, S, q_pos0=0, scale=0.0, ws=None, prof=None, out=None, span_stride=0):
    return _attention("sl_span_attention_prefill", OP_ATTENTION_PREFILL, Q, K, V, idx, S, q_pos0,
                      scale, ws, prof, out, span_stride)


def sl_span_attention_decode(Q, K, V, idx, S, q_pos0=None, scale=0.0, ws=None, prof=None, out=None, span_stride=0):
    q_pos0 = K.shape[1] - 1 if q_pos0 is None else q_pos0
    return _attention("sl_span_attention_decode", OP_ATTENTION_DECODE, Q, K, V, idx, S, q_pos0,
                      scale, ws, prof, out, span_stride)


class DecodeBatch:
    """The device array of sl_decode_seq records for B sequences, and the tensors it points at.

    Qs, Q: lists of [Hq, 1, D]; K, V: lists of [Hkv, L_b, D] (V with K's strides); Ks: list of packed
    span keys [Hkv, ceil(L_b / S), D] or None.  idx / scores / O / LSE are allocated here and filled
    by the two batched calls.  The kv head stride is passed to the library when every sequence has
    the same one (caches cut from one [B, Hkv, Lmax, D] buffer); otherwise every cache must be
    contiguous and the library takes L_b * D."""

    def __init__(self, Qs, Q, K, V, Ks, S, topk, want_scores=False, span_stride=0):
        B = len(Q)
        if not (len(Qs) == len(K) == len(V) == B) or (Ks is not None and len(Ks) != B) or B < 1:
            raise ValueError("one Qs, Q, K, V (and Ks) per sequence")
        dev, Hq, D = Q[0].device, Q[0].shape[0], Q[0].shape[2]
        self.B, self.S, self.topk = B, int(S), int(topk)
        self.tensors = (Qs, Q, K, V, Ks)  # kept alive: the records hold raw pointers
        self.idx = torch.empty((B, Hq, 1, topk), dtype=torch.int32, device=dev)
        self.scores = torch.empty((B, Hq, 1, topk), dtype=torch.float32, device=dev) if want_scores else None
        self.O = torch.empty((B, Hq, 1, D), dtype=Q[0].dtype, device=dev)
        self.LSE = torch.empty((B, Hq, 1), dtype=torch.float32, device=dev)
        self.longest = max(range(B), key=lambda b: K[b].shape[1])
        same = all(k.stride(0) == K[0].stride(0) for k in K)
        recs = (SlDecodeSeq * B)()
        for b in range(B):
            if (Q[b].shape != Q[0].shape or Qs[b].shape != Q[0].shape or Q[b].stride() != Q[0].stride()
                    or Qs[b].stride() != Q[0].stride() or Q[b].dtype != Q[0].dtype or K[b].dtype != Q[0].dtype):
                raise ValueError("queries of a batch share shape, strides and dtype")
            if (K[b].shape[0] != K[0].shape[0] or K[b].shape[2] != D or V[b].shape != K[b].shape
                    or V[b].stride() != K[b].stride() or K[b].stride(1) != K[0].stride(1) or K[b].stride(2) != 1):
                raise ValueError("caches of a batch share heads, D and the token stride; V has K's strides")
            if not same and not K[b].is_contiguous():
                raise ValueError("caches with different head strides must each be contiguous")
            Lb = K[b].shape[1]
            if Ks is not None and (tuple(Ks[b].shape) != (K[b].shape[0], -(-Lb // self.S), D)
                                   or not Ks[b].is_contiguous()):
                raise ValueError("Ks[b] must be contiguous [Hkv, ceil(L_b / S), D]")
            r = recs[b]
            r.Qs, r.Q, r.K, r.V = Qs[b].data_ptr(), Q[b].data_ptr(), K[b].data_ptr(), V[b].data_ptr()
            r.Ks = Ks[b].data_ptr() if Ks is not None else None
            r.idx = self.idx[b].data_ptr()
            r.scores = self.scores[b].data_ptr() if want_scores else None
            r.O, r.LSE, r.L = self.O[b].data_ptr(), self.LSE[b].data_ptr(), Lb
        host = torch.frombuffer(bytearray(bytes(recs)), dtype=torch.int64).clone()
        self.records = host.to(dev)
        m = self.longest
        self.params = make_params(Q[m], K[m], S, topk, K[m].shape[1] - 1, span_stride=span_stride)
        if not same:
            self.params.kv_stride_h = 0


def sl_span_search_decode_batched(batch: DecodeBatch):
    """Fills batch.idx (and batch.scores) for every sequence; returns them."""
    st = load().sl_span_search_decode_batched(ctypes.byref(batch.params), _ptr(batch.records), batch.B,
                                              _stream())
    _check(st, "sl_span_search_decode_batched")
    return (batch.idx, batch.scores) if batch.scores is not None else batch.idx


def sl_span_attention_decode_batched(batch: DecodeBatch, scale=0.0, ws=None):
    """Joint span-attention of every sequence on batch.idx; returns (batch.O, batch.LSE)."""
    lib = load()
    batch.params.scale = float(scale)
    need = _need(lib.sl_decode_batched_workspace_bytes(ctypes.byref(batch.params), batch.B))
    wptr, wbytes = _ws(ws).get(need)
    st = lib.sl_span_attention_decode_batched(ctypes.byref(batch.params), _ptr(batch.records), batch.B,
                                              wptr, wbytes, _stream())
    _check(st, "sl_span_attention_decode_batched")
    return batch.O, batch.LSE


def sl_span_attention_combined_decode_batched(batch: DecodeBatch, scale=0.0, ws=None):
    """Gated combination of every sequence on batch.idx / batch.scores; returns batch.O."""
    lib = load()
    if batch.scores is None:
        raise ValueError("the combination form needs the search scores: DecodeBatch(..., want_scores=True)")
    batch.params.scale = float(scale)
    need = _need(lib.sl_decode_batched_workspace_bytes(ctypes.byref(batch.params), batch.B))
    wptr, wbytes = _ws(ws).get(need)
    st = lib.sl_span_attention_combined_decode_batched(ctypes.byref(batch.params), _ptr(batch.records),
                                                       batch.B, wptr, wbytes, _stream())
    _check(st, "sl_span_attention_combined_decode_batched")
    return batch.O


def sl_anchor_search_decode_batched(batch: DecodeBatch, window, search_root=2):
    """Top-k anchors (token positions) of every sequence's last position into batch.idx / batch.scores."""
    g = SlAnchorGeometry(window, 0, 0, search_root, 0)
    st = load().sl_anchor_search_decode_batched(ctypes.byref(batch.params), ctypes.byref(g),
                                                _ptr(batch.records), batch.B, _stream())
    _check(st, "sl_anchor_search_decode_batched")
    return (batch.idx, batch.scores) if batch.scores is not None else batch.idx


def sl_anchor_attention_decode_batched(batch: DecodeBatch, window, backward_factor, forward_factor,
                                       scale=0.0, ws=None, search_root=2):
    """Algorithm 1's span-attention + combination for every sequence; returns batch.O."""
    lib = load()
    if batch.scores is None:
        raise ValueError("the combination needs the search scores: DecodeBatch(..., want_scores=True)")
    batch.params.scale = float(scale)
    g = SlAnchorGeometry(window, backward_factor, forward_factor, search_root, 0)
    need = _need(lib.sl_anchor_batched_workspace_bytes(ctypes.byref(batch.params), ctypes.byref(g), batch.B))
    wptr, wbytes = _ws(ws).get(need)
    st = lib.sl_anchor_attention_decode_batched(ctypes.byref(batch.params), ctypes.byref(g),
                                                _ptr(batch.records), batch.B, wptr, wbytes, _stream())
    _check(st, "sl_anchor_attention_decode_batched")
    return batch.O
