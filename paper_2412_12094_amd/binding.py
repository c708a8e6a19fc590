"""Thin ctypes binding of libsepattn.so: argument marshalling only.

Each function has the name and the semantics of the C entry point declared in include/sepattn.h and
takes torch tensors that already live on the GPU (torch is used for device memory and streams,
nothing else).  Workspaces are allocated here with torch and handed to the library, which never
allocates.  Every step of the computation runs in the library's HIP kernels; if the library is
missing this module raises at load time: there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SEPATTN_LIB names another build of the same library (the host-sanitizer build that a CPU test runs the
# argument-validation tests against); every build runs the same kernels
LIB_PATH = os.environ.get("SEPATTN_LIB") or os.path.join(_HERE, "libsepattn.so")

SEPATTN_BF16 = 0
SEPATTN_FP32 = 1

EXPORTS = (
    "sepattn_status_string",
    "sepattn_mark_separators",
    "sepattn_mark_interval",
    "sepattn_compact_workspace_bytes",
    "sepattn_compact_indices",
    "sepattn_mark_compact",
    "sepattn_forward_workspace_bytes",
    "sepattn_forward",
    "sepattn_forward_headwise",
    "sepattn_backward_headwise_workspace_bytes",
    "sepattn_backward_headwise",
    "sepattn_doc_bounds",
    "sepattn_forward_packed",
    "sepattn_backward_packed",
    "sepattn_backward_workspace_bytes",
    "sepattn_backward",
    "sepattn_decode_workspace_bytes",
    "sepattn_decode",
    "sepattn_decode_noalloc_scratch_bytes",
    "sepattn_decode_noalloc",
    "sepkv_evict_workspace_bytes",
    "sepkv_evict_window",
    "sepkv_fill_from_prefill",
    "sepkv_rope_table",
    "sepattn_decode_rope",
    "sepkv_append",
    "sepattn_kernel_name",
    "sepattn_profile_create",
    "sepattn_profile_attach",
    "sepattn_profile_detach",
    "sepattn_profile_read",
    "sepattn_profile_destroy",
)


class SepattnParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int), ("Hq", ctypes.c_int), ("Hkv", ctypes.c_int), ("L", ctypes.c_int),
                ("d", ctypes.c_int), ("a", ctypes.c_int), ("n", ctypes.c_int), ("scale", ctypes.c_float),
                ("dtype", ctypes.c_int), ("cap", ctypes.c_int)]


class SepkvParams(ctypes.Structure):
    _fields_ = [("S", ctypes.c_int), ("Hq", ctypes.c_int), ("Hkv", ctypes.c_int), ("d", ctypes.c_int),
                ("a", ctypes.c_int), ("s", ctypes.c_int), ("w", ctypes.c_int), ("c", ctypes.c_int),
                ("scale", ctypes.c_float), ("dtype", ctypes.c_int)]


class SepattnError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__(f"{fn} failed: status {status} ({status_string(status)})")


_lib = None


def load(path: Optional[str] = None):
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build it with `python -m paper_2412_12094_amd.build` (hipcc, gfx950)")
    lib = ctypes.CDLL(path)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.sepattn_status_string.restype = ctypes.c_char_p
    lib.sepattn_status_string.argtypes = [ci]
    lib.sepattn_mark_separators.restype = ci
    lib.sepattn_mark_separators.argtypes = [vp, ci, ci, vp, ci, vp, vp]
    lib.sepattn_mark_interval.restype = ci
    lib.sepattn_mark_interval.argtypes = [ci, ci, ci, ci, vp, vp]
    lib.sepattn_compact_workspace_bytes.restype = sz
    lib.sepattn_compact_workspace_bytes.argtypes = [ci, ci]
    lib.sepattn_compact_indices.restype = ci
    lib.sepattn_compact_indices.argtypes = [vp, ci, ci, vp, ci, vp, vp, vp, sz, vp]
    lib.sepattn_mark_compact.restype = ci
    lib.sepattn_mark_compact.argtypes = [vp, ci, ci, vp, ci, vp, vp, ci, vp, vp, vp, sz, vp]
    pp = ctypes.POINTER(SepattnParams)
    lib.sepattn_forward_workspace_bytes.restype = sz
    lib.sepattn_forward_workspace_bytes.argtypes = [pp]
    lib.sepattn_forward.restype = ci
    lib.sepattn_forward.argtypes = [pp] + [vp] * 9 + [sz, vp]
    lib.sepattn_forward_headwise.restype = ci
    lib.sepattn_forward_headwise.argtypes = [pp] + [vp] * 10 + [sz, vp]
    lib.sepattn_backward_headwise_workspace_bytes.restype = sz
    lib.sepattn_backward_headwise_workspace_bytes.argtypes = [pp, vp]
    lib.sepattn_backward_headwise.restype = ci
    lib.sepattn_backward_headwise.argtypes = [pp] + [vp] * 14 + [sz, vp]
    lib.sepattn_doc_bounds.restype = ci
    lib.sepattn_doc_bounds.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp]
    lib.sepattn_forward_packed.restype = ci
    lib.sepattn_forward_packed.argtypes = [pp] + [vp] * 11 + [sz, vp]
    lib.sepattn_backward_packed.restype = ci
    lib.sepattn_backward_packed.argtypes = [pp] + [vp] * 15 + [sz, vp]
    lib.sepattn_backward_workspace_bytes.restype = sz
    lib.sepattn_backward_workspace_bytes.argtypes = [pp]
    lib.sepattn_backward.restype = ci
    lib.sepattn_backward.argtypes = [pp] + [vp] * 13 + [sz, vp]
    kp = ctypes.POINTER(SepkvParams)
    lib.sepattn_decode_workspace_bytes.restype = sz
    lib.sepattn_decode_workspace_bytes.argtypes = [kp]
    lib.sepattn_decode.restype = ci
    lib.sepattn_decode.argtypes = [kp] + [vp] * 7 + [sz, vp]
    lib.sepattn_decode_noalloc_scratch_bytes.restype = sz
    lib.sepattn_decode_noalloc_scratch_bytes.argtypes = [kp]
    lib.sepattn_decode_noalloc.restype = ci
    lib.sepattn_decode_noalloc.argtypes = [kp] + [vp] * 7
    lib.sepkv_evict_workspace_bytes.restype = sz
    lib.sepkv_evict_workspace_bytes.argtypes = [kp]
    lib.sepkv_evict_window.restype = ci
    lib.sepkv_evict_window.argtypes = [kp] + [vp] * 5 + [sz, vp]
    lib.sepkv_fill_from_prefill.restype = ci
    lib.sepkv_fill_from_prefill.argtypes = [kp, ci, ci, vp, vp, vp, vp, ci, vp, vp, vp, vp, vp, vp]
    lib.sepkv_rope_table.restype = ci
    lib.sepkv_rope_table.argtypes = [ci, ci, ctypes.c_double, vp, vp]
    lib.sepattn_decode_rope.restype = ci
    lib.sepattn_decode_rope.argtypes = [kp, vp, vp, vp, vp, vp, ci, vp, vp, vp, sz, vp]
    lib.sepkv_append.restype = ci
    lib.sepkv_append.argtypes = [kp] + [vp] * 8
    lib.sepattn_kernel_name.restype = ctypes.c_char_p
    lib.sepattn_kernel_name.argtypes = [ci]
    lib.sepattn_profile_create.restype = ci
    lib.sepattn_profile_create.argtypes = [ci, ci, ctypes.POINTER(vp)]
    lib.sepattn_profile_attach.restype = ci
    lib.sepattn_profile_attach.argtypes = [vp]
    lib.sepattn_profile_detach.restype = ci
    lib.sepattn_profile_detach.argtypes = [vp]
    lib.sepattn_profile_read.restype = ci
    lib.sepattn_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ci, ctypes.POINTER(ctypes.c_int)]
    lib.sepattn_profile_destroy.restype = None
    lib.sepattn_profile_destroy.argtypes = [vp]
    if path == LIB_PATH or _lib is None:
        _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().sepattn_status_string(int(status)).decode()


KERNEL_IDS = {"mark": 0, "compact_count": 1, "compact_write": 2, "forward": 3, "bwd_dq": 4, "bwd_dkv": 5,
              "bwd_combine": 6, "decode_split": 7, "decode_merge": 8, "evict_sizes": 9, "evict_move": 10,
              "cache_fill": 11, "rope_table": 12, "cache_append": 13,
              "mark_interval": 14, "doc_bounds": 15, "mark_compact": 16}


def sepattn_kernel_name(kernel: int) -> str:
    return load().sepattn_kernel_name(int(kernel)).decode()


def sepattn_profile_begin(kernel: int, max_records: int):
    """Create a measurement handle for one kernel and attach it to this thread: the thread's next launches
    of that kernel are bracketed with HIP events on the launch stream.  Returns the handle."""
    lib = load()
    h = ctypes.c_void_p()
    _check("sepattn_profile_create", lib.sepattn_profile_create(int(kernel), int(max_records), ctypes.byref(h)))
    rc = lib.sepattn_profile_attach(h)
    if rc != 0:
        lib.sepattn_profile_destroy(h)
        raise SepattnError("sepattn_profile_attach", rc)
    return (h, int(max_records))


def sepattn_profile_end(handle):
    """Detach the handle, wait for the recorded events, free it; returns the per-launch durations in
    milliseconds."""
    lib = load()
    h, max_records = handle
    ms = (ctypes.c_float * max_records)()
    n = ctypes.c_int(0)
    rc = lib.sepattn_profile_detach(h)
    rc = rc or lib.sepattn_profile_read(h, ms, max_records, ctypes.byref(n))
    lib.sepattn_profile_destroy(h)
    _check("sepattn_profile_end", rc)
    return [float(ms[i]) for i in range(n.value)]


def _check(fn: str, rc: int) -> None:
    if rc != 0:
        raise SepattnError(fn, rc)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(t: torch.Tensor):
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def _ws(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return SEPATTN_BF16
    if t.dtype == torch.float32:
        return SEPATTN_FP32
    raise TypeError(f"unsupported dtype {t.dtype}: bf16 or fp32 expected")


def _dev(*ts: torch.Tensor) -> None:
    for t in ts:
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError("libsepattn works on GPU tensors only")
        if not t.is_contiguous():
            raise ValueError("tensors must be contiguous")


# ------------------------------------------------------------------------------------------------
def sepattn_mark_separators(token_ids: torch.Tensor, sep_ids, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """token_ids int32 [B,L] (GPU), sep_ids: host sequence of ints -> is_sep uint8 [B,L]."""
    _dev(token_ids, out)
    assert token_ids.dtype == torch.int32 and token_ids.dim() == 2
    B, L = token_ids.shape
    ids = (ctypes.c_int32 * len(sep_ids))(*[int(x) for x in sep_ids])
    if out is None:
        out = torch.empty((B, L), dtype=torch.uint8, device=token_ids.device)
    _check("sepattn_mark_separators",
           load().sepattn_mark_separators(_ptr(token_ids), B, L, ctypes.cast(ids, ctypes.c_void_p),
                                          len(sep_ids), _ptr(out), _stream(token_ids)))
    return out


def sepattn_mark_interval(B: int, L: int, delta: int, phase: int, device, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """-> is_sep uint8 [B,L] with is_sep[b, j] = (j % delta == phase): the fixed-interval variant's markers."""
    if out is None:
        out = torch.empty((int(B), int(L)), dtype=torch.uint8, device=device)
    _dev(out)
    _check("sepattn_mark_interval",
           load().sepattn_mark_interval(int(B), int(L), int(delta), int(phase), _ptr(out), _stream(out)))
    return out


def sepattn_compact_indices(is_sep: torch.Tensor, cap: Optional[int] = None, want_prefix: bool = True,
                            fill: int = -1, out=None, ws: Optional[torch.Tensor] = None
                            ) -> Tuple[torch.Tensor, torch.Tensor, Optional[torch.Tensor]]:
    """is_sep uint8 [B,L] -> (sep_idx int32 [B,cap], sep_count int32 [B], sep_prefix int32 [B,L+1]).

    Unless `out` = (sep_idx, sep_count, sep_prefix) is given, sep_idx is allocated and pre-filled
    with `fill` by torch; the library leaves entries beyond the count untouched.
    """
    _dev(is_sep)
    assert is_sep.dtype == torch.uint8 and is_sep.dim() == 2
    B, L = is_sep.shape
    dev = is_sep.device
    if out is None:
        cap = L if cap is None else int(cap)
        idx = torch.full((B, max(cap, 1)), fill, dtype=torch.int32, device=dev)
        cnt = torch.empty((B,), dtype=torch.int32, device=dev)
        pre = torch.empty((B, L + 1), dtype=torch.int32, device=dev) if want_prefix else None
    else:
        idx, cnt, pre = out
        _dev(idx, cnt, pre)
        cap = idx.shape[1]
    lib = load()
    if ws is None:
        ws = _ws(lib.sepattn_compact_workspace_bytes(B, L), dev)
    _check("sepattn_compact_indices",
           lib.sepattn_compact_indices(_ptr(is_sep), B, L, _ptr(idx), cap, _ptr(cnt), _ptr(pre), _ptr(ws),
                                       ws.numel(), _stream(is_sep)))
    return idx, cnt, pre


def sepattn_mark_compact(token_ids: torch.Tensor, sep_ids, cap: Optional[int] = None, want_prefix: bool = True,
                         fill: int = -1, out=None, ws: Optional[torch.Tensor] = None):
    """token_ids int32 [B,L] (GPU), sep_ids: host sequence of ints -> (is_sep uint8 [B,L], sep_idx int32 [B,cap],
    sep_count int32 [B], sep_prefix int32 [B,L+1]): marking and compaction in one call.

    Unless `out` = (is_sep, sep_idx, sep_count, sep_prefix) is given, the outputs are allocated and sep_idx is
    pre-filled with `fill` by torch; the library leaves entries beyond the count untouched.
    """
    _dev(token_ids)
    assert token_ids.dtype == torch.int32 and token_ids.dim() == 2
    B, L = token_ids.shape
    dev = token_ids.device
    ids = (ctypes.c_int32 * len(sep_ids))(*[int(x) for x in sep_ids])
    if out is None:
        cap = L if cap is None else int(cap)
        is_sep = torch.empty((B, L), dtype=torch.uint8, device=dev)
        idx = torch.full((B, max(cap, 1)), fill, dtype=torch.int32, device=dev)
        cnt = torch.empty((B,), dtype=torch.int32, device=dev)
        pre = torch.empty((B, L + 1), dtype=torch.int32, device=dev) if want_prefix else None
    else:
        is_sep, idx, cnt, pre = out
        _dev(is_sep, idx, cnt, pre)
        cap = idx.shape[1]
    lib = load()
    if ws is None:
        ws = _ws(lib.sepattn_compact_workspace_bytes(B, L), dev)
    _check("sepattn_mark_compact",
           lib.sepattn_mark_compact(_ptr(token_ids), B, L, ctypes.cast(ids, ctypes.c_void_p), len(sep_ids), _ptr(is_sep),
                                    _ptr(idx), cap, _ptr(cnt), _ptr(pre), _ptr(ws), ws.numel(), _stream(token_ids)))
    return is_sep, idx, cnt, pre


def _attn_params(Q, K, a, n, scale, cap) -> SepattnParams:
    B, Hq, L, d = Q.shape
    Hkv = K.shape[1]
    return SepattnParams(B, Hq, Hkv, L, d, int(a), int(n), float(scale), _dtype_code(Q), int(cap))


def sepattn_forward(Q, K, V, sep_idx, sep_count, sep_prefix, a: int, n: int, scale: float,
                    out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None, ws: Optional[torch.Tensor] = None):
    """Q [B,Hq,L,d], K,V [B,Hkv,L,d] -> (O like Q, LSE fp32 [B,Hq,L])."""
    _dev(Q, K, V, sep_idx, sep_count, sep_prefix)
    assert K.shape == V.shape and Q.dtype == K.dtype == V.dtype
    p = _attn_params(Q, K, a, n, scale, sep_idx.shape[1])
    lib = load()
    if out is None:
        O = torch.empty_like(Q)
        LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    else:
        O, LSE = out
    if ws is None:
        ws = _ws(lib.sepattn_forward_workspace_bytes(ctypes.byref(p)), Q.device)
    _check("sepattn_forward",
           lib.sepattn_forward(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(sep_idx), _ptr(sep_count),
                               _ptr(sep_prefix), _ptr(O), _ptr(LSE), _ptr(ws), ws.numel(), _stream(Q)))
    return O, LSE


def _head_windows(n_per_head, Hq: int):
    arr = (ctypes.c_int32 * Hq)(*[int(v) for v in n_per_head])
    assert len(n_per_head) == Hq
    return arr


def sepattn_forward_headwise(Q, K, V, sep_idx, sep_count, sep_prefix, a: int, n_per_head, scale: float,
                             out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None, ws: Optional[torch.Tensor] = None):
    """sepattn_forward with a neighbour window of its own for every query head (n_per_head: Hq ints, host)."""
    _dev(Q, K, V, sep_idx, sep_count, sep_prefix)
    assert K.shape == V.shape and Q.dtype == K.dtype == V.dtype
    p = _attn_params(Q, K, a, 1, scale, sep_idx.shape[1])
    nh = _head_windows(n_per_head, Q.shape[1])
    lib = load()
    if out is None:
        O = torch.empty_like(Q)
        LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    else:
        O, LSE = out
    if ws is None:
        ws = _ws(lib.sepattn_forward_workspace_bytes(ctypes.byref(p)), Q.device)
    _check("sepattn_forward_headwise",
           lib.sepattn_forward_headwise(ctypes.byref(p), nh, _ptr(Q), _ptr(K), _ptr(V), _ptr(sep_idx), _ptr(sep_count),
                                        _ptr(sep_prefix), _ptr(O), _ptr(LSE), _ptr(ws), ws.numel(), _stream(Q)))
    return O, LSE


def sepattn_backward_headwise(Q, K, V, O, LSE, dO, sep_idx, sep_count, sep_prefix, a: int, n_per_head, scale: float,
                              out: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None,
                              ws: Optional[torch.Tensor] = None):
    """sepattn_backward with per-head neighbour windows -> (dQ, dK, dV)."""
    _dev(Q, K, V, O, LSE, dO, sep_idx, sep_count, sep_prefix)
    p = _attn_params(Q, K, a, 1, scale, sep_idx.shape[1])
    nh = _head_windows(n_per_head, Q.shape[1])
    lib = load()
    if out is None:
        dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    else:
        dQ, dK, dV = out
    if ws is None:
        ws = _ws(lib.sepattn_backward_headwise_workspace_bytes(ctypes.byref(p), nh), Q.device)
    _check("sepattn_backward_headwise",
           lib.sepattn_backward_headwise(ctypes.byref(p), nh, _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO),
                                         _ptr(sep_idx), _ptr(sep_count), _ptr(sep_prefix), _ptr(dQ), _ptr(dK),
                                         _ptr(dV), _ptr(ws), ws.numel(), _stream(Q)))
    return dQ, dK, dV


def sepattn_doc_bounds(cu_seqlens: torch.Tensor, L: int, a: int = 0, is_sep_row: Optional[torch.Tensor] = None,
                       out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None):
    """One packed row: cu_seqlens int32 [n_docs+1] (GPU; cu[0] = 0, cu[-1] = L) -> (doc_start, doc_end) int32 [L].
    If is_sep_row (uint8 [L], one row of the marker bitmap) is given, the first a tokens of every
    document are marked in it, in place."""
    _dev(cu_seqlens, is_sep_row)
    assert cu_seqlens.dtype == torch.int32 and cu_seqlens.dim() == 1
    if out is None:
        out = (torch.empty((int(L),), dtype=torch.int32, device=cu_seqlens.device),
               torch.empty((int(L),), dtype=torch.int32, device=cu_seqlens.device))
    _dev(*out)
    _check("sepattn_doc_bounds",
           load().sepattn_doc_bounds(_ptr(cu_seqlens), int(cu_seqlens.numel()) - 1, int(L), int(a), _ptr(out[0]),
                                     _ptr(out[1]), _ptr(is_sep_row), _stream(cu_seqlens)))
    return out


def sepattn_forward_packed(Q, K, V, doc_start, doc_end, sep_idx, sep_count, sep_prefix, n: int, scale: float,
                           out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None, ws: Optional[torch.Tensor] = None):
    """Forward over rows of packed documents: doc_start, doc_end int32 [B,L] per-position bounds;
    the index arrays come from a bitmap in which every document's initial tokens are marked (a = 0 here)."""
    _dev(Q, K, V, doc_start, doc_end, sep_idx, sep_count, sep_prefix)
    assert doc_start.dtype == torch.int32 and doc_end.dtype == torch.int32
    assert tuple(doc_start.shape) == (Q.shape[0], Q.shape[2]) and doc_end.shape == doc_start.shape
    p = _attn_params(Q, K, 0, n, scale, sep_idx.shape[1])
    lib = load()
    if out is None:
        O = torch.empty_like(Q)
        LSE = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    else:
        O, LSE = out
    if ws is None:
        ws = _ws(lib.sepattn_forward_workspace_bytes(ctypes.byref(p)), Q.device)
    _check("sepattn_forward_packed",
           lib.sepattn_forward_packed(ctypes.byref(p), _ptr(doc_start), _ptr(doc_end), _ptr(Q), _ptr(K), _ptr(V),
                                      _ptr(sep_idx), _ptr(sep_count), _ptr(sep_prefix), _ptr(O), _ptr(LSE), _ptr(ws),
                                      ws.numel(), _stream(Q)))
    return O, LSE


def sepattn_backward_workspace_bytes(Q, K, a: int, n: int, scale: float, cap: int) -> int:
    p = _attn_params(Q, K, a, n, scale, cap)
    return int(load().sepattn_backward_workspace_bytes(ctypes.byref(p)))


def sepattn_backward(Q, K, V, O, LSE, dO, sep_idx, sep_count, sep_prefix, a: int, n: int, scale: float,
                     out: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None,
                     ws: Optional[torch.Tensor] = None):
    """-> (dQ like Q, dK like K, dV like V)."""
    _dev(Q, K, V, O, LSE, dO, sep_idx, sep_count, sep_prefix)
    p = _attn_params(Q, K, a, n, scale, sep_idx.shape[1])
    lib = load()
    if out is None:
        dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    else:
        dQ, dK, dV = out
    if ws is None:
        ws = _ws(lib.sepattn_backward_workspace_bytes(ctypes.byref(p)), Q.device)
    _check("sepattn_backward",
           lib.sepattn_backward(ctypes.byref(p), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO),
                                _ptr(sep_idx), _ptr(sep_count), _ptr(sep_prefix), _ptr(dQ), _ptr(dK),
                                _ptr(dV), _ptr(ws), ws.numel(), _stream(Q)))
    return dQ, dK, dV


def sepattn_backward_packed(Q, K, V, O, LSE, dO, doc_start, doc_end, sep_idx, sep_count, sep_prefix, n: int,
                            scale: float, out=None, ws: Optional[torch.Tensor] = None):
    """Backward over rows of packed documents -> (dQ, dK, dV); arguments as sepattn_forward_packed."""
    _dev(Q, K, V, O, LSE, dO, doc_start, doc_end, sep_idx, sep_count, sep_prefix)
    assert doc_start.dtype == torch.int32 and doc_end.dtype == torch.int32
    assert tuple(doc_start.shape) == (Q.shape[0], Q.shape[2]) and doc_end.shape == doc_start.shape
    p = _attn_params(Q, K, 0, n, scale, sep_idx.shape[1])
    lib = load()
    if out is None:
        dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    else:
        dQ, dK, dV = out
    if ws is None:
        ws = _ws(lib.sepattn_backward_workspace_bytes(ctypes.byref(p)), Q.device)
    _check("sepattn_backward_packed",
           lib.sepattn_backward_packed(ctypes.byref(p), _ptr(doc_start), _ptr(doc_end), _ptr(Q), _ptr(K), _ptr(V),
                                       _ptr(O), _ptr(LSE), _ptr(dO), _ptr(sep_idx), _ptr(sep_count), _ptr(sep_prefix),
                                       _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(ws), ws.numel(), _stream(Q)))
    return dQ, dK, dV


def _kv_params(q, Kc, a, s, w, scale) -> SepkvParams:
    S, Hq, d = q.shape
    _, Hkv, c, _ = Kc.shape
    return SepkvParams(S, Hq, Hkv, d, int(a), int(s), int(w), c, float(scale), _dtype_code(Kc))


def sepattn_decode(q, Kc, Vc, sizes, a: int, s: int, w: int, scale: float,
                   out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None, ws: Optional[torch.Tensor] = None):
    """q [S,Hq,d], Kc,Vc [S,Hkv,c,d], sizes int32 [S,6] -> (out [S,Hq,d], lse fp32 [S,Hq])."""
    _dev(q, Kc, Vc, sizes)
    assert sizes.dtype == torch.int32 and sizes.dim() == 2 and sizes.shape[1] == 6 and sizes.is_contiguous()
    p = _kv_params(q, Kc, a, s, w, scale)
    lib = load()
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    else:
        o, lse = out
    if ws is None:
        ws = _ws(lib.sepattn_decode_workspace_bytes(ctypes.byref(p)), q.device)
    _check("sepattn_decode",
           lib.sepattn_decode(ctypes.byref(p), _ptr(q), _ptr(Kc), _ptr(Vc), _ptr(sizes), _ptr(o), _ptr(lse),
                              _ptr(ws), ws.numel(), _stream(q)))
    return o, lse


def sepattn_decode_noalloc(q, Kc, Vc, sizes, a: int, s: int, w: int, scale: float,
                           out: Tuple[torch.Tensor, torch.Tensor]):
    """sepattn_decode without a workspace (the library's fixed scratch array is used); the caller passes
    the outputs (out [S,Hq,d], lse fp32 [S,Hq]), so nothing at all is allocated by the call."""
    _dev(q, Kc, Vc, sizes)
    assert sizes.dtype == torch.int32 and sizes.dim() == 2 and sizes.shape[1] == 6 and sizes.is_contiguous()
    p = _kv_params(q, Kc, a, s, w, scale)
    o, lse = out
    _check("sepattn_decode_noalloc",
           load().sepattn_decode_noalloc(ctypes.byref(p), _ptr(q), _ptr(Kc), _ptr(Vc), _ptr(sizes), _ptr(o), _ptr(lse),
                                         _stream(q)))
    return o, lse


def sepkv_rope_table(n_pos: int, d: int, base: float, device, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """-> fp32 [n_pos, 2, d/2]: cos, then sin, of position * base^(-2i/d)."""
    if out is None:
        out = torch.empty((int(n_pos), 2, int(d) // 2), dtype=torch.float32, device=device)
    _dev(out)
    _check("sepkv_rope_table", load().sepkv_rope_table(int(n_pos), int(d), float(base), _ptr(out), _stream(out)))
    return out


def sepattn_decode_rope(q, Kc, Vc, sizes, rope_table, a: int, s: int, w: int, scale: float,
                        out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None, ws: Optional[torch.Tensor] = None):
    """As sepattn_decode, with q and the cached keys stored without position encoding and turned by
    their positions within the cache inside the kernel; rope_table from sepkv_rope_table."""
    _dev(q, Kc, Vc, sizes, rope_table)
    assert sizes.dtype == torch.int32 and sizes.dim() == 2 and sizes.shape[1] == 6 and sizes.is_contiguous()
    assert rope_table.dtype == torch.float32
    assert rope_table.dim() == 3 and rope_table.shape[1] == 2 and rope_table.shape[2] * 2 == q.shape[2]
    p = _kv_params(q, Kc, a, s, w, scale)
    lib = load()
    if out is None:
        o = torch.empty_like(q)
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    else:
        o, lse = out
    if ws is None:
        ws = _ws(lib.sepattn_decode_workspace_bytes(ctypes.byref(p)), q.device)
    _check("sepattn_decode_rope",
           lib.sepattn_decode_rope(ctypes.byref(p), _ptr(q), _ptr(Kc), _ptr(Vc), _ptr(sizes), _ptr(rope_table),
                                   int(rope_table.shape[0]), _ptr(o), _ptr(lse), _ptr(ws), ws.numel(), _stream(q)))
    return o, lse


def sepkv_append(k_new, v_new, is_sep_new, Kc, Vc, win_is_sep, sizes, Hq: int, a: int, s: int, w: int) -> None:
    """In place: k_new, v_new [S,Hkv,d] and is_sep_new uint8 [S] enter Kc, Vc [S,Hkv,c,d], win_is_sep, sizes."""
    _dev(k_new, v_new, is_sep_new, Kc, Vc, win_is_sep, sizes)
    assert sizes.dtype == torch.int32 and sizes.dim() == 2 and sizes.shape[1] == 6 and sizes.is_contiguous()
    assert is_sep_new.dtype == torch.uint8 and win_is_sep.dtype == torch.uint8
    S, Hkv, c, d = Kc.shape
    assert tuple(k_new.shape) == (S, Hkv, d) and tuple(v_new.shape) == (S, Hkv, d) and k_new.dtype == Kc.dtype
    p = SepkvParams(S, int(Hq), Hkv, d, int(a), int(s), int(w), c, 1.0, _dtype_code(Kc))
    _check("sepkv_append",
           load().sepkv_append(ctypes.byref(p), _ptr(k_new), _ptr(v_new), _ptr(is_sep_new), _ptr(Kc), _ptr(Vc),
                               _ptr(win_is_sep), _ptr(sizes), _stream(Kc)))


def sepkv_evict_window(Kc, Vc, win_is_sep, sizes, Hq: int, a: int, s: int, w: int,
                       ws: Optional[torch.Tensor] = None) -> None:
    """In place on Kc, Vc [S,Hkv,c,d], win_is_sep uint8 [S,c-a-s], sizes int32 [S,6]."""
    _dev(Kc, Vc, win_is_sep, sizes)
    assert sizes.dtype == torch.int32 and sizes.dim() == 2 and sizes.shape[1] == 6 and sizes.is_contiguous()
    S, Hkv, c, d = Kc.shape
    p = SepkvParams(S, int(Hq), Hkv, d, int(a), int(s), int(w), c, 1.0, _dtype_code(Kc))
    lib = load()
    # the step needs no scratch memory: a workspace is passed on if the caller has one, NULL otherwise
    _check("sepkv_evict_window",
           lib.sepkv_evict_window(ctypes.byref(p), _ptr(Kc), _ptr(Vc), _ptr(win_is_sep), _ptr(sizes), _ptr(ws),
                                  0 if ws is None else ws.numel(), _stream(Kc)))


def sepkv_fill_from_prefill(K, V, is_sep, sep_idx, sep_prefix, Hq: int, a: int, s: int, w: int, c: int, nw: int,
                            out=None):
    """Prefill K, V [S,Hkv,L,d] -> (Kc, Vc [S,Hkv,c,d], win_is_sep uint8 [S,c-a-s], sizes int32 [S,6]).
    Freshly allocated outputs are zero-filled (the call leaves slots beyond the sizes untouched)."""
    _dev(K, V, is_sep, sep_idx, sep_prefix)
    S, Hkv, L, d = K.shape
    p = SepkvParams(S, int(Hq), Hkv, d, int(a), int(s), int(w), int(c), 1.0, _dtype_code(K))
    if out is None:
        Kc = torch.zeros((S, Hkv, c, d), dtype=K.dtype, device=K.device)
        Vc = torch.zeros_like(Kc)
        flags = torch.zeros((S, c - a - s), dtype=torch.uint8, device=K.device)
        sizes = torch.zeros((S, 6), dtype=torch.int32, device=K.device)
    else:
        Kc, Vc, flags, sizes = out
        _dev(Kc, Vc, flags, sizes)
        assert sizes.dtype == torch.int32 and tuple(sizes.shape) == (S, 6) and sizes.is_contiguous()
    _check("sepkv_fill_from_prefill",
           load().sepkv_fill_from_prefill(ctypes.byref(p), int(L), int(nw), _ptr(K), _ptr(V), _ptr(is_sep),
                                          _ptr(sep_idx), int(sep_idx.shape[1]), _ptr(sep_prefix), _ptr(Kc), _ptr(Vc),
                                          _ptr(flags), _ptr(sizes), _stream(K)))
    return Kc, Vc, flags, sizes
