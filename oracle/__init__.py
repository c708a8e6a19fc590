"""CPU oracle for SepAttention.  TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check
and by bench.py's cpu_baseline leg, never by the product package.

`sepattn_oracle.c` holds the arithmetic (dense, explicit mask; see its header for the passages it
follows).  This module compiles it with gcc into two shared objects (double and float builds) and
wraps them with numpy-in / numpy-out functions.  `cache_sim.py` is the host-only cache-size
simulator of Sec. 3.3; `sanitize_check.c` drives the C functions under the address and
undefined-behaviour sanitizers (tests/test_oracle_sanitizers.py).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sepattn_oracle.c")
_LIBS = {}


def lib_path(precision: str) -> str:
    return os.path.join(_HERE, f"liboracle_{precision}.so")


def build(force: bool = False) -> None:
    """Compile both builds of the oracle with gcc (no GPU toolchain involved)."""
    for precision, ctype in (("f64", "double"), ("f32", "float")):
        out = lib_path(precision)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", f"-DORACLE_REAL={ctype}",
               _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)
    # the memory-safety driver (tests build it again with the sanitizers switched on)
    chk = os.path.join(_HERE, "sanitize_check.c")
    exe = os.path.join(_HERE, "sanitize_check.o")
    if force or not os.path.exists(exe) or os.path.getmtime(exe) < max(os.path.getmtime(chk), os.path.getmtime(_SRC)):
        subprocess.run(["gcc", "-O1", "-std=c11", "-I", _HERE, "-c", chk, "-o", exe], check=True)


def _lib(precision: str):
    if precision not in _LIBS:
        if not os.path.exists(lib_path(precision)) or \
                os.path.getmtime(lib_path(precision)) < os.path.getmtime(_SRC):
            build()
        lib = ctypes.CDLL(lib_path(precision))
        want = 8 if precision == "f64" else 4
        assert lib.oracle_real_bytes() == want
        _LIBS[precision] = lib
    return _LIBS[precision]


def _real(precision: str):
    return np.float64 if precision == "f64" else np.float32


def _ptr(x: Optional[np.ndarray]):
    return None if x is None else x.ctypes.data_as(ctypes.c_void_p)


def _c(x, dtype) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=dtype)


def mark_separators(token_ids: np.ndarray, sep_ids: np.ndarray) -> np.ndarray:
    """uint8 [B,L]: 1 where the token id is in sep_ids (Sec. 4.1 "Parameter Setting")."""
    token_ids = _c(token_ids, np.int32)
    sep_ids = _c(sep_ids, np.int32)
    B, L = token_ids.shape
    out = np.zeros((B, L), dtype=np.uint8)
    _lib("f64").oracle_mark_separators(_ptr(token_ids), B, L, _ptr(sep_ids), int(sep_ids.size),
                                       _ptr(out))
    return out


def mark_interval(B: int, L: int, delta: int, phase: int) -> np.ndarray:
    """Markers of the fixed-interval variant (appendix "Fixed-Interval Variant"): one token in every
    `delta` takes the separators' place: position j iff j % delta == phase (the paper gives the
    interval only; the offset is a reading, [parity unpinned]).  uint8 [B, L]."""
    row = np.array([1 if j % delta == phase else 0 for j in range(L)], dtype=np.uint8)
    return np.tile(row, (B, 1))


def compact_indices(is_sep: np.ndarray, cap: Optional[int] = None
                    ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(sep_idx [B,cap] padded with -1, sep_count [B], sep_prefix [B,L+1])."""
    is_sep = _c(is_sep, np.uint8)
    B, L = is_sep.shape
    cap = L if cap is None else int(cap)
    idx = np.full((B, max(cap, 1)), -1, dtype=np.int32)
    cnt = np.zeros((B,), dtype=np.int32)
    pre = np.zeros((B, L + 1), dtype=np.int32)
    _lib("f64").oracle_compact_indices(_ptr(is_sep), B, L, _ptr(idx), cap, _ptr(cnt), _ptr(pre))
    return idx[:, :cap], cnt, pre


def mask(is_sep_row: np.ndarray, a: int, n: int, rows: Optional[np.ndarray] = None) -> np.ndarray:
    """Explicit boolean mask rows [n_rows, L] of one sequence (Sec. 3.1, Eq. 2)."""
    is_sep_row = _c(is_sep_row, np.uint8)
    L = is_sep_row.size
    rows = np.arange(L, dtype=np.int32) if rows is None else _c(rows, np.int32)
    M = np.zeros((rows.size, L), dtype=np.uint8)
    _lib("f64").oracle_mask_rows(_ptr(is_sep_row), L, int(a), int(n), _ptr(rows), int(rows.size),
                                 _ptr(M))
    return M.astype(bool)


def _n_head(n_head, Hq: int):
    if n_head is None:
        return None
    n_head = _c(n_head, np.int32)
    assert n_head.shape == (Hq,) and (n_head >= 1).all()
    return n_head


def forward(Q, K, V, is_sep, a: int, n: int, scale: float, rows: Optional[np.ndarray] = None,
            return_A: bool = False, precision: str = "f64", n_head=None):
    """Eq. 1 with the mask of Eq. 2.  Returns (O [B,Hq,R,d], LSE [B,Hq,R]) and A [B,Hq,R,L] if asked.

    rows (int32 list) restricts the computation to those query rows; R = len(rows) or L.
    n_head [Hq], if given, replaces n by a neighbour window of its own for every query head (the
    head-wise variant of Sec. 4.6).
    """
    rt = _real(precision)
    Q, K, V = _c(Q, rt), _c(K, rt), _c(V, rt)
    is_sep = _c(is_sep, np.uint8)
    B, Hq, L, d = Q.shape
    Hkv = K.shape[1]
    assert K.shape == (B, Hkv, L, d) and V.shape == K.shape and is_sep.shape == (B, L)
    if rows is not None:
        rows = _c(rows, np.int32)
        R = int(rows.size)
    else:
        R = L
    O = np.zeros((B, Hq, R, d), dtype=rt)
    LSE = np.zeros((B, Hq, R), dtype=rt)
    A = np.zeros((B, Hq, R, L), dtype=rt) if return_A else None
    fn = _lib(precision).oracle_forward
    fn.restype = ctypes.c_int
    rc = fn(_ptr(Q), _ptr(K), _ptr(V), _ptr(is_sep), B, Hq, Hkv, L, d, int(a), int(n),
            _ptr(_n_head(n_head, Hq)), ctypes.c_double(scale), _ptr(rows), R, _ptr(O), _ptr(LSE), _ptr(A))
    if rc != 0:
        raise ValueError(f"oracle_forward failed with code {rc}")
    return (O, LSE, A) if return_A else (O, LSE)


def backward(Q, K, V, dO, is_sep, a: int, n: int, scale: float, precision: str = "f64", n_head=None,
             return_term_rss: bool = False):
    """Analytic gradient of Eq. 1: returns (dQ [B,Hq,L,d], dK, dV [B,Hkv,L,d]).

    With return_term_rss also (eQ, eK, eV): for every gradient element the root of the sum of the
    squares of the terms it adds up (see oracle_backward), the scale of the error that rounding the
    attention weights to a short format before the sum must cause."""
    rt = _real(precision)
    Q, K, V, dO = _c(Q, rt), _c(K, rt), _c(V, rt), _c(dO, rt)
    is_sep = _c(is_sep, np.uint8)
    B, Hq, L, d = Q.shape
    Hkv = K.shape[1]
    assert dO.shape == Q.shape and V.shape == K.shape
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    eQ, eK, eV = (np.zeros_like(x) for x in (Q, K, V)) if return_term_rss else (None, None, None)
    fn = _lib(precision).oracle_backward
    fn.restype = ctypes.c_int
    rc = fn(_ptr(Q), _ptr(K), _ptr(V), _ptr(dO), _ptr(is_sep), B, Hq, Hkv, L, d, int(a), int(n),
            _ptr(_n_head(n_head, Hq)), ctypes.c_double(scale), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(eQ), _ptr(eK),
            _ptr(eV))
    if rc != 0:
        raise ValueError(f"oracle_backward failed with code {rc}")
    return (dQ, dK, dV, eQ, eK, eV) if return_term_rss else (dQ, dK, dV)


def decode(q, Kc, Vc, sizes, a: int, s: int, scale: float, precision: str = "f64"):
    """Single-query attention over every valid entry of the four-block cache (Sec. 3.2 / 3.3)."""
    rt = _real(precision)
    q, Kc, Vc = _c(q, rt), _c(Kc, rt), _c(Vc, rt)
    sizes = _c(sizes, np.int32)
    S, Hq, d = q.shape
    _, Hkv, c, _ = Kc.shape
    out = np.zeros((S, Hq, d), dtype=rt)
    lse = np.zeros((S, Hq), dtype=rt)
    fn = _lib(precision).oracle_decode
    fn.restype = ctypes.c_int
    rc = fn(_ptr(q), _ptr(Kc), _ptr(Vc), _ptr(sizes), S, Hq, Hkv, d, int(a), int(s), c,
            ctypes.c_double(scale), _ptr(out), _ptr(lse))
    if rc != 0:
        raise ValueError(f"oracle_decode failed with code {rc}")
    return out, lse


def evict_window(Kc: np.ndarray, Vc: np.ndarray, win_is_sep: np.ndarray, sizes: np.ndarray,
                 a: int, s: int):
    """Compression step of Sec. 3.3 on copies of the inputs; rows are moved as raw bytes.

    Kc, Vc: [S,Hkv,c,d] of any fixed-width dtype.  Returns (Kc', Vc', win_is_sep', sizes').
    Slots beyond the new sizes hold unspecified data.
    """
    Kc = np.array(Kc, copy=True, order="C")
    Vc = np.array(Vc, copy=True, order="C")
    fl = np.array(win_is_sep, dtype=np.uint8, copy=True, order="C")
    sz = np.array(sizes, dtype=np.int32, copy=True, order="C")
    S, Hkv, c, d = Kc.shape
    fn = _lib("f64").oracle_evict_window
    fn.restype = ctypes.c_int
    rc = fn(_ptr(Kc), _ptr(Vc), _ptr(fl), _ptr(sz), S, Hkv, int(a), int(s), c,
            ctypes.c_long(d * Kc.dtype.itemsize))
    if rc != 0:
        raise ValueError(f"oracle_evict_window failed with code {rc}")
    return Kc, Vc, fl, sz


def fill_from_prefill(K: np.ndarray, V: np.ndarray, is_sep: np.ndarray, a: int, s: int, w: int, c: int,
                      nw: int):
    """Hand-over from prefill to the four-block cache (Sec. 3.2 "Generation", Sec. 3.3): keep the
    initial tokens, the newest (at most s) separators older than the window, and the last nw tokens.

    K, V: [S,Hkv,L,d] of any fixed-width dtype; is_sep: [S,L].  Returns (Kc, Vc, win_is_sep, sizes,
    valid) with Kc, Vc [S,Hkv,c,d] (zero where no row was placed), win_is_sep uint8 [S,c-a-s],
    sizes int32 [S,4] and valid bool [S,c]: the slots that hold a row.
    """
    S, Hkv, L, d = K.shape
    wcap = c - a - s
    assert 0 <= nw <= min(wcap, L - min(a, L))
    Kc = np.zeros((S, Hkv, c, d), dtype=K.dtype)
    Vc = np.zeros((S, Hkv, c, d), dtype=V.dtype)
    flags = np.zeros((S, wcap), dtype=np.uint8)
    sizes = np.zeros((S, 4), dtype=np.int32)
    valid = np.zeros((S, c), dtype=bool)
    for q in range(S):
        n_init = min(a, L)
        wstart = L - nw
        old_seps = [j for j in range(n_init, wstart) if is_sep[q, j]]
        kept = old_seps[len(old_seps) - min(s, len(old_seps)):]
        placed = [(t, t) for t in range(n_init)]
        placed += [(a + k, j) for k, j in enumerate(kept)]
        placed += [(a + s + u, wstart + u) for u in range(nw)]
        for slot, j in placed:
            Kc[q, :, slot] = K[q, :, j]
            Vc[q, :, slot] = V[q, :, j]
            valid[q, slot] = True
        for u in range(nw):
            flags[q, u] = 1 if is_sep[q, wstart + u] else 0
        wl = min(w, nw)
        sizes[q] = (n_init, len(kept), nw - wl, wl)
    return Kc, Vc, flags, sizes, valid


def rope_rotate(x: np.ndarray, pos, base: float) -> np.ndarray:
    """Rotary position encoding of x [..., d] at position(s) `pos` (broadcast over x's leading axes).

    Sec. 3.3 "Positional Encoding" fixes which positions are used (those within the cache); the
    rotation itself is the one of the Llama / Pythia backbones the paper evaluates (Sec. 4.1): dimension
    i < d/2 is paired with i + d/2 and the pair is turned by pos * base**(-2i/d).  The paper prints
    neither the pairing nor the base: this reading is [parity unpinned] against the paper; the pins
    hold the function to the reading.
    """
    x = np.asarray(x, dtype=np.float64)
    d = x.shape[-1]
    h = d // 2
    theta = np.float64(base) ** (-2.0 * np.arange(h, dtype=np.float64) / d)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * theta
    co, si = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :h], x[..., h:]
    return np.concatenate([x1 * co - x2 * si, x2 * co + x1 * si], axis=-1)


def cache_slots(sizes_row: np.ndarray, a: int, s: int) -> np.ndarray:
    """Slots of the valid entries of one sequence, oldest first: Initial Cache, Separator Cache,
    Past Window Cache, Local Window Cache (Sec. 3.3)."""
    n_init, n_sep, n_past, n_loc = (int(v) for v in sizes_row)
    return np.concatenate([np.arange(n_init), a + np.arange(n_sep), a + s + np.arange(n_past + n_loc)]).astype(np.int64)


def decode_rope(q: np.ndarray, Kc: np.ndarray, Vc: np.ndarray, sizes: np.ndarray, a: int, s: int,
                scale: float, base: float):
    """Single-query attention over the cache with positions taken *within the cache* (Sec. 3.3
    "Positional Encoding"; Sec. 4.6, the ablation of the positional shifting): the valid entries, oldest
    first, are at positions 0 .. nv-1 and the query (the newest entry's token) at nv-1.  q and the
    cached keys are stored without position encoding.  Returns (out [S,Hq,d], lse [S,Hq]) in fp64.
    """
    q = np.asarray(q, dtype=np.float64)
    Kc = np.asarray(Kc, dtype=np.float64)
    Vc = np.asarray(Vc, dtype=np.float64)
    S, Hq, d = q.shape
    Hkv = Kc.shape[1]
    G = Hq // Hkv
    out = np.zeros((S, Hq, d))
    lse = np.full((S, Hq), -np.inf)
    for sq in range(S):
        slots = cache_slots(sizes[sq], a, s)
        nv = len(slots)
        if nv == 0:
            continue
        for h in range(Hq):
            kv = h // G
            Kr = rope_rotate(Kc[sq, kv, slots], np.arange(nv), base)
            qr = rope_rotate(q[sq, h], nv - 1, base)
            sc = scale * (Kr @ qr)
            m = sc.max()
            p = np.exp(sc - m)
            lse[sq, h] = m + np.log(p.sum())
            out[sq, h] = (p / p.sum()) @ Vc[sq, kv, slots]
    return out, lse


def append_token(Kc: np.ndarray, Vc: np.ndarray, win_is_sep: np.ndarray, sizes: np.ndarray,
                 k_new: np.ndarray, v_new: np.ndarray, is_sep_new: np.ndarray, a: int, s: int, w: int):
    """One new token per sequence enters the cache (Sec. 3.3 "Framework"): the Initial Cache takes the
    first a tokens; later tokens enter the Local Window Cache, whose oldest entry passes to the Past
    Window Cache once it holds more than w.  A sequence whose window region [a+s, c) is full is left
    as it is (the compression step has to run first).  Works on copies; k_new, v_new: [S,Hkv,d].
    """
    Kc = np.array(Kc, copy=True)
    Vc = np.array(Vc, copy=True)
    fl = np.array(win_is_sep, dtype=np.uint8, copy=True)
    sz = np.array(sizes, dtype=np.int32, copy=True)
    S, _, c, _ = Kc.shape
    wcap = c - a - s
    for sq in range(S):
        n_init, n_sep, n_past, n_loc = (int(v) for v in sz[sq])
        if n_init < a:
            Kc[sq, :, n_init] = k_new[sq]
            Vc[sq, :, n_init] = v_new[sq]
            sz[sq, 0] = n_init + 1
            continue
        u = n_past + n_loc
        if u >= wcap:
            continue
        Kc[sq, :, a + s + u] = k_new[sq]
        Vc[sq, :, a + s + u] = v_new[sq]
        fl[sq, u] = 1 if is_sep_new[sq] else 0
        n_loc += 1
        if n_loc > w:
            n_loc -= 1
            n_past += 1
        sz[sq, 2], sz[sq, 3] = n_past, n_loc
    return Kc, Vc, fl, sz


def doc_bounds(cu_seqlens: np.ndarray, L: int) -> Tuple[np.ndarray, np.ndarray]:
    """Packed documents in one row of L positions: document k covers [cu[k], cu[k+1]), cu[0] = 0,
    cu[-1] = L.  Returns, per position, the first position of its document and one past its last."""
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    assert cu[0] == 0 and cu[-1] == L and (np.diff(cu) > 0).all()
    start = np.zeros(L, dtype=np.int32)
    end = np.zeros(L, dtype=np.int32)
    for k in range(len(cu) - 1):
        start[cu[k]:cu[k + 1]] = cu[k]
        end[cu[k]:cu[k + 1]] = cu[k + 1]
    return start, end


def forward_packed(Q, K, V, is_sep, cu_seqlens, a: int, n: int, scale: float, precision: str = "f64"):
    """SepAttention over a row of packed documents: every document is a sequence of its own (its first
    a tokens are its initial tokens, a query sees nothing outside its document), i.e. Eq. 1 / Eq. 2
    applied to each slice [cu[k], cu[k+1]) separately.  cu_seqlens: one array per batch row."""
    Q, K, V = (np.asarray(x) for x in (Q, K, V))
    B, Hq, L, d = Q.shape
    O = np.zeros((B, Hq, L, d), dtype=np.float64 if precision == "f64" else np.float32)
    LSE = np.zeros((B, Hq, L), dtype=O.dtype)
    for b in range(B):
        cu = np.asarray(cu_seqlens[b], dtype=np.int64)
        for k in range(len(cu) - 1):
            s, e = int(cu[k]), int(cu[k + 1])
            o, l = forward(Q[b:b + 1, :, s:e], K[b:b + 1, :, s:e], V[b:b + 1, :, s:e], is_sep[b:b + 1, s:e], a, n,
                           scale, precision=precision)
            O[b, :, s:e], LSE[b, :, s:e] = o[0], l[0]
    return O, LSE


def backward_packed(Q, K, V, dO, is_sep, cu_seqlens, a: int, n: int, scale: float, precision: str = "f64",
                    return_term_rss: bool = False):
    """Gradients of forward_packed: document by document (with return_term_rss also eQ, eK, eV of
    `backward`)."""
    Q, K, V, dO = (np.asarray(x) for x in (Q, K, V, dO))
    rt = np.float64 if precision == "f64" else np.float32
    outs = [np.zeros(x.shape, dtype=rt) for x in (Q, K, V)] + \
           ([np.zeros(x.shape, dtype=rt) for x in (Q, K, V)] if return_term_rss else [])
    for b in range(Q.shape[0]):
        cu = np.asarray(cu_seqlens[b], dtype=np.int64)
        for k in range(len(cu) - 1):
            s, e = int(cu[k]), int(cu[k + 1])
            res = backward(Q[b:b + 1, :, s:e], K[b:b + 1, :, s:e], V[b:b + 1, :, s:e], dO[b:b + 1, :, s:e],
                           is_sep[b:b + 1, s:e], a, n, scale, precision=precision, return_term_rss=return_term_rss)
            for dst, src in zip(outs, res):
                dst[b, :, s:e] = src[0]
    return tuple(outs)


def mark_doc_initial(is_sep: np.ndarray, doc_start: np.ndarray, a: int) -> np.ndarray:
    """Marker bitmap with the first a tokens of every document added (they are visible to every later
    query of their document, exactly like its separators)."""
    pos = np.arange(is_sep.shape[1])[None, :]
    return (np.asarray(is_sep, dtype=bool) | (pos - doc_start < a)).astype(np.uint8)
