"""Seeded, synthetic stand-ins for the paper's workloads (input generation only).

The paper trains on Pile and evaluates on PG19 and others with Pythia / Llama-3 weights; none of
those are available, so every input here is random with the shapes and separator densities of
those workloads. Random numbers come from numpy's counter-based Philox generator keyed by an
explicit seed, so the CPU oracle and the GPU path are fed bit-identical arrays.

Nothing in this file computes a mask, an attention score or a compaction.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

VOCAB = 32000
# Nine arbitrary, distinct token ids standing for the nine separator strings of Sec. 4.1
# ("Parameter Setting"); the tokenizer itself is outside this build.
SEPARATOR_IDS = np.array([17, 402, 1999, 5003, 8191, 12000, 20480, 27777, 31999], dtype=np.int32)

BASE_SEED = 0x5E9A77


@dataclass(frozen=True)
class AttnConfig:
    """One training / prefill workload: shapes, mask hyper-parameters (a, n) and separator density p."""

    name: str
    B: int
    Hq: int
    Hkv: int
    L: int
    d: int
    a: int
    n: int
    p: float
    dtype: str  # "bf16" or "fp32"
    qkv_scale: float
    seed: int
    backward: bool

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))


@dataclass(frozen=True)
class CacheConfig:
    """One streaming-decode workload: S sequences, cache capacities (a, s, w, c)."""

    name: str
    S: int
    Hq: int
    Hkv: int
    d: int
    a: int
    s: int
    w: int
    c: int
    p: float
    dtype: str
    seed: int

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))

    @property
    def window_capacity(self) -> int:
        return self.c - self.a - self.s


CONFIGS: Dict[str, object] = {
    # tiny forward-only check, fp32 path
    "cfg1": AttnConfig("cfg1", B=1, Hq=1, Hkv=1, L=512, d=64, a=4, n=64, p=1.0 / 8, dtype="fp32",
                       qkv_scale=1.0, seed=BASE_SEED + 1, backward=False),
    # Pythia-160m-like training shape
    "cfg2": AttnConfig("cfg2", B=8, Hq=12, Hkv=12, L=2048, d=64, a=4, n=64, p=0.10, dtype="bf16",
                       qkv_scale=1.0, seed=BASE_SEED + 2, backward=True),
    # Llama-3-8B attention shape at 8K: the headline workload
    "cfg3": AttnConfig("cfg3", B=1, Hq=32, Hkv=8, L=8192, d=128, a=4, n=256, p=0.08, dtype="bf16",
                       qkv_scale=0.5, seed=BASE_SEED + 3, backward=True),
    # long-context prefill, forward only
    "cfg4": AttnConfig("cfg4", B=1, Hq=32, Hkv=8, L=65536, d=128, a=4, n=1024, p=0.08, dtype="bf16",
                       qkv_scale=0.5, seed=BASE_SEED + 4, backward=False),
    # streaming decode on the compressed cache: 4 + 2048 + 1024 + 256 entries
    "cfg5": CacheConfig("cfg5", S=32, Hq=32, Hkv=8, d=128, a=4, s=2048, w=256, c=3332, p=0.08,
                        dtype="bf16", seed=BASE_SEED + 5),
}


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed) & 0xFFFFFFFFFFFFFFFF, int(stream)]))


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even) and return them as fp32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def make_token_ids(B: int, L: int, p: float, seed: int, placement: str = "iid") -> np.ndarray:
    """int32 [B, L] token ids; a position holds one of SEPARATOR_IDS with probability p.

    placement "iid": independent Bernoulli(p) per position. placement "geometric": the gap to the
    next separator is drawn Geometric(p) on {1, 2, ...} (the same law written as segment
    lengths). Non-separator positions draw uniformly from the vocabulary minus SEPARATOR_IDS, so
    the separator density is exactly what the Bernoulli / geometric draw produced.
    """
    g = _rng(seed, 1)
    if placement == "iid":
        sep = g.random((B, L)) < p
    elif placement == "geometric":
        sep = np.zeros((B, L), dtype=bool)
        for b in range(B):
            if p <= 0.0:
                break
            pos = -1
            # enough gaps to cover L with overwhelming margin, redrawn if short
            while pos < L:
                gaps = g.geometric(p, size=max(16, int(2 * L * p) + 16))
                idx = pos + np.cumsum(gaps)
                sep[b, idx[idx < L]] = True
                pos = int(idx[-1])
    else:
        raise ValueError(f"unknown placement {placement!r}")
    non_sep_vocab = np.setdiff1d(np.arange(VOCAB, dtype=np.int32), SEPARATOR_IDS)
    ids = non_sep_vocab[g.integers(0, non_sep_vocab.size, size=(B, L))]
    which = SEPARATOR_IDS[g.integers(0, SEPARATOR_IDS.size, size=(B, L))]
    return np.where(sep, which, ids).astype(np.int32)


def _normal(shape, scale: float, seed: int, stream: int, dtype: str) -> np.ndarray:
    x = _rng(seed, stream).standard_normal(shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    if dtype == "bf16":
        x = bf16_round(x)
    return x


def make_qkv(B, Hq, Hkv, L, d, scale, seed, dtype):
    """Q [B,Hq,L,d], K and V [B,Hkv,L,d], N(0,1)*scale, already rounded to `dtype`, returned as fp32."""
    Q = _normal((B, Hq, L, d), scale, seed, 2, dtype)
    K = _normal((B, Hkv, L, d), scale, seed, 3, dtype)
    V = _normal((B, Hkv, L, d), scale, seed, 4, dtype)
    return Q, K, V


def make_dO(B, Hq, L, d, seed, dtype):
    """Upstream gradient dO [B,Hq,L,d] ~ N(0,1), rounded to `dtype`, returned as fp32."""
    return _normal((B, Hq, L, d), 1.0, seed, 5, dtype)


def config_inputs(cfg: AttnConfig, placement: Optional[str] = None) -> Dict[str, np.ndarray]:
    """All inputs of one AttnConfig."""
    if placement is None:
        placement = "geometric" if cfg.name in ("cfg3", "cfg4") else "iid"
    out = {"token_ids": make_token_ids(cfg.B, cfg.L, cfg.p, cfg.seed, placement)}
    out["Q"], out["K"], out["V"] = make_qkv(cfg.B, cfg.Hq, cfg.Hkv, cfg.L, cfg.d, cfg.qkv_scale,
                                            cfg.seed, cfg.dtype)
    if cfg.backward:
        out["dO"] = make_dO(cfg.B, cfg.Hq, cfg.L, cfg.d, cfg.seed, cfg.dtype)
    return out


def make_cache(cfg: CacheConfig, sizes: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """A KV cache in the four-region layout [initial | separator | window] with per-sequence sizes.

    Kc, Vc: fp32 [S, Hkv, c, d] (values rounded to cfg.dtype); q: [S, Hq, d];
    sizes: int32 [S, 4] = (Size_init, Size_sep, Size_past_w, Size_local_w), all regions full
    unless given; win_is_sep: uint8 [S, c-a-s], one Bernoulli(p) flag per window slot.
    """
    S, Hkv, c, d = cfg.S, cfg.Hkv, cfg.c, cfg.d
    Kc = _normal((S, Hkv, c, d), 1.0, cfg.seed, 2, cfg.dtype)
    Vc = _normal((S, Hkv, c, d), 1.0, cfg.seed, 3, cfg.dtype)
    q = _normal((S, cfg.Hq, d), 1.0, cfg.seed, 4, cfg.dtype)
    if sizes is None:
        wcap = cfg.window_capacity
        sizes = np.tile(np.array([cfg.a, cfg.s, wcap - cfg.w, cfg.w], dtype=np.int32), (S, 1))
    flags = (_rng(cfg.seed, 5).random((S, cfg.window_capacity)) < cfg.p).astype(np.uint8)
    return {"Kc": Kc, "Vc": Vc, "q": q, "sizes": np.ascontiguousarray(sizes, dtype=np.int32),
            "win_is_sep": flags}


def cache_to_ring(Kc, Vc, flags, sizes4, heads, a: int, s: int, fill=None):
    """The library's physical cache layout for a cache given in LINEAR layout (every block's valid entries
    at the start of its slot range, oldest first): the Separator Cache and the window region are rings,
    separator k in slot a + (head_sep + k) mod s, window entry u at window index (head_win + u) mod wcap.

    Kc, Vc [S,Hkv,c,d] (any dtype), flags uint8 [S,wcap], sizes4 int32 [S,4], heads int32 [S,2].
    Slots (and flags) that hold no valid entry keep what the linear arrays held there, or `fill`.
    Returns (Kc_ring, Vc_ring, flags_ring, sizes6).  Data movement only: no arithmetic of the method."""
    Kc, Vc, flags = np.asarray(Kc), np.asarray(Vc), np.asarray(flags)
    S, _, c, _ = Kc.shape
    wcap = c - a - s
    Kp, Vp, Fp = Kc.copy(), Vc.copy(), flags.copy()
    if fill is not None:
        Kp[...] = fill
        Vp[...] = fill
    sizes6 = np.zeros((S, 6), dtype=np.int32)
    for q in range(S):
        ni, ns, npast, nl = (int(v) for v in sizes4[q])
        hs, hw = int(heads[q][0]), int(heads[q][1])
        sizes6[q] = (ni, ns, npast, nl, hs, hw)
        Kp[q, :, :ni], Vp[q, :, :ni] = Kc[q, :, :ni], Vc[q, :, :ni]
        for k in range(ns):
            t = a + (hs + k) % s
            Kp[q, :, t], Vp[q, :, t] = Kc[q, :, a + k], Vc[q, :, a + k]
        for u in range(npast + nl):
            t = (hw + u) % wcap
            Kp[q, :, a + s + t], Vp[q, :, a + s + t] = Kc[q, :, a + s + u], Vc[q, :, a + s + u]
            Fp[q, t] = flags[q, u]
    return Kp, Vp, Fp, sizes6


def cache_from_ring(Kp, Vp, Fp, sizes6, a: int, s: int):
    """Inverse of cache_to_ring: (Kc, Vc, flags, sizes4) in linear layout; slots and flags without a valid
    entry are zero."""
    Kp, Vp, Fp = np.asarray(Kp), np.asarray(Vp), np.asarray(Fp)
    S, _, c, _ = Kp.shape
    wcap = c - a - s
    Kc, Vc, flags = np.zeros_like(Kp), np.zeros_like(Vp), np.zeros_like(Fp)
    for q in range(S):
        ni, ns, npast, nl, hs, hw = (int(v) for v in sizes6[q])
        Kc[q, :, :ni], Vc[q, :, :ni] = Kp[q, :, :ni], Vp[q, :, :ni]
        for k in range(ns):
            t = a + (hs + k) % s
            Kc[q, :, a + k], Vc[q, :, a + k] = Kp[q, :, t], Vp[q, :, t]
        for u in range(npast + nl):
            t = (hw + u) % wcap
            Kc[q, :, a + s + u], Vc[q, :, a + s + u] = Kp[q, :, a + s + t], Vp[q, :, a + s + t]
            flags[q, u] = Fp[q, t]
    return Kc, Vc, flags, np.ascontiguousarray(np.asarray(sizes6)[:, :4], dtype=np.int32)


def small_variant(cfg: AttnConfig, **kw) -> AttnConfig:
    """A copy of cfg with some fields replaced (used for reduced-size parity cases)."""
    return replace(cfg, **kw)
