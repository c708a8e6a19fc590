"""Host-side checks that need no GPU: the C-ABI library loads and exports every symbol the header
declares, argument validation returns the documented status codes before anything is launched,
workspace queries are consistent, and the benchmark's pair accounting agrees with the oracle's mask."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sepattn.h")


@pytest.fixture(scope="module")
def sp():
    import paper_2412_12094_amd as sp_

    if not os.path.exists(sp_.LIB_PATH):
        from paper_2412_12094_amd import build

        build.build()
    sp_.load()
    return sp_


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sep(?:attn|kv)_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(sp):
    lib = sp.load()
    names = declared_functions()
    assert len(names) >= 15
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(sp.EXPORTS)


def test_status_strings(sp):
    seen = {sp.status_string(k) for k in range(8)}
    assert len(seen) == 8 and sp.status_string(0) == "ok"
    assert sp.status_string(99) == "unknown status"


def attn_params(sp, **kw):
    base = dict(B=1, Hq=8, Hkv=2, L=1024, d=128, a=4, n=64, scale=0.088, dtype=0, cap=1024)
    base.update(kw)
    return sp.SepattnParams(*[base[k] for k in ("B", "Hq", "Hkv", "L", "d", "a", "n", "scale", "dtype", "cap")])


def kv_params(sp, **kw):
    base = dict(S=2, Hq=8, Hkv=2, d=128, a=4, s=64, w=32, c=200, scale=0.088, dtype=0)
    base.update(kw)
    return sp.SepkvParams(*[base[k] for k in ("S", "Hq", "Hkv", "d", "a", "s", "w", "c", "scale", "dtype")])


FAKE = ctypes.c_void_p(0x1000)  # never dereferenced: every call below fails validation first


def fwd(sp, p, q=FAKE):
    return sp.load().sepattn_forward(ctypes.byref(p), q, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None)


def test_forward_validation_codes(sp):
    assert fwd(sp, attn_params(sp), q=None) == 1                      # NULL
    assert fwd(sp, attn_params(sp, L=0)) == 2                         # shape
    assert fwd(sp, attn_params(sp, Hq=6, Hkv=4)) == 2                 # Hq % Hkv
    assert fwd(sp, attn_params(sp, n=0)) == 3                         # n >= 1
    assert fwd(sp, attn_params(sp, a=-1)) == 3
    assert fwd(sp, attn_params(sp, scale=float("nan"))) == 3
    assert fwd(sp, attn_params(sp, d=96)) == 4                        # head dim
    assert fwd(sp, attn_params(sp, dtype=7)) == 4
    assert fwd(sp, attn_params(sp, cap=0)) == 6
    assert fwd(sp, attn_params(sp), q=ctypes.c_void_p(0x1004)) == 3   # misaligned
    assert sp.load().sepattn_forward(None, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, None) == 1


def test_backward_needs_workspace(sp):
    lib = sp.load()
    p = attn_params(sp)
    need = lib.sepattn_backward_workspace_bytes(ctypes.byref(p))
    assert need > 1024 * 8 * 4 and need % 256 == 0
    args = [FAKE] * 13
    assert lib.sepattn_backward(ctypes.byref(p), *args, 0, None) == 5           # ws NULL
    args[-1] = FAKE
    assert lib.sepattn_backward(ctypes.byref(p), *args, need - 1, None) == 5    # too small
    assert lib.sepattn_backward_workspace_bytes(ctypes.byref(attn_params(sp, n=0))) == 0


def test_mark_and_compact_validation(sp):
    lib = sp.load()
    ids = (ctypes.c_int32 * 3)(1, 2, 3)
    idp = ctypes.cast(ids, ctypes.c_void_p)
    assert lib.sepattn_mark_separators(None, 1, 8, idp, 3, FAKE, None) == 1
    assert lib.sepattn_mark_separators(FAKE, 0, 8, idp, 3, FAKE, None) == 2
    assert lib.sepattn_mark_separators(FAKE, 1, 8, idp, 0, FAKE, None) == 3
    assert lib.sepattn_mark_separators(FAKE, 1, 8, idp, 65, FAKE, None) == 3
    assert lib.sepattn_compact_workspace_bytes(2, 5000) >= 2 * 3 * 4
    assert lib.sepattn_compact_indices(FAKE, 1, 8, FAKE, 0, FAKE, FAKE, FAKE, 256, None) == 6
    assert lib.sepattn_compact_indices(FAKE, 1, 8, FAKE, 8, FAKE, FAKE, None, 0, None) == 5
    assert lib.sepattn_compact_indices(None, 1, 8, FAKE, 8, FAKE, FAKE, FAKE, 256, None) == 1
    mc = lambda tok=FAKE, L=8, n=3, cap=8, ws=FAKE, wsb=256: lib.sepattn_mark_compact(
        tok, 1, L, idp, n, FAKE, FAKE, cap, FAKE, FAKE, ws, wsb, None)
    assert mc(tok=None) == 1 and mc(L=0) == 2 and mc(n=0) == 3 and mc(n=65) == 3
    assert mc(cap=0) == 6 and mc(ws=None, wsb=0) == 5 and mc(tok=ctypes.c_void_p(0x1004)) == 3


def test_cache_call_validation(sp):
    lib = sp.load()
    ok = kv_params(sp)
    assert lib.sepattn_decode_workspace_bytes(ctypes.byref(ok)) >= 2 * 8 * 130 * 4
    assert lib.sepkv_evict_workspace_bytes(ctypes.byref(ok)) == 0   # the compression step needs no scratch memory
    dec = lambda p, q=FAKE: lib.sepattn_decode(ctypes.byref(p), q, FAKE, FAKE, FAKE, FAKE, None, None, 0, None)
    assert dec(ok, None) == 1
    assert dec(kv_params(sp, a=100, s=80, w=32, c=200)) == 3   # a + s + w >= c
    assert dec(kv_params(sp, w=0)) == 3
    assert dec(kv_params(sp, d=100)) == 4
    assert dec(kv_params(sp, S=0)) == 2
    assert dec(kv_params(sp, c=(1 << 23) + 1)) == 2            # a slot's byte offset would not fit 32 bits
    assert dec(kv_params(sp, c=1 << 22)) == 5                  # the largest cache that does (then: no workspace)
    assert dec(ok) == 5                                        # workspace missing
    na = lambda p, q=FAKE: lib.sepattn_decode_noalloc(ctypes.byref(p), q, FAKE, FAKE, FAKE, FAKE, None, None)
    assert na(ok, None) == 1 and na(kv_params(sp, w=0)) == 3 and na(kv_params(sp, d=100)) == 4
    assert na(kv_params(sp, S=4096, Hq=8, Hkv=8, c=200)) == 5  # partial results beyond the fixed scratch array
    ev = lambda p, k=FAKE: lib.sepkv_evict_window(ctypes.byref(p), k, FAKE, FAKE, FAKE, None, 0, None)
    assert ev(ok, None) == 1 and ev(ok, ctypes.c_void_p(0x1004)) == 3   # NULL; misaligned cache
    assert ev(kv_params(sp, Hq=7, Hkv=2)) == 2


def test_profile_hook_argument_checks(sp):
    lib = sp.load()
    h = ctypes.c_void_p()
    assert lib.sepattn_profile_create(-1, 4, ctypes.byref(h)) == 3 and lib.sepattn_profile_create(3, 0, ctypes.byref(h)) == 3
    assert lib.sepattn_profile_create(3, 4, None) == 1 and not h
    assert lib.sepattn_profile_attach(None) == 1 and lib.sepattn_profile_detach(None) == 1
    n = ctypes.c_int(0)
    ms = (ctypes.c_float * 4)()
    assert lib.sepattn_profile_read(None, ms, 4, ctypes.byref(n)) == 1
    lib.sepattn_profile_destroy(None)  # a no-op
    names = {sp.sepattn_kernel_name(k) for k in range(17)}
    assert len(names) == 17 and sp.sepattn_kernel_name(17) == "unknown"


def test_binding_refuses_cpu_tensors(sp):
    import torch

    with pytest.raises(ValueError):
        sp.sepattn_mark_separators(torch.zeros((1, 8), dtype=torch.int32), [1, 2])


def test_bench_pair_accounting_matches_oracle_mask():
    import bench
    import oracle

    rng = np.random.default_rng(0)
    for L, a, n, p in ((300, 4, 64, 0.1), (257, 0, 1, 0.3), (100, 200, 7, 0.2), (64, 3, 500, 0.0)):
        flags = (rng.random(L) < p).astype(np.uint8)
        M = oracle.mask(flags, a, n)
        assert bench.count_visible_pairs(flags, min(a, L), min(n, L)) == int(M.sum())
        i, j = np.nonzero(M)
        assert bench.count_far_pairs(flags, min(a, L), min(n, L)) == int((i - j >= min(n, L)).sum())


def test_workload_generators_are_deterministic_and_shaped():
    import workloads as wl

    c = wl.CONFIGS["cfg1"]
    a, b = wl.config_inputs(c), wl.config_inputs(c)
    for k in a:
        assert np.array_equal(a[k], b[k])
    assert a["Q"].shape == (1, 1, 512, 64) and a["token_ids"].dtype == np.int32
    tok = wl.make_token_ids(2, 20000, 0.08, 3, "geometric")
    dens = np.isin(tok, wl.SEPARATOR_IDS).mean()
    assert abs(dens - 0.08) < 0.01
    x = wl.make_qkv(1, 2, 1, 16, 64, 0.5, 9, "bf16")[0]
    assert np.array_equal(wl.bf16_round(x), x)  # already on the bf16 grid
    cc = wl.CONFIGS["cfg5"]
    assert cc.a + cc.s + cc.w < cc.c and cc.window_capacity == 1280


def test_ring_layout_helpers_round_trip():
    """The test helpers that lay a linear cache out as the library's rings and back are inverse to each
    other on the valid entries, and with both heads at 0 the ring layout IS the linear one."""
    import workloads as wl

    rng = np.random.default_rng(0)
    S, Hkv, d, a, s, c = 3, 2, 4, 2, 5, 2 + 5 + 7
    Kc = rng.integers(0, 1000, size=(S, Hkv, c, d)).astype(np.int32)
    Vc = rng.integers(0, 1000, size=(S, Hkv, c, d)).astype(np.int32)
    fl = rng.integers(0, 2, size=(S, 7)).astype(np.uint8)
    sizes = np.array([[2, 5, 4, 3], [1, 2, 0, 2], [0, 0, 0, 0]], dtype=np.int32)
    heads = np.array([[3, 5], [4, 6], [0, 0]], dtype=np.int32)
    Kp, Vp, Fp, s6 = wl.cache_to_ring(Kc, Vc, fl, sizes, heads, a, s)
    assert np.array_equal(s6[:, :4], sizes) and np.array_equal(s6[:, 4:], heads)
    assert np.array_equal(Kp[0, :, a + (3 + 4) % 5], Kc[0, :, a + 4])            # newest separator wrapped to slot a+2
    assert np.array_equal(Vp[0, :, a + s + (5 + 6) % 7], Vc[0, :, a + s + 6])    # newest window entry wrapped
    K2, V2, F2, s4 = wl.cache_from_ring(Kp, Vp, Fp, s6, a, s)
    for q in range(S):
        ni, ns, npast, nl = sizes[q]
        for g, r in ((K2, Kc), (V2, Vc)):
            assert np.array_equal(g[q, :, :ni], r[q, :, :ni]) and np.array_equal(g[q, :, a:a + ns], r[q, :, a:a + ns])
            assert np.array_equal(g[q, :, a + s:a + s + npast + nl], r[q, :, a + s:a + s + npast + nl])
        assert np.array_equal(F2[q, :npast + nl], fl[q, :npast + nl])
    K0, V0, F0, _ = wl.cache_to_ring(Kc, Vc, fl, sizes, np.zeros((S, 2), np.int32), a, s)
    assert np.array_equal(K0, Kc) and np.array_equal(V0, Vc) and np.array_equal(F0, fl)
