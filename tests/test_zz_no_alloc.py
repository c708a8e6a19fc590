"""The decode entry point that allocates nothing (for callers under graph capture or in serving loops
that cannot call hipMalloc): its outputs must equal those of sepattn_decode, which runs the same
kernels with a caller-provided workspace, bit for bit; two calls in a row, the second on a smaller
cache batch, share the library's fixed scratch array.  Needs an MI355X."""
import ctypes

import numpy as np
import pytest

import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sp():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2412_12094_amd as sp_

    sp_.load()
    return sp_


def _case(S, Hq, Hkv, d, a, s, w, c, seed):
    cfg = wl.CacheConfig("noalloc", S, Hq, Hkv, d, a, s, w, c, 0.1, "bf16", seed=seed)
    rng = np.random.default_rng(seed)
    sizes = np.zeros((S, 4), dtype=np.int32)
    for q in range(S):
        tot = int(rng.integers(1, c - a - s + 1))
        sizes[q] = (a, int(rng.integers(0, s + 1)), tot - min(w, tot), min(w, tot))
    data = wl.make_cache(cfg, sizes)
    heads = np.stack([rng.integers(0, s, size=S), rng.integers(0, c - a - s, size=S)], axis=1)
    Kp, Vp, _, sizes6 = wl.cache_to_ring(data["Kc"], data["Vc"], data["win_is_sep"], sizes, heads, a, s)
    bf = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda().to(torch.bfloat16).contiguous()
    return cfg, bf(data["q"]), bf(Kp), bf(Vp), torch.from_numpy(sizes6).cuda()


def test_decode_noalloc_equals_decode_on_two_calls_in_a_row(sp):
    from paper_2412_12094_amd import binding as bd

    lib = bd.load()
    # several slices per cache, so that the partial results do go through the scratch array; the
    # second call is smaller in every dimension of the scratch layout (sequences, heads, slices)
    shapes = [(2, 32, 1, 128, 4, 500, 64, 900), (1, 8, 1, 64, 2, 100, 16, 300)]
    for i, (S, Hq, Hkv, d, a, s, w, c) in enumerate(shapes):
        cfg, q, Kc, Vc, sizes = _case(S, Hq, Hkv, d, a, s, w, c, 500 + i)
        p = bd._kv_params(q, Kc, a, s, w, cfg.scale)
        need = lib.sepattn_decode_noalloc_scratch_bytes(ctypes.byref(p))
        assert 2 * S * Hq * (d + 2) * 4 <= need <= (4 << 20), need  # at least two slices: the scratch array is in use
        want_o, want_l = sp.sepattn_decode(q, Kc, Vc, sizes, a, s, w, cfg.scale)
        out = (torch.full_like(q, 7.0), torch.full((S, Hq), 7.0, dtype=torch.float32, device="cuda"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        sp.sepattn_decode_noalloc(q, Kc, Vc, sizes, a, s, w, cfg.scale, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(out[0], want_o) and torch.equal(out[1], want_l), i


def test_decode_noalloc_rejects_what_does_not_fit(sp):
    from paper_2412_12094_amd import binding as bd

    lib = bd.load()
    # 512 sequences x 64 heads: the partial results of the slices exceed the fixed array
    S, Hq, Hkv, d, a, s, w, c = 512, 64, 64, 128, 4, 16, 8, 64
    q = torch.zeros((S, Hq, d), dtype=torch.bfloat16, device="cuda")
    Kc = torch.zeros((S, Hkv, c, d), dtype=torch.bfloat16, device="cuda")
    sizes = torch.zeros((S, 6), dtype=torch.int32, device="cuda")
    p = bd._kv_params(q, Kc, a, s, w, 0.1)
    assert lib.sepattn_decode_noalloc_scratch_bytes(ctypes.byref(p)) > (4 << 20)
    out = torch.empty_like(q)
    rc = lib.sepattn_decode_noalloc(ctypes.byref(p), bd._ptr(q), bd._ptr(Kc), bd._ptr(Kc), bd._ptr(sizes), bd._ptr(out),
                                    None, None)
    assert rc == 5
