"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU needed).

Each test holds the oracle to something other than itself: a value the paper prints, a closed
form, a special case that reduces to a textbook / library routine, or brute force on tiny inputs.
"""
import math
import os

import numpy as np
import pytest

import oracle
from oracle import cache_sim

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


def _flags(B, L, p, seed):
    return (np.random.default_rng(seed).random((B, L)) < p).astype(np.uint8)


# ----------------------------------------------------------------------------------------------
# independent helpers written for the tests only
# ----------------------------------------------------------------------------------------------
def visible_set(i, is_sep, a, n):
    """Sec. 3.1 in set language: Init ∪ Sep ∪ Nbr(i), restricted to keys not after i."""
    init = set(range(0, a))
    seps = {j for j, f in enumerate(is_sep) if f}
    nbr = set(range(i - n + 1, i + 1))
    return {j for j in (init | seps | nbr) if 0 <= j <= i}


def softmax_attention_dense(Q, K, V, allowed, scale):
    """Textbook masked attention for one head in numpy fp64. allowed: bool [L,L]."""
    S = (Q @ K.T) * scale
    S = np.where(allowed, S, -np.inf)
    m = S.max(axis=1, keepdims=True)
    P = np.exp(S - m)
    l = P.sum(axis=1, keepdims=True)
    return (P / l) @ V, (m + np.log(l))[:, 0]


def per_pair_forward(Q, K, V, is_sep, a, n, scale):
    """Pure-python per-pair evaluation of Eq. 1 / Eq. 2 for one head (tiny inputs only)."""
    L, d = Q.shape
    O = np.zeros((L, d))
    LSE = np.zeros(L)
    for i in range(L):
        vis = sorted(visible_set(i, is_sep, a, n))
        lam = [scale * sum(Q[i, k] * K[j, k] for k in range(d)) for j in vis]
        mx = max(lam)
        w = [math.exp(x - mx) for x in lam]
        den = sum(w)
        for jj, j in enumerate(vis):
            for k in range(d):
                O[i, k] += w[jj] / den * V[j, k]
        LSE[i] = mx + math.log(den)
    return O, LSE


# ----------------------------------------------------------------------------------------------
# mark / compact
# ----------------------------------------------------------------------------------------------
def test_mark_matches_numpy_isin():
    rng = np.random.default_rng(0)
    ids = rng.integers(0, 50, size=(3, 257)).astype(np.int32)
    seps = np.array([3, 7, 49, 0], dtype=np.int32)
    got = oracle.mark_separators(ids, seps)
    assert got.dtype == np.uint8
    assert np.array_equal(got.astype(bool), np.isin(ids, seps))


def test_compact_invariants_and_brute_force():
    is_sep = _flags(4, 300, 0.2, 1)
    is_sep[1] = 0  # a sequence with no separator
    is_sep[2] = 1  # a sequence of separators only
    idx, cnt, pre = oracle.compact_indices(is_sep)
    for b in range(4):
        want = [j for j in range(300) if is_sep[b, j]]
        assert cnt[b] == len(want) == pre[b, 300]
        assert list(idx[b, :cnt[b]]) == want
        assert np.all(np.diff(idx[b, :cnt[b]]) > 0)
        assert np.all(idx[b, cnt[b]:] == -1)
        assert list(pre[b]) == [int(is_sep[b, :j].astype(np.int64).sum()) for j in range(301)]
    # capacity smaller than the count: list is truncated, count stays true
    idx2, cnt2, _ = oracle.compact_indices(is_sep, cap=5)
    assert np.array_equal(cnt2, cnt)
    assert list(idx2[2]) == [0, 1, 2, 3, 4]


# ----------------------------------------------------------------------------------------------
# mask
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("L,a,n,p", [(1, 0, 1, 0.5), (17, 0, 1, 0.3), (40, 3, 5, 0.2), (64, 4, 16, 0.1),
                                     (33, 40, 2, 0.0), (29, 2, 64, 0.5), (50, 0, 7, 1.0)])
def test_mask_equals_set_membership(L, a, n, p):
    is_sep = _flags(1, L, p, L + a + n)[0]
    M = oracle.mask(is_sep, a, n)
    want = np.zeros((L, L), dtype=bool)
    for i in range(L):
        for j in visible_set(i, is_sep, a, n):
            want[i, j] = True
    assert np.array_equal(M, want)
    assert M.diagonal().all()  # n >= 1: every token sees itself
    assert not np.triu(M, 1).any()  # causal


def _golden_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_mask_reproduces_printed_attention_map_ratio_without_separators():
    """Table 'tab_flops', StrmLLM n=64 at L=2048: 6.43 % of the lower triangle is ones (a=3)."""
    printed = {(r[0], int(r[1])): float(r[2]) for r in _golden_rows("tab_flops_attention_ratio.txt")}
    L = 2048
    M = oracle.mask(np.zeros(L, dtype=np.uint8), 3, 64)
    ones = int(M.sum())
    assert ones == 135005
    ratio = 100.0 * ones / (L * (L + 1) // 2)
    assert round(ratio, 2) == printed[("StrmLLM", 64)]


def test_mask_ratio_with_separators_is_consistent_with_the_table():
    """Both SepLLM entries of 'tab_flops' (n=64: 17.21 %, n=128: 22.48 %) follow from ONE separator
    density; the n=64 entry fixes it (0.115) and the n=128 entry is then predicted."""
    printed = {(r[0], int(r[1])): float(r[2]) for r in _golden_rows("tab_flops_attention_ratio.txt")}
    L, a = 2048, 3
    tri = L * (L + 1) // 2

    def mean_ratio(n, p):
        vals = []
        for seed in range(6):
            is_sep = _flags(1, L, p, 100 + seed)[0]
            vals.append(100.0 * oracle.mask(is_sep, a, n).sum() / tri)
        return float(np.mean(vals))

    assert abs(mean_ratio(64, 0.1152) - printed[("SepLLM", 64)]) < 0.35
    assert abs(mean_ratio(128, 0.1152) - printed[("SepLLM", 128)]) < 0.35


def test_zero_query_probe_counts_visible_keys():
    """Q = 0 makes every row uniform: exp(LSE_i) is the number of visible keys and O_i their mean."""
    B, H, L, d, a, n = 1, 2, 96, 8, 3, 10
    is_sep = _flags(B, L, 0.15, 5)
    K, V = _rand((B, H, L, d), 6), _rand((B, H, L, d), 7)
    O, LSE = oracle.forward(np.zeros((B, H, L, d)), K, V, is_sep, a, n, 0.3)
    for i in range(L):
        vis = sorted(visible_set(i, is_sep[0], a, n))
        assert abs(math.exp(LSE[0, 0, i]) - len(vis)) < 1e-9
        assert np.allclose(O[0, 1, i], V[0, 1, vis].mean(axis=0), atol=1e-12)


# ----------------------------------------------------------------------------------------------
# forward
# ----------------------------------------------------------------------------------------------
def test_rows_of_A_sum_to_one_and_respect_mask():
    B, H, L, d, a, n = 2, 2, 70, 16, 2, 9
    is_sep = _flags(B, L, 0.2, 11)
    Q, K, V = _rand((B, H, L, d), 1), _rand((B, H, L, d), 2), _rand((B, H, L, d), 3)
    O, LSE, A = oracle.forward(Q, K, V, is_sep, a, n, 0.25, return_A=True)
    assert np.allclose(A.sum(-1), 1.0, atol=1e-12)
    for b in range(B):
        M = oracle.mask(is_sep[b], a, n)
        assert np.all(A[b][:, ~M] == 0.0)
        assert np.all(A[b][:, M] > 0.0)
    assert np.allclose(np.einsum("bhij,bhjk->bhik", A, V), O, atol=1e-12)


def test_constant_V_gives_constant_O():
    B, H, L, d = 1, 1, 50, 8
    is_sep = _flags(B, L, 0.2, 3)
    v = _rand((d,), 9)
    V = np.broadcast_to(v, (B, H, L, d)).copy()
    O, _ = oracle.forward(_rand((B, H, L, d), 1), _rand((B, H, L, d), 2), V, is_sep, 2, 5, 0.5)
    assert np.allclose(O, v, atol=1e-12)


@pytest.mark.parametrize("case", ["all_separators", "n_ge_L", "a_ge_L"])
def test_degenerate_cases_are_full_causal_attention(case):
    """Everything visible => plain causal attention (the hybrid full-attention layers of Sec. 4.3)."""
    import torch

    B, H, L, d = 1, 2, 61, 16
    Q, K, V = _rand((B, H, L, d), 1), _rand((B, H, L, d), 2), _rand((B, H, L, d), 3)
    is_sep = np.zeros((B, L), dtype=np.uint8)
    a, n = 0, 1
    if case == "all_separators":
        is_sep[:] = 1
    elif case == "n_ge_L":
        n = L
    else:
        a = L + 5
    scale = 1.0 / math.sqrt(d)
    O, LSE = oracle.forward(Q, K, V, is_sep, a, n, scale)
    causal = np.tril(np.ones((L, L), dtype=bool))
    for h in range(H):
        Oref, lref = softmax_attention_dense(Q[0, h], K[0, h], V[0, h], causal, scale)
        assert np.allclose(O[0, h], Oref, atol=1e-12)
        assert np.allclose(LSE[0, h], lref, atol=1e-12)
    # library routine (fp32 on CPU)
    t = lambda x: torch.from_numpy(x).float()
    Ot = torch.nn.functional.scaled_dot_product_attention(t(Q), t(K), t(V), is_causal=True)
    assert np.allclose(O, Ot.numpy(), atol=2e-5)


def test_no_separators_is_sink_plus_sliding_window():
    """Without separators the mask is the StreamingLLM pattern: a sinks + the n closest tokens."""
    B, H, L, d, a, n = 1, 1, 80, 8, 4, 12
    Q, K, V = _rand((B, H, L, d), 1), _rand((B, H, L, d), 2), _rand((B, H, L, d), 3)
    i = np.arange(L)[:, None]
    j = np.arange(L)[None, :]
    allowed = (j <= i) & ((j < a) | (j > i - n))
    O, LSE = oracle.forward(Q, K, V, np.zeros((B, L), np.uint8), a, n, 0.4)
    Oref, lref = softmax_attention_dense(Q[0, 0], K[0, 0], V[0, 0], allowed, 0.4)
    assert np.allclose(O[0, 0], Oref, atol=1e-12) and np.allclose(LSE[0, 0], lref, atol=1e-12)


def test_self_only_closed_form():
    """a=0, no separators, n=1: each token sees only itself => O = V, LSE_i = scale <Q_i,K_i>."""
    B, H, L, d = 2, 3, 20, 8
    Q, K, V = _rand((B, H, L, d), 1), _rand((B, H, L, d), 2), _rand((B, H, L, d), 3)
    O, LSE = oracle.forward(Q, K, V, np.zeros((B, L), np.uint8), 0, 1, 0.7)
    assert np.allclose(O, V, atol=1e-13)
    assert np.allclose(LSE, 0.7 * (Q * K).sum(-1), atol=1e-12)


@pytest.mark.parametrize("L,a,n,p", [(12, 2, 3, 0.3), (20, 0, 4, 0.2), (9, 1, 1, 0.5)])
def test_forward_equals_per_pair_python_loop(L, a, n, p):
    d = 4
    is_sep = _flags(1, L, p, 21)
    Q, K, V = _rand((1, 1, L, d), 1), _rand((1, 1, L, d), 2), _rand((1, 1, L, d), 3)
    O, LSE = oracle.forward(Q, K, V, is_sep, a, n, 0.6)
    Oref, lref = per_pair_forward(Q[0, 0], K[0, 0], V[0, 0], is_sep[0], a, n, 0.6)
    assert np.allclose(O[0, 0], Oref, atol=1e-12) and np.allclose(LSE[0, 0], lref, atol=1e-12)


def test_row_subset_matches_full_and_f32_build_is_close():
    B, H, L, d, a, n = 1, 2, 64, 8, 2, 6
    is_sep = _flags(B, L, 0.2, 4)
    Q, K, V = _rand((B, H, L, d), 1), _rand((B, H, L, d), 2), _rand((B, H, L, d), 3)
    O, LSE = oracle.forward(Q, K, V, is_sep, a, n, 0.5)
    rows = np.array([0, 5, 63, 17], dtype=np.int32)
    Or, Lr = oracle.forward(Q, K, V, is_sep, a, n, 0.5, rows=rows)
    assert np.array_equal(Or, O[:, :, rows]) and np.array_equal(Lr, LSE[:, :, rows])
    O32, L32 = oracle.forward(Q, K, V, is_sep, a, n, 0.5, precision="f32")
    assert O32.dtype == np.float32
    assert np.allclose(O32, O, atol=1e-5) and np.allclose(L32, LSE, atol=1e-5)


def test_gqa_equals_mha_with_repeated_kv_heads():
    B, Hq, Hkv, L, d, a, n = 1, 6, 2, 40, 8, 2, 5
    is_sep = _flags(B, L, 0.2, 8)
    Q, K, V = _rand((B, Hq, L, d), 1), _rand((B, Hkv, L, d), 2), _rand((B, Hkv, L, d), 3)
    dO = _rand((B, Hq, L, d), 4)
    G = Hq // Hkv
    Kr, Vr = np.repeat(K, G, axis=1), np.repeat(V, G, axis=1)  # head h reads KV head h // G
    O1, L1 = oracle.forward(Q, K, V, is_sep, a, n, 0.5)
    O2, L2 = oracle.forward(Q, Kr, Vr, is_sep, a, n, 0.5)
    assert np.allclose(O1, O2, atol=1e-13) and np.allclose(L1, L2, atol=1e-13)
    dQ1, dK1, dV1 = oracle.backward(Q, K, V, dO, is_sep, a, n, 0.5)
    dQ2, dK2, dV2 = oracle.backward(Q, Kr, Vr, dO, is_sep, a, n, 0.5)
    assert np.allclose(dQ1, dQ2, atol=1e-12)
    assert np.allclose(dK1, dK2.reshape(B, Hkv, G, L, d).sum(2), atol=1e-12)
    assert np.allclose(dV1, dV2.reshape(B, Hkv, G, L, d).sum(2), atol=1e-12)


# ----------------------------------------------------------------------------------------------
# backward
# ----------------------------------------------------------------------------------------------
def test_backward_matches_central_finite_differences():
    B, Hq, Hkv, L, d, a, n = 1, 2, 1, 24, 4, 2, 4
    is_sep = _flags(B, L, 0.25, 2)
    Q, K, V = _rand((B, Hq, L, d), 1), _rand((B, Hkv, L, d), 2), _rand((B, Hkv, L, d), 3)
    dO = _rand((B, Hq, L, d), 4)
    scale = 0.5
    dQ, dK, dV = oracle.backward(Q, K, V, dO, is_sep, a, n, scale)

    def loss(q, k, v):
        O, _ = oracle.forward(q, k, v, is_sep, a, n, scale)
        return float((O * dO).sum())

    rng = np.random.default_rng(0)
    eps = 1e-5
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(25):
            idx = tuple(rng.integers(0, s) for s in X.shape)
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += eps
            Xm[idx] -= eps
            args_p = {"Q": (Xp, K, V), "K": (Q, Xp, V), "V": (Q, K, Xp)}[name]
            args_m = {"Q": (Xm, K, V), "K": (Q, Xm, V), "V": (Q, K, Xm)}[name]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert abs(fd - G[idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, G[idx])


def test_backward_full_causal_matches_torch_autograd():
    import torch

    B, Hq, Hkv, L, d = 2, 4, 2, 33, 8
    Q, K, V = _rand((B, Hq, L, d), 1), _rand((B, Hkv, L, d), 2), _rand((B, Hkv, L, d), 3)
    dO = _rand((B, Hq, L, d), 4)
    scale = 1.0 / math.sqrt(d)
    is_sep = np.ones((B, L), dtype=np.uint8)
    dQ, dK, dV = oracle.backward(Q, K, V, dO, is_sep, 0, 1, scale)
    q = torch.tensor(Q, requires_grad=True)
    k = torch.tensor(K, requires_grad=True)
    v = torch.tensor(V, requires_grad=True)
    G = Hq // Hkv
    o = torch.nn.functional.scaled_dot_product_attention(
        q, k.repeat_interleave(G, dim=1), v.repeat_interleave(G, dim=1), is_causal=True)
    o.backward(torch.tensor(dO))
    assert np.allclose(dQ, q.grad.numpy(), atol=1e-10)
    assert np.allclose(dK, k.grad.numpy(), atol=1e-10)
    assert np.allclose(dV, v.grad.numpy(), atol=1e-10)


def test_backward_sparse_mask_matches_torch_autograd_with_explicit_mask():
    """The SepLLM mask itself (built by the independent set-membership helper) through autograd."""
    import torch

    B, H, L, d, a, n = 1, 2, 30, 4, 2, 3
    is_sep = _flags(B, L, 0.2, 12)
    Q, K, V, dO = (_rand((B, H, L, d), s) for s in (1, 2, 3, 4))
    allowed = np.zeros((L, L), dtype=bool)
    for i in range(L):
        allowed[i, list(visible_set(i, is_sep[0], a, n))] = True
    dQ, dK, dV = oracle.backward(Q, K, V, dO, is_sep, a, n, 0.5)
    q, k, v = (torch.tensor(x, requires_grad=True) for x in (Q, K, V))
    s = (q @ k.transpose(-1, -2)) * 0.5
    s = s.masked_fill(~torch.tensor(allowed), float("-inf"))
    o = torch.softmax(s, dim=-1) @ v
    o.backward(torch.tensor(dO))
    assert np.allclose(dQ, q.grad.numpy(), atol=1e-10)
    assert np.allclose(dK, k.grad.numpy(), atol=1e-10)
    assert np.allclose(dV, v.grad.numpy(), atol=1e-10)


def test_backward_closed_forms():
    B, H, L, d = 1, 2, 16, 4
    Q, K, V, dO = (_rand((B, H, L, d), s) for s in (1, 2, 3, 4))
    none = np.zeros((B, L), np.uint8)
    # each token sees only itself: O = V, so dV = dO and nothing flows to Q, K
    dQ, dK, dV = oracle.backward(Q, K, V, dO, none, 0, 1, 0.5)
    assert np.allclose(dV, dO, atol=1e-13) and np.all(dQ == 0) and np.all(dK == 0)
    # constant V: O does not depend on the scores => dQ = dK = 0
    is_sep = _flags(B, L, 0.3, 5)
    Vc = np.broadcast_to(_rand((d,), 7), V.shape).copy()
    dQ, dK, _ = oracle.backward(Q, K, Vc, dO, is_sep, 1, 3, 0.5)
    assert np.allclose(dQ, 0, atol=1e-12) and np.allclose(dK, 0, atol=1e-12)
    # constant K: dQ_i = scale * k * sum_j dLambda_ij and the softmax Jacobian rows sum to 0
    Kc = np.broadcast_to(_rand((d,), 8), K.shape).copy()
    dQ, _, _ = oracle.backward(Q, Kc, V, dO, is_sep, 1, 3, 0.5)
    assert np.allclose(dQ, 0, atol=1e-12)


# ----------------------------------------------------------------------------------------------
# head-wise windows (Sec. 4.6, the head-wise variant) and the term magnitudes of the gradients
# ----------------------------------------------------------------------------------------------
def test_per_head_windows_reduce_to_the_scalar_window_and_to_single_head_runs():
    """n_head with all heads equal is the scalar n; with different windows, query head h must equal a
    single-head run with n = n_head[h], and dK / dV of a KV head the sum of its heads' single runs."""
    B, Hq, Hkv, L, d, a = 2, 4, 2, 40, 4, 2
    is_sep = _flags(B, L, 0.2, 3)
    Q, K, V = _rand((B, Hq, L, d), 1), _rand((B, Hkv, L, d), 2), _rand((B, Hkv, L, d), 3)
    dO = _rand((B, Hq, L, d), 4)
    O0, L0 = oracle.forward(Q, K, V, is_sep, a, 5, 0.5)
    O1, L1 = oracle.forward(Q, K, V, is_sep, a, 99, 0.5, n_head=[5, 5, 5, 5])
    assert np.array_equal(O0, O1) and np.array_equal(L0, L1)
    g0 = oracle.backward(Q, K, V, dO, is_sep, a, 5, 0.5)
    g1 = oracle.backward(Q, K, V, dO, is_sep, a, 99, 0.5, n_head=[5, 5, 5, 5])
    assert all(np.array_equal(x, y) for x, y in zip(g0, g1))
    nh = [1, L + 7, 3, 12]                      # a full-attention head inside each group
    O, LSE = oracle.forward(Q, K, V, is_sep, a, 77, 0.5, n_head=nh)
    dQ, dK, dV = oracle.backward(Q, K, V, dO, is_sep, a, 77, 0.5, n_head=nh)
    sumK, sumV = np.zeros_like(K), np.zeros_like(V)
    G = Hq // Hkv
    for h in range(Hq):
        kv = h // G
        args = (Q[:, h:h + 1], K[:, kv:kv + 1], V[:, kv:kv + 1])
        o, l = oracle.forward(*args, is_sep, a, nh[h], 0.5)
        assert np.array_equal(O[:, h:h + 1], o) and np.array_equal(LSE[:, h:h + 1], l)
        gq, gk, gv = oracle.backward(*args, dO[:, h:h + 1], is_sep, a, nh[h], 0.5)
        assert np.array_equal(dQ[:, h:h + 1], gq)
        sumK[:, kv:kv + 1] += gk
        sumV[:, kv:kv + 1] += gv
    assert np.allclose(dK, sumK, atol=1e-13) and np.allclose(dV, sumV, atol=1e-13)
    # and the mask itself, brute force: the head with n_head = 1 and no initial tokens sees itself and separators
    _, _, A = oracle.forward(Q, K, V, is_sep, 0, 50, 0.5, n_head=[1, 50, 50, 50], return_A=True)
    for b in range(B):
        for i in range(L):
            want = {j for j in range(i + 1) if j == i or is_sep[b, j]}
            assert set(np.nonzero(A[b, 0, i])[0]) == want


def test_term_magnitudes_of_the_gradients():
    """eQ, eK, eV are root-sum-squares of the terms the gradients add up: pinned by the closed form
    of the self-only case, by building them from the attention matrix the forward returns, and by
    the inequalities |sum| <= sum|term| ... every sum of N terms obeys |sum| <= sqrt(N) * rss."""
    B, Hq, Hkv, L, d, a, n = 1, 4, 2, 28, 4, 2, 4
    Q, K, V = _rand((B, Hq, L, d), 1), _rand((B, Hkv, L, d), 2), _rand((B, Hkv, L, d), 3)
    dO = _rand((B, Hq, L, d), 4)
    none = np.zeros((B, L), np.uint8)
    # every token sees only itself: A = I, so dV_j = sum over the heads of dO_j, one term per head
    dQ, dK, dV, eQ, eK, eV = oracle.backward(Q, K, V, dO, none, 0, 1, 0.5, return_term_rss=True)
    G = Hq // Hkv
    want = np.sqrt((dO.reshape(B, Hkv, G, L, d) ** 2).sum(axis=2))
    assert np.allclose(eV, want, atol=1e-13) and np.all(eK == 0) and np.all(eQ == 0)
    # general case, from the attention matrix
    is_sep = _flags(B, L, 0.25, 9)
    scale = 0.7
    dQ, dK, dV, eQ, eK, eV = oracle.backward(Q, K, V, dO, is_sep, a, n, scale, return_term_rss=True)
    O, _, A = oracle.forward(Q, K, V, is_sep, a, n, scale, return_A=True)
    eV2, eK2 = np.zeros_like(V), np.zeros_like(K)
    for h in range(Hq):
        kv = h // G
        Ah = A[0, h]
        Drow = (dO[0, h] * O[0, h]).sum(axis=1)
        dS = Ah * (dO[0, h] @ V[0, kv].T - Drow[:, None])
        eV2[0, kv] += (Ah ** 2).T @ (dO[0, h] ** 2)
        eK2[0, kv] += scale ** 2 * (dS ** 2).T @ (Q[0, h] ** 2)
        assert np.allclose(eQ[0, h], scale * np.sqrt((dS ** 2) @ (K[0, kv] ** 2)), atol=1e-12)
    assert np.allclose(eV, np.sqrt(eV2), atol=1e-12) and np.allclose(eK, np.sqrt(eK2), atol=1e-12)
    # a sum of at most N terms is at most sqrt(N) times their root-sum-square
    assert (np.abs(dV) <= math.sqrt(G * L) * eV + 1e-12).all()
    assert (np.abs(dK) <= math.sqrt(G * L) * eK + 1e-12).all()
    assert (np.abs(dQ) <= math.sqrt(L) * eQ + 1e-12).all()
    # the gradients themselves do not change when the magnitudes are asked for
    g = oracle.backward(Q, K, V, dO, is_sep, a, n, scale)
    assert all(np.array_equal(x, y) for x, y in zip(g, (dQ, dK, dV)))


# ----------------------------------------------------------------------------------------------
# decode
# ----------------------------------------------------------------------------------------------
def test_decode_equals_prefill_row_under_fundamental_design_cache():
    """Sec. 3.2 "Generation": keeping initial + separator + n neighbouring KV reproduces row i."""
    B, Hq, Hkv, L, d, a, n = 1, 4, 2, 90, 8, 3, 7
    is_sep = _flags(B, L, 0.2, 31)
    Q, K, V = _rand((B, Hq, L, d), 1), _rand((B, Hkv, L, d), 2), _rand((B, Hkv, L, d), 3)
    O, LSE = oracle.forward(Q, K, V, is_sep, a, n, 0.35)
    s_cap, c = 40, 3 + 40 + 16
    for i in (0, 2, 9, 50, 89):
        init = [j for j in range(min(a, i + 1))]
        win = [j for j in range(max(a, i - n + 1), i + 1)]
        seps = [j for j in range(a, i - n + 1) if is_sep[0, j]]
        Kc = np.zeros((1, Hkv, c, d))
        Vc = np.zeros((1, Hkv, c, d))
        for slot0, lst in ((0, init), (a, seps), (a + s_cap, win)):
            Kc[0, :, slot0:slot0 + len(lst)] = K[0][:, lst]
            Vc[0, :, slot0:slot0 + len(lst)] = V[0][:, lst]
        past = max(0, len(win) - 4)
        sizes = np.array([[len(init), len(seps), past, len(win) - past]], dtype=np.int32)
        out, lse = oracle.decode(Q[:, :, i], Kc, Vc, sizes, a, s_cap, 0.35)
        assert np.allclose(out[0], O[0, :, i], atol=1e-12)
        assert np.allclose(lse[0], LSE[0, :, i], atol=1e-12)


def test_fill_from_prefill_reproduces_the_last_prefill_row():
    """Sec. 3.2 "Generation": the cache handed over after L tokens, with nw = n and room for every
    separator, holds exactly what row L-1 of the prefill sees, so decoding Q_{L-1} over it gives
    that row.  Pins the hand-over against the forward and the decode together."""
    B, Hq, Hkv, L, d, a, n = 2, 4, 2, 83, 8, 3, 11
    is_sep = _flags(B, L, 0.2, 5)
    Q, K, V = _rand((B, Hq, L, d), 1), _rand((B, Hkv, L, d), 2), _rand((B, Hkv, L, d), 3)
    O, LSE = oracle.forward(Q, K, V, is_sep, a, n, 0.35)
    s_cap, w = 60, 4
    c = a + s_cap + 16
    Kc, Vc, flags, sizes, valid = oracle.fill_from_prefill(K, V, is_sep, a, s_cap, w, c, n)
    out, lse = oracle.decode(Q[:, :, L - 1], Kc, Vc, sizes, a, s_cap, 0.35)
    assert np.allclose(out, O[:, :, L - 1], atol=1e-12)
    assert np.allclose(lse, LSE[:, :, L - 1], atol=1e-12)
    assert np.array_equal(flags[:, :n], is_sep[:, L - n:])
    assert (sizes[:, 2] + sizes[:, 3] == n).all() and (sizes[:, 3] == w).all()
    assert (valid.sum(1) == sizes.sum(1)).all()


def test_fill_from_prefill_agrees_with_the_streaming_policy():
    """The hand-over must land in the state the token-by-token policy of Sec. 3.3 reaches: with nw =
    the policy's n after L tokens, the separator count equals the simulator's Size_sep, the rows of
    the Separator Cache are the newest separators older than the window (oldest first), and a
    too-small Separator Cache keeps the newest s of them."""
    a, s, w, c = 2, 6, 5, 24
    L = 150
    is_sep = _flags(1, L, 0.25, 9)
    sim = cache_sim.simulate(is_sep[0], a, s, w, c)
    K = np.arange(L, dtype=np.float64).reshape(1, 1, L, 1) + 0.5  # a row is its position + 0.5
    for m in (1, 2, 7, 23, 24, 60, 149):
        Lm = m + 1
        nw = int(sim["n"][m])
        Kc, Vc, flags, sizes, valid = oracle.fill_from_prefill(K[:, :, :Lm], K[:, :, :Lm], is_sep[:, :Lm], a, s, w, c, nw)
        assert sizes[0, 0] == min(a, Lm)
        assert sizes[0, 2] + sizes[0, 3] == nw
        assert sizes[0, 1] == sim["size_sep"][m], (m, sizes[0], sim["size_sep"][m])
        assert sizes.sum() == sim["size_run"][m]
        kept = (Kc[0, 0, a:a + sizes[0, 1], 0] - 0.5).astype(int)
        want = [j for j in range(min(a, Lm), Lm - nw) if is_sep[0, j]][-s:] if s else []
        assert list(kept) == want[len(want) - sizes[0, 1]:]
        win = (Kc[0, 0, a + s:a + s + nw, 0] - 0.5).astype(int)
        assert list(win) == list(range(Lm - nw, Lm))


def test_decode_zero_query_probe_counts_entries():
    S, Hq, Hkv, d, a, s, c = 3, 2, 1, 4, 2, 5, 16
    Kc, Vc = _rand((S, Hkv, c, d), 1), _rand((S, Hkv, c, d), 2)
    sizes = np.array([[2, 5, 4, 5], [1, 0, 0, 1], [2, 3, 0, 9]], dtype=np.int32)
    out, lse = oracle.decode(np.zeros((S, Hq, d)), Kc, Vc, sizes, a, s, 1.0)
    assert np.allclose(np.exp(lse), sizes.sum(1, keepdims=True), atol=1e-9)
    slots = [0, 1, 2, 3, 4, 7, 8, 9, 10, 11, 12, 13, 14, 15][:]  # seq 2: init 0,1; sep 2,3,4; win 7..15
    assert np.allclose(out[2, 0], Vc[2, 0, slots].mean(0), atol=1e-12)


def test_mark_interval_worked_example_and_mask():
    """Fixed-interval variant: with delta = 4, phase = 1 the markers of 10 positions are 1, 5, 9; a row
    of the mask then sees the initial tokens, the marked positions and its neighbours, nothing else."""
    m = oracle.mark_interval(2, 10, 4, 1)
    assert m.dtype == np.uint8 and m.tolist() == [[0, 1, 0, 0, 0, 1, 0, 0, 0, 1]] * 2
    for L, delta, phase in ((37, 5, 0), (64, 8, 7), (5, 9, 3), (16, 1, 0)):
        f = oracle.mark_interval(1, L, delta, phase)[0]
        assert f.sum() == len(range(phase, L, delta)) and all(f[j] for j in range(phase, L, delta))
    L, a, n, delta = 40, 2, 4, 8
    M = oracle.mask(oracle.mark_interval(1, L, delta, 3)[0], a, n)
    for i in range(L):
        want = {j for j in range(i + 1) if j < a or j % delta == 3 or i - j < n}
        assert set(np.nonzero(M[i])[0]) == want


# ----------------------------------------------------------------------------------------------
# packed documents
# ----------------------------------------------------------------------------------------------
def _packed_mask(is_sep_row, start, a, n):
    L = len(is_sep_row)
    M = np.zeros((L, L), dtype=bool)
    for i in range(L):
        for j in range(i + 1):
            M[i, j] = start[j] == start[i] and (j - start[j] < a or bool(is_sep_row[j]) or i - j < n)
    return M


def test_packed_documents_against_an_explicit_mask():
    """Every document is a sequence of its own: forward and backward over the packed row must equal
    plain masked softmax attention (and its autograd gradient) under the explicit L x L mask
    "same document, and initial token of that document or separator or neighbour"."""
    torch = pytest.importorskip("torch")
    B, Hq, Hkv, L, d, a, n, scale = 2, 4, 2, 61, 8, 2, 5, 0.3
    cus = [np.array([0, 7, 8, 30, 61]), np.array([0, 61])]
    is_sep = _flags(B, L, 0.2, 21)
    Q, K, V, dO = _rand((B, Hq, L, d), 1), _rand((B, Hkv, L, d), 2), _rand((B, Hkv, L, d), 3), _rand((B, Hq, L, d), 4)
    O, LSE = oracle.forward_packed(Q, K, V, is_sep, cus, a, n, scale)
    dQ, dK, dV = oracle.backward_packed(Q, K, V, dO, is_sep, cus, a, n, scale)
    G = Hq // Hkv
    for b in range(B):
        start, end = oracle.doc_bounds(cus[b], L)
        assert (start <= np.arange(L)).all() and (np.arange(L) < end).all() and set(start) | {L} == set(cus[b])
        M = torch.from_numpy(_packed_mask(is_sep[b], start, a, n))
        q = torch.tensor(Q[b], dtype=torch.float64, requires_grad=True)
        k = torch.tensor(K[b], dtype=torch.float64, requires_grad=True)
        v = torch.tensor(V[b], dtype=torch.float64, requires_grad=True)
        sc = scale * torch.einsum("hid,hjd->hij", q, k.repeat_interleave(G, dim=0))
        sc = sc.masked_fill(~M, float("-inf"))
        out = torch.einsum("hij,hjd->hid", torch.softmax(sc, dim=-1), v.repeat_interleave(G, dim=0))
        out.backward(torch.from_numpy(dO[b]))
        assert np.allclose(O[b], out.detach().numpy(), atol=1e-12)
        assert np.allclose(LSE[b], torch.logsumexp(sc, dim=-1).detach().numpy(), atol=1e-12)
        assert np.allclose(dQ[b], q.grad.numpy(), atol=1e-11)
        assert np.allclose(dK[b], k.grad.numpy(), atol=1e-11)
        assert np.allclose(dV[b], v.grad.numpy(), atol=1e-11)
    # one document = the unpacked call
    O1, L1 = oracle.forward(Q[1:], K[1:], V[1:], is_sep[1:], a, n, scale)
    assert np.array_equal(O[1:], O1) and np.array_equal(LSE[1:], L1)
    # the markers with every document's initial tokens added
    start0, _ = oracle.doc_bounds(cus[0], L)
    m = oracle.mark_doc_initial(is_sep[:1], start0[None], a)[0]
    assert all(m[j] == (1 if (is_sep[0, j] or j in (0, 1, 7, 8, 9, 30, 31)) else 0) for j in range(L))


# ----------------------------------------------------------------------------------------------
# positions within the cache (Sec. 3.3 "Positional Encoding") and the append step
# ----------------------------------------------------------------------------------------------
def test_rope_rotation_worked_examples():
    """Pairing (i, i + d/2), direction and frequencies: unit vectors turn by pos * base**(-2i/d)."""
    for pos in (0, 1, 7, 1000):
        assert np.allclose(oracle.rope_rotate(np.array([1.0, 0.0]), pos, 123.0), [math.cos(pos), math.sin(pos)], atol=1e-12)
        assert np.allclose(oracle.rope_rotate(np.array([0.0, 1.0]), pos, 123.0), [-math.sin(pos), math.cos(pos)], atol=1e-12)
        # d = 4, base = 100: the second pair (dimensions 1 and 3) turns by 0.1 per position
        got = oracle.rope_rotate(np.array([0.0, 2.0, 0.0, 0.0]), pos, 100.0)
        assert np.allclose(got, [0.0, 2 * math.cos(0.1 * pos), 0.0, 2 * math.sin(0.1 * pos)], atol=1e-12)
    # d = 8, base = 10000: angles 1, 0.1, 0.01, 0.001 per position
    x = np.zeros(8)
    x[3] = 1.0
    assert np.allclose(oracle.rope_rotate(x, 500, 10000.0)[[3, 7]], [math.cos(0.5), math.sin(0.5)], atol=1e-12)
    # a rotation: lengths are kept, positions broadcast over rows
    X = _rand((5, 16), 3)
    assert np.allclose(np.linalg.norm(oracle.rope_rotate(X, np.arange(5), 10000.0), axis=1), np.linalg.norm(X, axis=1), atol=1e-12)


def test_decode_rope_matches_the_relative_position_form():
    """With rotary encoding a score depends on the distance only: in complex form, pairing dimension
    i with i + d/2, score = Re sum_i q_i conj(k_i) exp(1j (m - p) theta_i).  The query sits at the
    newest entry's position m = nv - 1 and entry e (oldest first) at p = e."""
    S, Hq, Hkv, d, a, s, c = 3, 4, 2, 8, 2, 5, 20
    base, scale = 50.0, 0.3
    Kc, Vc, q = _rand((S, Hkv, c, d), 1), _rand((S, Hkv, c, d), 2), _rand((S, Hq, d), 3)
    sizes = np.array([[2, 5, 4, 5], [1, 0, 0, 1], [2, 3, 0, 9]], dtype=np.int32)
    out, lse = oracle.decode_rope(q, Kc, Vc, sizes, a, s, scale, base)
    h = d // 2
    theta = np.array([base ** (-i / h) for i in range(h)])
    for sq in range(S):
        slots = list(range(sizes[sq, 0])) + [a + k for k in range(sizes[sq, 1])] + [a + s + u for u in range(sizes[sq, 2] + sizes[sq, 3])]
        nv = len(slots)
        for hq in range(Hq):
            kv = hq // (Hq // Hkv)
            zq = q[sq, hq, :h] + 1j * q[sq, hq, h:]
            sc = np.empty(nv)
            for e, sl in enumerate(slots):
                zk = Kc[sq, kv, sl, :h] + 1j * Kc[sq, kv, sl, h:]
                sc[e] = scale * np.real(np.sum(zq * np.conj(zk) * np.exp(1j * (nv - 1 - e) * theta)))
            pr = np.exp(sc - sc.max())
            assert np.allclose(out[sq, hq], (pr / pr.sum()) @ Vc[sq, kv, slots], atol=1e-12)
            assert np.isclose(lse[sq, hq], sc.max() + np.log(pr.sum()), atol=1e-12)


def test_decode_rope_special_cases():
    S, Hq, Hkv, d, a, s, c = 2, 2, 1, 8, 2, 4, 16
    Kc, Vc, q = _rand((S, Hkv, c, d), 4), _rand((S, Hkv, c, d), 5), _rand((S, Hq, d), 6)
    sizes = np.array([[2, 3, 2, 4], [2, 4, 0, 6]], dtype=np.int32)
    # (i) frequencies that vanish (huge base) leave only pair 0 turning; without that pair in the query
    #     the encoding drops out and the plain decode must come back
    q0 = q.copy()
    q0[..., 0] = 0.0
    q0[..., d // 2] = 0.0
    out, lse = oracle.decode_rope(q0, Kc, Vc, sizes, a, s, 0.4, 1e300)
    out_plain, lse_plain = oracle.decode(q0, Kc, Vc, sizes, a, s, 0.4)
    assert np.allclose(out, out_plain, atol=1e-12) and np.allclose(lse, lse_plain, atol=1e-12)
    # (ii) one entry: position 0 for key and query, no rotation at all
    one = np.array([[1, 0, 0, 0], [1, 0, 0, 0]], dtype=np.int32)
    out, lse = oracle.decode_rope(q, Kc, Vc, one, a, s, 0.4, 10000.0)
    assert np.allclose(out, np.repeat(Vc[:, :, 0], Hq, axis=1), atol=1e-12)
    assert np.allclose(lse, 0.4 * np.einsum("shd,sd->sh", q, Kc[:, 0, 0]), atol=1e-12)
    # (iii) positions are those within the cache, not slots: the same entries in the same order, split
    #      differently among the blocks, give the same result
    sizes_a = np.array([[2, 3, 0, 4]], dtype=np.int32)
    sizes_b = np.array([[2, 0, 0, 7]], dtype=np.int32)
    Kb, Vb = np.zeros_like(Kc[:1]), np.zeros_like(Vc[:1])
    src = [0, 1, a, a + 1, a + 2, a + s, a + s + 1, a + s + 2, a + s + 3]
    dst = [0, 1] + [a + s + u for u in range(7)]
    Kb[0, :, dst], Vb[0, :, dst] = Kc[0, :, src], Vc[0, :, src]
    oa, la = oracle.decode_rope(q[:1], Kc[:1], Vc[:1], sizes_a, a, s, 0.4, 10000.0)
    ob, lb = oracle.decode_rope(q[:1], Kb, Vb, sizes_b, a, s, 0.4, 10000.0)
    assert np.allclose(oa, ob, atol=1e-12) and np.allclose(la, lb, atol=1e-12)
    # (iv) an empty cache
    out, lse = oracle.decode_rope(q, Kc, Vc, np.zeros((S, 4), dtype=np.int32), a, s, 0.4, 10000.0)
    assert (out == 0).all() and np.isneginf(lse).all()


def _stream(is_sep, K, a, s, w, c, upto):
    """Tokens 0 .. upto-1 enter one by one; the compression step runs whenever the window region is full."""
    S, Hkv, L, d = K.shape
    Kc, Vc = np.zeros((S, Hkv, c, d)), np.zeros((S, Hkv, c, d))
    fl, sz = np.zeros((S, c - a - s), dtype=np.uint8), np.zeros((S, 4), dtype=np.int32)
    hist = []
    for m in range(upto):
        Kc, Vc, fl, sz = oracle.append_token(Kc, Vc, fl, sz, K[:, :, m], -K[:, :, m], is_sep[:, m], a, s, w)
        if sz[0, 2] + sz[0, 3] == c - a - s:
            Kc, Vc, fl, sz = oracle.evict_window(Kc, Vc, fl, sz, a, s)
        hist.append(sz[0].copy())
    return Kc, Vc, fl, sz, hist


def test_append_and_compress_reach_the_handover_state():
    """Sec. 3.2 / 3.3: streaming the tokens in one by one must leave the cache the hand-over from a
    prefill of the same tokens builds (same rows in the same slots, same flags and sizes)."""
    a, s, w, c, L = 2, 5, 4, 19, 90
    is_sep = _flags(1, L, 0.3, 11)
    K = _rand((1, 2, L, 3), 12)
    for upto in (1, 2, 3, 9, 14, 15, 40, 90):
        Kc, Vc, fl, sz, _ = _stream(is_sep, K, a, s, w, c, upto)
        nw = int(sz[0, 2] + sz[0, 3])
        Kf, Vf, ff, sf, valid = oracle.fill_from_prefill(K[:, :, :upto], -K[:, :, :upto], is_sep[:, :upto], a, s, w, c, nw)
        assert np.array_equal(sz, sf), (upto, sz, sf)
        assert np.array_equal(fl[:, :nw], ff[:, :nw])
        assert np.array_equal(Kc[0][:, valid[0]], Kf[0][:, valid[0]]) and np.array_equal(Vc[0][:, valid[0]], Vf[0][:, valid[0]])


def test_append_follows_the_size_state_machine():
    """Without a Separator Cache (s = 0) "window region full" and "Size_run = c" are the same event, so
    the sizes must follow the simulator of Sec. 3.3 token by token; the Local Window never exceeds w."""
    a, s, w, c, L = 3, 0, 4, 13, 60
    is_sep = _flags(1, L, 0.3, 13)
    K = _rand((1, 1, L, 2), 14)
    sim = cache_sim.simulate(is_sep[0], a, s, w, c)
    _, _, _, _, hist = _stream(is_sep, K, a, s, w, c, L)
    for m, h in enumerate(hist):
        assert h[0] == min(a, m + 1) and h[3] <= w
        assert h[2] + h[3] == sim["n"][m] and h.sum() == sim["size_run"][m]
    # a full window region refuses the token
    Kc, Vc = np.zeros((1, 1, 8, 2)), np.zeros((1, 1, 8, 2))
    sz = np.array([[1, 2, 2, 3]], dtype=np.int32)
    K2, V2, f2, s2 = oracle.append_token(Kc, Vc, np.zeros((1, 5), dtype=np.uint8), sz, np.ones((1, 1, 2)), np.ones((1, 1, 2)), np.array([1]), 1, 2, 3)
    assert np.array_equal(s2, sz) and (K2 == 0).all()


# ----------------------------------------------------------------------------------------------
# eviction and the cache-size state machine
# ----------------------------------------------------------------------------------------------
def test_evict_postconditions_and_rows_bit_exact():
    rng = np.random.default_rng(0)
    S, Hkv, d, a, s, c = 3, 2, 4, 2, 6, 2 + 6 + 12
    Kc = rng.integers(0, 2 ** 16, size=(S, Hkv, c, d)).astype(np.uint16)
    Vc = rng.integers(0, 2 ** 16, size=(S, Hkv, c, d)).astype(np.uint16)
    flags = (rng.random((S, 12)) < 0.5).astype(np.uint8)
    flags[1, :8] = 1  # forces separator-cache overflow for sequence 1
    sizes = np.array([[2, 1, 8, 4], [2, 5, 8, 4], [2, 0, 0, 3]], dtype=np.int32)
    K2, V2, f2, sz2 = oracle.evict_window(Kc, Vc, flags, sizes, a, s)
    for q in range(S):
        ni, ns, P, Lw = sizes[q]
        kept = [a + s + t for t in range(P) if flags[q, t]]
        src = ([a + k for k in range(ns)] + kept)[-s:] if (ns + len(kept)) > 0 else []
        assert list(sz2[q]) == [ni, min(s, ns + len(kept)), 0, Lw]
        for X, X2 in ((Kc, K2), (Vc, V2)):
            assert np.array_equal(X2[q, :, :a], X[q, :, :a])
            assert np.array_equal(X2[q, :, a:a + len(src)], X[q, :, src].transpose(1, 0, 2)
                                  if len(src) else X2[q, :, a:a])
            assert np.array_equal(X2[q, :, a + s:a + s + Lw], X[q, :, a + s + P:a + s + P + Lw])
        assert np.array_equal(f2[q, :Lw], flags[q, P:P + Lw])


def test_evict_preserves_attention_over_kept_entries():
    """Dropping is the only change: decode over the new cache = decode over the kept entries."""
    rng = np.random.default_rng(1)
    S, Hq, Hkv, d, a, s, c = 2, 2, 1, 4, 1, 4, 1 + 4 + 10
    Kc, Vc = _rand((S, Hkv, c, d), 1), _rand((S, Hkv, c, d), 2)
    flags = (rng.random((S, 10)) < 0.4).astype(np.uint8)
    sizes = np.array([[1, 2, 6, 4], [1, 4, 5, 3]], dtype=np.int32)
    q = _rand((S, Hq, d), 3)
    K2, V2, f2, sz2 = oracle.evict_window(Kc, Vc, flags, sizes, a, s)
    out2, lse2 = oracle.decode(q, K2, V2, sz2, a, s, 0.5)
    for sq in range(S):
        ni, ns, P, Lw = sizes[sq]
        kept = [a + s + t for t in range(P) if flags[sq, t]]
        sep_src = ([a + k for k in range(ns)] + kept)[-s:]
        slots = list(range(ni)) + sep_src + [a + s + P + t for t in range(Lw)]
        allowed = np.ones((1, len(slots)), dtype=bool)
        for h in range(Hq):
            o, l = softmax_attention_dense(q[sq, h][None], Kc[sq, 0, slots], Vc[sq, 0, slots], allowed, 0.5)
            assert np.allclose(out2[sq, h], o[0], atol=1e-12) and abs(lse2[sq, h] - l[0]) < 1e-12


def test_simulated_runtime_usage_reproduces_printed_rkv_values():
    """Sec. 3.3: after the Separator Cache fills, n(m) is a sawtooth on [w, c-a-s] of period
    c-a-s-w and mean Size_run -> (w+c+a+s)/2, which is what every r.KV the paper prints equals."""
    for a, s, w, c, rkv in (map(int, r) for r in _golden_rows("runtime_kv_usage.txt")):
        assert (w + c + a + s) / 2 == rkv
        period = c - a - s - w
        M = 40 * period + 6 * c + 40 * s
        is_sep = (np.random.default_rng(a + s + w + c).random(M) < 0.1)
        sim = cache_sim.simulate(is_sep, a, s, w, c)
        assert sim["size_run_pre"].max() == c
        full = np.flatnonzero(sim["size_sep"] == s)
        assert full.size, "separator cache never filled"
        fires = np.flatnonzero(sim["compressed"] & (np.arange(M) >= full[0]))
        assert np.all(np.diff(fires) == period)
        lo, hi = fires[1], fires[-1]  # whole periods
        n_steady = sim["n"][lo:hi]
        assert n_steady.min() == w and n_steady.max() == c - a - s - 1
        assert sim["size_run_pre"][lo:hi].max() == c
        mean_post = sim["size_run"][lo:hi].mean()
        mean_pre = sim["size_run_pre"][lo:hi].mean()
        assert abs(0.5 * (mean_post + mean_pre) - rkv) < 1e-9
        assert abs(n_steady.mean() + 0.5 - (w + c - a - s) / 2) < 1e-9
