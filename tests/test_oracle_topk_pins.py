"""Pins for the oracle's top-k compressor path (Section 5.1, second bullet), CPU only.

Hand cases, the tie rule, brute force against numpy's stable sort, exact error feedback, the special
case K = L (the compressor is then the identity, so the step is the momentum SGD the identity path
already pins), and the collapsed recursion of the supplement, which holds for any compressor.
"""
import numpy as np
import pytest

import oracle

F = np.float32


def topk_of(u, L, K, n=1):
    """Worker step arranged so that the compensated vector is exactly u (beta = 0, m = 0, delta = 0)."""
    u = np.ascontiguousarray(u, F).reshape(n, -1)
    d = u.shape[1]
    C = d // L
    idx, val = np.zeros((n, C, K), np.uint32), np.zeros((n, C, K), F)
    werr = np.zeros((n, d), F)
    oracle.topk_compress(d, n, L, K, np.zeros((n, d), F), u, werr, idx, val, 0.0)
    return idx, val, werr


def test_topk_hand_cases():
    L = 32
    u = np.zeros(L, F)
    u[[3, 7, 20, 31]] = [1.5, -4.0, 2.0, -3.0]
    idx, val, werr = topk_of(u, L, 2)
    assert idx[0, 0].tolist() == [7, 31] and val[0, 0].tolist() == [-4.0, -3.0]      # ascending index
    expect = u.copy()
    expect[[7, 31]] = 0.0
    assert np.array_equal(werr[0], expect)
    idx, val, _ = topk_of(u, L, 3)
    assert idx[0, 0].tolist() == [7, 20, 31] and val[0, 0].tolist() == [-4.0, 2.0, -3.0]


def test_topk_ties_keep_lower_index_first():
    L = 64
    u = np.zeros(L, F)
    u[[5, 9, 40, 41]] = [2.0, -2.0, 2.0, 7.0]            # three elements of magnitude 2
    idx, val, _ = topk_of(u, L, 3)
    assert idx[0, 0].tolist() == [5, 9, 41] and val[0, 0].tolist() == [2.0, -2.0, 7.0]
    idx, val, werr = topk_of(np.zeros(L, F), L, 4)        # everything ties at zero
    assert idx[0, 0].tolist() == [0, 1, 2, 3] and not val.any() and not werr.any()
    u = np.full(L, -0.0, F)
    u[10] = 0.0
    idx, _, _ = topk_of(u, L, 2)                          # -0.0 and +0.0 have the same magnitude
    assert idx[0, 0].tolist() == [0, 1]


@pytest.mark.parametrize("K", [1, 17, 256, 1024])
def test_topk_brute_force_against_numpy(K):
    rng = np.random.default_rng(K)
    L, C, n = 1024, 2, 2
    u = rng.normal(0, 1, (n, C * L)).astype(F)
    u[0, :200] = np.round(u[0, :200] * 4) / 4             # plenty of exact ties
    idx, val, werr = topk_of(u, L, K, n=n)
    for i in range(n):
        for k in range(C):
            uk = u[i, k * L:(k + 1) * L]
            order = np.argsort(-np.abs(uk), kind="stable")       # stable: lower index first among equals
            keep = np.sort(order[:K])
            assert np.array_equal(idx[i, k], keep.astype(np.uint32))
            assert np.array_equal(val[i, k], uk[keep])
            rest = uk.copy()
            rest[keep] = 0.0
            assert np.array_equal(werr[i, k * L:(k + 1) * L], rest)
            assert np.abs(uk[keep]).min() >= np.abs(rest).max()


def test_topk_error_feedback_is_exact_on_both_sides():
    """C[u] + delta' = u bit for bit: kept elements go out whole, the rest stay whole in the error."""
    rng = np.random.default_rng(3)
    d, n, L, K = 4096, 3, 1024, 37
    C = d // L
    beta = F(0.9)
    m = rng.normal(0, 1e-3, (n, d)).astype(F)
    g = rng.normal(0, 1e-2, (n, d)).astype(F)
    werr0 = rng.normal(0, 3e-3, (n, d)).astype(F)
    werr = werr0.copy()
    idx, val = np.zeros((n, C, K), np.uint32), np.zeros((n, C, K), F)
    oracle.topk_compress(d, n, L, K, m, g, werr, idx, val, beta)
    u64 = np.float64(beta) * m + np.float64(F(1) - beta) * g + werr0
    dense = np.zeros((n, d), F)
    for i in range(n):
        for k in range(C):
            dense[i, k * L + idx[i, k].astype(np.int64)] = val[i, k]
    np.testing.assert_allclose(dense.astype(np.float64) + werr, u64, rtol=0, atol=2e-9)
    assert np.all((dense == 0) | (werr == 0))
    serr0 = rng.normal(0, 1e-3, d).astype(F)
    serr = serr0.copy()
    sidx, sval = np.zeros((C, K), np.uint32), np.zeros((C, K), F)
    oracle.topk_server_reduce(d, n, L, K, idx, val, serr, sidx, sval)
    ubar64 = dense.astype(np.float64).mean(axis=0) + serr0
    sdense = np.zeros(d, F)
    for k in range(C):
        sdense[k * L + sidx[k].astype(np.int64)] = sval[k]
        assert np.all(np.diff(sidx[k].astype(np.int64)) > 0)
    np.testing.assert_allclose(sdense.astype(np.float64) + serr, ubar64, rtol=0, atol=2e-9)
    kept = sdense != 0
    assert np.abs(ubar64[kept]).min() >= np.abs(ubar64[~kept].reshape(C, -1)).max(axis=1).min() - 1e-12


def test_topk_with_k_equal_l_is_the_identity_compressor():
    """K = L keeps everything: the step must equal the identity-compressor path (momentum SGD), bit for bit."""
    rng = np.random.default_rng(4)
    d, n, L, T = 1024, 3, 256, 4
    x = rng.normal(0, 0.02, d).astype(F)
    m = np.tile(rng.normal(0, 1e-3, d).astype(F), (n, 1))
    v = np.exp(rng.normal(-12, 1, d)).astype(F)
    a = oracle.State(d, n, L, x, m, v)
    b = oracle.State(d, n, L, x, m, v)
    for t in range(T):
        g = rng.normal(0, 1e-2, (n, d)).astype(F)
        a.step_topk(g, L, 0.9, 1e-4, 1e-8)
        b.step(g, 0.9, 1e-4, 1e-8, compressor=oracle.IDENTITY)
        assert np.array_equal(a.x, b.x) and np.array_equal(a.m, b.m)
        assert not a.werr.any() and not a.serr.any()


def test_topk_collapsed_recursion_and_gather():
    """m_t + D_t = beta m_{t-1} + (1-beta) gbar_t + D_{t-1} (supplement) with the top-k compressor; the
    gathered momentum is zero outside the K positions the server kept and equal on all workers."""
    rng = np.random.default_rng(5)
    d, n, L, K, T = 2048, 4, 512, 16, 5
    x = rng.normal(0, 0.02, d).astype(F)
    m = np.tile(rng.normal(0, 1e-3, d).astype(F), (n, 1))
    v = np.exp(rng.normal(-12, 1, d)).astype(F)
    st = oracle.State(d, n, L, x, m, v)
    delta = lambda s: s.werr.astype(np.float64).mean(axis=0) + s.serr.astype(np.float64)
    for t in range(T):
        g = rng.normal(0, 1e-2, (n, d)).astype(F)
        m_prev, D_prev, x_prev = st.m[0].astype(np.float64), delta(st), st.x.copy()
        st.step_topk(g, K, 0.9, 1e-4, 1e-8)
        lhs = st.m[0].astype(np.float64) + delta(st)
        rhs = np.float64(F(0.9)) * m_prev + np.float64(F(1) - F(0.9)) * g.astype(np.float64).mean(axis=0) + D_prev
        np.testing.assert_allclose(lhs, rhs, rtol=0, atol=5e-9)
        assert np.count_nonzero(st.m[0]) == (d // L) * K
        for i in range(1, n):
            assert np.array_equal(st.m[i], st.m[0])
        moved = st.x != x_prev
        assert np.array_equal(moved, st.m[0] != 0)          # x moves exactly where the momentum is non-zero
        step64 = np.float64(F(1e-4)) * st.m[0].astype(np.float64) / (np.sqrt(v.astype(np.float64)) + 1e-8)
        np.testing.assert_allclose(st.x, x_prev.astype(np.float64) - step64, rtol=1e-6, atol=1e-9)
