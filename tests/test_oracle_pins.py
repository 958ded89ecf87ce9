"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without a GPU.

The paper prints no worked numeric example of the update, so the oracle is
held by invariants (error feedback, norm preservation), hand-derived closed
forms (tests/golden/onebit_hand_cases.txt), brute force on tiny inputs,
special cases that reduce to textbook routines (identity compressor ->
momentum SGD with a fixed preconditioner; warm-up -> torch.optim.Adam), the
collapsed recursion and the telescoping identity of the supplement, and
structural checks (chunk / worker independence).  Every expected value below
is computed in float64 numpy or pure Python written in this file; none comes
from the HIP path.
"""
import os

import numpy as np
import pytest

import oracle

F = np.float32
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "onebit_hand_cases.txt")


# ---------------------------------------------------------------- helpers ---

def bufs(d, n, L):
    C = d // L
    return dict(packed=np.zeros((n, d // 32), np.uint32), scales=np.zeros((n, C), F),
                spacked=np.zeros(d // 32, np.uint32), sscales=np.zeros(C, F))


def unpack(words, count):
    """Bit j&31 of word j>>5, for j < count, as a 0/1 array (pure numpy, LSB first)."""
    words = np.asarray(words, np.uint32).reshape(-1)
    j = np.arange(count)
    return ((words[j >> 5] >> (j & 31).astype(np.uint32)) & np.uint32(1)).astype(np.int64)


def decode(words, scales, L):
    """Dense +-scale vector from sign words and per-chunk scales, float64."""
    count = words.size * 32
    bits = unpack(words, count)
    s = np.repeat(np.asarray(scales, np.float64), L)
    return np.where(bits == 1, s, -s)


def compress_of(u, L, n=1):
    """Run the oracle's worker step so that the compensated vector is exactly u (beta = 0, m = 0, delta = 0)."""
    u = np.ascontiguousarray(u, F).reshape(n, -1)
    d = u.shape[1]
    b = bufs(d, n, L)
    werr = np.zeros((n, d), F)
    oracle.compress(d, n, L, np.zeros((n, d), F), u, werr, b["packed"], b["scales"], 0.0)
    return b["packed"], b["scales"], werr


def rand_state(rng, d, n, shared_m=False):
    x = rng.normal(0, 0.02, d).astype(F)
    m = rng.normal(0, 1e-3, (n, d)).astype(F)
    if shared_m:
        m[:] = m[0]
    v = np.exp(rng.normal(-12, 1, d)).astype(F)
    return x, m, v


# ------------------------------------------------- golden / closed forms ----

def _golden_cases():
    cases = []
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, L, spec, sumsq, scale, words = [p.strip() for p in line.split("|")]
            cases.append((name, int(L), spec, float(sumsq), float(scale),
                          [int(w, 16) for w in words.split(",")]))
    return cases


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c[0])
def test_golden_hand_cases(case):
    """Section 5.1: scale = ||u||_2 / sqrt(L), signs LSB-first, sign(0) = +1 (hand-derived fixture)."""
    name, L, spec, sumsq, scale, words = case
    u = np.zeros(L, F)
    if spec.startswith("*:"):
        u[:] = float(spec[2:])
    elif spec != "-":
        for item in spec.split(","):
            idx, val = item.split(":")
            u[int(idx)] = float(val)
    assert float(np.sum(u.astype(np.float64) ** 2)) == sumsq      # fixture self-consistency
    packed, scales, werr = compress_of(u, L)
    assert [int(w) for w in packed.reshape(-1)] == words
    assert scales[0, 0] == pytest.approx(scale, rel=2e-7, abs=0)
    # error feedback by hand: delta' = u - (+-scale)
    s = float(scales[0, 0])
    expect = u.astype(np.float64) - np.where(u >= 0, s, -s)
    np.testing.assert_allclose(werr.reshape(-1), expect, rtol=0, atol=1.2e-7 * max(1.0, abs(u).max()))
    if name in ("all_equal", "neg_equal", "zeros"):
        assert np.all(werr == 0)             # |u| constant => the compressor is lossless


def test_pack_patterns():
    """32 elements -> exactly one word; alternating signs from element 0 -> 0x55555555; -0.0 counts as +."""
    L = 64
    u = np.ones(L, F)
    u[1::2] = -1
    packed, scales, _ = compress_of(u, L)
    assert packed.shape == (1, 2) and packed.dtype == np.uint32
    assert [int(w) for w in packed[0]] == [0x55555555, 0x55555555]
    assert scales[0, 0] == 1.0
    u = np.full(L, -0.0, F)
    u[5] = -1.0
    packed, _, _ = compress_of(u, L)
    assert [int(w) for w in packed[0]] == [0xFFFFFFDF, 0xFFFFFFFF]
    u = -np.ones(L, F)
    u[33] = 2.0
    packed, _, _ = compress_of(u, L)
    assert [int(w) for w in packed[0]] == [0x00000000, 0x00000002]


def test_pack_roundtrip_random():
    """unpack(pack(sign(u))) = (u >= 0) with u = g + delta (one exact-sign addition)."""
    rng = np.random.default_rng(1)
    d, n, L = 4096, 3, 1024
    g = rng.normal(0, 1e-2, (n, d)).astype(F)
    werr = rng.normal(0, 1e-2, (n, d)).astype(F)
    g[0, :7] = 0.0
    werr[0, :7] = [0.0, -0.0, 1e-40, -1e-40, 0.0, 0.0, 0.0]      # zeros and denormals
    u64 = g.astype(np.float64) + werr.astype(np.float64)
    b = bufs(d, n, L)
    oracle.compress(d, n, L, np.zeros((n, d), F), g, werr, b["packed"], b["scales"], 0.0)
    for i in range(n):
        np.testing.assert_array_equal(unpack(b["packed"][i], d), (u64[i] >= 0).astype(np.int64))


def test_scale_is_l2_not_l1():
    """Section 5.1 'same magnitude': ||scale * sign(u)||_2 = ||u||_2, i.e. scale = rms(u), not mean|u|."""
    rng = np.random.default_rng(2)
    L = 8192
    u = rng.normal(0, 1e-2, 2 * L).astype(F)
    _, scales, _ = compress_of(u, L)
    for k in range(2):
        uk = u[k * L:(k + 1) * L].astype(np.float64)
        assert float(scales[0, k]) * np.sqrt(L) == pytest.approx(np.linalg.norm(uk), rel=2e-7)
        assert abs(float(scales[0, k]) - np.mean(np.abs(uk))) > 0.1 * float(scales[0, k])


def test_scale_rounding_is_single():
    """The scale is the correctly rounded fp32 of the fp64 value sqrt(exact sum / L) (math.fsum = exact sum)."""
    import math
    rng = np.random.default_rng(3)
    L = 32768
    u = (rng.normal(0, 1, L) * 10.0 ** rng.uniform(-6, 2, L)).astype(F)
    _, scales, _ = compress_of(u, L)
    exact = math.fsum(float(a) * float(a) for a in u)       # products exact in binary64
    assert scales[0, 0] == F(math.sqrt(exact / L))


# ----------------------------------------------------- error feedback (P1) --

def test_error_feedback_worker_and_server():
    """delta' = u - C[u] (Section 3.1; supplement steps 1-2): C[u] + delta' recovers u on both sides."""
    rng = np.random.default_rng(4)
    d, n, L = 8192, 3, 2048
    beta = F(0.9)
    x, m, v = rand_state(rng, d, n)
    g = rng.normal(0, 1e-2, (n, d)).astype(F)
    werr0 = rng.normal(0, 3e-3, (n, d)).astype(F)
    serr0 = rng.normal(0, 1e-3, d).astype(F)
    werr, serr = werr0.copy(), serr0.copy()
    b = bufs(d, n, L)
    oracle.compress(d, n, L, m, g, werr, b["packed"], b["scales"], beta)
    u64 = np.float64(beta) * m + np.float64(F(1) - beta) * g + werr0
    msgs = np.stack([decode(b["packed"][i], b["scales"][i], L) for i in range(n)])
    np.testing.assert_allclose(msgs + werr, u64, rtol=0, atol=2e-9)          # ~1 ulp of 1e-2
    assert np.abs(werr).max() > 1e-4                                          # the error is not trivially zero

    oracle.server_reduce(d, n, L, b["packed"], b["scales"], serr, b["spacked"], b["sscales"])
    ubar64 = msgs.mean(axis=0) + serr0
    smsg = decode(b["spacked"], b["sscales"], L)
    np.testing.assert_allclose(smsg + serr, ubar64, rtol=0, atol=2e-9)
    np.testing.assert_array_equal(unpack(b["spacked"], d), (ubar64 >= 0).astype(np.int64) |
                                  (np.abs(ubar64) < 1e-10))                   # signs, away from ties
    for k in range(d // L):
        sl = slice(k * L, (k + 1) * L)
        assert float(b["sscales"][k]) == pytest.approx(np.sqrt(np.mean(ubar64[sl] ** 2)), rel=1e-6)


# ----------------------------------------------------- brute force (P4) -----

@pytest.mark.parametrize("n", [1, 2, 3, 5])
def test_server_average_brute_force(n):
    """Server average of the n decoded messages + server error, against pure-Python loops (tiny d)."""
    rng = np.random.default_rng(10 + n)
    d, L = 64, 32
    packed = rng.integers(0, 2 ** 32, (n, d // 32), dtype=np.uint64).astype(np.uint32)
    scales = rng.uniform(0.5, 2.0, (n, d // L)).astype(F)
    serr0 = rng.normal(0, 0.3, d).astype(F)
    serr = serr0.copy()
    b = bufs(d, n, L)
    oracle.server_reduce(d, n, L, packed, scales, serr, b["spacked"], b["sscales"])
    ubar = []
    for j in range(d):
        tot = 0.0
        for i in range(n):
            bit = (int(packed[i, j // 32]) >> (j % 32)) & 1
            s = float(scales[i, j // L])
            tot += s if bit else -s
        ubar.append(tot / n + float(serr0[j]))
    ubar = np.array(ubar)
    for k in range(d // L):
        sl = slice(k * L, (k + 1) * L)
        s_expect = np.sqrt(np.mean(ubar[sl] ** 2))
        assert float(b["sscales"][k]) == pytest.approx(s_expect, rel=1e-6)
        for j in range(k * L, (k + 1) * L):
            bit = (int(b["spacked"][j // 32]) >> (j % 32)) & 1
            if abs(ubar[j]) > 1e-6:
                assert bit == (1 if ubar[j] >= 0 else 0)
            c = float(b["sscales"][k]) if bit else -float(b["sscales"][k])
            assert c + float(serr[j]) == pytest.approx(ubar[j], abs=5e-7)


# -------------------------------------------- identity compressor (P5) ------

def test_identity_compressor_is_momentum_sgd():
    """'APMSqueeze (Uncompressed)' of Section 5.3: with C = identity the step is momentum SGD
    preconditioned by the frozen v, and both errors stay exactly zero."""
    rng = np.random.default_rng(5)
    d, n, L, T = 2048, 4, 512, 6
    beta, lr, eps = F(0.9), F(1e-4), F(1e-8)
    x, m, v = rand_state(rng, d, n, shared_m=True)
    st = oracle.State(d, n, L, x, m, v)
    x64, m64 = x.astype(np.float64), m[0].astype(np.float64)
    P = 1.0 / (np.sqrt(v.astype(np.float64)) + np.float64(eps))
    for t in range(T):
        g = rng.normal(0, 1e-2, (n, d)).astype(F)
        st.step(g, beta, lr, eps, compressor=oracle.IDENTITY)
        m64 = np.float64(beta) * m64 + np.float64(F(1) - beta) * g.astype(np.float64).mean(axis=0)
        x64 = x64 - np.float64(lr) * m64 * P
        assert np.all(st.werr == 0) and np.all(st.serr == 0)
    np.testing.assert_allclose(st.m[0], m64, rtol=1e-5, atol=1e-9)
    np.testing.assert_allclose(st.x, x64, rtol=1e-5, atol=1e-7)
    for i in range(1, n):
        np.testing.assert_array_equal(st.m[i], st.m[0])


# ------------------------------------- collapsed recursion (P6) and P7 ------

def _delta(st):
    return st.werr.astype(np.float64).mean(axis=0) + st.serr.astype(np.float64)


@pytest.mark.parametrize("shared", [True, False])
def test_collapsed_recursion(shared):
    """Supplement, 'Proof to the Updating Form': m_t + D_t = beta m_{t-1} + (1-beta) gbar_t + D_{t-1},
    D = mean_i delta_i + delta_server, for the 1-bit compressor, step after step."""
    rng = np.random.default_rng(6)
    d, n, L, T = 4096, 4, 1024, 5
    beta, lr, eps = F(0.9), F(1e-4), F(1e-8)
    x, m, v = rand_state(rng, d, n, shared_m=shared)
    st = oracle.State(d, n, L, x, m, v)
    for t in range(T):
        g = rng.normal(0, 1e-2, (n, d)).astype(F)
        m_prev = st.m.astype(np.float64).mean(axis=0)
        D_prev = _delta(st)
        st.step(g, beta, lr, eps)
        lhs = st.m[0].astype(np.float64) + _delta(st)
        rhs = np.float64(beta) * m_prev + np.float64(F(1) - beta) * g.astype(np.float64).mean(axis=0) + D_prev
        np.testing.assert_allclose(lhs, rhs, rtol=0, atol=5e-9)
        assert np.abs(st.m[0]).max() > 1e-4


def test_telescoping_closed_form():
    """Supplement, proof of Lemma 2 (auxiliary sequence y_t): with constant lr and P = 1/(sqrt(v)+eps),
    z_t = x_t - lr P (beta m_t + D_t)/(1-beta) moves by exactly -lr P gbar_t per step, so the final x is
    fixed by x_0, m_0, the final momentum and errors, and the SUM of the averaged gradients."""
    rng = np.random.default_rng(7)
    d, n, L, T = 4096, 4, 512, 12
    beta, lr, eps = F(0.9), F(1e-4), F(1e-8)
    x0, m0, v = rand_state(rng, d, n, shared_m=True)
    st = oracle.State(d, n, L, x0, m0, v)
    gsum = np.zeros(d)
    for t in range(T):
        g = rng.normal(0, 1e-2, (n, d)).astype(F)
        gsum += g.astype(np.float64).mean(axis=0)
        st.step(g, beta, lr, eps)
    b64, omb = np.float64(beta), np.float64(F(1) - beta)
    P = 1.0 / (np.sqrt(v.astype(np.float64)) + np.float64(eps))
    lr64 = np.float64(lr)
    z0 = x0.astype(np.float64) - lr64 * P * (b64 * m0[0].astype(np.float64)) / omb
    zT = z0 - lr64 * P * gsum
    xT = zT + lr64 * P * (b64 * st.m[0].astype(np.float64) + _delta(st)) / omb
    correction = np.abs(xT - zT).max()
    np.testing.assert_allclose(st.x, xT, rtol=0, atol=2e-7)
    assert correction > 1e-5          # the identity is not vacuous at this tolerance


# ------------------------------------------------------ special cases -------

def test_single_worker_recompression_is_idempotent():
    """n = 1 and zero server error: C[C[u]] = C[u], so the server's signs equal the worker's, its scale
    equals the worker's to rounding and its new error is ~0."""
    rng = np.random.default_rng(8)
    d, L = 4096, 1024
    u = rng.normal(0, 1e-2, d).astype(F)
    packed, scales, _ = compress_of(u, L)
    serr = np.zeros(d, F)
    b = bufs(d, 1, L)
    oracle.server_reduce(d, 1, L, packed, scales, serr, b["spacked"], b["sscales"])
    np.testing.assert_array_equal(b["spacked"], packed[0])
    np.testing.assert_allclose(b["sscales"], scales[0], rtol=2e-7)
    assert np.abs(serr).max() <= 2e-7 * float(scales.max())


def test_apply_closed_form_and_gather():
    """Algorithm 1 lines 10-11: every worker's momentum becomes the decoded server message (a copy, bit
    for bit), and x moves by -lr * m / (sqrt(v) + eps)."""
    rng = np.random.default_rng(9)
    d, n, L = 4096, 3, 1024
    lr, eps = F(3e-4), F(1e-8)
    x0, m, v = rand_state(rng, d, n)
    spacked = rng.integers(0, 2 ** 32, d // 32, dtype=np.uint64).astype(np.uint32)
    sscales = rng.uniform(1e-4, 1e-2, d // L).astype(F)
    x = x0.copy()
    oracle.apply(d, n, L, spacked, sscales, v, x, m, lr, eps)
    bits = unpack(spacked, d)
    s32 = np.repeat(sscales, L)
    expect_m = np.where(bits == 1, s32, -s32).astype(F)
    for i in range(n):
        np.testing.assert_array_equal(m[i], expect_m)
    x64 = x0.astype(np.float64) - np.float64(lr) * expect_m.astype(np.float64) / (
        np.sqrt(v.astype(np.float64)) + np.float64(eps))
    np.testing.assert_allclose(x, x64, rtol=1e-6, atol=1e-9)
    assert np.abs(x - x0).max() > 1e-6
    # eps = 0 is the paper's literal update (division by sqrt(v))
    x = x0.copy()
    oracle.apply(d, n, L, spacked, sscales, v, x, m, lr, 0.0)
    np.testing.assert_allclose(x, x0.astype(np.float64) - np.float64(lr) * expect_m / np.sqrt(v.astype(np.float64)),
                               rtol=1e-6, atol=1e-9)


# -------------------------------------------------------- warm-up (P9) ------

@pytest.mark.parametrize("n", [1, 4])
def test_warmup_matches_torch_adam(n):
    """Section 3.2 'Original Adam': the warm-up step on the averaged gradient equals torch.optim.Adam (CPU, fp64)."""
    import torch
    rng = np.random.default_rng(11)
    d, T = 1024, 7
    lr, b1, b2, eps = 1e-3, 0.9, 0.999, 1e-8
    x0 = rng.normal(0, 0.02, d).astype(F)
    x, m, v = x0.copy(), np.zeros(d, F), np.zeros(d, F)
    p = torch.tensor(x0.astype(np.float64), requires_grad=True)
    opt = torch.optim.Adam([p], lr=lr, betas=(float(F(b1)), float(F(b2))), eps=eps)
    for t in range(1, T + 1):
        g = rng.normal(0, 1e-2, (n, d)).astype(F)
        oracle.warmup_step(d, n, x, m, v, g, lr, b1, b2, eps, t)
        p.grad = torch.tensor(g.astype(np.float64).mean(axis=0))
        opt.step()
    state = opt.state[p]
    np.testing.assert_allclose(x, p.detach().numpy(), rtol=1e-5, atol=1e-7)
    np.testing.assert_allclose(m, state["exp_avg"].numpy(), rtol=1e-5, atol=1e-9)
    np.testing.assert_allclose(v, state["exp_avg_sq"].numpy(), rtol=1e-5, atol=1e-12)
    assert np.abs(x - x0).max() > 1e-3          # seven steps of size ~lr each


def test_freeze_handover():
    """Algorithm 1 initialisation + line 3: errors start at zero, every worker starts from the warm-up momentum."""
    rng = np.random.default_rng(12)
    d, n = 256, 3
    m_warm = rng.normal(0, 1e-3, d).astype(F)
    m = rng.normal(0, 1, (n, d)).astype(F)
    werr = rng.normal(0, 1, (n, d)).astype(F)
    serr = rng.normal(0, 1, d).astype(F)
    oracle.freeze(d, n, m_warm, m, werr, serr)
    for i in range(n):
        np.testing.assert_array_equal(m[i], m_warm)
    assert not werr.any() and not serr.any()


# ----------------------------------------------- structure / indexing -------

def test_chunks_and_workers_are_independent():
    """The method is a parameter server per chunk (supplement, first paragraph): a chunk's result depends
    only on that chunk's elements, and a worker's message only on that worker's slices.  Running every
    (worker, chunk) as its own d = L, n = 1 problem must give the same bits."""
    rng = np.random.default_rng(13)
    d, n, L = 3 * 512, 3, 512
    beta = F(0.9)
    _, m, _ = rand_state(rng, d, n)
    g = rng.normal(0, 1e-2, (n, d)).astype(F)
    werr0 = rng.normal(0, 1e-3, (n, d)).astype(F)
    werr = werr0.copy()
    b = bufs(d, n, L)
    oracle.compress(d, n, L, m, g, werr, b["packed"], b["scales"], beta)
    for i in range(n):
        for k in range(d // L):
            sl = slice(k * L, (k + 1) * L)
            e = werr0[i, sl].copy().reshape(1, L)
            bb = bufs(L, 1, L)
            oracle.compress(L, 1, L, m[i, sl].copy().reshape(1, L), g[i, sl].copy().reshape(1, L), e,
                            bb["packed"], bb["scales"], beta)
            np.testing.assert_array_equal(bb["packed"][0], b["packed"][i, k * L // 32:(k + 1) * L // 32])
            assert bb["scales"][0, 0] == b["scales"][i, k]
            np.testing.assert_array_equal(e[0], werr[i, sl])
    # server: chunk k alone
    serr0 = rng.normal(0, 1e-3, d).astype(F)
    serr = serr0.copy()
    oracle.server_reduce(d, n, L, b["packed"], b["scales"], serr, b["spacked"], b["sscales"])
    for k in range(d // L):
        sl = slice(k * L, (k + 1) * L)
        wsl = slice(k * L // 32, (k + 1) * L // 32)
        e = serr0[sl].copy()
        bb = bufs(L, n, L)
        oracle.server_reduce(L, n, L, np.ascontiguousarray(b["packed"][:, wsl]),
                             np.ascontiguousarray(b["scales"][:, k:k + 1]), e, bb["spacked"], bb["sscales"])
        np.testing.assert_array_equal(bb["spacked"], b["spacked"][wsl])
        assert bb["sscales"][0] == b["sscales"][k]
        np.testing.assert_array_equal(e, serr[sl])


def test_momentum_and_gradient_are_not_swapped():
    """u = beta*m + (1-beta)*g + delta: with beta = 0.75, m = 4, g = 8, delta = 1 every element is
    0.75*4 + 0.25*8 + 1 = 6 exactly (swapping m and g would give 8)."""
    d, L = 64, 32
    m = np.full((1, d), 4.0, F)
    g = np.full((1, d), 8.0, F)
    werr = np.full((1, d), 1.0, F)
    b = bufs(d, 1, L)
    oracle.compress(d, 1, L, m, g, werr, b["packed"], b["scales"], 0.75)
    assert np.all(b["scales"] == 6.0) and np.all(werr == 0.0) and np.all(b["packed"] == 0xFFFFFFFF)


def test_determinism():
    rng = np.random.default_rng(14)
    d, n, L = 4096, 4, 1024
    x, m, v = rand_state(rng, d, n)
    gs = [rng.normal(0, 1e-2, (n, d)).astype(F) for _ in range(3)]
    outs = []
    for _ in range(2):
        st = oracle.State(d, n, L, x, m, v)
        for g in gs:
            st.step(g, 0.9, 1e-4, 1e-8)
        outs.append((st.x.copy(), st.m.copy(), st.werr.copy(), st.serr.copy(), st.packed.copy(),
                     st.spacked.copy(), st.scales.copy(), st.sscales.copy()))
    for a, b_ in zip(*outs):
        np.testing.assert_array_equal(a, b_)


@pytest.mark.parametrize("shape", [(4096, 4, 1024), (3 * 2048, 3, 2048 * 3), (8 * 160, 5, 160)],
                         ids=["4chunks", "1chunk", "8chunks"])
def test_thread_count_does_not_change_a_bit(shape):
    """Only independent work is spread over threads (whole (worker, chunk) problems, whole chunks, elements of
    loops with no carried value), so any thread count gives the bits of the serial run: warm-up, hand-over and
    compressed steps, more chunks than threads and fewer."""
    d, n, L = shape
    rng = np.random.default_rng(15)
    x, _, _ = rand_state(rng, d, n)
    gs = [rng.normal(0, 1e-2, (n, d)).astype(F) for _ in range(5)]
    outs = []
    try:
        for threads in (1, 2, 5):
            oracle.set_threads(threads)
            xw, mw, vw = x.copy(), np.zeros(d, F), np.zeros(d, F)
            for t in (1, 2):
                oracle.warmup_step(d, n, xw, mw, vw, gs[t - 1], 1e-3, 0.9, 0.999, 1e-8, t)
            m = np.zeros((n, d), F)
            oracle.freeze(d, n, mw, m, np.zeros((n, d), F), np.zeros(d, F))
            st = oracle.State(d, n, L, xw, m, vw)
            for g in gs[2:]:
                st.step(g, 0.9, 1e-4, 1e-8)
            outs.append((st.x.copy(), st.m.copy(), st.werr.copy(), st.serr.copy(), st.packed.copy(),
                         st.spacked.copy(), st.scales.copy(), st.sscales.copy()))
    finally:
        oracle.set_threads(1)
    for other in outs[1:]:
        for a, b_ in zip(outs[0], other):
            np.testing.assert_array_equal(a, b_)


def test_empty_input():
    """d = 0 is a valid, empty problem: nothing is read or written."""
    e = np.zeros((1, 0), F)
    oracle.compress(0, 1, 32, e, e, e.copy(), np.zeros((1, 0), np.uint32), np.zeros((1, 0), F), 0.9)
    oracle.server_reduce(0, 1, 32, np.zeros((1, 0), np.uint32), np.zeros((1, 0), F), np.zeros(0, F),
                         np.zeros(0, np.uint32), np.zeros(0, F))
    oracle.apply(0, 1, 32, np.zeros(0, np.uint32), np.zeros(0, F), np.zeros(0, F), np.zeros(0, F), e.copy(),
                 1e-4, 1e-8)


# ------------------------------------------- APGSqueeze variant (Sec. 5.3) ---

def test_apgsqueeze_identity_is_momentum_sgd_and_recursion_holds():
    """Section 5.3 item 4: error-compensated compression of the gradient.  With C = identity it is momentum
    SGD preconditioned by the frozen v; with the 1-bit compressor the double error feedback telescopes:
    ghat_t + D_t = gbar_t + D_{t-1}, D = mean_i delta_i + delta_server, ghat = decoded server message."""
    rng = np.random.default_rng(21)
    d, n, L, T = 2048, 4, 512, 6
    beta, lr, eps = F(0.9), F(1e-4), F(1e-8)
    x, m, v = rand_state(rng, d, n, shared_m=True)
    ident = oracle.State(d, n, L, x, m, v)
    onebit = oracle.State(d, n, L, x, m, v)
    x64, m64 = x.astype(np.float64), m[0].astype(np.float64)
    P = 1.0 / (np.sqrt(v.astype(np.float64)) + np.float64(eps))
    for t in range(T):
        g = rng.normal(0, 1e-2, (n, d)).astype(F)
        gbar = g.astype(np.float64).mean(axis=0)
        ident.step_gradient(g, beta, lr, eps, compressor=oracle.IDENTITY)
        m64 = np.float64(beta) * m64 + np.float64(F(1) - beta) * gbar
        x64 = x64 - np.float64(lr) * m64 * P
        assert not ident.werr.any() and not ident.serr.any()
        D_prev = _delta(onebit)
        m_prev = onebit.m[0].astype(np.float64)
        onebit.step_gradient(g, beta, lr, eps)
        ghat = decode(onebit.spacked, onebit.sscales, L)
        np.testing.assert_allclose(ghat + _delta(onebit), gbar + D_prev, rtol=0, atol=5e-9)
        np.testing.assert_allclose(onebit.m[0], np.float64(beta) * m_prev + np.float64(F(1) - beta) * ghat,
                                   rtol=1e-6, atol=1e-10)
        for i in range(1, n):
            np.testing.assert_array_equal(onebit.m[i], onebit.m[0])
    np.testing.assert_allclose(ident.m[0], m64, rtol=1e-5, atol=1e-9)
    np.testing.assert_allclose(ident.x, x64, rtol=1e-5, atol=1e-7)
    assert np.abs(onebit.x - x).max() > 1e-6


def test_apgsqueeze_hand_values():
    """u = g + delta = 3 everywhere -> scale 3, error 0; then m = 0.75*4 + 0.25*3 = 3.75 and, with v = 1,
    eps = 0.25, lr = 0.5: x = 1 - 0.5*3.75/1.25 = -0.5, all exact."""
    d, L, n = 64, 32, 2
    g = np.full((n, d), 2.0, F)
    werr = np.full((n, d), 1.0, F)
    b = bufs(d, n, L)
    oracle.compress(d, n, L, None, g, werr, b["packed"], b["scales"], 0.0)
    assert np.all(b["scales"] == 3.0) and np.all(werr == 0) and np.all(b["packed"] == 0xFFFFFFFF)
    serr = np.zeros(d, F)
    oracle.server_reduce(d, n, L, b["packed"], b["scales"], serr, b["spacked"], b["sscales"])
    assert np.all(b["sscales"] == 3.0) and not serr.any()
    m = np.full((n, d), 4.0, F)
    x = np.ones(d, F)
    oracle.apply_gradient(d, n, L, b["spacked"], b["sscales"], np.ones(d, F), x, m, 0.5, 0.75, 0.25)
    assert np.all(m == 3.75) and np.all(x == -0.5)


# ------------------------------------------------- 16-bit gradient inputs ---

def test_widen_f16_all_patterns_against_numpy():
    """Every one of the 65536 binary16 patterns widens to the value numpy's float16 gives it."""
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.widen_g16(bits, oracle.GRAD_F16)
    want = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))     # incl. the sign of zero
    assert got[0x0001] == 2.0 ** -24 and got[0x3C00] == 1.0 and got[0xC000] == -2.0 and got[0x7BFF] == 65504.0


def test_widen_bf16_all_patterns_against_torch():
    """Every bfloat16 pattern widens to the value torch's bfloat16 gives it (= the pattern shifted left by 16)."""
    import torch
    bits = np.arange(65536, dtype=np.uint16)
    got = oracle.widen_g16(bits, oracle.GRAD_BF16)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))
    assert np.array_equal(got[~nan].view(np.uint32), (bits.astype(np.uint32) << 16)[~nan])
    with pytest.raises(ValueError):
        oracle.widen_g16(bits, 7)

