"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Bar (from the build's target): sign words bit-exact; scales, errors, momenta and parameters within
rtol 1e-5 / atol 1e-7.  Scales are additionally expected to be bit-equal except where the binary64
sum lands next to a binary32 rounding boundary (the two sides add in different orders).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2008_11343_amd import binding as B
from paper_2008_11343_amd import workloads as W
from paper_2008_11343_amd.runner import DeviceRun, from_host_state

pytestmark = pytest.mark.gpu

F = np.float32
RTOL, ATOL = 1e-5, 1e-7
DEV = "cuda:0"


def say(msg):
    print("[parity] " + msg, flush=True)


def host(t):
    a = t.detach().cpu().numpy()
    return a.view(np.uint32) if a.dtype == np.int32 else a


def close(a, b, what):
    np.testing.assert_allclose(a, b, rtol=RTOL, atol=ATOL, err_msg=what)


def same_words(a, b, what):
    a, b = np.asarray(a).reshape(-1), np.asarray(b).reshape(-1)
    bad = np.flatnonzero(a != b)
    assert bad.size == 0, "%s: %d sign words differ, first at word %d: %08x vs %08x" % (
        what, bad.size, bad[0], a[bad[0]], b[bad[0]])


def oracle_state(d, n, L, st):
    return oracle.State(d, n, L, st["x"], st["m"], st["v"], st["werr"], st["serr"])


MODES = [0, B.APMS_DEFER_ERRORS, B.APMS_DEFER_GATHER, B.APMS_DEFER_ERRORS | B.APMS_DEFER_GATHER]
MODE_IDS = ["eager", "defer-errors", "defer-gather", "defer-all"]


def compare_momentum(run, om, sscales_equal, tag):
    # the gathered momentum is a copy of +-sscale: exact given equal server scales
    gm = host(run.m)
    close(gm, om, tag + " m")
    if sscales_equal:
        assert np.array_equal(gm, om), tag + " m must be a bit-exact copy"


def compare_all(run, ost, tag, errors=True, momentum=True):
    same_words(host(run.packed), ost.packed, tag + " packed")
    same_words(host(run.spacked), ost.spacked, tag + " spacked")
    close(host(run.scales), ost.scales, tag + " scales")
    close(host(run.sscales), ost.sscales, tag + " sscales")
    close(host(run.x), ost.x, tag + " x")
    if momentum:
        compare_momentum(run, ost.m, np.array_equal(host(run.sscales), ost.sscales), tag)
    if errors:
        close(host(run.werr), ost.werr, tag + " worker_err")
        close(host(run.serr), ost.serr, tag + " server_err")


def random_case(seed, d, n, L, err_scale=3e-3):
    rng = np.random.default_rng(seed)
    st = dict(
        x=rng.normal(0, 0.02, d).astype(F),
        m=rng.normal(0, 1e-3, (n, d)).astype(F),
        v=np.exp(rng.normal(-12, 1, d)).astype(F),
        werr=rng.normal(0, err_scale, (n, d)).astype(F),
        serr=rng.normal(0, err_scale / 3, d).astype(F),
    )
    g = rng.normal(0, 1e-2, (n, d)).astype(F)
    return st, g


SHAPES = [
    # (n, L, C): one ragged word-tail tile, chunks not a multiple of the tile, several tiles per block
    (1, 32, 1),
    (3, 160, 2),
    (2, 4096, 2),
    (3, 4096 * 9 + 32 * 5, 3),
    (5, 4096 * 17, 2),
    (4, 65536, 4),
    (16, 4096 * 3 + 1024, 2),
]


@pytest.mark.parametrize("n,L,C", SHAPES)
@pytest.mark.parametrize("deferred", MODES, ids=MODE_IDS)
def test_stagewise_parity(n, L, C, deferred):
    """Each call fed the oracle's inputs for that stage: signs must match exactly.  A second compress then
    consumes whatever the first step left pending (errors in u form, the gather not yet written)."""
    d = L * C
    say("stagewise n=%d L=%d C=%d deferred=%s" % (n, L, C, deferred))
    st, g = random_case(100 + n + L, d, n, L)
    st["werr"][0, :8] = [0.0, -0.0, 1e-40, -1e-40, 0.0, 0.0, 0.0, 0.0]
    g[0, :8] = 0.0
    st["m"][0, :8] = 0.0
    ost = oracle_state(d, n, L, st)
    run = DeviceRun(d, n, L, DEV, deferred=deferred, state={k: torch.from_numpy(v) for k, v in st.items()})
    gd = torch.from_numpy(g).to(DEV)
    beta, lr, eps = 0.9, 1e-4, 1e-8

    run.compress(gd, beta)
    oracle.compress(d, n, L, ost.m, g, ost.werr, ost.packed, ost.scales, beta)
    same_words(host(run.packed), ost.packed, "packed")
    close(host(run.scales), ost.scales, "scales")
    # stage 2 consumes the ORACLE's messages
    run.packed.copy_(torch.from_numpy(ost.packed.view(np.int32)))
    run.scales.copy_(torch.from_numpy(ost.scales))
    run.server_reduce()
    oracle.server_reduce(d, n, L, ost.packed, ost.scales, ost.serr, ost.spacked, ost.sscales)
    same_words(host(run.spacked), ost.spacked, "spacked")
    close(host(run.sscales), ost.sscales, "sscales")
    run.spacked.copy_(torch.from_numpy(ost.spacked.view(np.int32)))
    run.sscales.copy_(torch.from_numpy(ost.sscales))
    run.apply(lr, eps)
    oracle.apply(d, n, L, ost.spacked, ost.sscales, ost.v, ost.x, ost.m, lr, eps)
    close(host(run.x), ost.x, "x")
    # second worker step: reads the (possibly pending) error and momentum left by the first
    g2 = np.ascontiguousarray(g[::-1] * F(0.5))
    run.compress(torch.from_numpy(g2).to(DEV), beta)
    m_after_gather = ost.m.copy()
    oracle.compress(d, n, L, ost.m, g2, ost.werr, ost.packed, ost.scales, beta)
    assert np.array_equal(host(run.m), m_after_gather), "gathered momentum must be a bit-exact copy"
    same_words(host(run.packed), ost.packed, "packed (second step)")
    close(host(run.scales), ost.scales, "scales (second step)")
    run.finalize()
    close(host(run.werr), ost.werr, "worker_err")
    close(host(run.serr), ost.serr, "server_err")
    torch.cuda.synchronize()
    run.close()


@pytest.mark.parametrize("deferred", MODES, ids=MODE_IDS)
def test_tiny_trajectory(deferred):
    """Config 'tiny' (d = 2^20, n = 4, chunk 2^16): 10 compressed steps, every buffer, every step.
    Pending buffers are compared where they become final: the momentum right after the compress that
    writes it, the errors at a mid-run and at the closing finalize."""
    wl = W.TINY
    st = W.host_state(wl)
    ost = oracle_state(wl.d_pad, wl.n, wl.L, st)
    run = from_host_state(wl, st, DEV, deferred=deferred)
    gd = torch.empty(wl.n, wl.d_pad, dtype=torch.float32, device=DEV)
    equal_scales = 0
    sscales_equal = True
    for step in range(wl.steps):
        say("tiny trajectory step %d mode=%d" % (step, deferred))
        g = W.host_grad(wl, step)
        gd.copy_(torch.from_numpy(g))
        run.compress(gd, wl.beta)
        compare_momentum(run, ost.m, sscales_equal, "after compress of step %d" % step)
        run.server_reduce()
        run.apply(wl.lr, wl.eps)
        ost.step(g, wl.beta, wl.lr, wl.eps)
        final = step in (4, wl.steps - 1)
        if final:
            run.finalize()                   # mid-run and at the end: pending -> final, then carry on
        compare_all(run, ost, "step %d" % step, errors=final or not (deferred & B.APMS_DEFER_ERRORS),
                    momentum=final or not (deferred & B.APMS_DEFER_GATHER))
        sscales_equal = np.array_equal(host(run.sscales), ost.sscales)
        equal_scales += int(np.array_equal(host(run.scales), ost.scales))
    assert equal_scales >= wl.steps - 1
    run.close()


@pytest.mark.parametrize("n", [1, 3, 5, 64])
def test_worker_counts(n):
    """n = 1, non-power-of-two n and the 64-worker case of the worker-scaling config, three steps each."""
    L, C = 4096 * 2 + 96, 2
    d = L * C
    st, _ = random_case(7 + n, d, n, L, err_scale=0.0)
    ost = oracle_state(d, n, L, st)
    run = DeviceRun(d, n, L, DEV, deferred=True, state={k: torch.from_numpy(v) for k, v in st.items()})
    wl = W.scaled(W.WORKER_SCALING, d, n=n, chunk=L)
    for step in range(3):
        say("worker count n=%d step %d" % (n, step))
        g = W.host_grad(wl, step)
        run.step(torch.from_numpy(g).to(DEV), 0.9, 1e-4, 1e-8)
        ost.step(g, 0.9, 1e-4, 1e-8)
    run.finalize()
    compare_all(run, ost, "n=%d" % n)
    run.close()


def sweep_cases():
    """Twenty seeded draws of (workers, chunk length, chunks, deferral mode): chunk lengths from one sign word
    to six tiles, mostly ragged."""
    rng = np.random.default_rng(20080811)
    cases = []
    for i in range(20):
        n = int(rng.integers(1, 10))
        L = 32 * int(rng.integers(1, 2 if i % 7 == 0 else 700))
        C = int(rng.integers(1, 6))
        cases.append((i, n, L, C, MODES[int(rng.integers(0, len(MODES)))]))
    return cases


@pytest.mark.parametrize("case,n,L,C,deferred", sweep_cases(), ids=lambda v: str(v))
def test_random_shape_sweep(case, n, L, C, deferred):
    """Four steps on each drawn shape with gradients of a drawn scale (every fifth case heavy-tailed), sign words
    compared after every step, every buffer after the closing finalize."""
    d = L * C
    rng = np.random.default_rng(1000 + case)
    st, _ = random_case(500 + case, d, n, L, err_scale=float(10.0 ** rng.uniform(-5, -2)))
    ost = oracle_state(d, n, L, st)
    run = DeviceRun(d, n, L, DEV, deferred=deferred, state={k: torch.from_numpy(v) for k, v in st.items()})
    sigma = float(10.0 ** rng.uniform(-4, -1))
    for step in range(4):
        say("sweep case %d n=%d L=%d C=%d mode=%d step %d" % (case, n, L, C, deferred, step))
        g = (rng.standard_t(3, (n, d)) if case % 5 == 0 else rng.normal(0, 1, (n, d))).astype(F) * F(sigma)
        run.step(torch.from_numpy(g).to(DEV), 0.9, 1e-3, 1e-8)
        ost.step(g, 0.9, 1e-3, 1e-8)
        same_words(host(run.packed), ost.packed, "case %d step %d packed" % (case, step))
        same_words(host(run.spacked), ost.spacked, "case %d step %d spacked" % (case, step))
    run.finalize()
    compare_all(run, ost, "sweep case %d" % case)
    run.close()


def test_degenerate_values():
    """All-zero input (scale 0, all signs +), denormals, huge and tiny magnitudes side by side."""
    n, L, C = 2, 4096 + 64, 2
    d = L * C
    z = np.zeros
    st = dict(x=z(d, F), m=z((n, d), F), v=np.ones(d, F), werr=z((n, d), F), serr=z(d, F))
    g = z((n, d), F)
    g[1, L:L + 6] = [1e-38, -1e-38, 1e-42, -1e-42, 3e3, -3e3]     # chunk 1 of worker 1 only
    ost = oracle_state(d, n, L, st)
    run = DeviceRun(d, n, L, DEV, state={k: torch.from_numpy(v) for k, v in st.items()})
    for step in range(2):
        say("degenerate values step %d" % step)
        run.step(torch.from_numpy(g).to(DEV), 0.9, 1e-4, 1e-8)
        ost.step(g, 0.9, 1e-4, 1e-8)
        compare_all(run, ost, "degenerate step %d" % step)
    assert host(run.scales)[0, 0] == 0.0 and host(run.scales)[1, 1] > 0.0
    run.close()


def test_empty_problem_on_device():
    run = DeviceRun(0, 3, 64, DEV)
    g = torch.empty(3, 0, dtype=torch.float32, device=DEV)
    run.step(g, 0.9, 1e-4, 1e-8)
    run.finalize()
    torch.cuda.synchronize()
    run.close()


def test_determinism_and_tile_plan_independence():
    """Same inputs -> same bits; a different tiles-per-block plan changes only the summation tree
    (scales within 1 ulp), never a sign word of the same step."""
    n, L, C = 4, 4096 * 13, 2
    d = L * C
    st, g = random_case(55, d, n, L)
    outs = []
    for tiles in (8, 8, 1, 5):
        run = DeviceRun(d, n, L, DEV, state={k: torch.from_numpy(v) for k, v in st.items()})
        B.apms_set_tiles_per_block(run.ctx, tiles, tiles)
        say("determinism tiles_per_block=%d" % tiles)
        run.step(torch.from_numpy(g).to(DEV), 0.9, 1e-4, 1e-8)
        outs.append({k: host(getattr(run, k)).copy() for k in
                     ("packed", "scales", "spacked", "sscales", "x", "m", "werr", "serr")})
        run.close()
    for k, v in outs[0].items():
        assert np.array_equal(v, outs[1][k]), k
    for other in outs[2:]:
        same_words(other["packed"], outs[0]["packed"], "packed across plans")
        np.testing.assert_allclose(other["scales"], outs[0]["scales"], rtol=2e-7)


def test_pending_buffer_state_machine():
    """Deferred modes remember which buffer is pending; a call that would lose or read pending state is
    refused until apms_finalize."""
    n, L, C = 2, 4096, 1
    d = L * C
    st, g = random_case(77, d, n, L)
    run = DeviceRun(d, n, L, DEV, deferred=True, state={k: torch.from_numpy(v) for k, v in st.items()})
    gd = torch.from_numpy(g).to(DEV)
    run.compress(gd, 0.9)
    other = torch.zeros_like(run.werr)
    with pytest.raises(B.ApmsError) as ei:
        B.apms_compress(run.ctx, run.m, gd, other, run.packed, run.scales, 0.9)
    assert ei.value.status == B.APMS_ESTATE
    run.finalize()
    B.apms_compress(run.ctx, run.m, gd, other, run.packed, run.scales, 0.9)    # now fine
    B.apms_finalize(run.ctx, other, None, None)
    # gather pending after apply: the sign words must survive, m must be the same buffer
    run.server_reduce()
    run.apply(1e-4, 1e-8)
    other_m = torch.zeros_like(run.m)
    for call in (lambda: run.server_reduce(),
                 lambda: B.apms_compress(run.ctx, other_m, gd, run.werr, run.packed, run.scales, 0.9),
                 lambda: run.freeze(),
                 lambda: run.warmup_step(gd, 1e-3, 0.9, 0.999, 1e-8, 1)):
        with pytest.raises(B.ApmsError) as ei:
            call()
        assert ei.value.status == B.APMS_ESTATE
    run.finalize()
    run.server_reduce()                                                        # now fine
    run.finalize()
    torch.cuda.synchronize()
    run.close()


def test_side_stream():
    """Work is queued on the caller's stream."""
    n, L, C = 2, 4096 * 2, 2
    d = L * C
    st, g = random_case(88, d, n, L)
    ost = oracle_state(d, n, L, st)
    run = DeviceRun(d, n, L, DEV, state={k: torch.from_numpy(v) for k, v in st.items()})
    gd = torch.from_numpy(g).to(DEV)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    run.step(gd, 0.9, 1e-4, 1e-8, stream=s)
    s.synchronize()
    ost.step(g, 0.9, 1e-4, 1e-8)
    compare_all(run, ost, "side stream")
    run.close()


def test_warmup_freeze_then_compressed():
    """The full pipeline at reduced size: a BERT-style tensor list (LayerNorm gradients 10x smaller),
    5 Adam warm-up steps on the averaged gradient, freeze, then 6 compressed steps."""
    tensors = tuple(W.bert_large_tensors(layers=2, hidden=64, ffn=256, vocab=500, positions=32))
    total = sum(s for _, s, _ in tensors)
    wl = W.Workload("pipeline-small", W.FULL_PIPELINE.index, d=total, n=4, steps=6, warmup_steps=5,
                    tensors=tensors)
    d, n, L = wl.d_pad, wl.n, wl.L
    st = W.host_state(wl, warm_start=True)
    run = DeviceRun(d, n, L, DEV, deferred=True)
    run.x.copy_(torch.from_numpy(st["x"]))
    run.v.zero_()
    # rubbish in what freeze must overwrite
    run.m[1:].fill_(3.0)
    run.werr.fill_(1.0)
    run.serr.fill_(-1.0)
    ox, om, ov = st["x"].copy(), st["m"].copy(), st["v"].copy()
    lr_w = 1e-3
    for t in range(1, wl.warmup_steps + 1):
        say("pipeline warm-up step %d" % t)
        g = W.host_grad(wl, t - 1)
        run.warmup_step(torch.from_numpy(g).to(DEV), lr_w, wl.beta, wl.beta2, wl.eps, t)
        oracle.warmup_step(d, n, ox, om, ov, g, lr_w, wl.beta, wl.beta2, wl.eps, t)
        close(host(run.x), ox, "warm-up x")
        close(host(run.m[0]), om, "warm-up m")
        np.testing.assert_allclose(host(run.v), ov, rtol=RTOL, atol=1e-12, err_msg="warm-up v")
    run.freeze()
    omn, owerr, oserr = np.empty((n, d), F), np.ones((n, d), F), np.ones(d, F)
    oracle.freeze(d, n, om, omn, owerr, oserr)
    assert np.array_equal(host(run.werr), owerr) and np.array_equal(host(run.serr), oserr)
    for i in range(n):
        assert np.array_equal(host(run.m[i]), host(run.m[0]))
    # continue both sides from the GPU's frozen state (one copy of the bits)
    ost = oracle.State(d, n, L, host(run.x), host(run.m), host(run.v))
    for step in range(wl.steps):
        say("pipeline compressed step %d" % step)
        g = W.host_grad(wl, wl.warmup_steps + step)
        run.step(torch.from_numpy(g).to(DEV), wl.beta, wl.lr, wl.eps)
        ost.step(g, wl.beta, wl.lr, wl.eps)
        compare_all(run, ost, "pipeline step %d" % step, errors=False, momentum=False)
    run.finalize()
    compare_all(run, ost, "pipeline end")
    run.close()


@pytest.mark.parametrize("n,L,C", [(4, 65536, 2), (3, 4096 * 9 + 160, 3), (2, 32, 4), (5, 4096, 1), (2, 65536 + 4096, 1)],
                         ids=["max-onepass", "ragged", "one-word-rows", "one-tile", "just-too-long"])
def test_eager_one_pass_has_the_bits_of_the_two_pass_route(n, L, C):
    """With eager errors a chunk of up to 65536 elements is compressed in ONE pass (u held on chip, the finished
    error written directly); longer chunks take two passes.  Both must give the bits of the deferred route
    (partials per tile + scales kernel): sign words, scales, errors, every step; and match the oracle."""
    d = L * C
    wl = W.Workload("onepass", 1, d=d, n=n, chunk=L, steps=4)
    st = W.host_state(wl)
    ost = oracle_state(wl.d_pad, wl.n, wl.L, st)
    eager = from_host_state(wl, st, DEV, deferred=False)
    later = from_host_state(wl, st, DEV, deferred=True)
    mixed = from_host_state(wl, st, DEV, deferred=B.APMS_DEFER_GATHER)       # eager errors, gather pending
    gd = torch.empty(wl.n, wl.d_pad, dtype=torch.float32, device=DEV)
    for step in range(wl.steps):
        say("one pass n=%d L=%d C=%d step %d" % (n, L, C, step))
        g = W.host_grad(wl, step)
        gd.copy_(torch.from_numpy(g))
        ost.step(g, wl.beta, wl.lr, wl.eps)
        for r in (eager, later, mixed):
            r.step(gd, wl.beta, wl.lr, wl.eps)
        torch.cuda.synchronize()
        for r, tag in ((later, "deferred"), (mixed, "eager errors + deferred gather")):
            for name in ("packed", "scales", "spacked", "sscales", "x"):
                assert torch.equal(getattr(eager, name), getattr(r, name)), "step %d, %s: %s" % (step, tag, name)
        assert torch.equal(eager.werr, mixed.werr) and torch.equal(eager.serr, mixed.serr), "step %d: errors" % step
        compare_all(eager, ost, "eager, step %d" % step, errors=True, momentum=True)
    for r in (later, mixed):
        r.finalize()
    torch.cuda.synchronize()
    for r in (later, mixed):
        for name in ("m", "werr", "serr"):
            assert torch.equal(getattr(eager, name), getattr(r, name)), name
    for r in (eager, later, mixed):
        r.close()


def test_gather_forms_agree_and_auto_decides():
    """The pending gather can be carried out by a fill of its own (split) or inside the worker kernel (fused);
    APMS_GATHER_AUTO times both on its first gathers and keeps the faster.  All three give the same bits in
    every buffer, and the automatic choice is made without the library ever waiting."""
    wl = W.scaled(W.TINY, 4096 * 24 + 4096 * 3 * 4, chunk=4096 * 3 + 0)
    st = W.host_state(wl)
    ost = oracle_state(wl.d_pad, wl.n, wl.L, st)
    runs = {mode: from_host_state(wl, st, DEV, deferred=True)
            for mode in (B.APMS_GATHER_SPLIT, B.APMS_GATHER_FUSED, B.APMS_GATHER_AUTO)}
    for mode, r in runs.items():
        assert B.apms_get_plan(r.ctx)["gather_mode"] == B.APMS_GATHER_AUTO      # the default
        B.apms_set_gather_mode(r.ctx, mode)
        plan = B.apms_get_plan(r.ctx)
        assert plan["gather_mode"] == mode
        assert plan["gather_choice"] == (-1 if mode == B.APMS_GATHER_AUTO else mode)
    gd = torch.empty(wl.n, wl.d_pad, dtype=torch.float32, device=DEV)
    steps = 11                                  # step 0 has no gather; gather 0 untimed, 1-6 timed, 7 decides, then the choice
    for step in range(steps):
        say("gather forms step %d" % step)
        g = W.host_grad(wl, step)
        gd.copy_(torch.from_numpy(g))
        ost.step(g, wl.beta, wl.lr, wl.eps)
        for r in runs.values():
            r.step(gd, wl.beta, wl.lr, wl.eps)
        torch.cuda.synchronize()
        ref = runs[B.APMS_GATHER_SPLIT]
        for mode, r in runs.items():
            for name in ("packed", "scales", "spacked", "sscales", "x"):
                assert torch.equal(getattr(r, name), getattr(ref, name)), "step %d mode %d: %s" % (step, mode, name)
        same_words(host(ref.packed), ost.packed, "worker signs, step %d" % step)
        same_words(host(ref.spacked), ost.spacked, "server signs, step %d" % step)
    plan = B.apms_get_plan(runs[B.APMS_GATHER_AUTO].ctx)
    assert plan["gather_choice"] in (B.APMS_GATHER_SPLIT, B.APMS_GATHER_FUSED), plan
    assert all(ms > 0.0 for ms in plan["gather_ms"]), plan
    for r in runs.values():
        r.finalize()
    torch.cuda.synchronize()
    ref = runs[B.APMS_GATHER_SPLIT]
    compare_all(ref, ost, "after %d steps" % steps, errors=True, momentum=True)
    for mode, r in runs.items():
        for name in ("m", "werr", "serr"):
            assert torch.equal(getattr(r, name), getattr(ref, name)), "mode %d: %s" % (mode, name)
        r.close()


def test_hip_graph_replay_matches_eager():
    """The step allocates nothing, never synchronises and records no memset, so a steady-state step can be
    captured in a HIP graph: replays (with fresh gradients in the same buffer, and the program's own
    eager work and synchronisations in between) must give the bits of the eager path, every time."""
    wl = W.scaled(W.TINY, 4096 * 40, chunk=4096 * 10)
    st = W.host_state(wl)
    runs = [from_host_state(wl, st, DEV, deferred=True) for _ in range(2)]
    graphed, eager = runs
    gd = torch.empty(wl.n, wl.d_pad, dtype=torch.float32, device=DEV)
    for step in range(2):                       # reach the steady state: errors and gather pending
        gd.copy_(torch.from_numpy(W.host_grad(wl, step)))
        for r in runs:
            r.step(gd, wl.beta, wl.lr, wl.eps)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        graphed.step(gd, wl.beta, wl.lr, wl.eps)
    torch.cuda.synchronize()
    scratch = torch.empty(1 << 20, device=DEV)
    for step in range(2, 7):
        say("graph replay for step %d" % step)
        gd.copy_(torch.from_numpy(W.host_grad(wl, step)))
        torch.cuda.synchronize()
        graph.replay()
        scratch.normal_()                       # unrelated eager work between replays
        eager.step(gd, wl.beta, wl.lr, wl.eps)
        torch.cuda.synchronize()
        for name in ("packed", "scales", "spacked", "sscales", "x"):
            assert torch.equal(getattr(graphed, name), getattr(eager, name)), "replay of step %d: %s" % (step, name)
    for r in runs:
        r.finalize()
    torch.cuda.synchronize()
    for name in ("m", "werr", "serr"):
        assert torch.equal(getattr(graphed, name), getattr(eager, name)), name
    for r in runs:
        r.close()


@pytest.mark.parametrize("deferred", [True, False, B.APMS_DEFER_GATHER], ids=["deferred", "eager", "eager-errors"])
@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_sixteen_bit_gradients(fmt, deferred):
    """16-bit gradient inputs (binary16 / bfloat16, widened exactly): 3 Adam warm-up steps, freeze, 5
    compressed steps, ragged chunks; subnormal, zero and extreme 16-bit values planted in the first step.
    Fully deferred (two-pass worker kernel), eager and eager errors with the gather deferred (the one-pass
    worker kernel reading m, and decoding the pending gather)."""
    ofmt = {"f16": oracle.GRAD_F16, "bf16": oracle.GRAD_BF16}[fmt]
    wl = W.Workload("g16", 0, d=3 * (4096 * 3 + 96), n=3, chunk=4096 * 3 + 96, steps=5, warmup_steps=3)
    d, n, L = wl.d_pad, wl.n, wl.L
    st = W.host_state(wl, warm_start=True)
    run = DeviceRun(d, n, L, DEV, deferred=deferred)
    flags = run.deferral
    run.x.copy_(torch.from_numpy(st["x"]))
    run.v.zero_()
    ox, om, ov = st["x"].copy(), st["m"].copy(), st["v"].copy()
    special = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x03FF, 0x0400, 0x7BFF, 0xFBFF] if fmt == "f16" else
                       [0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x4F00, 0xCF00], np.uint16)
    for t in range(1, wl.warmup_steps + 1):
        say("g16 %s warm-up step %d" % (fmt, t))
        bits = W.host_grad_g16(wl, t - 1, fmt)
        if t == 1:
            bits[1, 5:5 + special.size] = special
        run.warmup_step(W.g16_bits_to_tensor(bits, fmt, DEV), 1e-3, wl.beta, wl.beta2, wl.eps, t)
        oracle.warmup_step(d, n, ox, om, ov, oracle.widen_g16(bits, ofmt), 1e-3, wl.beta, wl.beta2, wl.eps, t)
        close(host(run.x), ox, "warm-up x")
        close(host(run.m[0]), om, "warm-up m")
        np.testing.assert_allclose(host(run.v), ov, rtol=RTOL, atol=1e-12, err_msg="warm-up v")
    run.freeze()
    ost = oracle.State(d, n, L, host(run.x), host(run.m), host(run.v))
    for step in range(wl.steps):
        say("g16 %s compressed step %d" % (fmt, step))
        bits = W.host_grad_g16(wl, wl.warmup_steps + step, fmt)
        if step == 0:
            bits[2, L + 7:L + 7 + special.size] = special
        run.step(W.g16_bits_to_tensor(bits, fmt, DEV), wl.beta, wl.lr, wl.eps)
        ost.step(oracle.widen_g16(bits, ofmt), wl.beta, wl.lr, wl.eps)
        compare_all(run, ost, "g16 %s step %d" % (fmt, step), errors=not (flags & B.APMS_DEFER_ERRORS),
                    momentum=not (flags & B.APMS_DEFER_GATHER))
    run.finalize()
    compare_all(run, ost, "g16 %s end" % fmt)
    run.close()


def test_implicit_momentum_mode():
    """APMS_IMPLICIT_MOMENTUM: the momentum lives only in the server's sign words and scales; steps never
    touch m[n][d], yet every output matches the oracle, and apms_finalize right after apms_apply still
    materialises the gathered momentum on demand."""
    wl = W.scaled(W.TINY, 4 * (4096 * 5 + 160), chunk=4096 * 5 + 160)
    st = W.host_state(wl)
    ost = oracle_state(wl.d_pad, wl.n, wl.L, st)
    flags = B.APMS_DEFER_ERRORS | B.APMS_DEFER_GATHER | B.APMS_IMPLICIT_MOMENTUM
    run = from_host_state(wl, st, DEV, deferred=flags)
    m_before = run.m.clone()
    for step in range(6):
        say("implicit momentum step %d" % step)
        g = W.host_grad(wl, step)
        run.step(torch.from_numpy(g).to(DEV), wl.beta, wl.lr, wl.eps)
        ost.step(g, wl.beta, wl.lr, wl.eps)
        compare_all(run, ost, "implicit step %d" % step, errors=False, momentum=False)
        if step < 3:
            assert torch.equal(run.m, m_before), "a step wrote m in implicit mode"
        elif step == 3:
            B.apms_finalize(run.ctx, None, None, run.m)        # on demand, between apply and the next compress
            compare_momentum(run, ost.m, np.array_equal(host(run.sscales), ost.sscales), "implicit, materialised")
            m_before = run.m.clone()
        else:
            assert torch.equal(run.m, m_before)
    run.finalize()
    compare_all(run, ost, "implicit end")
    run.close()


@pytest.mark.parametrize("deferred", [0, B.APMS_DEFER_ERRORS], ids=["eager", "defer-errors"])
@pytest.mark.parametrize("fmt", ["f32", "bf16"])
def test_gradient_variant(deferred, fmt):
    """APGSqueeze variant (Section 5.3): the gradient is compensated and compressed, every worker forms the
    momentum from the decoded average.  6 steps on ragged chunks, every buffer against the oracle."""
    wl = W.Workload("apg", 1, d=2 * (4096 * 4 + 224), n=5, chunk=4096 * 4 + 224, steps=6)
    d, n, L = wl.d_pad, wl.n, wl.L
    st = W.host_state(wl)
    st["m"][:] = st["m"][0]                      # workers share the momentum, as after a warm-up
    ost = oracle_state(d, n, L, st)
    run = from_host_state(wl, st, DEV, deferred=deferred)
    for step in range(wl.steps):
        say("gradient variant %s step %d mode=%d" % (fmt, step, deferred))
        if fmt == "f32":
            g = W.host_grad(wl, step)
            gd = torch.from_numpy(g).to(DEV)
        else:
            bits = W.host_grad_g16(wl, step, fmt)
            g = oracle.widen_g16(bits, oracle.GRAD_BF16)
            gd = W.g16_bits_to_tensor(bits, fmt, DEV)
        run.step_gradient(gd, wl.beta, wl.lr, wl.eps)
        ost.step_gradient(g, wl.beta, wl.lr, wl.eps)
        compare_all(run, ost, "apg step %d" % step, errors=not deferred, momentum=False)
        close(host(run.m), ost.m, "apg momentum")
    run.finalize()
    compare_all(run, ost, "apg end", momentum=False)
    close(host(run.m), ost.m, "apg momentum")
    run.close()
