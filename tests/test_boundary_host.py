"""Host-side tests of the C-ABI boundary: no GPU, no compute.

The library must load, export every function include/apms.h declares, and turn every invalid call into
a status code before anything is launched.  A context created with APMS_DEVICE_NONE validates only.
"""
import ctypes
import os
import re

import pytest

from paper_2008_11343_amd import binding as B
from paper_2008_11343_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = 0x10000          # fake, well-aligned "device addresses": validation never dereferences them
STEP = 0x10000000


def fake(i):
    return A + i * STEP


@pytest.fixture
def ctx():
    c = B.apms_create(d=8192, n=2, chunk_elems=4096, device=B.APMS_DEVICE_NONE)
    yield c
    B.apms_destroy(c)


def status_of(fn, *args, **kw):
    try:
        fn(*args, **kw)
    except B.ApmsError as e:
        return e.status
    return B.APMS_OK


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "apms.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(apms_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    lib = ctypes.CDLL(B.library_path())
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror_covers_all_codes():
    texts = {B.apms_strerror(code) for code in range(0, -10, -1)}
    assert len(texts) == 10 and "unknown apms status" not in texts
    assert B.apms_strerror(-99) == "unknown apms status"


@pytest.mark.parametrize("d,n,chunk,expect", [
    (8192, 0, 4096, B.APMS_EINVAL),
    (-32, 1, 32, B.APMS_EINVAL),
    (8192, 1, 0, B.APMS_ESHAPE),
    (8192, 4097, 4096, B.APMS_ESHAPE),     # more workers than the server kernel stages scales for
    (8192, 1, 48, B.APMS_ESHAPE),          # not a multiple of 32
    (8192, 1, 4096 * 3, B.APMS_ESHAPE),    # does not divide d
    (8192, 1, 16, B.APMS_ESHAPE),
    (0, 3, 32, B.APMS_OK),                 # empty problem
    (96, 5, 32, B.APMS_OK),
])
def test_create_validation(d, n, chunk, expect):
    try:
        c = B.apms_create(d, n, chunk, B.APMS_DEVICE_NONE)
    except B.ApmsError as e:
        assert e.status == expect
    else:
        assert expect == B.APMS_OK
        B.apms_destroy(c)


def test_create_rejects_bad_device_and_null_out():
    assert status_of(B.apms_create, 8192, 1, 4096, -7) == B.APMS_EINVAL
    assert B.load().apms_create(None, 8192, 1, 4096, B.APMS_DEVICE_NONE) == B.APMS_EINVAL
    assert B.load().apms_destroy(None) == B.APMS_OK


def test_valid_calls_on_validation_only_context_report_no_device(ctx):
    """No CPU fallback: with nothing to run on, a valid call fails loudly."""
    assert status_of(B.apms_compress, ctx, fake(0), fake(1), fake(2), fake(3), fake(4), 0.9) == B.APMS_ENODEV
    assert status_of(B.apms_server_reduce, ctx, fake(0), fake(1), fake(2), fake(3), fake(4)) == B.APMS_ENODEV
    assert status_of(B.apms_apply, ctx, fake(0), fake(1), fake(2), fake(3), fake(4), 1e-4, 1e-8) == B.APMS_ENODEV
    assert status_of(B.apms_warmup_step, ctx, fake(0), fake(1), fake(2), fake(3), 1e-3, 0.9, 0.999, 1e-8, 1) == \
        B.APMS_ENODEV
    assert status_of(B.apms_freeze, ctx, fake(0), fake(1), fake(2)) == B.APMS_ENODEV
    assert status_of(B.apms_finalize, ctx, fake(0), fake(1), fake(2)) == B.APMS_ENODEV


def test_null_misaligned_and_overlapping_arrays(ctx):
    good = [fake(i) for i in range(5)]
    for pos in range(5):
        args = list(good)
        args[pos] = None
        assert status_of(B.apms_compress, ctx, *args, 0.9) == B.APMS_EINVAL
        assert status_of(B.apms_server_reduce, ctx, *args) == B.APMS_EINVAL
        assert status_of(B.apms_apply, ctx, *args, 1e-4, 1e-8) == B.APMS_EINVAL
        args[pos] = good[pos] + 4
        assert status_of(B.apms_compress, ctx, *args, 0.9) == B.APMS_EALIGN
        assert status_of(B.apms_server_reduce, ctx, *args) == B.APMS_EALIGN
        assert status_of(B.apms_apply, ctx, *args, 1e-4, 1e-8) == B.APMS_EALIGN
    # worker_err overlapping the tail of m ([n][d] floats = 65536 bytes)
    args = list(good)
    args[2] = good[0] + 65536 - 16
    assert status_of(B.apms_compress, ctx, *args, 0.9) == B.APMS_EALIAS
    args[2] = good[0] + 65536                      # touching, not overlapping
    assert status_of(B.apms_compress, ctx, *args, 0.9) == B.APMS_ENODEV
    # apply: x aliasing v
    assert status_of(B.apms_apply, ctx, good[0], good[1], good[2], good[2], good[4], 1e-4, 1e-8) == B.APMS_EALIAS
    assert status_of(B.apms_warmup_step, ctx, good[0], good[0], good[2], good[3], 1e-3, 0.9, 0.999, 1e-8, 1) == \
        B.APMS_EALIAS


def test_scalar_ranges(ctx):
    good = [fake(i) for i in range(5)]
    for beta in (-0.1, 1.0, 1.5, float("nan")):
        assert status_of(B.apms_compress, ctx, *good, beta) == B.APMS_EINVAL
    assert status_of(B.apms_compress, ctx, *good, 0.0) == B.APMS_ENODEV
    w = good[:4]
    assert status_of(B.apms_warmup_step, ctx, *w, 1e-3, 0.9, 0.999, 1e-8, 0) == B.APMS_EINVAL
    assert status_of(B.apms_warmup_step, ctx, *w, 1e-3, 1.0, 0.999, 1e-8, 1) == B.APMS_EINVAL
    assert status_of(B.apms_warmup_step, ctx, *w, 1e-3, 0.9, -0.5, 1e-8, 1) == B.APMS_EINVAL
    assert status_of(B.apms_warmup_step, ctx, *w, float("nan"), 0.9, 0.999, 1e-8, 1) == B.APMS_EINVAL
    assert status_of(B.apms_apply, ctx, *good, float("nan"), 1e-8) == B.APMS_EINVAL
    assert status_of(B.apms_set_deferral, ctx, 8) == B.APMS_EINVAL
    assert status_of(B.apms_set_deferral, ctx, B.APMS_IMPLICIT_MOMENTUM) == B.APMS_EINVAL      # needs DEFER_GATHER
    assert status_of(B.apms_set_deferral, ctx, B.APMS_DEFER_GATHER | B.APMS_IMPLICIT_MOMENTUM) == B.APMS_OK
    assert status_of(B.apms_set_deferral, ctx, B.APMS_DEFER_ERRORS | B.APMS_DEFER_GATHER) == B.APMS_OK
    assert status_of(B.apms_set_tiles_per_block, ctx, -1, 0) == B.APMS_EINVAL
    assert status_of(B.apms_set_occupancy_pad, ctx, B.APMS_KERNEL_COUNT, 0) == B.APMS_EINVAL
    assert status_of(B.apms_set_occupancy_pad, ctx, B.APMS_KERNEL_WARMUP, 32768) == B.APMS_OK
    assert status_of(B.apms_set_occupancy_pad, ctx, B.APMS_KERNEL_APPLY, 200 * 1024) == B.APMS_EINVAL
    assert status_of(B.apms_set_occupancy_pad, ctx, B.APMS_KERNEL_APPLY, 4096) == B.APMS_OK
    assert B.apms_get_plan(ctx)["occupancy_pad"][B.APMS_KERNEL_APPLY] == 4096
    # the worker kernel's pad defaults to "by variant"; only that kernel accepts the value
    assert B.apms_get_plan(ctx)["occupancy_pad"][B.APMS_KERNEL_COMPRESS] == B.APMS_PAD_AUTO
    assert status_of(B.apms_set_occupancy_pad, ctx, B.APMS_KERNEL_COMPRESS, 65536) == B.APMS_OK
    assert status_of(B.apms_set_occupancy_pad, ctx, B.APMS_KERNEL_COMPRESS, B.APMS_PAD_AUTO) == B.APMS_OK
    assert status_of(B.apms_set_occupancy_pad, ctx, B.APMS_KERNEL_APPLY, B.APMS_PAD_AUTO) == B.APMS_EINVAL
    assert status_of(B.apms_set_occupancy_pad, ctx, B.APMS_KERNEL_COMPRESS, -2) == B.APMS_EINVAL


def test_sixteen_bit_gradient_entry_points(ctx):
    good = [fake(i) for i in range(5)]
    m, g, e, p, sc = good
    for fmt in (B.APMS_GRAD_F16, B.APMS_GRAD_BF16):
        assert status_of(B.apms_compress_g16, ctx, m, g, fmt, e, p, sc, 0.9) == B.APMS_ENODEV
        assert status_of(B.apms_warmup_step_g16, ctx, m, g, e, p, fmt, 1e-3, 0.9, 0.999, 1e-8, 1) == B.APMS_ENODEV
    for fmt in (0, 3, -1):
        assert status_of(B.apms_compress_g16, ctx, m, g, fmt, e, p, sc, 0.9) == B.APMS_EINVAL
        assert status_of(B.apms_warmup_step_g16, ctx, m, g, e, p, fmt, 1e-3, 0.9, 0.999, 1e-8, 1) == B.APMS_EINVAL
    assert status_of(B.apms_compress_g16, ctx, m, None, B.APMS_GRAD_F16, e, p, sc, 0.9) == B.APMS_EINVAL
    assert status_of(B.apms_compress_g16, ctx, m, g + 2, B.APMS_GRAD_F16, e, p, sc, 0.9) == B.APMS_EALIGN
    # g is [n][d] 16-bit values = 32768 bytes here: a buffer right behind it does not overlap, one inside does
    assert status_of(B.apms_compress_g16, ctx, m, g, B.APMS_GRAD_BF16, g + 32768, p, sc, 0.9) == B.APMS_ENODEV
    assert status_of(B.apms_compress_g16, ctx, m, g, B.APMS_GRAD_BF16, g + 32768 - 16, p, sc, 0.9) == B.APMS_EALIAS
    assert status_of(B.apms_compress, ctx, m, g, g + 32768, p, sc, 0.9) == B.APMS_EALIAS      # fp32 g is twice as long


def test_gradient_variant_entry_points(ctx):
    g, e, p, sc, m = [fake(i) for i in range(5)]
    for fmt in (0, B.APMS_GRAD_F16, B.APMS_GRAD_BF16):
        assert status_of(B.apms_compress_gradient, ctx, g, fmt, e, p, sc) == B.APMS_ENODEV
    assert status_of(B.apms_compress_gradient, ctx, g, 9, e, p, sc) == B.APMS_EINVAL
    assert status_of(B.apms_compress_gradient, ctx, None, 0, e, p, sc) == B.APMS_EINVAL
    assert status_of(B.apms_compress_gradient, ctx, g, 0, g + 16, p, sc) == B.APMS_EALIAS
    assert status_of(B.apms_apply_gradient, ctx, p, sc, g, e, m, 1e-4, 0.9, 1e-8) == B.APMS_ENODEV
    assert status_of(B.apms_apply_gradient, ctx, p, sc, g, e, m, 1e-4, 1.0, 1e-8) == B.APMS_EINVAL
    assert status_of(B.apms_apply_gradient, ctx, p, sc, g, e, e, 1e-4, 0.9, 1e-8) == B.APMS_EALIAS
    assert status_of(B.apms_apply_gradient, ctx, p, sc, g, e, m + 8, 1e-4, 0.9, 1e-8) == B.APMS_EALIGN


def test_gather_mode_knob(ctx):
    assert B.apms_get_plan(ctx)["gather_mode"] == B.APMS_GATHER_AUTO
    for mode in (B.APMS_GATHER_SPLIT, B.APMS_GATHER_FUSED, B.APMS_GATHER_AUTO):
        B.apms_set_gather_mode(ctx, mode)
        assert B.apms_get_plan(ctx)["gather_mode"] == mode
    assert status_of(B.apms_set_gather_mode, ctx, 3) == B.APMS_EINVAL
    assert status_of(B.apms_set_gather_mode, ctx, -1) == B.APMS_EINVAL
    assert status_of(B.apms_set_gather_mode, None, 0) == B.APMS_EINVAL


def test_topk_entry_points(ctx):
    a = [fake(i) for i in range(6)]
    m, g, e, idx, val, x = a
    assert status_of(B.apms_topk_compress, ctx, m, g, e, idx, val, 40, 0.9) == B.APMS_ENODEV
    assert status_of(B.apms_topk_compress, ctx, m, g, e, idx, val, 0, 0.9) == B.APMS_EINVAL
    assert status_of(B.apms_topk_compress, ctx, m, g, e, idx, val, 4097, 0.9) == B.APMS_EINVAL      # K > chunk
    assert status_of(B.apms_topk_compress, ctx, m, g, e, idx, val, 40, 1.0) == B.APMS_EINVAL
    assert status_of(B.apms_topk_compress, ctx, m, g, e, None, val, 40, 0.9) == B.APMS_EINVAL
    assert status_of(B.apms_topk_compress, ctx, m, g, e, idx, idx + 16, 40, 0.9) == B.APMS_EALIAS
    assert status_of(B.apms_topk_compress, ctx, m, g, e, idx + 4, val, 40, 0.9) == B.APMS_EALIGN
    assert status_of(B.apms_topk_server_reduce, ctx, idx, val, 40, e, m, g) == B.APMS_ENODEV
    assert status_of(B.apms_topk_server_reduce, ctx, idx, val, -1, e, m, g) == B.APMS_EINVAL
    assert status_of(B.apms_topk_apply, ctx, idx, val, 40, g, x, m, 1e-4, 1e-8) == B.APMS_ENODEV
    assert status_of(B.apms_topk_apply, ctx, idx, val, 40, g, x, x, 1e-4, 1e-8) == B.APMS_EALIAS
    assert status_of(B.apms_topk_apply, ctx, idx, val, 40, g, x, m, float("nan"), 1e-8) == B.APMS_EINVAL
    # the set-up call that sizes the selection's scratch
    assert status_of(B.apms_topk_reserve, ctx, 40) == B.APMS_ENODEV
    assert status_of(B.apms_topk_reserve, ctx, 0) == B.APMS_EINVAL
    assert status_of(B.apms_topk_reserve, ctx, 4097) == B.APMS_EINVAL
    assert status_of(B.apms_topk_reserve, None, 40) == B.APMS_EINVAL


def test_topk_list_positions_must_fit_32_bits():
    """K = chunk_elems = 2^31 passes the range check on K but not the kernels' 32-bit list positions."""
    big = 1 << 31
    c = B.apms_create(d=big, n=1, chunk_elems=big, device=B.APMS_DEVICE_NONE)
    try:
        far = [A + i * (1 << 40) for i in range(6)]
        m, g, e, idx, val, x = far
        assert status_of(B.apms_topk_reserve, c, big) == B.APMS_ESHAPE
        assert status_of(B.apms_topk_compress, c, m, g, e, idx, val, big, 0.9) == B.APMS_ESHAPE
        assert status_of(B.apms_topk_server_reduce, c, idx, val, big, e, m, g) == B.APMS_ESHAPE
        assert status_of(B.apms_topk_apply, c, idx, val, big, g, x, m, 1e-4, 1e-8) == B.APMS_ESHAPE
        assert status_of(B.apms_topk_compress, c, m, g, e, idx, val, big - 1, 0.9) == B.APMS_ENODEV
    finally:
        B.apms_destroy(c)


def test_static_server_reduce_validates_before_touching_the_device():
    """The context-free entry point checks geometry, its fixed scratch limit and the arrays on the host."""
    p, sc, e, sp, ssc = (fake(i) for i in range(5))
    call = B.apms_server_reduce_static
    assert status_of(call, 8192, 0, 4096, p, sc, e, sp, ssc) == B.APMS_EINVAL
    assert status_of(call, -32, 1, 32, p, sc, e, sp, ssc) == B.APMS_EINVAL
    assert status_of(call, 8192, 2, 48, p, sc, e, sp, ssc) == B.APMS_ESHAPE
    assert status_of(call, 8192, 2, 4096 * 3, p, sc, e, sp, ssc) == B.APMS_ESHAPE
    assert status_of(call, 8192, 2, 4096, None, sc, e, sp, ssc) == B.APMS_EINVAL
    assert status_of(call, 8192, 2, 4096, p + 4, sc, e, sp, ssc) == B.APMS_EALIGN
    assert status_of(call, 8192, 2, 4096, p, sc, e, e + 64, ssc) == B.APMS_EALIAS
    limit_blocks = B.APMS_STATIC_SCRATCH_BYTES // 8            # binary64 partials the fixed array holds
    assert status_of(call, (limit_blocks + 1) * 32, 1, 32, p, sc, e, sp, ssc) == B.APMS_ELIMIT
    assert status_of(call, 0, 3, 64, None, None, None, None, None) == B.APMS_OK
    header = open(os.path.join(ROOT, "include", "apms.h")).read()
    assert re.search(r"#define\s+APMS_STATIC_SCRATCH_BYTES\s+\(1 << 20\)", header) and B.APMS_STATIC_SCRATCH_BYTES == 1 << 20


def function_body(source, signature_start):
    """Text of the function whose definition starts with `signature_start`, braces matched."""
    at = source.index(signature_start)
    open_brace = source.index("{", source.index(")", at))
    depth, i = 0, open_brace
    while True:
        depth += {"{": 1, "}": -1}.get(source[i], 0)
        if depth == 0:
            return source[at:i + 1]
        i += 1


def test_static_server_reduce_holds_no_allocating_call():
    """The entry point for callers that cannot allocate, the helper that resolves its scratch array and the three
    launchers it queues contain no call that allocates or frees device or pinned memory (read off the source: on
    a GPU the device's free memory also moves with the runtime's own pools, so it is no measure of this)."""
    csrc = os.path.join(ROOT, "paper_2008_11343_amd", "csrc")
    api = open(os.path.join(csrc, "api.hip")).read()
    kernels = open(os.path.join(csrc, "kernels.hip")).read()
    bodies = [function_body(api, "int apms_server_reduce_static("), function_body(api, "hipError_t static_scratch("),
              function_body(kernels, "hipError_t launch_server_reduce("), function_body(kernels, "hipError_t launch_scales("),
              function_body(kernels, "hipError_t launch_finalize(")]
    for body in bodies:
        assert len(body) > 200
        body = re.sub(r"//[^\n]*", "", body)                  # comments may say "new"
        assert not re.search(r"hip\w*(Malloc|Free|Alloc|MemPool)\w*\s*\(|\bnew\b|\bmalloc\s*\(|std::vector", body), body[:80]
    entry = bodies[0]
    assert "static_scratch(device, &base)" in entry and "launch_server_reduce(" in entry
    assert "HIP_SYMBOL(scratch)" in bodies[1] and re.search(
        r"static __device__ __align__\(256\) unsigned char scratch\[APMS_STATIC_SCRATCH_BYTES\];", api)


def test_empty_problem_is_ok_without_a_device():
    c = B.apms_create(0, 4, 64, B.APMS_DEVICE_NONE)
    try:
        B.apms_compress(c, None, None, None, None, None, 0.9)
        B.apms_server_reduce(c, None, None, None, None, None)
        B.apms_apply(c, None, None, None, None, None, 1e-4, 1e-8)
        B.apms_warmup_step(c, None, None, None, None, 1e-3, 0.9, 0.999, 1e-8, 1)
        B.apms_freeze(c, None, None, None)
        plan = B.apms_get_plan(c)
        assert plan["chunks"] == 0 and plan["compress_grid"] == 0 and plan["apply_grid"] == 0
    finally:
        B.apms_destroy(c)


@pytest.mark.parametrize("wl", W.CONFIGS, ids=lambda w: w.name)
def test_launch_plan_of_every_config(wl):
    """Host launch planning: grids cover every tile exactly once and fit a 1-D launch."""
    c = B.apms_create(wl.d_pad, wl.n, wl.L, B.APMS_DEVICE_NONE)
    try:
        p = B.apms_get_plan(c)
        assert p["d"] == wl.d_pad and p["n"] == wl.n and p["chunk_elems"] == wl.L and p["chunks"] == wl.C
        for kind in ("compress", "server"):
            tile, tpb, bpc = p[kind + "_tile_elems"], p[kind + "_tiles_per_block"], p[kind + "_blocks_per_chunk"]
            assert tile % 1024 == 0
            tiles = -(-wl.L // tile)
            assert (bpc - 1) * tpb < tiles <= bpc * tpb
        assert p["compress_grid"] == wl.n * wl.C * p["compress_blocks_per_chunk"] < 2 ** 31
        assert p["server_grid"] == wl.C * p["server_blocks_per_chunk"]
        assert p["apply_grid"] == wl.n * wl.C * -(-wl.L // p["apply_tile_elems"]) < 2 ** 31
        assert p["scratch_bytes"] < 64 << 20
        B.apms_set_tiles_per_block(c, 3, 5)
        q = B.apms_get_plan(c)
        assert q["compress_tiles_per_block"] == 3 and q["server_tiles_per_block"] == 5
        assert q["compress_blocks_per_chunk"] == -(-(-(-wl.L // p["compress_tile_elems"])) // 3)
    finally:
        B.apms_destroy(c)


def test_maximum_sizes():
    """Sizes whose launch grids would not fit a 1-D launch are refused at creation; the largest that fit
    are planned without 32-bit overflow."""
    assert status_of(B.apms_create, 1 << 40, 64, 1 << 34, B.APMS_DEVICE_NONE) == B.APMS_ESHAPE
    assert status_of(B.apms_create, 1 << 42, 1, 1 << 42, B.APMS_DEVICE_NONE) == B.APMS_ESHAPE
    c = B.apms_create(1 << 36, 8, 1 << 33, B.APMS_DEVICE_NONE)       # 64 G elements, 8 workers, 8 chunks
    try:
        p = B.apms_get_plan(c)
        assert p["chunks"] == 8
        assert p["compress_grid"] == 8 * 8 * ((1 << 33) // p["compress_tile_elems"]) < 2 ** 31
        assert p["apply_grid"] == 8 * 8 * ((1 << 33) // p["apply_tile_elems"]) < 2 ** 31
        assert p["scratch_bytes"] > 0
    finally:
        B.apms_destroy(c)


def test_ragged_chunk_plan():
    c = B.apms_create(3 * (4096 * 2 + 160), 2, 4096 * 2 + 160, B.APMS_DEVICE_NONE)
    try:
        p = B.apms_get_plan(c)
        assert p["chunks"] == 3
        assert p["compress_blocks_per_chunk"] * p["compress_tiles_per_block"] * p["compress_tile_elems"] >= 4096 * 2 + 160
    finally:
        B.apms_destroy(c)


def test_workload_recipes():
    """The synthetic configurations: padded sizes, chunk lengths and the tensor-list bucket."""
    sizes = {w.name: (w.d_pad, w.n, w.L, w.C) for w in W.CONFIGS}
    assert sizes["tiny"] == (1 << 20, 4, 1 << 16, 16)
    assert sizes["bert-base-flat"] == (110_002_176, 8, 13_750_272, 8)
    assert sizes["bert-large-flat"] == (340_000_768, 16, 21_250_048, 16)
    assert sizes["worker-scaling"] == (110_100_480, 64, 1_720_320, 64)
    assert sizes["bert-large-tensor-list"] == (335_151_104, 16, 20_946_944, 16)
    t = W.bert_large_tensors()
    assert len(t) == 391 and sum(s for _, s, _ in t) == 335_141_888
    assert sum(1 for _, _, ln in t if ln) == 2 * (1 + 2 * 24)
    small = W.scaled(W.FULL_PIPELINE, 4096 * 16, n=2)
    g0, g1 = W.host_grad(small, 0), W.host_grad(small, 1)
    assert g0.shape == (2, small.d_pad) and not (g0 == g1).all()
    assert (W.host_grad(small, 0) == g0).all()                 # seeded: same key, same bits
    st = W.host_state(W.scaled(W.TINY, 5000, chunk=4096))
    assert st["x"].shape == (8192,) and (st["x"][5000:] == 0).all() and (st["v"][5000:] == 1).all()
    assert (st["m"][:, 5000:] == 0).all() and not st["werr"].any() and not st["serr"].any()


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is a one-GPU program: --gpus N with N > 1 exits with a message that says so."""
    import subprocess
    import sys
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert out.returncode != 0 and "ONE GPU" in out.stderr and out.stdout.strip() == ""
