"""apms_server_reduce_static, the server step for callers that cannot allocate device memory: its kernels' scratch
(the binary64 norm partials) lives in a fixed array inside the library's device image.  Checked through the C ABI
against apms_server_reduce on an eager context (same kernels, same tiling: every output bit-equal) and against the
CPU oracle, on two calls in a row, the second with a smaller problem, so that whatever the first call left in the
shared array must not matter.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2008_11343_amd import binding as B

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
RTOL, ATOL = 1e-5, 1e-7


def problem(d, n, L, seed):
    """Worker messages (sign words + scales) and a non-zero server error for one server step."""
    C = d // L
    gen = torch.Generator(device=DEV).manual_seed(seed)
    f = dict(dtype=torch.float32, device=DEV)
    m = torch.empty(n, d, **f).normal_(0.0, 1e-3, generator=gen)
    g = torch.empty(n, d, **f).normal_(0.0, 1e-2, generator=gen)
    werr = torch.empty(n, d, **f).normal_(0.0, 2e-3, generator=gen)
    serr = torch.empty(d, **f).normal_(0.0, 1e-3, generator=gen)
    packed = torch.zeros(n, d // 32, dtype=torch.int32, device=DEV)
    scales = torch.zeros(n, C, **f)
    ctx = B.apms_create(d, n, L, 0)
    try:
        B.apms_compress(ctx, m, g, werr, packed, scales, 0.9)
        torch.cuda.synchronize()
    finally:
        B.apms_destroy(ctx)
    return packed, scales, serr


def outputs(d, L):
    return (torch.zeros(d // 32, dtype=torch.int32, device=DEV),
            torch.zeros(d // L, dtype=torch.float32, device=DEV))


def check_one(d, n, L, seed):
    print("[no-alloc] d=%d n=%d chunk=%d seed=%d" % (d, n, L, seed), flush=True)
    C = d // L
    packed, scales, serr0 = problem(d, n, L, seed)
    # existing entry point, eager context
    serr_ctx = serr0.clone()
    spacked_ctx, sscales_ctx = outputs(d, L)
    ctx = B.apms_create(d, n, L, 0)
    try:
        B.apms_server_reduce(ctx, packed, scales, serr_ctx, spacked_ctx, sscales_ctx)
        torch.cuda.synchronize()
    finally:
        B.apms_destroy(ctx)
    # the allocation-free one: every tensor exists before the call; the call itself must not allocate
    serr_st = serr0.clone()
    spacked_st, sscales_st = outputs(d, L)
    # (that the entry point's code holds no allocating call is checked on its source, in test_boundary_host.py: the
    # device's free memory is no measure of it, the runtime's own pools move it by megabytes when memory is short)
    # the count of allocations ever made: a tensor of an earlier case released meanwhile does not move it
    allocations = lambda: torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    torch.cuda.synchronize()
    before = allocations()
    B.apms_server_reduce_static(d, n, L, packed, scales, serr_st, spacked_st, sscales_st)
    torch.cuda.synchronize()
    assert allocations() == before, "the call went through torch's allocator"
    assert torch.equal(spacked_st, spacked_ctx), "server sign words differ from apms_server_reduce"
    assert torch.equal(sscales_st, sscales_ctx), "server scales differ from apms_server_reduce"
    assert torch.equal(serr_st, serr_ctx), "server error differs from apms_server_reduce"
    # and the oracle, to the parity bar
    o_serr = serr0.cpu().numpy().copy()
    o_spacked, o_sscales = np.zeros(d // 32, np.uint32), np.zeros(C, np.float32)
    oracle.server_reduce(d, n, L, packed.cpu().numpy().view(np.uint32), scales.cpu().numpy(), o_serr, o_spacked,
                         o_sscales)
    assert np.array_equal(spacked_st.cpu().numpy().view(np.uint32), o_spacked)
    np.testing.assert_allclose(sscales_st.cpu().numpy(), o_sscales, rtol=RTOL, atol=ATOL)
    np.testing.assert_allclose(serr_st.cpu().numpy(), o_serr, rtol=RTOL, atol=ATOL)


def test_static_server_reduce_two_calls_second_smaller():
    check_one(d=3 * (4096 * 9 + 160), n=5, L=4096 * 9 + 160, seed=31)      # several tiles, ragged tail, odd n
    check_one(d=2 * 4096, n=3, L=4096, seed=32)                            # smaller: reuses the array's low end


def test_static_server_reduce_limits_and_validation():
    z = lambda *s, dt=torch.float32: torch.zeros(*s, dtype=dt, device=DEV)
    d, n, L = 8192, 2, 4096
    packed, scales, serr = z(n, d // 32, dt=torch.int32), z(n, 2), z(d)
    spacked, sscales = outputs(d, L)

    def status(*args):
        try:
            B.apms_server_reduce_static(*args)
        except B.ApmsError as e:
            return e.status
        return B.APMS_OK

    assert status(d, n, L, packed, scales, serr, spacked, sscales) == B.APMS_OK
    assert status(d, 0, L, packed, scales, serr, spacked, sscales) == B.APMS_EINVAL
    assert status(d, n, 48, packed, scales, serr, spacked, sscales) == B.APMS_ESHAPE
    assert status(d, n, L, None, scales, serr, spacked, sscales) == B.APMS_EINVAL
    assert status(d, n, L, packed, scales, serr, spacked, serr) == B.APMS_EALIAS
    assert status(d, n, L, packed, scales, serr.data_ptr() + 4, spacked, sscales) == B.APMS_EALIGN
    # more chunk-blocks than the fixed array holds: refused on the host, nothing is dereferenced
    huge_chunks = (B.APMS_STATIC_SCRATCH_BYTES // 8 + 1)
    assert status(huge_chunks * 32, 1, 32, packed, scales, serr, spacked, sscales) == B.APMS_ELIMIT
    assert status(0, 1, 32, None, None, None, None, None) == B.APMS_OK
    torch.cuda.synchronize()
