"""Device-side plumbing around the C ABI: buffers for one workload and the call sequence of a step.

Holds no arithmetic: every value is produced by libapms kernels through `binding`.  Used by the
tests, the smoke check and the benchmark so that all three drive the library the same way.
"""
from __future__ import annotations

import torch

from . import binding as B


class DeviceRun:
    """State of the compression stage for n simulated workers, resident in HBM.

    x [d], m [n][d], v [d], werr [n][d], serr [d] fp32; packed [n][d/32], spacked [d/32] uint32 (stored
    as int32 tensors, same bits); scales [n][C], sscales [C] fp32; g [n][d] is the caller's input.
    """

    def __init__(self, d, n, L, device="cuda:0", deferred=False, state=None, place=False, grad_dtype=None):
        """deferred: False (everything eager), True (errors and gather deferred) or an int of APMS_DEFER_* flags.
        state: dict of tensors (x, m, v, werr, serr) copied into the run's own buffers.
        grad_dtype: also allocate the gradient input `self.g` [n][d] of that dtype.
        place: choose where the worker error and the gradient lie in HBM by timing (see `_allocate`)."""
        self.d, self.n, self.L = d, n, L
        self.C = d // L if L else 0
        self.device = torch.device(device)
        idx = self.device.index if self.device.index is not None else torch.cuda.current_device()
        self.ctx = B.apms_create(d, n, L, idx)
        self.deferral = (B.APMS_DEFER_ERRORS | B.APMS_DEFER_GATHER) if deferred is True else int(deferred)
        if self.deferral:
            B.apms_set_deferral(self.ctx, self.deferral)
        self.placement = self._allocate(place, grad_dtype)
        if state is not None:
            self.x.copy_(state["x"].reshape(d))
            self.m.copy_(state["m"].reshape(n, d))
            self.v.copy_(state["v"].reshape(d))
            self.werr.copy_(state["werr"].reshape(n, d))
            self.serr.copy_(state["serr"].reshape(d))
        else:
            self.x.zero_()
            self.m.zero_()
            self.v.fill_(1.0)
            self.werr.zero_()
            self.serr.zero_()
        for t in (self.packed, self.scales, self.spacked, self.sscales):
            t.zero_()

    # MI355X: its 288 GiB of HBM behave as three regions of 96 GiB.  The fused form of the gather-carrying
    # worker kernel writes two [n][d] streams (momentum, error) and reads two (error, gradient); measured on
    # the chip with BERT-Large-sized buffers, it runs 10-15 % faster when the momentum lies in a different
    # region than the error and the gradient than with all three in one (where inside a region a buffer
    # lies, and address skews, make no difference; buffers of 1 GB do not show the effect).  The library's
    # default (APMS_GATHER_AUTO) copes with any placement by timing its split form against the fused one;
    # `place` goes one step further and looks for a placement on which the fused form wins.  Where the
    # driver puts an allocation cannot be asked or steered from here, so it finds one by trying.
    PLACE_MIN_BYTES = 4 << 30          # smaller [n][d] buffers are not worth placing

    def _allocate(self, place, grad_dtype):
        """Allocates every buffer of the run.  With `place` (float32 gradients only) further [n][d]
        buffers are allocated one after the other, the fused worker kernel is timed with each adjacent pair
        of them as (worker error, gradient), the fastest pair is kept and the rest freed.  Returns a dict
        that describes what was done (None if nothing was placed)."""
        d, n, dev = self.d, self.n, self.device
        f = dict(dtype=torch.float32, device=dev)
        i = dict(dtype=torch.int32, device=dev)
        self.m = torch.empty(n, d, **f)
        self.werr = torch.empty(n, d, **f)
        self.g = torch.empty(n, d, dtype=grad_dtype, device=dev) if grad_dtype is not None else None
        self.x = torch.empty(d, **f)
        self.v = torch.empty(d, **f)
        self.serr = torch.empty(d, **f)
        self.packed = torch.empty(n, d // 32, **i)
        self.scales = torch.empty(n, self.C, **f)
        self.spacked = torch.empty(d // 32, **i)
        self.sscales = torch.empty(self.C, **f)
        big = n * d * 4
        if (not place or big < self.PLACE_MIN_BYTES or grad_dtype != torch.float32
                or not self.deferral & B.APMS_DEFER_GATHER):
            return None
        torch.cuda.empty_cache()
        free, _ = torch.cuda.mem_get_info(dev)
        extra = min(8, int((free - (16 << 30)) // big))
        if extra < 1:
            return None
        cands = [self.werr, self.g] + [torch.empty(n, d, **f) for _ in range(extra)]
        probe = B.apms_create(d, n, self.L, dev.index or 0)

        def worker_ms(werr, g):
            best = None
            for step in range(3):                             # the 1st call has no gather to carry out
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                B.apms_compress(probe, self.m, g, werr, self.packed, self.scales, 0.9)
                b.record()
                B.apms_server_reduce(probe, self.packed, self.scales, self.serr, self.spacked, self.sscales)
                B.apms_apply(probe, self.spacked, self.sscales, self.v, self.x, self.m, 1e-4, 1e-8)
                b.synchronize()
                if step:
                    ms = a.elapsed_time(b)
                    best = ms if best is None else min(best, ms)
            B.apms_finalize(probe, werr, self.serr, self.m)
            return best

        try:
            B.apms_set_deferral(probe, self.deferral)
            B.apms_set_gather_mode(probe, B.APMS_GATHER_FUSED)     # the form whose speed depends on the placement
            self.v.fill_(1.0)
            for t in [self.m, self.x, self.serr] + cands:
                t.zero_()
            times = [worker_ms(cands[k], cands[k + 1]) for k in range(len(cands) - 1)]
            k = min(range(len(times)), key=times.__getitem__)
            self.werr, self.g = cands[k], cands[k + 1]
            del cands
            torch.cuda.empty_cache()
            torch.cuda.synchronize()
        finally:
            B.apms_destroy(probe)
        return {"policy": "worker error and gradient = the adjacent pair of %d successively allocated buffers that "
                          "the fused worker kernel runs fastest on (HBM regions); which form of the kernel then "
                          "runs is the library's own choice (APMS_GATHER_AUTO)" % (len(times) + 1),
                "chosen_pair": k, "fused_worker_kernel_ms_by_pair": [round(t, 3) for t in times]}

    def close(self):
        if self.ctx is not None:
            B.apms_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # the three calls of one compressed step (Algorithm 1 lines 6-11)
    @staticmethod
    def _grad_format(g):
        """0 for float32 gradients, APMS_GRAD_F16 / APMS_GRAD_BF16 for torch.float16 / torch.bfloat16."""
        return {torch.float32: 0, torch.float16: B.APMS_GRAD_F16, torch.bfloat16: B.APMS_GRAD_BF16}[g.dtype]

    def compress(self, g, beta, stream=None):
        fmt = self._grad_format(g)
        if fmt:
            B.apms_compress_g16(self.ctx, self.m, g, fmt, self.werr, self.packed, self.scales, beta, stream)
        else:
            B.apms_compress(self.ctx, self.m, g, self.werr, self.packed, self.scales, beta, stream)

    def server_reduce(self, stream=None):
        B.apms_server_reduce(self.ctx, self.packed, self.scales, self.serr, self.spacked, self.sscales, stream)

    def apply(self, lr, eps, stream=None):
        B.apms_apply(self.ctx, self.spacked, self.sscales, self.v, self.x, self.m, lr, eps, stream)

    def step(self, g, beta, lr, eps, stream=None):
        self.compress(g, beta, stream)
        self.server_reduce(stream)
        self.apply(lr, eps, stream)

    def step_topk(self, g, K, beta, lr, eps, stream=None):
        """One compressed step with the top-k compressor (Section 5.1): K kept elements per chunk."""
        if getattr(self, "idx", None) is None or self.idx.shape[-1] != K:
            i = dict(dtype=torch.int32, device=self.device)
            f = dict(dtype=torch.float32, device=self.device)
            self.idx, self.val = torch.zeros(self.n, self.C, K, **i), torch.zeros(self.n, self.C, K, **f)
            self.sidx, self.sval = torch.zeros(self.C, K, **i), torch.zeros(self.C, K, **f)
            B.apms_topk_reserve(self.ctx, K)        # set-up: sizes the selection's scratch (no-op if it suffices)
        B.apms_topk_compress(self.ctx, self.m, g, self.werr, self.idx, self.val, K, beta, stream)
        B.apms_topk_server_reduce(self.ctx, self.idx, self.val, K, self.serr, self.sidx, self.sval, stream)
        B.apms_topk_apply(self.ctx, self.sidx, self.sval, K, self.v, self.x, self.m, lr, eps, stream)

    def step_gradient(self, g, beta, lr, eps, stream=None):
        """One step of the APGSqueeze variant (Section 5.3): the gradient is what gets compressed."""
        B.apms_compress_gradient(self.ctx, g, self._grad_format(g), self.werr, self.packed, self.scales, stream)
        self.server_reduce(stream)
        B.apms_apply_gradient(self.ctx, self.spacked, self.sscales, self.v, self.x, self.m, lr, beta, eps, stream)

    def finalize(self, stream=None):
        """Bring every pending buffer (both errors, the momentum) to its final contents."""
        B.apms_finalize(self.ctx, self.werr, self.serr, self.m, stream)

    # warm-up (Algorithm 1 line 2) works on worker 0's momentum slice
    def warmup_step(self, g, lr, beta1, beta2, eps, t, stream=None):
        fmt = self._grad_format(g)
        if fmt:
            B.apms_warmup_step_g16(self.ctx, self.x, self.m[0], self.v, g, fmt, lr, beta1, beta2, eps, t, stream)
        else:
            B.apms_warmup_step(self.ctx, self.x, self.m[0], self.v, g, lr, beta1, beta2, eps, t, stream)

    def freeze(self, stream=None):
        B.apms_freeze(self.ctx, self.m, self.werr, self.serr, stream)


def from_host_state(wl, st, device="cuda:0", deferred=False) -> DeviceRun:
    """DeviceRun for workload `wl` initialised from numpy arrays (workloads.host_state)."""
    state = {k: torch.from_numpy(v) for k, v in st.items() if k in ("x", "m", "v", "werr", "serr")}
    return DeviceRun(wl.d_pad, wl.n, wl.L, device=device, deferred=deferred, state=state)
