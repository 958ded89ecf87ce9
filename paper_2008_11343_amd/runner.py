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

    def __init__(self, d, n, L, device="cuda:0", deferred=False, state=None):
        """deferred: False (everything eager), True (errors and gather deferred) or an int of APMS_DEFER_* flags."""
        self.d, self.n, self.L = d, n, L
        self.C = d // L if L else 0
        self.device = torch.device(device)
        idx = self.device.index if self.device.index is not None else torch.cuda.current_device()
        self.ctx = B.apms_create(d, n, L, idx)
        self.deferral = (B.APMS_DEFER_ERRORS | B.APMS_DEFER_GATHER) if deferred is True else int(deferred)
        if self.deferral:
            B.apms_set_deferral(self.ctx, self.deferral)
        f = dict(dtype=torch.float32, device=self.device)
        i = dict(dtype=torch.int32, device=self.device)
        if state is not None:
            self.x = state["x"].to(**f).contiguous()
            self.m = state["m"].to(**f).reshape(n, d).contiguous()
            self.v = state["v"].to(**f).contiguous()
            self.werr = state["werr"].to(**f).reshape(n, d).contiguous()
            self.serr = state["serr"].to(**f).contiguous()
        else:
            self.x = torch.zeros(d, **f)
            self.m = torch.zeros(n, d, **f)
            self.v = torch.ones(d, **f)
            self.werr = torch.zeros(n, d, **f)
            self.serr = torch.zeros(d, **f)
        self.packed = torch.zeros(n, d // 32, **i)
        self.scales = torch.zeros(n, self.C, **f)
        self.spacked = torch.zeros(d // 32, **i)
        self.sscales = torch.zeros(self.C, **f)

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
