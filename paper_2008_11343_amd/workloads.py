"""Seeded synthetic workloads for the APMSqueeze compression stage.

This module only produces INPUTS (shapes, sizes, random values).  It holds
none of the method's arithmetic and is the one piece of code that both the
HIP path's tests/benchmark and the CPU oracle's tests are fed from: whatever
is generated here is handed, as the same bits, to both sides.

The buffers stand in for the paper's BERT pre-training runs (Section 5.2:
BERT-Base, 110M parameters; BERT-Large, 340M parameters, L=24, H=1024); only
the parameter counts, the tensor shapes and the worker counts are borrowed,
no dataset and no trained weight.

Distributions (second argument of N(.,.) is the standard deviation):
  x ~ N(0, 0.02), m_i ~ N(0, 1e-3) per worker, g_i ~ N(0, 1e-2) fresh each
  step (or 1e-2 * Student-t with 3 degrees of freedom), v = exp(N(-12, 1)),
  worker and server errors zero.  Padding elements (index >= d) are ordinary
  elements of the flat buffer with g = m = x = 0 and v = 1.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

BASE_SEED = 200811343

_KIND = {"x": 1, "m": 2, "v": 3, "g": 4, "aux": 5}


def pad_to(d: int, multiple: int) -> int:
    return (d + multiple - 1) // multiple * multiple


def bert_large_tensors(layers: int = 24, hidden: int = 1024, ffn: int = 4096,
                       vocab: int = 30522, positions: int = 512,
                       token_types: int = 2) -> List[Tuple[str, int, bool]]:
    """(name, element count, is_layernorm) for every weight and bias of a BERT encoder
    with a pooler, in bucketing order (Section 5.2 gives L=24, H=1024 for BERT-Large)."""
    t: List[Tuple[str, int, bool]] = []
    t.append(("embeddings.word", vocab * hidden, False))
    t.append(("embeddings.position", positions * hidden, False))
    t.append(("embeddings.token_type", token_types * hidden, False))
    t.append(("embeddings.ln.weight", hidden, True))
    t.append(("embeddings.ln.bias", hidden, True))
    for l in range(layers):
        p = "layer%d." % l
        for proj in ("q", "k", "v", "o"):
            t.append((p + "attn.%s.weight" % proj, hidden * hidden, False))
            t.append((p + "attn.%s.bias" % proj, hidden, False))
        t.append((p + "attn.ln.weight", hidden, True))
        t.append((p + "attn.ln.bias", hidden, True))
        t.append((p + "ffn.in.weight", hidden * ffn, False))
        t.append((p + "ffn.in.bias", ffn, False))
        t.append((p + "ffn.out.weight", ffn * hidden, False))
        t.append((p + "ffn.out.bias", hidden, False))
        t.append((p + "out.ln.weight", hidden, True))
        t.append((p + "out.ln.bias", hidden, True))
    t.append(("pooler.weight", hidden * hidden, False))
    t.append(("pooler.bias", hidden, False))
    return t


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration: flat fp32 buffer of d parameters, n simulated workers."""
    name: str
    index: int                      # position in the benchmark's config list (part of the seed key)
    d: int                          # unpadded parameter count
    n: int                          # simulated workers
    chunk: Optional[int] = None     # chunk length L; None -> d_pad / n (one chunk per worker, as in the paper)
    steps: int = 10                 # compressed steps
    warmup_steps: int = 0           # Adam warm-up steps before the freeze
    grad: str = "normal"            # "normal" | "student_t3"
    beta: float = 0.9
    beta2: float = 0.999
    lr: float = 1e-4
    eps: float = 1e-8
    tensors: Optional[tuple] = field(default=None, compare=False)   # (name, size, is_layernorm) list

    @property
    def d_pad(self) -> int:
        if self.chunk is not None:
            return pad_to(self.d, self.chunk)
        return pad_to(self.d, self.n * 4096)

    @property
    def L(self) -> int:
        return self.chunk if self.chunk is not None else self.d_pad // self.n

    @property
    def C(self) -> int:
        return self.d_pad // self.L

    def layernorm_segments(self) -> List[Tuple[int, int]]:
        """(offset, size) of every LayerNorm tensor inside the flat buffer."""
        segs, off = [], 0
        for _, size, is_ln in (self.tensors or ()):
            if is_ln:
                segs.append((off, size))
            off += size
        return segs


def _bert_large_count() -> int:
    return sum(s for _, s, _ in bert_large_tensors())


TINY = Workload("tiny", 0, d=1 << 20, n=4, chunk=1 << 16, steps=10)
BERT_BASE = Workload("bert-base-flat", 1, d=110_000_000, n=8, steps=100)
BERT_LARGE = Workload("bert-large-flat", 2, d=340_000_000, n=16, steps=50)
WORKER_SCALING = Workload("worker-scaling", 3, d=110_000_000, n=64, steps=20, grad="student_t3")
FULL_PIPELINE = Workload("bert-large-tensor-list", 4, d=_bert_large_count(), n=16, steps=80,
                         warmup_steps=20, tensors=tuple(bert_large_tensors()))
CONFIGS = [TINY, BERT_BASE, BERT_LARGE, WORKER_SCALING, FULL_PIPELINE]


def scaled(wl: Workload, d: int, name: Optional[str] = None, **kw) -> Workload:
    """Same recipe at another size (for parity cases the oracle finishes in seconds)."""
    args = dict(name=name or "%s@d=%d" % (wl.name, d), index=wl.index, d=d, n=wl.n, chunk=wl.chunk,
                steps=wl.steps, warmup_steps=wl.warmup_steps, grad=wl.grad, beta=wl.beta, beta2=wl.beta2,
                lr=wl.lr, eps=wl.eps, tensors=None)
    args.update(kw)
    return Workload(**args)


def _seed_seq(wl: Workload, kind: str, worker: int, step: int, seed: int) -> np.random.SeedSequence:
    return np.random.SeedSequence([seed, wl.index, _KIND[kind], worker + 1, step + 1])


def _host_rng(wl, kind, worker=0, step=0, seed=BASE_SEED) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(_seed_seq(wl, kind, worker, step, seed)))


def _device_seed(wl, kind, worker=0, step=0, seed=BASE_SEED) -> int:
    return int(_seed_seq(wl, kind, worker, step, seed).generate_state(1, np.uint64)[0] >> np.uint64(1))


# ----------------------------------------------------------------------------
# Host (numpy) generation: small cases, generated once and uploaded.
# ----------------------------------------------------------------------------

def host_state(wl: Workload, seed: int = BASE_SEED, warm_start: bool = False) -> dict:
    """Initial state as numpy arrays: x [d_pad], m [n][d_pad], v [d_pad], werr [n][d_pad], serr [d_pad].

    warm_start=True gives the state BEFORE an Adam warm-up instead (m = v = 0, m of shape [d_pad])."""
    d, dp, n = wl.d, wl.d_pad, wl.n
    f = np.float32
    x = np.zeros(dp, f)
    x[:d] = _host_rng(wl, "x", seed=seed).normal(0.0, 0.02, d).astype(f)
    if warm_start:
        return dict(x=x, m=np.zeros(dp, f), v=np.zeros(dp, f))
    m = np.zeros((n, dp), f)
    for i in range(n):
        m[i, :d] = _host_rng(wl, "m", i, seed=seed).normal(0.0, 1e-3, d).astype(f)
    v = np.ones(dp, f)
    v[:d] = np.exp(_host_rng(wl, "v", seed=seed).normal(-12.0, 1.0, d)).astype(f)
    return dict(x=x, m=m, v=v, werr=np.zeros((n, dp), f), serr=np.zeros(dp, f))


def host_grad(wl: Workload, step: int, seed: int = BASE_SEED) -> np.ndarray:
    """Per-worker gradients [n][d_pad] of one step (padding elements zero)."""
    d, dp, n = wl.d, wl.d_pad, wl.n
    g = np.zeros((n, dp), np.float32)
    for i in range(n):
        rng = _host_rng(wl, "g", i, step, seed)
        if wl.grad == "normal":
            vals = rng.normal(0.0, 1e-2, d)
        elif wl.grad == "student_t3":
            vals = 1e-2 * rng.standard_t(3.0, d)
        else:
            raise ValueError(wl.grad)
        g[i, :d] = vals.astype(np.float32)
    for off, size in wl.layernorm_segments():
        g[:, off:off + size] *= np.float32(0.1)
    return g


# ----------------------------------------------------------------------------
# Device (torch) generation: large cases, generated in HBM; the chunks an
# oracle check needs are copied back to the host, so both sides see one copy
# of the bits.  torch is imported lazily so host-only users do not need it.
# ----------------------------------------------------------------------------

def _gen(device, seed_int):
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed_int)
    return gen


def device_state(wl: Workload, device="cuda", seed: int = BASE_SEED, warm_start: bool = False) -> dict:
    """Initial state as torch tensors on `device` (same layout as host_state, different random bits)."""
    import torch
    dp, n = wl.d_pad, wl.n
    kw = dict(dtype=torch.float32, device=device)
    if warm_start:
        st = dict(x=torch.empty(dp, **kw), m=torch.empty(dp, **kw), v=torch.empty(dp, **kw))
    else:
        st = dict(x=torch.empty(dp, **kw), m=torch.empty(n, dp, **kw), v=torch.empty(dp, **kw),
                  werr=torch.empty(n, dp, **kw), serr=torch.empty(dp, **kw))
    return device_state_(wl, st, seed=seed, warm_start=warm_start)


def device_state_(wl: Workload, st: dict, seed: int = BASE_SEED, warm_start: bool = False) -> dict:
    """Fill the tensors of `st` (x, m, v and, unless warm_start, werr, serr; already on the GPU, shapes as
    device_state returns them) with the initial state, in place."""
    import torch
    d, dp, n = wl.d, wl.d_pad, wl.n
    x, m, v = st["x"], st["m"], st["v"]
    device = x.device
    x.zero_()
    x[:d].normal_(0.0, 0.02, generator=_gen(device, _device_seed(wl, "x", seed=seed)))
    if warm_start:
        m.zero_()
        v.zero_()
        return st
    assert m.shape == (n, dp)
    m.zero_()
    for i in range(n):
        m[i, :d].normal_(0.0, 1e-3, generator=_gen(device, _device_seed(wl, "m", i, seed=seed)))
    v.fill_(1.0)
    v[:d].normal_(-12.0, 1.0, generator=_gen(device, _device_seed(wl, "v", seed=seed))).exp_()
    st["werr"].zero_()
    st["serr"].zero_()
    return st


def device_grad_(wl: Workload, step: int, out, seed: int = BASE_SEED):
    """Fill `out` ([n][d_pad] float32 tensor on the GPU) with the gradients of one step, in place."""
    import torch
    d, dp, n = wl.d, wl.d_pad, wl.n
    assert out.shape == (n, dp) and out.dtype == torch.float32
    dev = out.device
    for i in range(n):
        gen = _gen(dev, _device_seed(wl, "g", i, step, seed))
        row = out[i, :d]
        if wl.grad == "normal":
            row.normal_(0.0, 1e-2, generator=gen)
        elif wl.grad == "student_t3":
            row.normal_(0.0, 1.0, generator=gen)
            chi = torch.zeros(d, dtype=torch.float32, device=dev)
            tmp = torch.empty(d, dtype=torch.float32, device=dev)
            for _ in range(3):
                tmp.normal_(0.0, 1.0, generator=gen)
                chi.addcmul_(tmp, tmp)
            chi.div_(3.0).sqrt_()
            row.div_(chi).mul_(1e-2)
            del chi, tmp
        else:
            raise ValueError(wl.grad)
    if dp > d:
        out[:, d:].zero_()
    for off, size in wl.layernorm_segments():
        out[:, off:off + size].mul_(0.1)
    return out


# ----------------------------------------------------------------------------
# 16-bit gradient inputs: the same draws, rounded to binary16 / bfloat16 (round to nearest even).
# Returned as raw uint16 bit patterns so that both sides widen them by their own means.
# ----------------------------------------------------------------------------

def host_grad_g16(wl: Workload, step: int, fmt: str, seed: int = BASE_SEED) -> np.ndarray:
    """Per-worker gradients [n][d_pad] of one step as 'f16' or 'bf16' bit patterns (uint16)."""
    g = host_grad(wl, step, seed)
    if fmt == "f16":
        return g.astype(np.float16).view(np.uint16)
    if fmt == "bf16":
        import torch
        return torch.from_numpy(g).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    raise ValueError(fmt)


def g16_bits_to_tensor(bits: np.ndarray, fmt: str, device="cuda"):
    """uint16 bit patterns -> torch tensor of dtype float16 / bfloat16 on `device` (same bits)."""
    import torch
    t = torch.from_numpy(bits.view(np.int16)).to(device)
    return t.view(torch.float16 if fmt == "f16" else torch.bfloat16)
