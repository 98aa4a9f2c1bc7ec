"""Seeded synthetic inputs for the linear-recurrence kernels (shared by tests, smoke and bench).

This module only draws random tensors; it contains none of the recurrence's arithmetic and imports
neither the oracle nor the GPU library, so both sides can consume the very same fp32 bits.

The five workloads mirror the shapes the paper measures on (arXiv 1709.04057: Table 1's sequence
lengths up to 65 536, Table 2's 256 hidden units, Section 4.2's one-million-step sequences of width
64-128, and the gated form h_t = a_t*h_{t-1} + (1-a_t)*x_t of Section 3.1); the paper's own inputs
were a random stream fed through TensorFlow models, so synthetic lambda/x of the same shape stand in.

All tensors are fp32, contiguous, time-major ``[T, B, n]`` (``h0`` is ``[B, n]``).  Seeds follow
``17090405 + 1000*cfg + k`` with k = 0 (lambda), 1 (x or z), 2 (h0), 3 (grad_h), 4 (mixture class).
"""
from __future__ import annotations

import torch

SEED_BASE = 17090405

#: cfg -> full-size shape and which passes are exercised
CONFIGS = {
    1: dict(T=1024, B=2, n=32, backward=False,
            note="forward only; lambda=sigmoid(N(0,1)), x~N(0,1), h0=0"),
    2: dict(T=65536, B=4, n=256, backward=True,
            note="lambda=sigmoid(N(2,1)), x~N(0,1), h0~N(0,1), grad_h~N(0,1)"),
    3: dict(T=1048576, B=1, n=128, backward=True,
            note="lambda=1-10^U(-4,-1), x~N(0,sd 0.1), h0=0, grad_h nonzero only in the last row"),
    4: dict(T=4096, B=16, n=1024, backward=True,
            note="lambda=sigmoid(N(0,1)), x=(1-lambda)*z, z~N(0,1), h0=0, grad_h~N(0,1)"),
    5: dict(T=262144, B=8, n=512, backward=True,
            note="lambda: 50% sigmoid(N(0,1)), 25% exactly 0, 25% fp32(1-1e-6); x,h0,grad_h~N(0,1)"),
}


def _gen(device, cfg, k):
    g = torch.Generator(device=device)
    g.manual_seed(SEED_BASE + 1000 * int(cfg) + k)
    return g


def _randn(shape, device, cfg, k, mean=0.0, std=1.0):
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(mean, std, generator=_gen(device, cfg, k))
    return t


def _rand(shape, device, cfg, k):
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.uniform_(0.0, 1.0, generator=_gen(device, cfg, k))
    return t


def make_inputs(cfg, T=None, B=None, n=None, device="cpu", per_channel=False):
    """Draw the inputs of workload ``cfg`` (1..5), optionally at a reduced shape.

    ``per_channel=True`` gives the accuracy-stress variants of workloads 3 and 5 in which lambda (or
    its mixture class) is drawn once per column and held along T, i.e. true long memory.

    Returns a dict with ``lam, x, h0, grad_h`` (``h0``/``grad_h`` may be None) and ``T, B, n``.
    """
    cfg = int(cfg)
    spec = CONFIGS[cfg]
    T = spec["T"] if T is None else int(T)
    B = spec["B"] if B is None else int(B)
    n = spec["n"] if n is None else int(n)
    dev = torch.device(device)
    shape = (T, B, n)
    lam_shape = (1, B, n) if per_channel else shape
    h0 = None
    grad_h = None

    if cfg == 1:
        lam = torch.sigmoid(_randn(lam_shape, dev, cfg, 0))
        x = _randn(shape, dev, cfg, 1)
    elif cfg == 2:
        lam = torch.sigmoid(_randn(lam_shape, dev, cfg, 0, mean=2.0))
        x = _randn(shape, dev, cfg, 1)
        h0 = _randn((B, n), dev, cfg, 2)
        grad_h = _randn(shape, dev, cfg, 3)
    elif cfg == 3:
        u = _rand(lam_shape, dev, cfg, 0)
        lam = 1.0 - torch.pow(10.0, -4.0 + 3.0 * u)
        x = _randn(shape, dev, cfg, 1, std=0.1)
        grad_h = torch.zeros(shape, dtype=torch.float32, device=dev)
        if T > 0:
            grad_h[T - 1] = _randn((B, n), dev, cfg, 3)
    elif cfg == 4:
        lam = torch.sigmoid(_randn(lam_shape, dev, cfg, 0))
        z = _randn(shape, dev, cfg, 1)
        x = (1.0 - lam) * z
        del z
        grad_h = _randn(shape, dev, cfg, 3)
    elif cfg == 5:
        lam = torch.sigmoid(_randn(lam_shape, dev, cfg, 0))
        cls = _rand(lam_shape, dev, cfg, 4)
        near_one = torch.tensor(1.0 - 1e-6, dtype=torch.float32).item()  # fp32-rounded 1-1e-6
        lam = torch.where(cls < 0.5, lam, torch.where(cls < 0.75, torch.zeros_like(lam),
                                                      torch.full_like(lam, near_one)))
        del cls
        x = _randn(shape, dev, cfg, 1)
        h0 = _randn((B, n), dev, cfg, 2)
        grad_h = _randn(shape, dev, cfg, 3)
    else:
        raise KeyError(cfg)

    if per_channel:
        lam = lam.expand(shape)
    lam = lam.contiguous()
    x = x.contiguous()
    return dict(cfg=cfg, T=T, B=B, n=n, lam=lam, x=x, h0=h0, grad_h=grad_h, backward=spec["backward"])


def make_generic(T, B, n, seed, device="cpu", lam_kind="sigmoid", with_h0=True):
    """Small general-purpose cases for edge-shape tests: lambda in (0,1), [-1,1] or with exact 0/1."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(SEED_BASE + 7 * int(seed) + 1)
    shape = (T, B, n)

    def randn(s):
        t = torch.empty(s, dtype=torch.float32, device=dev)
        return t.normal_(0.0, 1.0, generator=g)

    def rand(s):
        t = torch.empty(s, dtype=torch.float32, device=dev)
        return t.uniform_(0.0, 1.0, generator=g)

    if lam_kind == "sigmoid":
        lam = torch.sigmoid(randn(shape))
    elif lam_kind == "signed":
        lam = 2.0 * rand(shape) - 1.0
    elif lam_kind == "mixed":
        lam = torch.sigmoid(randn(shape))
        cls = rand(shape)
        lam = torch.where(cls < 0.2, torch.zeros_like(lam), lam)
        lam = torch.where(cls > 0.8, torch.ones_like(lam), lam)
        lam = torch.where((cls > 0.45) & (cls < 0.55), -lam, lam)
    else:
        raise KeyError(lam_kind)
    x = randn(shape)
    h0 = randn((B, n)) if with_h0 else None
    grad_h = randn(shape)
    return dict(T=T, B=B, n=n, lam=lam.contiguous(), x=x, h0=h0, grad_h=grad_h, backward=True)


#: gated-layer workloads (Section 3.1): pre-activations in, as a matrix product would leave them
GATED = {
    "g4": dict(T=4096, B=16, n=1024, gate_mean=0.0, gate_std=1.0,
               note="workload 4's shape and gate distribution, activations applied in the kernel"),
    "g2": dict(T=65536, B=4, n=256, gate_mean=2.0, gate_std=1.0, note="workload 2's shape, gates sigmoid(N(2,1))"),
    "g3": dict(T=1048576, B=1, n=128, gate_mean=7.0, gate_std=2.0,
               note="one million steps, gates mostly within 1e-2..1e-5 of one (long memory)"),
    "g5": dict(T=262144, B=8, n=512, gate_mean=1.0, gate_std=1.5,
               note="workload 5's shape (1.07e9 elements): the layer at the size the headline is measured on"),
}


def make_gated(T, B, n, seed, device="cpu", gate_mean=0.0, gate_std=1.0, with_h0=True, per_channel=False):
    """Pre-activations ``g_pre ~ N(gate_mean, gate_std)``, ``i_pre ~ N(0,1)``, ``h0, grad_h ~ N(0,1)``.

    ``per_channel=True`` holds g_pre constant along T in every column (a fixed decay rate: errors in
    the gate cannot average out)."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(SEED_BASE + 7 * int(seed) + 3)
    shape = (T, B, n)

    def randn(s, mean=0.0, std=1.0):
        t = torch.empty(s, dtype=torch.float32, device=dev)
        return t.normal_(mean, std, generator=g)

    g_pre = randn((1, B, n) if per_channel else shape, gate_mean, gate_std)
    if per_channel:
        g_pre = g_pre.expand(shape).contiguous()
    i_pre = randn(shape)
    h0 = randn((B, n)) if with_h0 else None
    grad_h = randn(shape)
    return dict(T=T, B=B, n=n, g_pre=g_pre, i_pre=i_pre, h0=h0, grad_h=grad_h)


#: LSTM-cell workloads (Section 3.2's GILR-LSTM cell): four pre-activation tensors in
LSTM = {
    "l4": dict(T=4096, B=16, n=1024, forget_mean=1.0, note="workload 4's shape; forget gates sigmoid(N(1,1))"),
    "l2": dict(T=65536, B=4, n=256, forget_mean=2.0, note="workload 2's shape; forget gates sigmoid(N(2,1))"),
    "l5": dict(T=262144, B=8, n=512, forget_mean=1.5, note="workload 5's shape (1.07e9 elements)"),
}


def make_lstm(T, B, n, seed, device="cpu", forget_mean=1.0, forget_std=1.0, with_c0=True):
    """``f_pre ~ N(forget_mean, forget_std)``; ``i_pre, z_pre, o_pre, c0, grad_h ~ N(0,1)``."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(SEED_BASE + 7 * int(seed) + 5)
    shape = (T, B, n)

    def randn(s, mean=0.0, std=1.0):
        t = torch.empty(s, dtype=torch.float32, device=dev)
        return t.normal_(mean, std, generator=g)

    return dict(T=T, B=B, n=n, f_pre=randn(shape, forget_mean, forget_std), i_pre=randn(shape), z_pre=randn(shape),
                o_pre=randn(shape), c0=randn((B, n)) if with_c0 else None, grad_h=randn(shape))
