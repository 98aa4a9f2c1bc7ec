"""Shared helpers of the GPU parity tests: run liblinrec through its Python binding (which only
marshals into the C ABI) and compare element by element with the fp64 oracle on the same fp32 bits.

Tolerances (stated by the build's target): forward max|err| <= 1e-5 * (1 + max|h_ref|); each gradient
tensor ||err||_inf <= 1e-4 * ||ref||_inf.
"""
import sys

import numpy as np
import torch

import oracle
import paper_1709_04057_amd as lr

FWD_TOL = 1e-5
GRAD_TOL = 1e-4
ORACLE_THREADS = 8


def say(msg):
    print("[parity] " + msg, flush=True)
    sys.stdout.flush()


def _np(t):
    return None if t is None else t.detach().cpu().numpy()


def run_forward(inp, h_out=None):
    return lr.linrec_forward(inp["lam"], inp["x"], inp["h0"], h_out=h_out)


def check_forward(inp, h_gpu, label=""):
    """Element-wise comparison of h_gpu with the oracle (streamed in slabs). Returns the error record."""
    lam, x, h0 = _np(inp["lam"]), _np(inp["x"]), _np(inp["h0"])
    T, B, n = lam.shape
    r = oracle.forward_compare(lam.reshape(T, B * n), x.reshape(T, B * n), None if h0 is None else h0.reshape(-1),
                               _np(h_gpu).reshape(T, B * n), threads=ORACLE_THREADS)
    tol = FWD_TOL * (1.0 + r["max_abs_ref"])
    assert r["max_abs_err"] <= tol, (
        f"{label}: forward max|err| {r['max_abs_err']:.3e} > {tol:.3e} (max|h| {r['max_abs_ref']:.3e}) "
        f"at (t, c) = {r['worst_index']}")
    return r


def reruns_agree(a, b, exact=False):
    """Do two GPU runs of the same call agree?  Bit for bit when ``exact`` (the three-phase, walk and
    serial variants); the single pass composes a carry-in from whichever predecessor summaries are
    published when it looks, so its repeats may differ in the last bit or two of a row: a fifth of the
    tolerance against the oracle (and one unit in the last place of bf16 storage) is allowed."""
    if a is None or b is None:
        return a is b
    if a.shape != b.shape or a.dtype != b.dtype:
        return False
    if torch.equal(a, b):
        return True
    if exact:
        return False
    af, bf = a.float(), b.float()
    slack = 2e-6 * (1.0 + float(af.abs().max()))
    if a.dtype == torch.bfloat16:
        return bool(((af - bf).abs() <= 2.0 ** -7 * torch.maximum(af.abs(), bf.abs()) + slack).all())
    return bool(((af - bf).abs() <= slack).all())


def run_backward(inp, h, **kw):
    return lr.linrec_backward(inp["lam"], h, inp["h0"], inp["grad_h"], **kw)


def check_backward(inp, h, gx, gl, gh0, label=""):
    lam, h0, e, hh = _np(inp["lam"]), _np(inp["h0"]), _np(inp["grad_h"]), _np(h)
    T, B, n = lam.shape
    C = B * n
    zeros_tc = None
    if gx is None or gl is None:
        zeros_tc = np.zeros((T, C), np.float32)
    r = oracle.backward_compare(lam.reshape(T, C), hh.reshape(T, C), None if h0 is None else h0.reshape(-1),
                                e.reshape(T, C),
                                zeros_tc if gx is None else _np(gx).reshape(T, C),
                                zeros_tc if gl is None else _np(gl).reshape(T, C),
                                None if gh0 is None else _np(gh0).reshape(-1), threads=ORACLE_THREADS)
    for name, got in (("grad_x", gx), ("grad_lambda", gl), ("grad_h0", gh0)):
        if got is None:
            continue
        ref = max(r[name]["max_abs_ref"], 1e-30)
        assert r[name]["max_abs_err"] <= GRAD_TOL * ref, (
            f"{label}: {name} ||err||_inf {r[name]['max_abs_err']:.3e} > {GRAD_TOL:.0e} * ||ref||_inf {ref:.3e}")
    return r


def fwd_bwd_check(inp, label):
    """Forward, then (if the workload has an upstream gradient) backward on the GPU's own h; both checked."""
    say(f"{label}: forward T={inp['T']} B={inp['B']} n={inp['n']}")
    h = run_forward(inp)
    torch.cuda.synchronize()
    check_forward(inp, h, label)
    if inp.get("grad_h") is not None:
        say(f"{label}: backward")
        gx, gl, gh0 = run_backward(inp, h)
        torch.cuda.synchronize()
        check_backward(inp, h, gx, gl, gh0, label)
    lr.linrec_check()


def check_norms(r, label, forward_names=("h", "c")):
    """Folded error norms (oracle.*_compare) against the tolerances: state tensors to
    FWD_TOL*(1 + max|ref|), gradient tensors to GRAD_TOL*max|ref|."""
    for name, rec in r.items():
        ref = rec["max_abs_ref"]
        tol = FWD_TOL * (1.0 + ref) if name in forward_names else GRAD_TOL * max(ref, 1e-30)
        assert rec["max_abs_err"] <= tol, (
            f"{label}: {name} error {rec['max_abs_err']:.3e} > {tol:.3e} (max|ref| {ref:.3e})")
    return {k: v["max_abs_err"] for k, v in r.items()}


def host_f32(t, T=None, C=None):
    """A device tensor (fp32 or bf16: bf16 widens exactly) as a float32 numpy array [T, C] or [C]."""
    if t is None:
        return None
    a = t.detach().float().cpu().numpy()
    return a.reshape(-1) if T is None else a.reshape(T, C)


class options:
    """Context manager: set liblinrec options, restore the previous values on exit."""

    def __init__(self, **kw):
        self.kw = kw
        self.ids = dict(variant=lr.OPT_VARIANT, tile=lr.OPT_TILE, chunk_tiles=lr.OPT_CHUNK_TILES,
                        spin_limit=lr.OPT_SPIN_LIMIT, hprev_late=lr.OPT_HPREV_LATE, taper=lr.OPT_TAPER, persistent=lr.OPT_PERSISTENT, grid_cap=lr.OPT_GRID_CAP,
                        stagger=lr.OPT_STAGGER)

    def __enter__(self):
        self.old = {k: lr.linrec_get_option(self.ids[k]) for k in self.kw}
        for k, v in self.kw.items():
            lr.linrec_set_option(self.ids[k], v)
        return self

    def __exit__(self, *exc):
        for k, v in self.old.items():
            lr.linrec_set_option(self.ids[k], v)
        return False


def one_column_tiles(family):
    """Ids of the family's tile shapes with one column per thread (usable whatever C and the alignment)."""
    return [i for i, info in all_tiles(family) if info["cols_per_thread"] == 1]


def all_tiles(family=None):
    """(id, description) of every tile shape the library has kernels of -- for entry-point family ``family``
    (lr.ENTRY_*) when given, else for any (ids are stable, so there are gaps)."""
    return [(i, info) for i in range(1, 129) if (info := lr.linrec_tile_info(i)) is not None
            and (family is None or lr.linrec_tile_has(i, family))]
