"""GPU parity of the bf16-storage entry points against the fp64 oracle, through the C ABI.

The inputs are bf16 values; widened to fp32 they are exact, so the fp64 oracle of the plain recurrence
(arXiv 1709.04057, Sections 2 and 2.2) run on those fp32 values IS the reference.  The library computes
as its fp32 entry points do and rounds each result to the nearest bf16, hence per element
    |got - ref| <= 2^-8 * |ref|  +  the fp32 path's tolerance
(2^-8 |ref| bounds half a unit in the last place of a bf16 with 8 significant bits; the fp32 path's
tolerance is 1e-5 * (1 + max|ref|) forward, 1e-4 * ||ref||_inf for each gradient).
"""
import numpy as np
import pytest
import torch

import linrec_workloads as wl
import oracle
import paper_1709_04057_amd as lr
from parity import FWD_TOL, GRAD_TOL, ORACLE_THREADS, all_tiles, check_norms, host_f32, options, say, reruns_agree

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
BF16_TILES = [i for i, _ in all_tiles(lr.ENTRY_BF16)]
HALF_ULP = 2.0 ** -8


def _f32(t):
    """bf16 tensor -> the same values as a float32 numpy array (exact)."""
    return None if t is None else t.detach().float().cpu().numpy()


def to_bf16(inp):
    out = dict(inp)
    for k in ("lam", "x", "h0", "grad_h"):
        if inp.get(k) is not None:
            out[k] = inp[k].to(torch.bfloat16).contiguous()
    return out


def bf16_check(inp, label, cols=None):
    T, B, n = inp["T"], inp["B"], inp["n"]
    C = B * n
    say(f"{label}: bf16 forward T={T} B={B} n={n}")
    h = lr.linrec_forward(inp["lam"], inp["x"], inp["h0"])
    assert h.dtype == torch.bfloat16
    torch.cuda.synchronize()
    sel = slice(None) if cols is None else torch.as_tensor(cols, device=h.device)

    def pick(t, rows=True):
        if t is None:
            return None
        t2 = t.reshape(T, C) if rows else t.reshape(C)
        return np.ascontiguousarray(_f32(t2[:, sel] if rows else t2[sel]))

    lam, x, h0 = pick(inp["lam"]), pick(inp["x"]), pick(inp["h0"], rows=False)
    href = oracle.forward(lam, x, h0, threads=ORACLE_THREADS)
    hg = pick(h)
    assert np.all(np.isfinite(hg))
    mag = np.abs(href).max() if href.size else 0.0
    bound = HALF_ULP * np.abs(href) + FWD_TOL * (1 + mag)
    worst = (np.abs(hg - href) / bound).max() if href.size else 0.0
    assert worst <= 1.0, f"{label}: forward error is {worst:.3f} of its bound"
    out = {"fwd": worst}
    if inp.get("grad_h") is not None:
        say(f"{label}: bf16 backward")
        gx, gl, gh0 = lr.linrec_backward(inp["lam"], h, inp["h0"], inp["grad_h"])
        torch.cuda.synchronize()
        rx, rl, rh0 = oracle.backward(lam, hg, h0, pick(inp["grad_h"]), threads=ORACLE_THREADS)
        for name, got, ref in (("grad_x", pick(gx), rx), ("grad_lambda", pick(gl), rl),
                               ("grad_h0", pick(gh0, rows=False), rh0)):
            assert np.all(np.isfinite(got)), f"{label}: {name} has non-finite values"
            m = max(np.abs(ref).max(), 1e-30) if ref.size else 1.0
            b = HALF_ULP * np.abs(ref) + GRAD_TOL * m
            w = (np.abs(got - ref) / b).max() if ref.size else 0.0
            assert w <= 1.0, f"{label}: {name} error is {w:.3f} of its bound"
            out[name] = w
    lr.linrec_check()
    return out


@pytest.mark.parametrize("tile", BF16_TILES)
def test_every_bf16_tile_ragged_shapes(tile):
    info = lr.linrec_tile_info(tile)
    v = info["cols_per_thread"]
    T = 2 * info["rows"] + info["rows"] // 2 + 3
    C = 2 * info["cols"] + 3 * v                     # ragged along the columns, still a multiple of v
    inp = to_bf16(wl.make_generic(T, 1, C, seed=300 + tile, device=DEV))
    with options(variant=lr.VARIANT_LOOKBACK, tile=tile):
        bf16_check(inp, f"tile {tile}")


@pytest.mark.parametrize("T,B,n", [(1, 1, 2), (2, 3, 4), (7, 1, 64), (513, 2, 34), (4096, 1, 16), (3000, 2, 100),
                                   (100, 1, 7), (900, 3, 11)])
@pytest.mark.parametrize("variant", ["auto", "serial"])
def test_small_and_degenerate_shapes(T, B, n, variant):
    # odd B*n (the last two shapes) has no 4-byte rows: the library falls back to its serial kernel
    inp = to_bf16(wl.make_generic(T, B, n, seed=T + n, device=DEV, lam_kind="mixed"))
    with options(variant=lr.VARIANT_AUTO if variant == "auto" else lr.VARIANT_SERIAL):
        bf16_check(inp, f"{variant} {T}x{B}x{n}")


def test_unaligned_views_and_optional_outputs():
    T, B, n = 1200, 2, 64
    inp = to_bf16(wl.make_generic(T, B, n, seed=8, device=DEV, with_h0=False))
    want = lr.linrec_forward(inp["lam"], inp["x"], None)
    # the same tensors placed 2 bytes off a 4-byte boundary: serial fallback, same values up to rounding order
    def shifted(t):
        buf = torch.empty(t.numel() + 1, dtype=torch.bfloat16, device=DEV)
        v = buf[1:].view(t.shape)
        v.copy_(t)
        return v
    got = lr.linrec_forward(shifted(inp["lam"]), shifted(inp["x"]), None, h_out=shifted(want))
    torch.cuda.synchronize()
    assert (got.float() - want.float()).abs().max() <= 2.0 ** -7 * want.float().abs().max()
    bf16_check(inp, "no h0")
    gx, gl, gh0 = lr.linrec_backward(inp["lam"], want, None, inp["grad_h"], want_grad_lambda=False, want_grad_h0=False)
    full = lr.linrec_backward(inp["lam"], want, None, inp["grad_h"])
    torch.cuda.synchronize()
    assert gl is None and gh0 is None and reruns_agree(gx, full[0])
    # in place on x, and grad_x in place on grad_h
    xb = inp["x"].clone()
    assert reruns_agree(lr.linrec_forward(inp["lam"], xb, None, h_out=xb), want)
    eb = inp["grad_h"].clone()
    assert reruns_agree(lr.linrec_backward(inp["lam"], want, None, eb, grad_x=eb)[0], full[0])
    # empty problems
    e = torch.empty((0, 2, 64), dtype=torch.bfloat16, device=DEV)
    g0 = torch.ones((2, 64), dtype=torch.bfloat16, device=DEV)
    lr.linrec_backward(e, e, None, e, grad_h0=g0)
    torch.cuda.synchronize()
    assert torch.count_nonzero(g0) == 0


def test_lambda_zero_is_a_copy_and_lambda_one_a_prefix_sum():
    T, B, n = 2000, 1, 64
    g = torch.Generator(device=DEV)
    g.manual_seed(5)
    x = torch.randint(-8, 9, (T, B, n), device=DEV, generator=g).to(torch.bfloat16)   # small integers: exact sums
    zero, one = torch.zeros_like(x), torch.ones_like(x)
    h = lr.linrec_forward(zero, x, None)
    torch.cuda.synchronize()
    assert torch.equal(h, x)
    h = lr.linrec_forward(one, x, None)
    torch.cuda.synchronize()
    ref = torch.cumsum(x.float(), dim=0)
    assert ref.abs().max() < 2 ** 24
    assert torch.equal(h, ref.to(torch.bfloat16))                                     # the only error is the final rounding


@pytest.mark.parametrize("cfg", [2, 4])
def test_full_size_workloads_every_element(cfg):
    # every element, through the oracle's slab-streaming comparison on the exactly widened bf16 values, each
    # allowed half a bf16 unit in the last place of its reference on top of the fp32 path's tolerance
    spec = wl.CONFIGS[cfg]
    inp = to_bf16(wl.make_inputs(cfg, device=DEV))
    T, C = spec["T"], spec["B"] * spec["n"]
    say(f"workload {cfg} in bf16: forward + backward")
    h = lr.linrec_forward(inp["lam"], inp["x"], inp["h0"])
    gx, gl, gh0 = lr.linrec_backward(inp["lam"], h, inp["h0"], inp["grad_h"])
    torch.cuda.synchronize()
    lr.linrec_check()
    assert all(t.dtype == torch.bfloat16 for t in (h, gx, gl, gh0))
    f = lambda t: host_f32(t, T, C)
    lam, hh, h0 = f(inp["lam"]), f(h), host_f32(inp["h0"])
    r = {"h": oracle.forward_compare(lam, f(inp["x"]), h0, hh, threads=ORACLE_THREADS, rel=HALF_ULP)}
    r.update(oracle.backward_compare(lam, hh, h0, f(inp["grad_h"]), f(gx), f(gl), host_f32(gh0), threads=ORACLE_THREADS,
                                     rel=HALF_ULP))
    say(f"workload {cfg} bf16: {check_norms(r, f'workload {cfg} bf16')}")
