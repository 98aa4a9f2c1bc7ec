"""GPU parity of the gated layer and the LSTM cell on bf16 storage against the fp64 oracle, through the C ABI.

arXiv 1709.04057, Sections 3.1 and 3.2 (the paper computes in fp32, Section 2.3; bf16 storage is a
bandwidth option).  The inputs are bf16 values; widened to fp32 they are exact, so the fp64 oracles of
the two forms run on those fp32 values ARE the reference.  The library computes as its fp32 entry points
do and rounds each result to the nearest bf16, hence per element
    |got - ref| <= 2^-8 * |ref|  +  the fp32 path's tolerance
(half a unit in the last place of a bf16; 1e-5 * (1 + max|ref|) forward, 1e-4 * ||ref||_inf per gradient).
The backward passes are given the ROUNDED h (c) of the forward pass, and so is the oracle.
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
HALF_ULP = 2.0 ** -8
PRE = ("f_pre", "i_pre", "z_pre", "o_pre")


GATED16_TILES = [i for i, _ in all_tiles(lr.ENTRY_GILR_BF16)]
CELL16_TILES = [i for i, _ in all_tiles(lr.ENTRY_LSTM_CELL_BF16)]


def to_bf16(inp):
    return {k: (v.to(torch.bfloat16).contiguous() if torch.is_tensor(v) else v) for k, v in inp.items()}


def _picker(T, C, cols, device):
    sel = slice(None) if cols is None else torch.as_tensor(cols, device=device)

    def pick(t, rows=True):  # the sampled columns as float32 on the host (exact for bf16 values)
        if t is None:
            return None
        t2 = t.reshape(T, C) if rows else t.reshape(C)
        return np.ascontiguousarray((t2[:, sel] if rows else t2[sel]).detach().float().cpu().numpy())

    return pick


def _within(got, ref, tol, label, name):
    assert np.all(np.isfinite(got)), f"{label}: {name} has non-finite values"
    if not ref.size:
        return 0.0
    mag = max(np.abs(ref).max(), 1e-30)
    bound = HALF_ULP * np.abs(ref) + (tol * (1 + mag) if tol == FWD_TOL else tol * mag)
    worst = (np.abs(got - ref) / bound).max()
    assert worst <= 1.0, f"{label}: {name} error is {worst:.3f} of its bound"
    return worst


def gated16_check(inp, tau, label, cols=None):
    T, B, n = inp["T"], inp["B"], inp["n"]
    pick = _picker(T, B * n, cols, inp["g_pre"].device)
    say(f"{label}: bf16 gilr forward T={T} B={B} n={n} tau={tau}")
    h = lr.linrec_gilr_forward(inp["g_pre"], inp["i_pre"], inp["h0"], tau=tau)
    assert h.dtype == torch.bfloat16
    torch.cuda.synchronize()
    gp, ip, h0 = pick(inp["g_pre"]), pick(inp["i_pre"]), pick(inp["h0"], rows=False)
    hg = pick(h)
    out = {"h": _within(hg, oracle.gilr_forward(gp, ip, h0, tau, threads=ORACLE_THREADS), FWD_TOL, label, "h")}
    say(f"{label}: bf16 gilr backward")
    grads = lr.linrec_gilr_backward(inp["g_pre"], inp["i_pre"], h, inp["h0"], inp["grad_h"], tau=tau)
    torch.cuda.synchronize()
    refs = oracle.gilr_backward(gp, ip, hg, h0, pick(inp["grad_h"]), tau, threads=ORACLE_THREADS)
    for k, name in enumerate(("grad_g_pre", "grad_i_pre", "grad_h0")):
        assert grads[k].dtype == torch.bfloat16
        out[name] = _within(pick(grads[k], rows=(k < 2)), refs[k], GRAD_TOL, label, name)
    lr.linrec_check()
    return out


def cell16_check(inp, label, cols=None):
    T, B, n = inp["T"], inp["B"], inp["n"]
    pick = _picker(T, B * n, cols, inp["f_pre"].device)
    say(f"{label}: bf16 lstm cell forward T={T} B={B} n={n}")
    c, h = lr.linrec_lstm_cell_forward(*(inp[k] for k in PRE), inp["c0"])
    assert c.dtype == torch.bfloat16 and h.dtype == torch.bfloat16
    torch.cuda.synchronize()
    pre = [pick(inp[k]) for k in PRE]
    c0 = pick(inp["c0"], rows=False)
    cref, href = oracle.lstm_forward(*pre, c0, threads=ORACLE_THREADS)
    cg = pick(c)
    out = {"c": _within(cg, cref, FWD_TOL, label, "c"), "h": _within(pick(h), href, FWD_TOL, label, "h")}
    say(f"{label}: bf16 lstm cell backward")
    grads = lr.linrec_lstm_cell_backward(*(inp[k] for k in PRE), c, inp["c0"], inp["grad_h"])
    torch.cuda.synchronize()
    refs = oracle.lstm_backward(*pre, cg, c0, pick(inp["grad_h"]), threads=ORACLE_THREADS)
    for k, name in enumerate(("grad_f_pre", "grad_i_pre", "grad_z_pre", "grad_o_pre", "grad_c0")):
        assert grads[k].dtype == torch.bfloat16
        out[name] = _within(pick(grads[k], rows=(k < 4)), refs[k], GRAD_TOL, label, name)
    lr.linrec_check()
    return out


def _ragged(info):
    T = 2 * info["rows"] + info["rows"] // 2 + 3
    C = 2 * info["cols"] + 5 * info["cols_per_thread"]   # ragged against the tile, whole accesses
    if info["cols_per_thread"] == 1:
        C += (C + 1) % 2                                  # an odd number of columns: rows 2 bytes off alignment
    return T, C


@pytest.mark.parametrize("variant", ["lookback", "walk"])
@pytest.mark.parametrize("tile", GATED16_TILES)
def test_every_gated_tile_ragged_shapes(tile, variant):
    T, C = _ragged(lr.linrec_tile_info(tile))
    inp = to_bf16(wl.make_gated(T, 1, C, seed=600 + tile, device=DEV, gate_mean=1.0, gate_std=2.0))
    with options(variant=getattr(lr, "VARIANT_" + variant.upper()), tile=tile):
        assert lr.linrec_plan_for(lr.ENTRY_GILR_BF16, T, 1, C, backward=True, alignment=8)[1] == tile
        gated16_check(inp, lr.TAU_TANH if tile % 2 else lr.TAU_IDENTITY, f"tile {tile} {variant}")


@pytest.mark.parametrize("variant", ["lookback", "walk"])
@pytest.mark.parametrize("tile", CELL16_TILES)
def test_every_cell_tile_ragged_shapes(tile, variant):
    T, C = _ragged(lr.linrec_tile_info(tile))
    inp = to_bf16(wl.make_lstm(T, 1, C, seed=700 + tile, device=DEV, forget_mean=1.0, forget_std=2.0))
    with options(variant=getattr(lr, "VARIANT_" + variant.upper()), tile=tile):
        assert lr.linrec_plan_for(lr.ENTRY_LSTM_CELL_BF16, T, 1, C, backward=True, alignment=8)[1] == tile
        cell16_check(inp, f"tile {tile} {variant}")


@pytest.mark.parametrize("T,B,n", [(1, 1, 2), (2, 3, 4), (7, 1, 64), (513, 2, 34), (4096, 1, 16), (3000, 2, 100),
                                   (100, 1, 7), (900, 3, 11)])
@pytest.mark.parametrize("variant", ["auto", "serial"])
def test_small_and_degenerate_shapes(T, B, n, variant):
    # odd B*n (the last two shapes) has no 4-byte rows: the one-column shapes, with 2-byte accesses
    with options(variant=lr.VARIANT_AUTO if variant == "auto" else lr.VARIANT_SERIAL):
        gated16_check(to_bf16(wl.make_gated(T, B, n, seed=T + n, device=DEV, gate_mean=0.5, gate_std=1.5)), lr.TAU_TANH,
                      f"gated {variant} {T}x{B}x{n}")
        cell16_check(to_bf16(wl.make_lstm(T, B, n, seed=T + n, device=DEV)), f"cell {variant} {T}x{B}x{n}")


def test_optional_outputs_no_initial_state_and_empty_problems():
    inp = to_bf16(wl.make_lstm(2500, 2, 48, seed=5, device=DEV, with_c0=False))
    cell16_check(inp, "no c0")
    pre = [inp[k] for k in PRE]
    c, h = lr.linrec_lstm_cell_forward(*pre, None)
    c_only, none = lr.linrec_lstm_cell_forward(*pre, None, want_h=False)
    full = lr.linrec_lstm_cell_backward(*pre, c, None, inp["grad_h"], want_grad_c0=False)
    part = lr.linrec_lstm_cell_backward(*pre, c, None, inp["grad_h"], want=(True, False, False, True), want_grad_c0=False)
    torch.cuda.synchronize()
    assert none is None and reruns_agree(c_only, c)
    assert part[1] is None and part[2] is None and reruns_agree(part[0], full[0]) and reruns_agree(part[3], full[3])
    g = to_bf16(wl.make_gated(1800, 2, 48, seed=6, device=DEV, with_h0=False))
    gated16_check(g, lr.TAU_TANH, "no h0")
    # T == 0: nothing is launched but the state gradient, which is zero
    e = torch.empty((0, 2, 48), dtype=torch.bfloat16, device=DEV)
    gh0 = torch.full((2, 48), 7.0, dtype=torch.bfloat16, device=DEV)
    lr.linrec_gilr_backward(e, e, e, None, e, grad_h0=gh0)
    gc0 = torch.full((2, 48), 7.0, dtype=torch.bfloat16, device=DEV)
    lr.linrec_lstm_cell_backward(e, e, e, e, e, None, e, grad_c0=gc0)
    torch.cuda.synchronize()
    assert not gh0.any() and not gc0.any()
    assert lr.linrec_gilr_forward(e, e, None).shape == (0, 2, 48)


def test_gates_close_to_one_keep_their_decay_rate():
    # 200 000 steps with a per-channel constant gate around sigmoid(9): the complement 1-g is formed from the
    # pre-activation in fp32, so bf16 storage costs the stored values their last bits and nothing else
    inp = to_bf16(wl.make_gated(200_000, 1, 64, seed=11, device=DEV, gate_mean=9.0, gate_std=1.5, per_channel=True))
    gated16_check(inp, lr.TAU_TANH, "long memory")


@pytest.mark.parametrize("name", ["g2", "g4", "l2", "l4"])
def test_full_size_workloads_every_element(name):
    # The benchmarked shapes on bf16 storage, every element of every output: the oracle runs on the exactly
    # widened inputs in blocks of whole columns, and each element is allowed half a bf16 unit in the last
    # place of its reference value on top of the fp32 path's tolerance.
    gated = name[0] == "g"
    spec = (wl.GATED if gated else wl.LSTM)[name]
    T, B, n = spec["T"], spec["B"], spec["n"]
    C = B * n
    f = lambda t: host_f32(t, T, C)
    if gated:
        inp = to_bf16(wl.make_gated(T, B, n, seed=sum(map(ord, name)), device=DEV, gate_mean=spec["gate_mean"],
                                    gate_std=spec["gate_std"]))
        say(f"workload {name} bf16: gilr forward + backward T={T} B={B} n={n}")
        h = lr.linrec_gilr_forward(inp["g_pre"], inp["i_pre"], inp["h0"], tau=lr.TAU_TANH)
        gg, gi, gh0 = lr.linrec_gilr_backward(inp["g_pre"], inp["i_pre"], h, inp["h0"], inp["grad_h"], tau=lr.TAU_TANH)
        torch.cuda.synchronize()
        lr.linrec_check()
        assert all(t.dtype == torch.bfloat16 for t in (h, gg, gi, gh0))
        r = oracle.gilr_compare(f(inp["g_pre"]), f(inp["i_pre"]), host_f32(inp["h0"]), f(inp["grad_h"]), f(h), f(gg), f(gi),
                                host_f32(gh0), lr.TAU_TANH, threads=ORACLE_THREADS, rel=HALF_ULP)
    else:
        inp = to_bf16(wl.make_lstm(T, B, n, seed=sum(map(ord, name)), device=DEV, forget_mean=spec["forget_mean"]))
        say(f"workload {name} bf16: lstm cell forward + backward T={T} B={B} n={n}")
        c, h = lr.linrec_lstm_cell_forward(*(inp[k] for k in PRE), inp["c0"])
        grads = lr.linrec_lstm_cell_backward(*(inp[k] for k in PRE), c, inp["c0"], inp["grad_h"])
        torch.cuda.synchronize()
        lr.linrec_check()
        assert all(t.dtype == torch.bfloat16 for t in (c, h) + tuple(grads))
        r = oracle.lstm_compare(*(f(inp[k]) for k in PRE), host_f32(inp["c0"]), f(inp["grad_h"]), f(c), f(h),
                                [f(g) for g in grads[:4]], host_f32(grads[4]), threads=ORACLE_THREADS, rel=HALF_ULP)
    say(f"workload {name} bf16: {check_norms(r, 'workload ' + name + ' bf16')}")


def test_autograd_wrappers_take_bf16():
    inp = to_bf16(wl.make_gated(700, 2, 64, seed=9, device=DEV))
    g_pre, i_pre = inp["g_pre"].requires_grad_(), inp["i_pre"].requires_grad_()
    h = lr.gilr(g_pre, i_pre, inp["h0"])
    (h.float() * inp["grad_h"].float()).sum().backward()
    want = lr.linrec_gilr_backward(g_pre.detach(), i_pre.detach(), h.detach(), inp["h0"], inp["grad_h"])
    torch.cuda.synchronize()
    assert h.dtype == torch.bfloat16 and reruns_agree(g_pre.grad, want[0]) and reruns_agree(i_pre.grad, want[1])
