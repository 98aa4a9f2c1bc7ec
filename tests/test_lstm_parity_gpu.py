"""GPU parity of the LSTM-cell entry points against the fp64 oracle, through the C ABI.

arXiv 1709.04057, Section 3.2 (the GILR-LSTM's cell): c_t = f_t*c_{t-1} + i_t*z_t, h_t = o_t*c_t, the
gates and the candidate from their pre-activations inside the scan kernel.  Tolerances as for the plain
recurrence: forward outputs max|err| <= 1e-5*(1 + max|ref|), each gradient ||err||_inf <= 1e-4*||ref||_inf.
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
CELL_TILES = [i for i, _ in all_tiles(lr.ENTRY_LSTM_CELL)]
PRE = ("f_pre", "i_pre", "z_pre", "o_pre")


def _np(t):
    return None if t is None else t.detach().cpu().numpy()


def cell_check(inp, label, cols=None):
    T, B, n = inp["T"], inp["B"], inp["n"]
    C = B * n
    say(f"{label}: lstm cell forward T={T} B={B} n={n}")
    c, h = lr.linrec_lstm_cell_forward(*(inp[k] for k in PRE), inp["c0"])
    torch.cuda.synchronize()
    sel = slice(None) if cols is None else torch.as_tensor(cols, device=c.device)

    def pick(t, rows=True):
        if t is None:
            return None
        t2 = t.reshape(T, C) if rows else t.reshape(C)
        return np.ascontiguousarray(_np(t2[:, sel] if rows else t2[sel]))

    pre = [pick(inp[k]) for k in PRE]
    c0 = pick(inp["c0"], rows=False)
    cref, href = oracle.lstm_forward(*pre, c0, threads=ORACLE_THREADS)
    cg, hg = pick(c), pick(h)
    out = {}
    for name, got, want in (("c", cg, cref), ("h", hg, href)):
        assert np.all(np.isfinite(got))
        err, ref = (np.abs(got - want).max(), np.abs(want).max()) if want.size else (0.0, 0.0)
        assert err <= FWD_TOL * (1 + ref), f"{label}: {name} max|err| {err:.3e} > {FWD_TOL * (1 + ref):.3e}"
        out[name] = err
    say(f"{label}: lstm cell backward")
    grads = lr.linrec_lstm_cell_backward(*(inp[k] for k in PRE), c, inp["c0"], inp["grad_h"])
    torch.cuda.synchronize()
    refs = oracle.lstm_backward(*pre, cg, c0, pick(inp["grad_h"]), threads=ORACLE_THREADS)
    for k, name in enumerate(("grad_f_pre", "grad_i_pre", "grad_z_pre", "grad_o_pre", "grad_c0")):
        got = pick(grads[k], rows=(k < 4))
        assert np.all(np.isfinite(got)), f"{label}: {name} has non-finite values"
        e, r = (np.abs(got - refs[k]).max(), max(np.abs(refs[k]).max(), 1e-30)) if refs[k].size else (0.0, 1.0)
        assert e <= GRAD_TOL * r, f"{label}: {name} ||err||_inf {e:.3e} > {GRAD_TOL:.0e} * {r:.3e}"
        out[name] = e / r
    lr.linrec_check()
    return out


@pytest.mark.parametrize("tile", CELL_TILES)
def test_every_cell_tile_ragged_shapes(tile):
    info = lr.linrec_tile_info(tile)
    T = 2 * info["rows"] + info["rows"] // 2 + 3
    C = 2 * info["cols"] + 5 * info["cols_per_thread"]   # ragged against the tile, whole accesses
    inp = wl.make_lstm(T, 1, C, seed=200 + tile, device=DEV, forget_mean=1.0, forget_std=2.0)
    with options(variant=lr.VARIANT_LOOKBACK, tile=tile):
        cell_check(inp, f"tile {tile}")


WIDE_CELL_TILES = [i for i in CELL_TILES if lr.linrec_tile_info(i)["cols_per_thread"] > 1]


@pytest.mark.parametrize("variant", ["lookback", "walk"])
@pytest.mark.parametrize("tile", WIDE_CELL_TILES)
def test_multi_column_tiles_over_many_tiles(tile, variant):
    """The shapes with 8- and 16-byte accesses on a problem of many tiles and workgroups, whole tile
    widths of adjacent columns among the sampled ones: the four-column backward kernels once stored a
    few lanes' next-row temporaries (a 128-bit store's data registers were overwritten too early), which
    small problems did not show."""
    T, B, n = 2048, 4, 1024
    C = B * n
    inp = wl.make_lstm(T, B, n, seed=400 + tile, device=DEV)
    rng = np.random.default_rng(tile)
    cols = np.unique(np.concatenate([np.arange(0, 256), np.arange(C - 256, C), 1536 + np.arange(256),
                                     rng.choice(C, size=128, replace=False)]))
    with options(variant=getattr(lr, "VARIANT_" + variant.upper()), tile=tile):
        for rep in range(2):
            cell_check(inp, f"tile {tile} {variant} pass {rep}", cols=cols)


def test_a_tile_the_cell_does_not_have_falls_back_to_one_it_has():
    # a shape the library has, but not for the cell (which exists for at most 32 elements per thread and is built
    # for the shapes its plans use): the request is ignored, not an error
    other = next(i for i, _ in all_tiles() if not lr.linrec_tile_has(i, lr.ENTRY_LSTM_CELL))
    inp = wl.make_lstm(3000, 1, 70, seed=3, device=DEV)
    with options(variant=lr.VARIANT_LOOKBACK, tile=other):
        assert lr.linrec_plan_for(lr.ENTRY_LSTM_CELL, 3000, 1, 70)[1] in CELL_TILES
        cell_check(inp, f"tile {other} requested")


@pytest.mark.parametrize("T,B,n", [(1, 1, 1), (2, 3, 5), (7, 1, 64), (513, 2, 33), (4096, 1, 16), (3000, 2, 100)])
@pytest.mark.parametrize("variant", ["lookback", "serial"])
def test_small_and_degenerate_shapes(T, B, n, variant):
    inp = wl.make_lstm(T, B, n, seed=T + n, device=DEV)
    with options(variant=lr.VARIANT_LOOKBACK if variant == "lookback" else lr.VARIANT_SERIAL):
        cell_check(inp, f"{variant} {T}x{B}x{n}")


def test_no_initial_state_and_optional_outputs():
    inp = wl.make_lstm(2500, 2, 48, seed=5, device=DEV, with_c0=False)
    cell_check(inp, "no c0")
    pre = [inp[k] for k in PRE]
    c, h = lr.linrec_lstm_cell_forward(*pre, None)
    c_only, none_h = lr.linrec_lstm_cell_forward(pre[0], pre[1], pre[2], None, None, want_h=False)
    none_c, h_only = lr.linrec_lstm_cell_forward(*pre, None, want_c=False)
    torch.cuda.synchronize()
    assert none_h is None and none_c is None and reruns_agree(c_only, c) and reruns_agree(h_only, h)
    full = lr.linrec_lstm_cell_backward(*pre, c, None, inp["grad_h"])
    for k in range(4):
        want = [j == k for j in range(4)]
        part = lr.linrec_lstm_cell_backward(*pre, c, None, inp["grad_h"], want=want, want_grad_c0=(k == 0))
        torch.cuda.synchronize()
        assert all(part[j] is None for j in range(4) if j != k) and reruns_agree(part[k], full[k])
        if k == 0:
            assert reruns_agree(part[4], full[4])
    # T == 0: grad_c0 is zero-filled; B*n == 0: nothing at all
    e = torch.empty((0, 2, 48), device=DEV)
    gc0 = torch.full((2, 48), 3.0, device=DEV)
    lr.linrec_lstm_cell_backward(e, e, e, e, e, None, e, grad_c0=gc0)
    torch.cuda.synchronize()
    assert torch.count_nonzero(gc0) == 0
    z = torch.empty((4, 0, 8), device=DEV)
    lr.linrec_lstm_cell_forward(z, z, z, z, None)


def test_long_memory_forget_gates_close_to_one():
    # forget pre-activations constant along T per column, N(9, 2): 1-f down to 1e-7; 200 000 steps
    T, B, n = 200_000, 1, 64
    inp = wl.make_lstm(T, B, n, seed=21, device=DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(77)
    inp["f_pre"] = torch.empty((1, B, n), device=DEV).normal_(9.0, 2.0, generator=g).expand(T, B, n).contiguous()
    # keep the cell bounded: a weak input gate
    inp["i_pre"] = inp["i_pre"] - 6.0
    r = cell_check(inp, "long memory")
    say(f"long memory: {r}")


@pytest.mark.parametrize("variant", ["lookback", "serial"])
def test_non_finite_pre_activations_stay_in_their_column(variant):
    T, B, n = 3000, 1, 80
    inp = wl.make_lstm(T, B, n, seed=11, device=DEV)
    pre = [inp[k].clone() for k in PRE]
    pre[0][100, 0, 40] = float("nan")      # forget gate: the cell is NaN from there on
    pre[3][200, 0, 41] = float("nan")      # output gate: only h[200] is NaN
    pre[2][300, 0, 42] = float("inf")      # candidate: tanh(inf) = 1, stays finite
    with options(variant=lr.VARIANT_LOOKBACK if variant == "lookback" else lr.VARIANT_SERIAL):
        c, h = lr.linrec_lstm_cell_forward(*pre, inp["c0"])
        cr, hr = lr.linrec_lstm_cell_forward(*(inp[k] for k in PRE), inp["c0"])
        torch.cuda.synchronize()
        lr.linrec_check()
    assert torch.isnan(c[100:, 0, 40]).all() and torch.isfinite(c[:100, 0, 40]).all()
    assert torch.isfinite(c[:, 0, 41]).all() and torch.isnan(h[200, 0, 41]) and torch.isfinite(h[201:, 0, 41]).all()
    assert torch.isfinite(c[:, 0, 42]).all()
    keep = [k for k in range(n) if k not in (40, 41, 42)]
    assert reruns_agree(c[:, 0, keep], cr[:, 0, keep]) and reruns_agree(h[:, 0, keep], hr[:, 0, keep])


@pytest.mark.parametrize("name", sorted(k for k in wl.LSTM if k != "l5"))
def test_full_size_workloads_every_element(name):
    # the benchmarked shapes in their launch configuration, every element of every output
    spec = wl.LSTM[name]
    T, B, n = spec["T"], spec["B"], spec["n"]
    C = B * n
    inp = wl.make_lstm(T, B, n, seed=sum(map(ord, name)), device=DEV, forget_mean=spec["forget_mean"])
    say(f"workload {name}: lstm cell forward + backward T={T} B={B} n={n}")
    c, h = lr.linrec_lstm_cell_forward(*(inp[k] for k in PRE), inp["c0"])
    grads = lr.linrec_lstm_cell_backward(*(inp[k] for k in PRE), c, inp["c0"], inp["grad_h"])
    torch.cuda.synchronize()
    lr.linrec_check()
    say(f"workload {name}: oracle on all {C} columns")
    r = oracle.lstm_compare(*(host_f32(inp[k], T, C) for k in PRE), host_f32(inp["c0"]), host_f32(inp["grad_h"], T, C),
                            host_f32(c, T, C), host_f32(h, T, C), [host_f32(g, T, C) for g in grads[:4]],
                            host_f32(grads[4]), threads=ORACLE_THREADS)
    say(f"workload {name}: {check_norms(r, 'workload ' + name)}")


def test_workload_5_shape_on_sampled_columns():
    # the largest benchmarked shape (1.07e9 elements) in its launch configuration; the oracle takes whole
    # blocks of adjacent columns at both ends and in the middle of a row (columns are independent recurrences)
    spec = wl.LSTM["l5"]
    T, B, n = spec["T"], spec["B"], spec["n"]
    C = B * n
    inp = wl.make_lstm(T, B, n, seed=sum(map(ord, "l5")), device=DEV, forget_mean=spec["forget_mean"])
    say(f"workload l5: lstm cell forward + backward T={T} B={B} n={n}")
    c, h = lr.linrec_lstm_cell_forward(*(inp[k] for k in PRE), inp["c0"])
    grads = lr.linrec_lstm_cell_backward(*(inp[k] for k in PRE), c, inp["c0"], inp["grad_h"])
    torch.cuda.synchronize()
    lr.linrec_check()
    for a in (0, C // 2 - 37, C - 64):
        cut = lambda t: t.reshape(-1, C)[:, a:a + 64].contiguous().cpu().numpy()
        say(f"workload l5: oracle on columns {a} .. {a + 63}")
        r = oracle.lstm_compare(*(cut(inp[k]) for k in PRE), cut(inp["c0"]).reshape(-1), cut(inp["grad_h"]), cut(c), cut(h),
                                [cut(g) for g in grads[:4]], cut(grads[4]).reshape(-1), threads=ORACLE_THREADS)
        say(f"workload l5: {check_norms(r, 'workload l5 columns from ' + str(a))}")
