"""The gated layer, the LSTM cell and the bf16-storage entry points share the single-pass kernel's
device-resident call state: they must be deterministic, safe on side streams that interleave with
other calls of the library, and replayable from a HIP graph."""
import pytest
import torch

import linrec_workloads as wl
import paper_1709_04057_amd as lr
from parity import options, reruns_agree, say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
PRE = ("f_pre", "i_pre", "z_pre", "o_pre")


def _calls():
    """name -> (function enqueuing forward+backward on the current stream, list of its output tensors)."""
    g = wl.make_gated(12000, 2, 96, seed=1, device=DEV, gate_mean=1.5)
    c = wl.make_lstm(12000, 2, 96, seed=2, device=DEV)
    b = {k: (v.to(torch.bfloat16).contiguous() if torch.is_tensor(v) else v)
         for k, v in wl.make_inputs(2, T=12000, B=2, n=96, device=DEV).items()}
    out = {}

    hg = torch.empty_like(g["g_pre"]); gg = torch.empty_like(hg); gi = torch.empty_like(hg)
    gh0 = torch.empty_like(g["h0"])

    def gated():
        lr.linrec_gilr_forward(g["g_pre"], g["i_pre"], g["h0"], h_out=hg)
        lr.linrec_gilr_backward(g["g_pre"], g["i_pre"], hg, g["h0"], g["grad_h"], grad_g_pre=gg, grad_i_pre=gi,
                                grad_h0=gh0)
    out["gated"] = (gated, [hg, gg, gi, gh0])

    pre = [c[k] for k in PRE]
    cs = torch.empty_like(pre[0]); hs = torch.empty_like(cs)
    grads = [torch.empty_like(cs) for _ in range(4)]
    gc0 = torch.empty_like(c["c0"])

    def cell():
        lr.linrec_lstm_cell_forward(*pre, c["c0"], c_out=cs, h_out=hs)
        lr.linrec_lstm_cell_backward(*pre, cs, c["c0"], c["grad_h"], grads=grads, grad_c0=gc0)
    out["lstm"] = (cell, [cs, hs] + grads + [gc0])

    hb = torch.empty_like(b["x"]); gx = torch.empty_like(hb); gl = torch.empty_like(hb)
    gb0 = torch.empty_like(b["h0"])

    def bf16():
        lr.linrec_forward(b["lam"], b["x"], b["h0"], h_out=hb)
        lr.linrec_backward(b["lam"], hb, b["h0"], b["grad_h"], grad_x=gx, grad_lambda=gl, grad_h0=gb0)
    out["bf16"] = (bf16, [hb, gx, gl, gb0])

    half = lambda d: {k: (v.to(torch.bfloat16).contiguous() if torch.is_tensor(v) else v) for k, v in d.items()}
    g16, c16 = half(g), half(c)
    hg16 = torch.empty_like(g16["g_pre"]); gg16 = torch.empty_like(hg16); gi16 = torch.empty_like(hg16)
    gh16 = torch.empty_like(g16["h0"])

    def gated_bf16():
        lr.linrec_gilr_forward(g16["g_pre"], g16["i_pre"], g16["h0"], h_out=hg16)
        lr.linrec_gilr_backward(g16["g_pre"], g16["i_pre"], hg16, g16["h0"], g16["grad_h"], grad_g_pre=gg16,
                                grad_i_pre=gi16, grad_h0=gh16)
    out["gated_bf16"] = (gated_bf16, [hg16, gg16, gi16, gh16])

    pre16 = [c16[k] for k in PRE]
    cs16 = torch.empty_like(pre16[0]); hs16 = torch.empty_like(cs16)
    grads16 = [torch.empty_like(cs16) for _ in range(4)]
    gc16 = torch.empty_like(c16["c0"])

    def cell_bf16():
        lr.linrec_lstm_cell_forward(*pre16, c16["c0"], c_out=cs16, h_out=hs16)
        lr.linrec_lstm_cell_backward(*pre16, cs16, c16["c0"], c16["grad_h"], grads=grads16, grad_c0=gc16)
    out["lstm_bf16"] = (cell_bf16, [cs16, hs16] + grads16 + [gc16])
    return out


def _same(a, b):
    # Bit-identical (NaN-safe), or -- these are repeats of the single pass, whose carry-in is composed from
    # whichever predecessor summaries are published when a tile looks -- equal to rounding.
    if torch.equal(a.view(torch.int16 if a.dtype == torch.bfloat16 else torch.int32),
                   b.view(torch.int16 if b.dtype == torch.bfloat16 else torch.int32)):
        return True
    return reruns_agree(a, b)


@pytest.mark.parametrize("name", ["gated", "lstm", "bf16", "gated_bf16", "lstm_bf16"])
def test_deterministic_on_interleaved_streams(name):
    calls = _calls()
    fn, outs = calls[name]
    fn()
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]
    others = [calls[k][0] for k in calls if k != name]
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        for t in outs:
            t.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(s1):
            fn()
        with torch.cuda.stream(s2):          # other entry points of the library at the same time, own workspace
            for o in others:
                o()
        s1.synchronize(); s2.synchronize()
        assert all(_same(a, b) for a, b in zip(outs, ref)), f"{name}: run {rep} differs"
    for s in (s1, s2, torch.cuda.current_stream()):
        lr.linrec_check(s)


def test_host_threads_on_streams_of_their_own():
    """One host thread per entry point, each enqueuing on its own stream at the same time (the binding's calls
    run without the interpreter lock): the library's workspace table and plan cache are shared, the results
    must be those of the same calls made alone."""
    import threading
    calls = _calls()
    ref = {}
    for name, (fn, outs) in calls.items():
        fn()
        torch.cuda.synchronize()
        ref[name] = [t.clone() for t in outs]
        for t in outs:
            t.zero_()
    torch.cuda.synchronize()
    errors = []
    start = threading.Barrier(len(calls))

    def worker(name):
        try:
            torch.cuda.set_device(0)
            s = torch.cuda.Stream()
            start.wait(timeout=60)
            with torch.cuda.stream(s):
                for _ in range(20):
                    calls[name][0]()
            lr.linrec_check(s)
        except Exception as e:  # reported by the main thread
            errors.append(f"{name}: {e!r}")

    threads = [threading.Thread(target=worker, args=(name,)) for name in calls]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not any(t.is_alive() for t in threads), "a host thread did not finish"
    assert not errors, errors
    torch.cuda.synchronize()
    lr.linrec_check()
    for name, (fn, outs) in calls.items():
        assert all(_same(a, b) for a, b in zip(outs, ref[name])), f"{name}: differs from the call made alone"
    lr.linrec_release_workspace()


@pytest.mark.parametrize("name", ["gated", "lstm", "bf16", "gated_bf16", "lstm_bf16"])
def test_hip_graph_replay(name):
    fn, outs = _calls()[name]
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with options(variant=lr.VARIANT_LOOKBACK), torch.cuda.stream(s):
        for _ in range(2):                   # allocates the stream's workspace: not capturable
            fn()
        s.synchronize()
        ref = [t.clone() for t in outs]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            fn()
        for rep in range(3):
            say(f"{name}: graph replay {rep}")
            for t in outs:
                t.zero_()
            g.replay()
            s.synchronize()
            assert all(_same(a, b) for a, b in zip(outs, ref)), f"{name}: replay {rep} differs from eager"
            fn()                             # eager work on the same stream between replays
            s.synchronize()
        lr.linrec_check(s)


@pytest.mark.parametrize("taper", [2, 8])
def test_tapered_tail_tiles_every_entry_point(taper):
    """LINREC_OPT_TAPER (off by default) ends the sequence on half- and quarter-height tiles: same results
    to tolerance for every entry point that runs the single-pass kernel."""
    from parity import fwd_bwd_check
    from test_bf16_parity_gpu import bf16_check, to_bf16
    from test_gilr_parity_gpu import gated_check
    from test_lstm_parity_gpu import cell_check
    from test_forms_bf16_parity_gpu import cell16_check, gated16_check
    from test_forms_bf16_parity_gpu import to_bf16 as forms_to_bf16

    T = 40_000          # enough tiles per column for the tapered region to hold several short tiles
    with options(variant=lr.VARIANT_LOOKBACK, taper=taper):
        fwd_bwd_check(wl.make_generic(T, 1, 70, seed=31, device=DEV), f"taper {taper} plain")
        gated_check(wl.make_gated(T, 1, 70, seed=32, device=DEV, gate_mean=1.0), lr.TAU_TANH, f"taper {taper} gated")
        cell_check(wl.make_lstm(T, 1, 70, seed=33, device=DEV), f"taper {taper} lstm")
        bf16_check(to_bf16(wl.make_generic(T, 1, 72, seed=34, device=DEV)), f"taper {taper} bf16")
        gated16_check(forms_to_bf16(wl.make_gated(T, 1, 72, seed=35, device=DEV, gate_mean=1.0)), lr.TAU_TANH,
                      f"taper {taper} gated bf16")
        cell16_check(forms_to_bf16(wl.make_lstm(T, 1, 72, seed=36, device=DEV)), f"taper {taper} lstm bf16")


@pytest.mark.parametrize("family", ["gated", "lstm", "bf16"])
def test_walk_variant_every_tile_shape(family):
    """LINREC_VARIANT_WALK (one workgroup per column group goes through the sequence, no look-back) for the
    gated layer, the cell and bf16 storage: every tile shape the family has, ragged rows and columns, several
    tiles per column group, and the initial state."""
    from test_bf16_parity_gpu import BF16_TILES, bf16_check, to_bf16
    from test_gilr_parity_gpu import GATED_TILES, gated_check
    from test_lstm_parity_gpu import CELL_TILES, cell_check

    tiles = {"gated": GATED_TILES, "lstm": CELL_TILES, "bf16": BF16_TILES}[family]
    for tile in tiles:
        info = lr.linrec_tile_info(tile)
        T = 2 * info["rows"] + 37                      # three tiles per column group, the last one ragged
        C = 2 * info["cols"] + 4 * info["cols_per_thread"]
        with options(variant=lr.VARIANT_WALK, tile=tile):
            label = f"walk {family} tile {tile} T={T} C={C}"
            say(label)
            if family == "gated":
                assert lr.linrec_plan_for(lr.ENTRY_GILR, T, 1, C) == (lr.VARIANT_WALK, tile)
                gated_check(wl.make_gated(T, 1, C, seed=tile, device=DEV, gate_mean=1.0), lr.TAU_TANH, label)
            elif family == "lstm":
                assert lr.linrec_plan_for(lr.ENTRY_LSTM_CELL, T, 1, C) == (lr.VARIANT_WALK, tile)
                cell_check(wl.make_lstm(T, 1, C, seed=tile, device=DEV), label)
            else:
                assert lr.linrec_plan_for(lr.ENTRY_BF16, T, 1, C, alignment=8) == (lr.VARIANT_WALK, tile)
                bf16_check(to_bf16(wl.make_generic(T, 1, C, seed=tile, device=DEV)), label)


def test_short_wide_problems_walk_in_every_family():
    """The automatic plan of every family on short, wide problems is the walk wherever the plan table has it
    ahead of the single pass: each family takes it for several of these shapes, and is right where it does."""
    from parity import fwd_bwd_check
    from test_bf16_parity_gpu import bf16_check, to_bf16
    from test_gilr_parity_gpu import gated_check
    from test_lstm_parity_gpu import cell_check
    from test_forms_bf16_parity_gpu import cell16_check, gated16_check
    from test_forms_bf16_parity_gpu import to_bf16 as forms_to_bf16
    import numpy as np

    shapes = [(128, 16, 1024), (500, 4, 4100), (1000, 8, 4096), (64, 16, 1024), (250, 4, 1100), (1000, 4, 3072),
              (2048, 8, 4096), (77, 2, 9000), (2000, 16, 4096)]
    walked = {fam: 0 for fam in range(6)}
    for i, (T, B, n) in enumerate(shapes):
        C = B * n
        # (the larger problems on sampled columns: whole column groups of the widest tiles at both ends of a row)
        cols = None
        if T * C > 1 << 24:
            cols = np.unique(np.concatenate([np.arange(0, 256), np.arange(C - 256, C), np.arange(5, C, 997)]))
        checks = {
            lr.ENTRY_PLAIN: lambda: fwd_bwd_check(wl.make_inputs(2, T=T, B=B, n=n, device=DEV), f"auto walk plain {T}x{B}x{n}"),
            lr.ENTRY_GILR: lambda: gated_check(wl.make_gated(T, B, n, seed=51 + i, device=DEV, gate_mean=1.0), lr.TAU_TANH,
                                               f"auto walk gated {T}x{B}x{n}", cols=cols),
            lr.ENTRY_LSTM_CELL: lambda: cell_check(wl.make_lstm(T, B, n, seed=52 + i, device=DEV), f"auto walk lstm {T}x{B}x{n}", cols=cols),
            lr.ENTRY_BF16: lambda: bf16_check(to_bf16(wl.make_generic(T, B, n, seed=53 + i, device=DEV)),
                                              f"auto walk bf16 {T}x{B}x{n}", cols=cols),
            lr.ENTRY_GILR_BF16: lambda: gated16_check(forms_to_bf16(wl.make_gated(T, B, n, seed=54 + i, device=DEV, gate_mean=1.0)),
                                                      lr.TAU_TANH, f"auto walk gated bf16 {T}x{B}x{n}", cols=cols),
            lr.ENTRY_LSTM_CELL_BF16: lambda: cell16_check(forms_to_bf16(wl.make_lstm(T, B, n, seed=55 + i, device=DEV)),
                                                          f"auto walk lstm bf16 {T}x{B}x{n}", cols=cols),
        }
        for fam, check in checks.items():
            plans = [lr.linrec_plan_for(fam, T, B, n, backward=bwd, alignment=8) for bwd in (False, True)]
            if any(v == lr.VARIANT_WALK for v, _ in plans):
                say(f"family {fam} [{T}, {B}, {n}]: plans {plans}")
                walked[fam] += 1
                check()
    assert all(k >= 3 for k in walked.values()), walked
    # long sequences never walk
    for fam in range(6):
        assert lr.linrec_plan_for(fam, 65536, 4, 4096, alignment=8)[0] == lr.VARIANT_LOOKBACK


def test_automatic_tapered_tail_in_every_family():
    """Where the static plan cuts the end of a launch into shorter tiles by itself (no option set), the results are
    right: per family, the first few problems of a list whose plan has a tapered tail."""
    from parity import fwd_bwd_check
    from test_bf16_parity_gpu import bf16_check, to_bf16
    from test_gilr_parity_gpu import gated_check
    from test_lstm_parity_gpu import cell_check
    from test_forms_bf16_parity_gpu import cell16_check, gated16_check
    from test_forms_bf16_parity_gpu import to_bf16 as forms_to_bf16

    assert lr.linrec_get_option(lr.OPT_TAPER) == -1
    shapes = [(2 ** lt, 1, C) for lt in range(10, 16) for C in (96, 256, 768, 1024, 2048, 4096)]
    total = 0
    for fam in range(6):
        hits = [s for s in shapes if lr.linrec_plan_taper(fam, *s, backward=False) or lr.linrec_plan_taper(fam, *s, backward=True)]
        for i, (T, B, n) in enumerate(hits[:3]):
            label = f"automatic taper, family {fam} [{T}, {n}]"
            say(label)
            total += 1
            if fam == lr.ENTRY_PLAIN:
                fwd_bwd_check(wl.make_inputs(2, T=T, B=B, n=n, device=DEV), label)
            elif fam == lr.ENTRY_GILR:
                gated_check(wl.make_gated(T, B, n, seed=61 + i, device=DEV, gate_mean=1.0), lr.TAU_TANH, label)
            elif fam == lr.ENTRY_LSTM_CELL:
                cell_check(wl.make_lstm(T, B, n, seed=62 + i, device=DEV), label)
            elif fam == lr.ENTRY_BF16:
                bf16_check(to_bf16(wl.make_generic(T, B, n, seed=63 + i, device=DEV)), label)
            elif fam == lr.ENTRY_GILR_BF16:
                gated16_check(forms_to_bf16(wl.make_gated(T, B, n, seed=64 + i, device=DEV, gate_mean=1.0)), lr.TAU_TANH, label)
            else:
                cell16_check(forms_to_bf16(wl.make_lstm(T, B, n, seed=65 + i, device=DEV)), label)
    assert total >= 6


def test_staggered_start_changes_timing_only():
    """LINREC_OPT_STAGGER delays every other workgroup of the first round: bit-identical results for every
    entry point, whatever the delay, on a problem several rounds of workgroups long."""
    T, B, n = 49_152, 4, 256
    plain = wl.make_inputs(2, T=T, B=B, n=n, device=DEV)
    gated = wl.make_gated(T, B, n, seed=41, device=DEV, gate_mean=1.0)
    cell = wl.make_lstm(T, B, n, seed=42, device=DEV)
    pre = [cell[k] for k in ("f_pre", "i_pre", "z_pre", "o_pre")]
    half = {k: (v.to(torch.bfloat16) if torch.is_tensor(v) else v) for k, v in plain.items()}
    gated16 = {k: (v.to(torch.bfloat16) if torch.is_tensor(v) else v) for k, v in gated.items()}
    cell16 = {k: (v.to(torch.bfloat16) if torch.is_tensor(v) else v) for k, v in cell.items()}
    pre16 = [cell16[k] for k in ("f_pre", "i_pre", "z_pre", "o_pre")]

    def run_all():
        h = lr.linrec_forward(plain["lam"], plain["x"], plain["h0"])
        out = [h, *lr.linrec_backward(plain["lam"], h, plain["h0"], plain["grad_h"])]
        hg = lr.linrec_gilr_forward(gated["g_pre"], gated["i_pre"], gated["h0"])
        out += [hg, *lr.linrec_gilr_backward(gated["g_pre"], gated["i_pre"], hg, gated["h0"], gated["grad_h"])]
        c, hc = lr.linrec_lstm_cell_forward(*pre, cell["c0"])
        out += [c, hc, *lr.linrec_lstm_cell_backward(*pre, c, cell["c0"], cell["grad_h"])]
        hb = lr.linrec_forward(half["lam"], half["x"], half["h0"])
        out += [hb, *lr.linrec_backward(half["lam"], hb, half["h0"], half["grad_h"])]
        hg16 = lr.linrec_gilr_forward(gated16["g_pre"], gated16["i_pre"], gated16["h0"])
        out += [hg16, *lr.linrec_gilr_backward(gated16["g_pre"], gated16["i_pre"], hg16, gated16["h0"], gated16["grad_h"])]
        c16, hc16 = lr.linrec_lstm_cell_forward(*pre16, cell16["c0"])
        out += [c16, hc16, *lr.linrec_lstm_cell_backward(*pre16, c16, cell16["c0"], cell16["grad_h"])]
        torch.cuda.synchronize()
        lr.linrec_check()
        return out

    with options(variant=lr.VARIANT_LOOKBACK, stagger=0):
        ref = run_all()
    for stagger in (3, 16):
        with options(variant=lr.VARIANT_LOOKBACK, stagger=stagger):
            got = run_all()
        assert all(_same(a, b) for a, b in zip(got, ref)), f"stagger {stagger} changed a result"


def test_rows_too_long_for_32_bit_tile_offsets_fall_back_to_the_serial_kernel():
    """A tile addresses its rows with 32-bit byte offsets; when rows*C*4 does not fit, every entry point
    must take the serial kernel by itself (and still be right)."""
    from parity import fwd_bwd_check
    from test_bf16_parity_gpu import bf16_check, to_bf16
    from test_gilr_parity_gpu import gated_check
    from test_lstm_parity_gpu import cell_check
    from test_forms_bf16_parity_gpu import cell16_check, gated16_check
    from test_forms_bf16_parity_gpu import to_bf16 as forms_to_bf16

    big = 1 << 25                           # 128 MiB rows: no tile shape can address even 32 of them
    assert lr.linrec_plan(4, 1, big)[0] == lr.VARIANT_SERIAL
    fwd_bwd_check(wl.make_generic(4, 1, big, seed=41, device=DEV), "long rows plain")
    gated_check(wl.make_gated(4, 1, big, seed=42, device=DEV), lr.TAU_TANH, "long rows gated",
                cols=list(range(0, big, big // 64)))
    cell_check(wl.make_lstm(4, 1, big, seed=43, device=DEV), "long rows lstm", cols=list(range(0, big, big // 64)))
    bf16_check(to_bf16(wl.make_generic(4, 1, big, seed=44, device=DEV)), "long rows bf16",
               cols=list(range(0, big, big // 64)))
    big16 = 1 << 26                         # (2-byte elements: twice the columns for the same row length)
    assert lr.linrec_plan_for(lr.ENTRY_GILR_BF16, 4, 1, big16)[0] == lr.VARIANT_SERIAL
    gated16_check(forms_to_bf16(wl.make_gated(4, 1, big16, seed=45, device=DEV)), lr.TAU_TANH, "long rows gated bf16",
                  cols=list(range(0, big16, big16 // 64)))
    cell16_check(forms_to_bf16(wl.make_lstm(4, 1, big16, seed=46, device=DEV)), "long rows lstm bf16",
                 cols=list(range(0, big16, big16 // 64)))


def test_tuned_plans_of_every_family_are_used_and_correct():
    """linrec_tune_for() times the candidate shapes of a family on scratch tensors; later calls with that
    shape use the winner (linrec_plan_for reports it) and stay correct whatever it picked."""
    from parity import fwd_bwd_check
    from test_bf16_parity_gpu import bf16_check, to_bf16
    from test_gilr_parity_gpu import gated_check
    from test_lstm_parity_gpu import cell_check
    from test_forms_bf16_parity_gpu import cell16_check, gated16_check
    from test_forms_bf16_parity_gpu import to_bf16 as forms_to_bf16

    T, B, n = 20000, 2, 96
    for family in (lr.ENTRY_PLAIN, lr.ENTRY_GILR, lr.ENTRY_LSTM_CELL, lr.ENTRY_BF16, lr.ENTRY_GILR_BF16,
                   lr.ENTRY_LSTM_CELL_BF16):
        for bwd in (False, True):
            lr.linrec_tune_for(family, T, B, n, backward=bwd)
            v, t = lr.linrec_plan_for(family, T, B, n, backward=bwd, alignment=16)
            say(f"family {family} backward={bwd}: tuned tile {t}")
            assert v == lr.VARIANT_LOOKBACK and lr.linrec_tile_info(t) is not None
    fwd_bwd_check(wl.make_inputs(2, T=T, B=B, n=n, device=DEV), "tuned plain")
    gated_check(wl.make_gated(T, B, n, seed=51, device=DEV, gate_mean=1.0), lr.TAU_TANH, "tuned gated")
    cell_check(wl.make_lstm(T, B, n, seed=52, device=DEV), "tuned lstm")
    bf16_check(to_bf16(wl.make_inputs(2, T=T, B=B, n=n, device=DEV)), "tuned bf16")
    gated16_check(forms_to_bf16(wl.make_gated(T, B, n, seed=53, device=DEV, gate_mean=1.0)), lr.TAU_TANH, "tuned gated bf16")
    cell16_check(forms_to_bf16(wl.make_lstm(T, B, n, seed=54, device=DEV)), "tuned lstm bf16")
    with pytest.raises(lr.LinrecError):
        lr.linrec_tune_for(7, T, B, n)


def test_stream_probes_compute_what_the_header_says():
    """The measurement kernels are not part of the recurrence, but a probe that skipped or doubled part of its
    arrays would time the wrong number of bytes: every element is checked, in both geometries."""
    T, C = 96, 1024
    g = torch.Generator(device=DEV)
    g.manual_seed(7)
    a, b, c = (torch.rand((T, C), device=DEV, generator=g) + 0.5 for _ in range(3))
    for rows in (False, True):
        call = (lambda *t: lr.linrec_stream_probe_rows(*t, T, C)) if rows else lr.linrec_stream_probe
        for ins, n_out in (((a, None, None), 1), ((a, b, None), 1), ((a, b, c), 2)):
            o0, o1 = torch.full_like(a, float("nan")), torch.full_like(a, float("nan"))
            call(*ins, o0, o1 if n_out == 2 else None)
            torch.cuda.synchronize()
            want = ins[0] * (ins[1] if ins[1] is not None else 1.0) + (ins[2] if ins[2] is not None else 0.0)
            # (the kernels may fuse the multiply and the add: one rounding less than torch's two)
            torch.testing.assert_close(o0, want, rtol=1e-6, atol=0)
            if n_out == 2:
                torch.testing.assert_close(o1, want * want, rtol=1e-6, atol=0)
        o0 = torch.full_like(a, float("nan"))
        call(None, None, None, o0, None)                          # write-only: every element is written
        call(a, None, None, None, None)                           # read-only: runs, writes nothing
        torch.cuda.synchronize()
        assert bool(torch.isfinite(o0).all())
