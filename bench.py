#!/usr/bin/env python3
"""Benchmark of the linear-recurrence hot path on one MI355X.

A step is one forward pass plus one backward pass of h_t = lambda_t*h_{t-1} + x_t over one batch of
synthetic, HBM-resident inputs.  The headline workload is the largest of the five that fits one GPU,
workload 5 ([T=262144, B=8, n=512] fp32, 1.07e9 elements); workloads 2 and 3 (the other two with
T >= 65536: 65536 steps at 256 hidden units, and the one-million-step regime of Section 4.2) and workload 4
(4096 steps of a wide layer) are timed in the same run and reported beside it.  Prints ONE JSON line:

  value         elements/s of forward+backward together on the headline workload, E / ms_per_step, E = T*B*n
                (K steps, wall clock between two device synchronisations, nothing else on the stream)
  roofline      the dominant kernel (the backward pass, 20 B/element) against the 8 TB/s HBM peak, its
                duration measured with HIP events on the launch stream over a second run of the K steps;
                frac_of_stream_probe relates it to what the library's pure streaming kernel reaches on this machine with the
                same streams in and out (flat arrays, or rows of 256 lanes like a wide tile: whichever is faster),
                frac_of_read_write_ceiling to what the box allows this mix of reads and writes (bytes read at the
                rate of a read-only kernel plus bytes written at the rate of a write-only one)
  per_workload  forward / backward time and fraction of the HBM peak for workloads 2, 3, 4 and 5
  cpu_baseline  the fp64 oracle timed on the host cores on the headline workload (at most 2^30 elements of it), streamed
                in slabs of rows with a carried fp64 state, once on one thread and once on all the cores this
                process may use (a baseline, not a target)

The library's static plan is what is timed: no tuning run precedes the measurement (--tune adds one).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
VARIANT_NAMES = {1: "threephase", 2: "lookback", 3: "serial", 4: "walk"}    # LINREC_VARIANT_*
FWD_BYTES_PER_EL = 12.0   # read lambda, x; write h
BWD_BYTES_PER_EL = 20.0   # read lambda, h, grad_h; write grad_x, grad_lambda


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5, help="headline workload 1..5 (default 5, the largest)")
    ap.add_argument("--also", default="auto",
                    help="comma-separated workloads timed beside the headline one and reported in per_workload "
                         "(default: 2,3,4 when the headline is workload 5 in fp32, else none; '' for none)")
    ap.add_argument("--variant", default="auto", choices=["auto", "threephase", "lookback", "serial", "walk"])
    ap.add_argument("--tile-fwd", type=int, default=0, help="pin this tile shape for the headline workload's forward pass")
    ap.add_argument("--tile-bwd", type=int, default=0, help="pin this tile shape for the headline workload's backward pass")
    ap.add_argument("--hprev-late", type=int, default=-1)
    ap.add_argument("--tune", action="store_true",
                    help="run linrec_tune() on every timed shape first and time the plan it remembers "
                         "(default: the library's static plan)")
    ap.add_argument("--no-tune", action="store_true", help="accepted for older command lines; the default now")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-threads", type=int, default=0)
    ap.add_argument("--cpu-sample-elements", type=int, default=1 << 30,
                    help="elements of the headline workload (whole rows from row 0) the oracle is timed on; the default "
                         "covers all of workload 5 (a few seconds of host time per leg)")
    ap.add_argument("--walk-grid", action="store_true",
                    help="short, wide problems: the walk variant against the single pass, and what the plan takes")
    ap.add_argument("--table1", action="store_true",
                    help="instead of the workload benchmark, time the parallel (single-pass) kernel against the "
                         "serial-over-T kernel on the grid of the paper's Table 1 (minibatch 1; 4, 32, 128 features; "
                         "T = 16 ... 65536) and print the speed-up ratios as one JSON line")
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"],
                    help="storage type of the tensors (bf16: linrec_forward_bf16 / linrec_backward_bf16, 6 and 10 "
                         "bytes per element; the arithmetic is fp32 either way)")
    ap.add_argument("--gated", default="", choices=["", "g2", "g3", "g4", "g5"],
                    help="time the gated (GILR) entry points on this workload instead (sigmoid / tanh applied in the "
                         "scan kernel: 12 B/element forward, 24 backward), next to the unfused sequence "
                         "elementwise kernels + linrec_forward")
    ap.add_argument("--lstm", default="", choices=["", "l2", "l4", "l5"],
                    help="time the LSTM-cell entry points on this workload instead (24 B/element forward, 40 backward), "
                         "next to the unfused forward")
    ap.add_argument("--probe", action="store_true", help="accepted for older command lines; the default now")
    ap.add_argument("--no-probe", action="store_true",
                    help="skip the library's pure streaming kernels (copy, 2-in/1-out, 3-in/2-out); the copy doubles "
                         "as the calibration kernel for byte counters, so counter runs keep it")
    return ap.parse_args()


def host_cores():
    """(cores of the box, cores this process may run on, threads the oracle's all-core leg uses)."""
    box = os.cpu_count() or 1
    mine = len(os.sched_getaffinity(0))
    return box, mine, max(1, min(16, mine))


def cpu_baseline(inp, h_gpu, threads, sample_elements):
    """Times the fp64 oracle (forward + backward) on the host over the first rows of the workload, streamed
    in slabs of rows with the fp64 state carried from slab to slab (so no full-size fp64 tensor exists), once
    on one thread and once on `threads`.  Only the time inside the oracle's C loops is counted.  The sample is
    treated as a sequence of its own (the backward pass starts at its last row)."""
    import numpy as np

    import oracle
    T, B, n = inp["T"], inp["B"], inp["n"]
    C = B * n
    Ts = max(1, min(T, sample_elements // C))
    f = lambda t: None if t is None else t[:Ts].float().cpu().numpy().reshape(Ts, C)   # (bf16 values widen exactly)
    lam, x, e, h32 = f(inp["lam"]), f(inp["x"]), f(inp["grad_h"]), f(h_gpu)
    h0 = None if inp["h0"] is None else inp["h0"].float().cpu().numpy().reshape(-1)
    oracle.build()
    slab = max(1, min(Ts, (1 << 24) // C))
    href = np.empty((slab, C), np.float64)
    gx, gl = np.empty((slab + 2, C), np.float64), np.empty((slab + 2, C), np.float64)

    def one_pass(nthreads):
        state = np.zeros(C, np.float64) if h0 is None else h0.astype(np.float64)
        t_fwd = t_bwd = 0.0
        for t0 in range(0, Ts, slab):
            t1 = min(Ts, t0 + slab)
            t = time.perf_counter()
            oracle.forward_slab(lam[t0:t1], x[t0:t1], state, href, 0, t1 - t0, nthreads)
            t_fwd += time.perf_counter() - t
        if e is not None:
            g, gh0 = np.zeros(C, np.float64), np.zeros(C, np.float64)
            t1 = Ts
            while t1 > 0:
                t0 = max(0, t1 - slab)
                base, top = max(t0 - 1, 0), min(t1 + 1, Ts)     # one row of halo either side (lambda[t+1], h[t-1])
                t = time.perf_counter()
                oracle.backward_slab(lam[base:top], h32[base:top], h0 if t0 == 0 else None, e[base:top], g, gx, gl, gh0,
                                     t0 - base, t1 - base, nthreads)
                t_bwd += time.perf_counter() - t
                t1 = t0
        return t_fwd, t_bwd

    f1, b1 = one_pass(1)
    fa, ba = one_pass(threads)
    box, mine, _ = host_cores()
    Es = Ts * C
    return {"value": Es / (fa + ba), "unit": "elements/s", "cores": threads, "kind": "oracle",
            "value_1thread": Es / (f1 + b1), "host_cores": box, "cores_available_to_this_process": mine,
            "sample": f"rows 0..{Ts - 1} of the workload ({Es} of {T * C} elements, all {C} columns), one forward + one "
                      f"backward pass of the fp64 oracle streamed in slabs of {slab} rows with a carried fp64 state; "
                      f"{threads} threads (columns split): forward {fa:.3f} s, backward {ba:.3f} s; "
                      f"1 thread: forward {f1:.3f} s, backward {b1:.3f} s"}


def measured_traffic(cfg, direction, form="", expect=None, kernel="lookback"):
    """HBM bytes per launch of the look-back kernel (or the walk) from the committed rocprofv3 counter summary
    (profiles/hbm_traffic_cfg<N>.json or hbm_traffic_<gated/lstm workload>.json, written by
    profile_summary.py traffic), or None.  `expect` is the tile geometry "vec, rows, wc, wt" of the plan
    that was just timed: a summary taken on another kernel instance says nothing about this run and is not
    reported."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{cfg}.json" if form else f"hbm_traffic_cfg{cfg}.json")
    try:
        with open(path) as f:
            d = json.load(f)
        k = d["kernels"][form + "k_" + kernel + "/" + direction]
        if expect is not None and f"Geo<{expect}," not in k["name"]:
            return None
        return k["hbm_bytes"]
    except (OSError, KeyError, ValueError):
        return None


def tile_geometry(lr, tile_id):
    """ "vec, rows per thread, threads along columns, threads along time" as the kernel names spell it."""
    i = lr.linrec_tile_info(tile_id)
    return None if i is None else f"{i['cols_per_thread']}, {i['rows_per_thread']}, {i['threads_cols']}, {i['threads_time']}"


def stream_probe(lr, torch, E, stream, iters=10):
    """GB/s of the library's streaming kernels on E-element arrays (no recurrence, same access instructions)."""
    bufs = [torch.rand(E, device="cuda:0") for _ in range(3)] + [torch.empty(E, device="cuda:0") for _ in range(2)]
    a, b, c, o0, o1 = bufs
    res = {}
    for name, argv, nbytes in (("copy_1in_1out", (a, None, None, o0, None), 8), ("fwd_like_2in_1out", (a, b, None, o0, None), 12),
                               ("bwd_like_3in_2out", (a, b, c, o0, o1), 20), ("read_only", (a, None, None, None, None), 4),
                               ("write_only", (None, None, None, o0, None), 4)):
        for _ in range(2):
            lr.linrec_stream_probe(*argv, stream=stream)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
        ev[0].record(stream)
        for i in range(iters):
            lr.linrec_stream_probe(*argv, stream=stream)
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        ms = sum(ev[i].elapsed_time(ev[i + 1]) for i in range(iters)) / iters
        res[name] = {"avg_ms": ms, "GB/s": nbytes * E / (ms * 1e-3) / 1e9, "bytes_per_element": nbytes}
    # the same mixes in the geometry of a tile ([T, 4096] arrays; 256 lanes side by side, 16 rows per thread)
    C = 4096
    T = E // C // 32 * 32
    if T > 0:
        view = [t[:T * C] for t in bufs]
        a, b, c, o0, o1 = view
        for name, argv, nbytes in (("rows_fwd_like_2in_1out", (a, b, None, o0, None), 12), ("rows_bwd_like_3in_2out", (a, b, c, o0, o1), 20),
                                   ("rows_read_only", (a, None, None, None, None), 4), ("rows_write_only", (None, None, None, o0, None), 4)):
            for _ in range(2):
                lr.linrec_stream_probe_rows(*argv, T, C, stream=stream)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
            ev[0].record(stream)
            for i in range(iters):
                lr.linrec_stream_probe_rows(*argv, T, C, stream=stream)
                ev[i + 1].record(stream)
            torch.cuda.synchronize()
            ms = sum(ev[i].elapsed_time(ev[i + 1]) for i in range(iters)) / iters
            res[name] = {"avg_ms": ms, "GB/s": nbytes * T * C / (ms * 1e-3) / 1e9, "bytes_per_element": nbytes}
    res["elements"] = E
    return res


def read_write_ceiling(probe, read_bytes, write_bytes):
    """What this box's memory allows a kernel that moves `read_bytes` in and `write_bytes` out per element: its bytes
    read at the rate of a kernel that only reads plus its bytes written at the rate of one that only writes (on an
    MI355X writes stream at about 80 % of the rate of reads, so no mix reaches what reads alone do)."""
    best = lambda k: max(probe[k]["GB/s"], probe.get("rows_" + k, probe[k])["GB/s"])     # the faster of the two geometries
    return (read_bytes + write_bytes) / (read_bytes / best("read_only") + write_bytes / best("write_only"))


def like_probe(probe, key):
    """The streaming rate the dominant kernel is measured against: the probe with the kernel's mix of streams in
    and out, in whichever of its two geometries (flat arrays, or the tiles' rows) is faster on this machine."""
    return max(probe[key]["GB/s"], probe.get("rows_" + key, probe[key])["GB/s"])


def table1(lr, torch):
    """Parallel / serial kernel throughput ratio on the paper's Table-1 grid (forward pass, b = 1)."""
    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    grid = {}
    for T in (16, 256, 4096, 65536):
        for m in (4, 32, 128):
            g = torch.Generator(device=dev)
            g.manual_seed(1709 + T + m)
            lam = torch.sigmoid(torch.randn((T, 1, m), device=dev, generator=g))
            x = torch.randn((T, 1, m), device=dev, generator=g)
            h = torch.empty_like(x)
            times = {}
            for name, variant in (("parallel", lr.VARIANT_LOOKBACK), ("serial", lr.VARIANT_SERIAL)):
                lr.linrec_set_option(lr.OPT_VARIANT, variant)
                iters = 200 if T <= 4096 else 30
                for _ in range(5):
                    lr.linrec_forward(lam, x, None, h_out=h, stream=stream)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(iters):
                    lr.linrec_forward(lam, x, None, h_out=h, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                times[name] = e0.elapsed_time(e1) / iters * 1e3   # microseconds per launch, back to back
            grid[f"T={T},m={m}"] = {"parallel_us": times["parallel"], "serial_us": times["serial"],
                                    "speedup": times["serial"] / times["parallel"],
                                    "parallel_events_per_s": T / (times["parallel"] * 1e-6)}
    lr.linrec_set_option(lr.OPT_VARIANT, lr.VARIANT_AUTO)
    return grid


def walk_grid(lr, torch, wl):
    """Short, wide problems: the walk (one workgroup per column group, no look-back) against the single pass,
    each with the shape the library picks for it; microseconds per launch, forward / backward, and what the
    automatic plan takes.  Plain fp32 recurrence, workload 2's value distributions."""
    dev = "cuda:0"
    stream = torch.cuda.current_stream()
    names = {lr.VARIANT_LOOKBACK: "lookback", lr.VARIANT_WALK: "walk"}
    grid = {}
    for T in (256, 512, 1024, 2048, 4096, 8192):
        for C in (4096, 8192, 16384, 32768, 65536):
            if T * C > 1 << 27:
                continue
            B, n = 4, C // 4
            inp = wl.make_inputs(2, T=T, B=B, n=n, device=dev)
            h = torch.empty_like(inp["x"])
            gx, gl = torch.empty_like(h), torch.empty_like(h)
            gh0 = torch.empty((B, n), device=dev)
            fwd = lambda: lr.linrec_forward(inp["lam"], inp["x"], inp["h0"], h_out=h, stream=stream)
            bwd = lambda: lr.linrec_backward(inp["lam"], h, inp["h0"], inp["grad_h"], grad_x=gx, grad_lambda=gl,
                                             grad_h0=gh0, stream=stream)
            rec = {"auto_plan": [names.get(lr.linrec_plan(T, B, n, backward=b)[0], "other") for b in (False, True)]}
            for variant in (lr.VARIANT_LOOKBACK, lr.VARIANT_WALK):
                lr.linrec_set_option(lr.OPT_VARIANT, variant)
                us = []
                for call in (fwd, bwd):
                    for _ in range(3):
                        call()
                    torch.cuda.synchronize()
                    ev = [torch.cuda.Event(enable_timing=True) for _ in range(11)]
                    ev[0].record(stream)
                    for i in range(10):
                        call()
                        ev[i + 1].record(stream)
                    torch.cuda.synchronize()
                    us.append(sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(10))[5] * 1e3)
                rec[names[variant] + "_us"] = us
                rec[names[variant] + "_tile"] = [lr.linrec_plan(T, B, n, backward=b)[1] for b in (False, True)]
            lr.linrec_set_option(lr.OPT_VARIANT, lr.VARIANT_AUTO)
            rec["walk_speedup"] = [rec["lookback_us"][i] / rec["walk_us"][i] for i in (0, 1)]
            grid[f"T={T},C={C}"] = rec
    return grid


def gated_bench(args, lr, torch, wl):
    """One JSON line for the gated entry points: per-pass times, GB/s against the 12 / 24 algorithmic
    bytes per element, and the unfused forward (activation kernels, then the plain scan) beside it."""
    dev = "cuda:0"
    spec = wl.GATED[args.gated]
    T, B, n = spec["T"], spec["B"], spec["n"]
    E = T * B * n
    inp = wl.make_gated(T, B, n, seed=sum(map(ord, args.gated)), device=dev, gate_mean=spec["gate_mean"],
                        gate_std=spec["gate_std"])
    bf16 = args.dtype == "bf16"   # bf16 storage: half the bytes, the same arithmetic
    if bf16:
        inp = {k: (v.to(torch.bfloat16).contiguous() if torch.is_tensor(v) else v) for k, v in inp.items()}
    g_pre, i_pre, h0, e = inp["g_pre"], inp["i_pre"], inp["h0"], inp["grad_h"]
    h = torch.empty_like(g_pre)
    gg, gi = torch.empty_like(g_pre), torch.empty_like(g_pre)
    gh0 = torch.empty_like(h0)
    lam, x = torch.empty_like(g_pre), torch.empty_like(g_pre)
    stream = torch.cuda.current_stream()
    K = args.steps
    family = lr.ENTRY_GILR_BF16 if bf16 else lr.ENTRY_GILR
    bpe_f, bpe_b = (6.0, 12.0) if bf16 else (12.0, 24.0)

    if args.tune:
        lr.linrec_tune_for(family, T, B, n, backward=False, stream=stream)
        lr.linrec_tune_for(family, T, B, n, backward=True, stream=stream)

    def fused_fwd():
        lr.linrec_gilr_forward(g_pre, i_pre, h0, h_out=h, stream=stream)

    def fused_bwd():
        lr.linrec_gilr_backward(g_pre, i_pre, h, h0, e, grad_g_pre=gg, grad_i_pre=gi, grad_h0=gh0, stream=stream)

    def unfused_fwd():  # what a framework does without the fused kernel: 3 elementwise kernels, then the scan
        torch.sigmoid(g_pre, out=lam)
        torch.tanh(i_pre, out=x)
        torch.addcmul(x, lam, x, value=-1.0, out=x)      # x = (1 - lam) * tanh(i_pre)
        lr.linrec_forward(lam, x, h0, h_out=h, stream=stream)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
        torch.cuda.synchronize()
        ev[0].record(stream)
        for i in range(K):
            fn()
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(K))
        return sum(ms) / K, ms[0]

    f_avg, f_min = timed(fused_fwd)
    b_avg, b_min = timed(fused_bwd)
    u_avg, u_min = timed(unfused_fwd)
    lr.linrec_check(stream)
    gbs = lambda bpe, ms: bpe * E / (ms * 1e-3) / 1e9
    out = {
        "metric": "gated linrec (GILR) fwd+bwd elements/sec and achieved HBM GB/s (% of MI355X peak)",
        "value": E / ((f_avg + b_avg) * 1e-3), "unit": "elements/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": f_avg + b_avg, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 arithmetic on bf16 storage" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.gated}: gated forward+backward, {'bf16 storage' if bf16 else 'fp32'}, time-major "
                               f"[T={T}, B={B}, n={n}], tau=tanh; " + spec["note"],
                   "variant_fwd": VARIANT_NAMES.get(lr.linrec_plan_for(family, T, B, n, backward=False)[0], "?"),
                   "tile_fwd": lr.linrec_plan_for(family, T, B, n, backward=False)[1],
                   "variant_bwd": VARIANT_NAMES.get(lr.linrec_plan_for(family, T, B, n, backward=True)[0], "?"),
                   "tile_bwd": lr.linrec_plan_for(family, T, B, n, backward=True)[1]},
        "forward": {"avg_ms": f_avg, "min_ms": f_min, "GB/s": gbs(bpe_f, f_avg), "frac_of_peak": gbs(bpe_f, f_avg) / HBM_PEAK_GBS},
        "backward": {"avg_ms": b_avg, "min_ms": b_min, "GB/s": gbs(bpe_b, b_avg), "frac_of_peak": gbs(bpe_b, b_avg) / HBM_PEAK_GBS},
        "unfused_forward": {"avg_ms": u_avg, "min_ms": u_min, "speedup_of_fused": u_avg / f_avg,
                            "what": "torch.sigmoid, torch.tanh, torch.addcmul, then linrec_forward"},
        "roofline": {"bound": "hbm",
                     "kernel": "gated backward pass (%s kernel)" % VARIANT_NAMES.get(lr.linrec_plan_for(family, T, B, n, backward=True)[0], "?"),
                     "achieved": gbs(bpe_b, b_avg),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs(bpe_b, b_avg) / HBM_PEAK_GBS, "traffic": None,
                     "bytes_per_element": bpe_b, "algorithmic_bytes": bpe_b * E, "avg_ms": b_avg},
        "cpu_baseline": None,
    }
    if not bf16:
        out["roofline"]["traffic"] = measured_traffic(args.gated, "backward", "gated:",
                                                      tile_geometry(lr, out["config"]["tile_bwd"]),
                                                      kernel=out["config"]["variant_bwd"])
    if not args.no_probe:
        out["stream_probe"] = stream_probe(lr, torch, min(E, 1 << 28), stream)
        ceiling = read_write_ceiling(out["stream_probe"], 4.0, 2.0)      # backward: four tensors in, two out
        out["roofline"]["read_write_ceiling_GB/s"] = ceiling
        out["roofline"]["frac_of_read_write_ceiling"] = out["roofline"]["achieved"] / ceiling
    if not args.no_cpu_baseline:
        import oracle
        threads = args.cpu_threads or min(16, len(os.sched_getaffinity(0)))
        C = B * n
        Ts = min(T, (1 << 27) // C)               # a bounded sample: the first rows, at most 2^27 elements
        f = lambda t: t[:Ts].float().cpu().numpy().reshape(-1, C)
        gp, ip, ee, hh = f(g_pre), f(i_pre), f(e), f(h)
        h0v = h0.float().cpu().numpy().reshape(-1)
        oracle.build()
        t0 = time.perf_counter()
        oracle.gilr_forward(gp, ip, h0v, threads=threads)
        t1 = time.perf_counter()
        oracle.gilr_backward(gp, ip, hh, h0v, ee, threads=threads)
        t2 = time.perf_counter()
        out["cpu_baseline"] = {"value": Ts * C / (t2 - t0), "unit": "elements/s", "cores": threads, "kind": "oracle",
                               "sample": f"{'the full workload' if Ts == T else f'the first {Ts} of {T} rows'}, one forward + one "
                                         f"backward pass of the fp64 oracle of the gated layer over {threads} host threads; "
                                         f"forward {t1 - t0:.3f} s, backward {t2 - t1:.3f} s"}
    print(json.dumps(out), flush=True)


def lstm_bench(args, lr, torch, wl):
    """One JSON line for the LSTM-cell entry points (Section 3.2's GILR-LSTM cell)."""
    dev = "cuda:0"
    spec = wl.LSTM[args.lstm]
    T, B, n = spec["T"], spec["B"], spec["n"]
    E = T * B * n
    inp = wl.make_lstm(T, B, n, seed=sum(map(ord, args.lstm)), device=dev, forget_mean=spec["forget_mean"])
    bf16 = args.dtype == "bf16"   # bf16 storage: half the bytes, the same arithmetic
    if bf16:
        inp = {k: (v.to(torch.bfloat16).contiguous() if torch.is_tensor(v) else v) for k, v in inp.items()}
    pre = [inp[k] for k in ("f_pre", "i_pre", "z_pre", "o_pre")]
    c0, e = inp["c0"], inp["grad_h"]
    c, h = torch.empty_like(e), torch.empty_like(e)
    grads = [torch.empty_like(e) for _ in range(4)]
    gc0 = torch.empty_like(c0)
    lam, x, og = torch.empty_like(e), torch.empty_like(e), torch.empty_like(e)
    stream = torch.cuda.current_stream()
    K = args.steps
    family = lr.ENTRY_LSTM_CELL_BF16 if bf16 else lr.ENTRY_LSTM_CELL
    bpe_f, bpe_b = (12.0, 20.0) if bf16 else (24.0, 40.0)

    if args.tune:
        lr.linrec_tune_for(family, T, B, n, backward=False, stream=stream)
        lr.linrec_tune_for(family, T, B, n, backward=True, stream=stream)

    def fused_fwd():
        lr.linrec_lstm_cell_forward(*pre, c0, c_out=c, h_out=h, stream=stream)

    def fused_bwd():
        lr.linrec_lstm_cell_backward(*pre, c, c0, e, grads=grads, grad_c0=gc0, stream=stream)

    def unfused_fwd():  # 6 elementwise kernels around the plain scan
        torch.sigmoid(pre[0], out=lam)
        torch.sigmoid(pre[1], out=x)
        torch.tanh(pre[2], out=og)
        torch.mul(x, og, out=x)
        lr.linrec_forward(lam, x, c0, h_out=c, stream=stream)
        torch.sigmoid(pre[3], out=og)
        torch.mul(og, c, out=h)

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
        torch.cuda.synchronize()
        ev[0].record(stream)
        for i in range(K):
            fn()
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(K))
        return sum(ms) / K, ms[0]

    f_avg, f_min = timed(fused_fwd)
    b_avg, b_min = timed(fused_bwd)
    u_avg, u_min = timed(unfused_fwd)
    lr.linrec_check(stream)
    gbs = lambda bpe, ms: bpe * E / (ms * 1e-3) / 1e9
    out = {
        "metric": "LSTM-cell linrec fwd+bwd elements/sec and achieved HBM GB/s (% of MI355X peak)",
        "value": E / ((f_avg + b_avg) * 1e-3), "unit": "elements/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": f_avg + b_avg, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 arithmetic on bf16 storage" if bf16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.lstm}: LSTM cell forward+backward, {'bf16 storage' if bf16 else 'fp32'}, time-major "
                               f"[T={T}, B={B}, n={n}]; " + spec["note"],
                   "variant_fwd": VARIANT_NAMES.get(lr.linrec_plan_for(family, T, B, n, backward=False)[0], "?"),
                   "tile_fwd": lr.linrec_plan_for(family, T, B, n, backward=False)[1],
                   "variant_bwd": VARIANT_NAMES.get(lr.linrec_plan_for(family, T, B, n, backward=True)[0], "?"),
                   "tile_bwd": lr.linrec_plan_for(family, T, B, n, backward=True)[1]},
        "forward": {"avg_ms": f_avg, "min_ms": f_min, "GB/s": gbs(bpe_f, f_avg), "frac_of_peak": gbs(bpe_f, f_avg) / HBM_PEAK_GBS},
        "backward": {"avg_ms": b_avg, "min_ms": b_min, "GB/s": gbs(bpe_b, b_avg), "frac_of_peak": gbs(bpe_b, b_avg) / HBM_PEAK_GBS},
        "unfused_forward": {"avg_ms": u_avg, "min_ms": u_min, "speedup_of_fused": u_avg / f_avg,
                            "what": "torch sigmoid x3, tanh, mul x2 around linrec_forward"},
        "roofline": {"bound": "hbm",
                     "kernel": "LSTM-cell backward pass (%s kernel)" % VARIANT_NAMES.get(lr.linrec_plan_for(family, T, B, n, backward=True)[0], "?"),
                     "achieved": gbs(bpe_b, b_avg),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs(bpe_b, b_avg) / HBM_PEAK_GBS, "traffic": None,
                     "bytes_per_element": bpe_b, "algorithmic_bytes": bpe_b * E, "avg_ms": b_avg},
        "cpu_baseline": None,
    }
    if not bf16:
        out["roofline"]["traffic"] = measured_traffic(args.lstm, "backward", "lstm:",
                                                      tile_geometry(lr, out["config"]["tile_bwd"]),
                                                      kernel=out["config"]["variant_bwd"])
    if not args.no_probe:
        out["stream_probe"] = stream_probe(lr, torch, min(E, 1 << 28), stream)
        ceiling = read_write_ceiling(out["stream_probe"], 6.0, 4.0)      # backward: six tensors in, four out
        out["roofline"]["read_write_ceiling_GB/s"] = ceiling
        out["roofline"]["frac_of_read_write_ceiling"] = out["roofline"]["achieved"] / ceiling
    if not args.no_cpu_baseline:
        import oracle
        threads = args.cpu_threads or min(16, len(os.sched_getaffinity(0)))
        C = B * n
        Ts = min(T, (1 << 27) // C)               # a bounded sample: the first rows, at most 2^27 elements
        f = lambda t: t[:Ts].float().cpu().numpy().reshape(-1, C)
        pp = [f(p) for p in pre]
        c0v = c0.float().cpu().numpy().reshape(-1)
        ee, cc = f(e), f(c)
        oracle.build()
        t0 = time.perf_counter()
        oracle.lstm_forward(*pp, c0v, threads=threads)
        t1 = time.perf_counter()
        oracle.lstm_backward(*pp, cc, c0v, ee, threads=threads)
        t2 = time.perf_counter()
        out["cpu_baseline"] = {"value": Ts * C / (t2 - t0), "unit": "elements/s", "cores": threads, "kind": "oracle",
                               "sample": f"{'the full workload' if Ts == T else f'the first {Ts} of {T} rows'}, one forward + one "
                                         f"backward pass of the fp64 oracle of the LSTM cell over {threads} host threads; "
                                         f"forward {t1 - t0:.3f} s, backward {t2 - t1:.3f} s"}
    print(json.dumps(out), flush=True)


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import linrec_workloads as wl
    import paper_1709_04057_amd as lr

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    if not os.path.exists(lr.lib_path()):   # load what is built; build only if nothing is
        from paper_1709_04057_amd import build as _build
        _build.build()
    lr.lib()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    variant = {"auto": lr.VARIANT_AUTO, "threephase": lr.VARIANT_THREEPHASE, "lookback": lr.VARIANT_LOOKBACK,
               "serial": lr.VARIANT_SERIAL, "walk": lr.VARIANT_WALK}[args.variant]
    lr.linrec_set_option(lr.OPT_VARIANT, variant)
    lr.linrec_set_option(lr.OPT_HPREV_LATE, args.hprev_late)

    if args.walk_grid:
        print(json.dumps({"metric": "walk vs single-pass kernel on short, wide problems (median microseconds per launch, "
                                    "[forward, backward], HIP events)", "walk_grid": walk_grid(lr, torch, wl)}), flush=True)
        return
    if args.table1:
        print(json.dumps({"metric": "parallel / serial linear-recurrence kernel throughput ratio (paper's Table 1 grid, "
                                    "minibatch 1, forward pass, launches back to back)",
                          "paper_values_for_context": {"hardware": "NVIDIA GPU of 2017 (K80 named for 'all experiments')",
                                                       "T=16": [0.06, 0.06, 0.05], "T=256": [0.22, 0.22, 0.86],
                                                       "T=4096": [1.02, 2.94, 3.36], "T=65536": [38.5, 41.8, 17.5],
                                                       "columns": "m = 4, 32, 128"},
                          "table1": table1(lr, torch)}), flush=True)
        return

    if args.gated:
        gated_bench(args, lr, torch, wl)
        return
    if args.lstm:
        lstm_bench(args, lr, torch, wl)
        return

    bf16 = args.dtype == "bf16"
    family = lr.ENTRY_BF16 if bf16 else lr.ENTRY_PLAIN
    fwd_bpe, bwd_bpe = (FWD_BYTES_PER_EL / 2, BWD_BYTES_PER_EL / 2) if bf16 else (FWD_BYTES_PER_EL, BWD_BYTES_PER_EL)
    stream = torch.cuda.current_stream()
    K = args.steps
    plan_kind = "tuned (linrec_tune ran first)" if args.tune else "static (no tuning run)"

    def time_workload(cfg, headline):
        """Generates workload `cfg` on the device, times K steps (wall clock, then once more with HIP events
        around every launch) and returns its record; the tensors are freed on return unless `headline`."""
        inp = wl.make_inputs(cfg, device=dev)
        if bf16:
            for k in ("lam", "x", "h0", "grad_h"):
                if inp[k] is not None:
                    inp[k] = inp[k].to(torch.bfloat16).contiguous()
        T, B, n = inp["T"], inp["B"], inp["n"]
        E = T * B * n
        lam, x, h0, e = inp["lam"], inp["x"], inp["h0"], inp["grad_h"]
        do_bwd = e is not None
        h = torch.empty_like(x)
        gx = torch.empty_like(x) if do_bwd else None
        gl = torch.empty_like(x) if do_bwd else None
        gh0 = torch.empty((B, n), device=dev, dtype=x.dtype) if do_bwd else None

        def fwd():
            lr.linrec_forward(lam, x, h0, h_out=h, stream=stream)

        def bwd():
            lr.linrec_backward(lam, h, h0, e, grad_x=gx, grad_lambda=gl, grad_h0=gh0, stream=stream)

        # the plan: pinned by --tile-fwd/--tile-bwd (headline only), tuned on request, else the library's own
        if headline and args.tile_fwd:
            lr.linrec_pin_plan(family, T, B, n, False, lr.VARIANT_LOOKBACK, args.tile_fwd)
        if headline and args.tile_bwd and do_bwd:
            lr.linrec_pin_plan(family, T, B, n, True, lr.VARIANT_LOOKBACK, args.tile_bwd)
        if args.tune and args.variant in ("auto", "lookback"):
            if not (headline and args.tile_fwd):
                lr.linrec_tune_for(family, T, B, n, backward=False, stream=stream)
            if do_bwd and not (headline and args.tile_bwd):
                lr.linrec_tune_for(family, T, B, n, backward=True, stream=stream)
        for _ in range(args.warmup):
            fwd()
            if do_bwd:
                bwd()
        # Timed region: exactly K steps, nothing but the library's launches on the stream.
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            fwd()
            if do_bwd:
                bwd()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        lr.linrec_check(stream)
        ms_per_step = (t1 - t0) * 1e3 / K
        # Per-kernel durations: the same K steps again with HIP events on the launch stream around each
        # launch (the event records themselves put ~5 us between consecutive kernels, which is why this is
        # a region of its own and not the one the throughput comes from).
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(K)]
        torch.cuda.synchronize()
        for i in range(K):
            ev[i][0].record(stream)
            fwd()
            ev[i][1].record(stream)
            if do_bwd:
                bwd()
            ev[i][2].record(stream)
        torch.cuda.synchronize()
        lr.linrec_check(stream)
        fwd_ms = sorted(ev[i][0].elapsed_time(ev[i][1]) for i in range(K))
        bwd_ms = sorted(ev[i][1].elapsed_time(ev[i][2]) for i in range(K))
        fwd_avg, bwd_avg = sum(fwd_ms) / K, sum(bwd_ms) / K
        gbs = lambda bpe, ms: bpe * E / (ms * 1e-3) / 1e9
        vf, tf = lr.linrec_plan_for(family, T, B, n, backward=False)
        vb, tb = lr.linrec_plan_for(family, T, B, n, backward=True)
        names = {lr.VARIANT_LOOKBACK: "lookback", lr.VARIANT_WALK: "walk", lr.VARIANT_THREEPHASE: "threephase",
                 lr.VARIANT_SERIAL: "serial"}
        rec = {
            "workload": f"cfg{cfg}: forward{'+backward' if do_bwd else ''}, {'bf16 storage' if bf16 else 'fp32'}, time-major "
                        f"[T={T}, B={B}, n={n}]; {wl.CONFIGS[cfg]['note']}",
            "T": T, "B": B, "n": n, "elements": E, "ms_per_step": ms_per_step, "elements/s": E / (ms_per_step * 1e-3),
            "kernel_fwd": names.get(vf, "?"), "tile_fwd": tf, "kernel_bwd": names.get(vb, "?") if do_bwd else None,
            "tile_bwd": tb if do_bwd else None,
            "forward": {"avg_ms": fwd_avg, "min_ms": fwd_ms[0], "median_ms": fwd_ms[K // 2], "GB/s": gbs(fwd_bpe, fwd_avg),
                        "frac_of_peak": gbs(fwd_bpe, fwd_avg) / HBM_PEAK_GBS, "elements/s": E / (fwd_avg * 1e-3)},
            "backward": None if not do_bwd else {
                "avg_ms": bwd_avg, "min_ms": bwd_ms[0], "median_ms": bwd_ms[K // 2], "GB/s": gbs(bwd_bpe, bwd_avg),
                "frac_of_peak": gbs(bwd_bpe, bwd_avg) / HBM_PEAK_GBS, "elements/s": E / (bwd_avg * 1e-3)},
            "combined_GB/s": (fwd_bpe + (bwd_bpe if do_bwd else 0)) * E / (ms_per_step * 1e-3) / 1e9,
        }
        if headline and (args.tile_fwd or args.tile_bwd):   # (pins are for this run only)
            lr.linrec_pin_plan(family, T, B, n, False, lr.VARIANT_LOOKBACK, 0)
            lr.linrec_pin_plan(family, T, B, n, True, lr.VARIANT_LOOKBACK, 0)
        return rec, (inp, h) if headline else None

    head, kept = time_workload(args.config, True)
    inp, h_gpu = kept
    E = head["elements"]
    do_bwd = head["backward"] is not None
    also = ("2,3,4" if args.config == 5 and not bf16 else "") if args.also == "auto" else args.also
    per = {f"cfg{args.config}": head}
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(inp, h_gpu, args.cpu_threads or host_cores()[2], args.cpu_sample_elements)
    del inp, h_gpu, kept
    torch.cuda.empty_cache()
    for c in [int(v) for v in also.split(",") if v.strip()]:
        if c != args.config:
            per[f"cfg{c}"] = time_workload(c, False)[0]
            torch.cuda.empty_cache()

    probe = None if args.no_probe else stream_probe(lr, torch, min(E, 1 << 28), stream)
    dom = "backward" if do_bwd else "forward"
    bpe = bwd_bpe if do_bwd else fwd_bpe
    tile = head["tile_bwd"] if do_bwd else head["tile_fwd"]
    kernel = head["kernel_bwd"] if do_bwd else head["kernel_fwd"]
    traffic = None
    if not bf16 and kernel in ("lookback", "walk"):
        traffic = measured_traffic(args.config, dom, expect=tile_geometry(lr, tile), kernel=kernel)
    roof = {"bound": "hbm", "kernel": f"{dom} pass ({kernel} kernel, tile shape {tile})", "achieved": head[dom]["GB/s"],
            "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": head[dom]["GB/s"] / HBM_PEAK_GBS, "traffic": traffic,
            "bytes_per_element": bpe, "algorithmic_bytes": bpe * E, "avg_ms": head[dom]["avg_ms"]}
    if probe is not None:
        like = like_probe(probe, "bwd_like_3in_2out" if do_bwd else "fwd_like_2in_1out")
        roof["stream_probe_GB/s"] = like
        roof["frac_of_stream_probe"] = head[dom]["GB/s"] / like
        rd, wr = (12.0, 8.0) if do_bwd else (8.0, 4.0)
        ceiling = read_write_ceiling(probe, rd, wr)          # (the ratio of reads to writes is what matters)
        roof["read_write_ceiling_GB/s"] = ceiling
        roof["frac_of_read_write_ceiling"] = head[dom]["GB/s"] / ceiling

    short = lambda r: {"T": r["T"], "B": r["B"], "n": r["n"], "elements": r["elements"],
                       "forward_ms": r["forward"]["avg_ms"], "forward_frac_of_peak": r["forward"]["frac_of_peak"],
                       "backward_ms": r["backward"] and r["backward"]["avg_ms"],
                       "backward_frac_of_peak": r["backward"] and r["backward"]["frac_of_peak"],
                       "ms_per_step": r["ms_per_step"], "elements/s": r["elements/s"], "combined_GB/s": r["combined_GB/s"],
                       "kernel_fwd": r["kernel_fwd"], "tile_fwd": r["tile_fwd"], "kernel_bwd": r["kernel_bwd"],
                       "tile_bwd": r["tile_bwd"]}
    out = {
        "metric": "linrec fwd+bwd elements/sec and achieved HBM GB/s (% of MI355X peak)",
        "value": head["elements/s"], "unit": "elements/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 arithmetic on bf16 storage" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "variant": args.variant, "plan": plan_kind,
                   "tile_fwd": head["tile_fwd"], "tile_bwd": head["tile_bwd"]},
        "forward": head["forward"], "backward": head["backward"], "combined_GB/s": head["combined_GB/s"],
        "roofline": roof,
        "per_workload": {k: short(r) for k, r in sorted(per.items())},
        # context only (another machine, a ratio not a rate): the paper's Table 1, parallel kernel over serial kernel
        "paper_context": {"source": "arXiv 1709.04057, Table 1 (Section 4.1.1): parallel / serial kernel throughput, minibatch 1, "
                                    "NVIDIA GPU of 2017 (a K80 is named for 'all experiments' in Section 4.2)",
                          "speedup_at_T=65536_for_m=4,32,128": [38.5, 41.8, 17.5],
                          "ours": "bench.py --table1 measures the same grid on the MI355X (profiles/table1_parallel_vs_serial_mi355x.txt)"},
        "cpu_baseline": cpu,
    }
    if probe is not None:
        out["stream_probe"] = dict(probe, elements=min(E, 1 << 28))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
