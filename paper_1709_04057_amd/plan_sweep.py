"""Measures which tile shape and variant run a [T, C] problem fastest, and writes the library's static plans.

A first call on a shape takes its plan -- variant and tile shape -- from a table of measurements, and the
library is built for the tile shapes that table uses and no others.  Both are generated here, in two steps:

    LINREC_EXTRA_FLAGS=-DLINREC_ALL_SHAPES LINREC_BUILD_OUT=$PWD/liblinrec_all.so python paper_1709_04057_amd/build.py
    LINREC_LIB_PATH=$PWD/liblinrec_all.so python -m paper_1709_04057_amd.plan_sweep measure --out sweep.jsonl
    python -m paper_1709_04057_amd.plan_sweep table sweep.jsonl         # anywhere; then build again
(``measure --families a,b`` times some families only, ``--min-columns n`` the wide cells only; ``table`` takes several
files, a later file's timing of a plan replacing an earlier one's, so a change to one family's kernels, or shapes
added for one region of the grid, need that family or region measured again and no more.
``measure`` also times the tapered tail, LINREC_OPT_TAPER = 2, on the three fastest single-pass shapes of every
cell; ``measure --taper-only sweep.jsonl ...`` does just that on the shapes an earlier sweep found.)

``measure`` (on the GPU, a few minutes, with a library that has every kernel the catalogue of shapes allows)
times every tile shape of every entry-point family, single pass and -- for short, wide problems -- walk,
forward and backward, on a grid of problem sizes (powers of two in T, half octaves in C) with seeded synthetic
inputs.  ``table`` picks, per family, the smallest set of shapes that stays within half a percent of the best
measured shape on average (``csrc/linrec_tile_set.inc``: what the build instantiates), and per grid cell and
widest access the caller's alignment allows (one, two or four columns per thread) the fastest plan among them
(``csrc/linrec_plan_table.inc``).  After a change of driver, compiler or clocks, run the three steps again.
"""
import argparse
import collections
import json
import math
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(HERE))

FAMILIES = {"plain": 0, "gilr": 1, "lstm_cell": 2, "bf16": 3, "gilr_bf16": 4, "lstm_cell_bf16": 5}  # LINREC_ENTRY_*
LT_MIN, LT_MAX = 6, 20                          # T = 64 .. 1048576, powers of two
LC_MIN, LC_MAX = 4, 16                          # C = 16 .. 65536, in half octaves (16, 24, 32, 48, ...)
T_GRID = [2 ** k for k in range(LT_MIN, LT_MAX + 1)]
C_GRID = sorted({2 ** k for k in range(LC_MIN, LC_MAX + 1)} | {3 * 2 ** (k - 1) for k in range(LC_MIN, LC_MAX)})
E_MIN = 2 ** 13
E_MAX = {"plain": 2 ** 30, "bf16": 2 ** 30}     # (the other families: 2^28 elements, up to eleven tensors each)
VARIANT_LOOKBACK, VARIANT_WALK = 2, 4


def grid(fam):
    return [(T, C) for T in T_GRID for C in C_GRID if E_MIN <= T * C <= E_MAX.get(fam, 2 ** 28)]


def measure(args):
    import torch
    import linrec_workloads as wl
    import paper_1709_04057_amd as lr

    def timeit(call, it):
        """Median microseconds per call, from events around each of `it` eager calls."""
        for _ in range(2):
            call()
        torch.cuda.synchronize()
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(it + 1)]
        evs[0].record()
        for i in range(it):
            call()
            evs[i + 1].record()
        torch.cuda.synchronize()
        return sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(it))[it // 2] * 1e3

    side = torch.cuda.Stream()

    def timeit_graph(call, reserve, reps=20, it=7):
        """The same for launches too short to time one by one (the host needs about 10 us to make a call): `reps`
        calls recorded into a HIP graph on a side stream, the graph replayed `it` times."""
        with torch.cuda.stream(side):
            reserve(side)                           # (a captured call cannot grow the stream's workspace)
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            g.capture_begin()
            for _ in range(reps):
                call()
            g.capture_end()
            g.replay()
            side.synchronize()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(it + 1)]
            evs[0].record()
            for i in range(it):
                g.replay()
                evs[i + 1].record()
            side.synchronize()
        del g
        return sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(it))[it // 2] * 1e3 / reps

    tiles = [i for i in range(1, 129) if lr.linrec_tile_info(i) is not None]
    fams = args.families.split(",") if args.families else list(FAMILIES)
    out = open(args.out, "a")
    prior = load(args.taper_only)[0] if args.taper_only else None   # (only the tapered tail is measured)
    lr.linrec_set_option(lr.OPT_TAPER, 0)
    for fam in fams:
        ep = FAMILIES[fam]
        bf16 = fam.endswith("bf16")
        cv = (lambda t: t.to(torch.bfloat16).contiguous() if torch.is_tensor(t) else t) if bf16 else (lambda t: t)
        for T, C in grid(fam):
            if C < args.min_columns:
                continue
            B, n = 1, C
            if fam.startswith("gilr"):
                inp = {k: cv(v) for k, v in wl.make_gated(T, B, n, seed=1, device="cuda:0", gate_mean=2.0).items()}
                h = torch.empty_like(inp["g_pre"])
                o1, o2 = torch.empty_like(h), torch.empty_like(h)
                s0 = torch.empty((B, n), device="cuda:0", dtype=h.dtype)
                fwd = lambda: lr.linrec_gilr_forward(inp["g_pre"], inp["i_pre"], inp["h0"], h_out=h)
                bwd = lambda: lr.linrec_gilr_backward(inp["g_pre"], inp["i_pre"], h, inp["h0"], inp["grad_h"],
                                                      grad_g_pre=o1, grad_i_pre=o2, grad_h0=s0)
            elif fam.startswith("lstm"):
                inp = {k: cv(v) for k, v in wl.make_lstm(T, B, n, seed=1, device="cuda:0").items()}
                pre = [inp[k] for k in ("f_pre", "i_pre", "z_pre", "o_pre")]
                c = torch.empty_like(pre[0])
                h = torch.empty_like(c)
                grads = [torch.empty_like(c) for _ in range(4)]
                s0 = torch.empty((B, n), device="cuda:0", dtype=c.dtype)
                fwd = lambda: lr.linrec_lstm_cell_forward(*pre, inp["c0"], c_out=c, h_out=h)
                bwd = lambda: lr.linrec_lstm_cell_backward(*pre, c, inp["c0"], inp["grad_h"], grads=grads, grad_c0=s0)
            else:
                inp = {k: cv(v) for k, v in wl.make_inputs(2, T=T, B=B, n=n, device="cuda:0").items()}
                h = torch.empty_like(inp["x"])
                o1, o2 = torch.empty_like(h), torch.empty_like(h)
                s0 = torch.empty((B, n), device="cuda:0", dtype=h.dtype)
                fwd = lambda: lr.linrec_forward(inp["lam"], inp["x"], inp["h0"], h_out=h)
                bwd = lambda: lr.linrec_backward(inp["lam"], h, inp["h0"], inp["grad_h"], grad_x=o1, grad_lambda=o2,
                                                 grad_h0=s0)
            lr.linrec_set_option(lr.OPT_VARIANT, lr.VARIANT_AUTO)
            lr.linrec_set_option(lr.OPT_TILE, 0)
            fwd()                                   # (the backward pass reads what the forward pass wrote)
            torch.cuda.synchronize()
            for which, call in (("fwd", fwd), ("bwd", bwd)):
                backward = which == "bwd"
                lr.linrec_set_option(lr.OPT_VARIANT, lr.VARIANT_AUTO)
                lr.linrec_set_option(lr.OPT_TILE, 0)
                short = timeit(call, 3) < 60.0      # the whole cell is timed one way
                best = None
                single = {}                         # single pass: {(tile, columns per thread): microseconds}
                variants = [VARIANT_LOOKBACK] + ([VARIANT_WALK] if (T <= 4096 and C >= 2048) or C >= 16384 else [])
                if prior is not None:
                    variants = []
                    single = {(t, vec): us for (var, t, vec), us in prior.get((ep, backward, T, C), {}).items()
                              if var == VARIANT_LOOKBACK}
                for variant in variants:
                    for tile in tiles:
                        info = lr.linrec_tile_info(tile)
                        if info["rows"] > 2 * T and info["rows"] > 64:
                            continue
                        lr.linrec_set_option(lr.OPT_VARIANT, variant)
                        lr.linrec_set_option(lr.OPT_TILE, tile)
                        # (a family that has no such kernel plans something else)
                        if lr.linrec_plan_for(ep, T, B, n, backward=backward) != (variant, tile):
                            continue
                        if short:
                            us = timeit_graph(call, lambda st: lr.linrec_reserve_workspace(ep, T, B, n, backward=backward,
                                                                                          stream=st))
                        else:
                            us = timeit(call, 9 if T * C <= 2 ** 26 else 5)
                        out.write(json.dumps(dict(fam=fam, T=T, C=C, p=which, var=variant, tile=tile,
                                                  vec=info["cols_per_thread"], us=us, graph=int(short))) + "\n")
                        if best is None or us < best[0]:
                            best = (us, variant, tile)
                        if variant == VARIANT_LOOKBACK:
                            single[(tile, info["cols_per_thread"])] = us
                # The tapered tail (LINREC_OPT_TAPER = 2: a quarter of the last round of tiles cut into shorter ones)
                # on the three fastest single-pass shapes of each access width (the table may settle on any of them),
                # each against the same shape timed again without.
                cand = set()
                for w in (1, 2, 4):
                    cand.update(sorted((k for k in single if k[1] <= w), key=single.get)[:3])
                for key in sorted(cand):
                    tile, info = key[0], lr.linrec_tile_info(key[0])
                    if info["rows_per_thread"] % 4 or info["rows_per_thread"] < 8 or T < 4 * info["rows"]:
                        continue
                    lr.linrec_set_option(lr.OPT_VARIANT, VARIANT_LOOKBACK)
                    lr.linrec_set_option(lr.OPT_TILE, tile)
                    if lr.linrec_plan_for(ep, T, B, n, backward=backward) != (VARIANT_LOOKBACK, tile):
                        continue
                    pair = []
                    for taper in (2, 0):
                        lr.linrec_set_option(lr.OPT_TAPER, taper)
                        if short:
                            pair.append(timeit_graph(call, lambda st: lr.linrec_reserve_workspace(ep, T, B, n, backward=backward,
                                                                                                 stream=st)))
                        else:
                            pair.append(timeit(call, 9 if T * C <= 2 ** 26 else 5))
                    out.write(json.dumps(dict(fam=fam, T=T, C=C, p=which, var=VARIANT_LOOKBACK, tile=tile, taper=2,
                                              vec=info["cols_per_thread"], us=pair[0], us0=pair[1], graph=int(short))) + "\n")
                out.flush()
                if best is not None:
                    print(f"{fam} T={T} C={C} {which}: variant {best[1]} tile {best[2]} {best[0]:.1f} us", flush=True)
                else:
                    print(f"{fam} T={T} C={C} {which}: tapered tails timed", flush=True)
            lr.linrec_check()
            del inp
    lr.linrec_set_option(lr.OPT_VARIANT, lr.VARIANT_AUTO)
    lr.linrec_set_option(lr.OPT_TILE, 0)
    lr.linrec_set_option(lr.OPT_TAPER, -1)


def load_tapers(sweeps):
    """{(family id, backward, T, C): {tile: (microseconds with the tapered tail, without it in the same run)}}"""
    tapers = collections.defaultdict(dict)
    for f in sweeps:
        for line in open(f):
            r = json.loads(line)
            if r.get("taper"):
                tapers[(FAMILIES[r["fam"]], r["p"] == "bwd", r["T"], r["C"])][r["tile"]] = (r["us"], r["us0"])
    return tapers


def load(sweeps):
    """{(family id, backward, T, C): {(variant, tile, columns per thread): microseconds}}"""
    cells = collections.defaultdict(dict)
    n = 0
    for f in sweeps:
        for line in open(f):
            r = json.loads(line)
            if r.get("taper"):
                continue
            cells[(FAMILIES[r["fam"]], r["p"] == "bwd", r["T"], r["C"])][(r["var"], r["tile"], r["vec"])] = r["us"]
            n += 1
    return cells, n


SLACK_US = 0.3      # differences below this are launch noise, not a property of the shape


def loss(us, best):
    return max(0.0, (us - SLACK_US) / best - 1.0)


def choose_shapes(cells, ep, mean_target, cell_target, max_shapes):
    """The shapes family `ep` is built for.  Greedily, the shape that lowers the mean loss against the best
    measured choice most, over every cell, pass and access width, until the mean is below `mean_target`; then
    the shape that repairs the most cells still more than `cell_target` behind their best (cells of at least
    30 us: below that the differences are launch latency), until none is left."""
    demands = []
    for (e, _, _, _), v in cells.items():
        if e != ep:
            continue
        for width in (1, 2, 4):
            ok = {k: us for k, us in v.items() if k[2] <= width}
            if not ok:
                continue
            per_tile = {}
            for (_, tile, _), us in ok.items():
                per_tile[tile] = min(per_tile.get(tile, 1e30), us)
            demands.append((min(ok.values()), per_tile))
    tiles = sorted({t for _, pt in demands for t in pt})

    def score(chosen):
        missing, behind, total = 0, 0, 0.0
        for best, pt in demands:
            have = [pt[t] for t in chosen if t in pt]
            if have:
                cell_loss = loss(min(have), best)
                total += cell_loss
                behind += best >= 30.0 and cell_loss > cell_target
            else:
                missing += 1
        return missing, total / max(1, len(demands)), behind

    chosen = []
    while len(chosen) < max_shapes:
        missing, mean, behind = score(chosen) if chosen else (1, 1.0, 0)
        if missing == 0 and mean < mean_target and behind == 0:
            break
        rest = [t for t in tiles if t not in chosen]
        if not rest:
            break
        if missing or mean >= mean_target:
            chosen.append(min(rest, key=lambda t: score(chosen + [t])[:2]))
        else:
            chosen.append(min(rest, key=lambda t: (score(chosen + [t])[2], score(chosen + [t])[1])))
    return sorted(chosen), score(chosen)


def choose_cell(cells, key, width, allowed, variant):
    """The fastest shape of `allowed` for one cell, access width and variant, judged on the cell's own timing
    and, at a quarter of the weight each, on its four neighbours' (a median of nine launches is good to 2-3 %);
    never a shape that measured more than OWN_LIMIT behind the cell's own best."""
    ep, bwd, T, C = key
    ci = C_GRID.index(C)
    mine = {t: us for (var, t, vec), us in cells[key].items() if var == variant and vec <= width and t in allowed}
    if not mine:
        return 0, None
    best_here = min(mine.values())
    neighbours = [(ep, bwd, T * 2, C), (ep, bwd, T // 2, C)]
    neighbours += [(ep, bwd, T, C_GRID[k]) for k in (ci - 1, ci + 1) if 0 <= k < len(C_GRID)]
    score = {}
    for t, us in mine.items():
        sc = us / best_here
        for nb in neighbours:
            theirs = {tt: u for (var, tt, vec), u in cells.get(nb, {}).items()
                      if var == variant and vec <= width and tt in allowed}
            sc += 0.25 * (theirs[t] / min(theirs.values()) if t in theirs else us / best_here)
        score[t] = sc
    t = min(score, key=score.get)
    # The neighbours smooth noise, they do not overrule the cell: a shape that measured more than OWN_LIMIT behind
    # the cell's own best (launch-latency differences aside) is a real loss there, whatever it does next door.
    if loss(mine[t], best_here) > OWN_LIMIT:
        t = min(mine, key=mine.get)
    return t, mine[t]


OWN_LIMIT = 0.05        # what a cell's plan may lose against the cell's own best measurement for its neighbours' sake


WALK_MARGIN = 0.97      # the walk is taken where it measured at least 3 % ahead of the single pass


TAPER_MARGIN = 0.98     # the tapered tail is taken where it measured at least 2 % ahead of the same shape without


def make_table(cells, shapes, tapers={}):
    """{(ep, bwd, lt, ci): ([single-pass tile per width], [walk tile per width or 0], [tapered eighths per width])}"""
    out = {}
    for key in cells:
        ep, bwd, T, C = key
        lb, walk, taper = [], [], []
        for width in (1, 2, 4):
            t, us = choose_cell(cells, key, width, shapes[ep], VARIANT_LOOKBACK)
            wt, wus = choose_cell(cells, key, width, shapes[ep], VARIANT_WALK)
            lb.append(t)
            walk.append(wt if wt and t and wus < WALK_MARGIN * us else 0)
            tapered, plain = tapers.get(key, {}).get(t, (1.0, 1.0))
            taper.append(2 if tapered < TAPER_MARGIN * plain and not walk[-1] else 0)
        out[(ep, bwd, int(math.log2(T)), C_GRID.index(C))] = (lb, walk, taper)
    return out


def table_loss(cells, tab):
    """Mean and worst loss of the table's choices against the best measured choice, per family."""
    res = collections.defaultdict(list)
    for (ep, bwd, T, C), v in cells.items():
        lb, walk, _ = tab[(ep, bwd, int(math.log2(T)), C_GRID.index(C))]
        for w, width in enumerate((1, 2, 4)):
            ok = {k: us for k, us in v.items() if k[2] <= width}
            if not ok:
                continue
            pick = (VARIANT_WALK, walk[w]) if walk[w] else (VARIANT_LOOKBACK, lb[w])
            us = [u for (var, t, _), u in ok.items() if (var, t) == pick]
            res[ep].append(loss(us[0], min(ok.values())))
    return {ep: (sum(x) / len(x), max(x)) for ep, x in res.items()}


def table(args):
    cells, n = load(args.sweeps)
    names = {v: k for k, v in FAMILIES.items()}
    shapes = {}
    for ep in sorted(names):
        shapes[ep], (missing, mean, behind) = choose_shapes(cells, ep, args.mean_loss, args.cell_loss, args.max_shapes)
        print(f"{names[ep]}: {len(shapes[ep])} shapes {shapes[ep]} (mean loss {100 * mean:.2f} %, {behind} cells more than "
              f"{100 * args.cell_loss:.0f} % behind, {missing} without a kernel)")
    tab = make_table(cells, shapes, load_tapers(args.sweeps))
    for ep in shapes:   # (a shape that, with the neighbours' weight, no cell takes in the end is not built)
        used = {t for (e, _, _, _), (lb, walk, _) in tab.items() if e == ep for t in lb + walk} - {0}
        if set(shapes[ep]) - used:
            print(f"{names[ep]}: not used by any cell after all, dropped: {sorted(set(shapes[ep]) - used)}")
        shapes[ep] = sorted(used)
    print("tapered tail taken in %d of %d cell-widths" % (sum(sum(1 for x in v[2] if x) for v in tab.values()), 3 * len(tab)))
    for ep, (mean, worst) in sorted(table_loss(cells, tab).items()):
        print(f"{names[ep]}: table within {100 * mean:.2f} % of the best measured choice on average, {100 * worst:.0f} % at worst")
    csrc = args.out or os.path.join(HERE, "csrc")
    stamp = f"// Written by plan_sweep.py from {n} timings on one MI355X; regenerate rather than edit.\n"
    every = sorted({t for s in shapes.values() for t in s})
    with open(os.path.join(csrc, "linrec_tile_set.inc"), "w") as f:
        f.write("// The tile shapes the library is built for, and for which entry-point families each has kernels:\n"
                "// (tile id, mask with bit LINREC_ENTRY_* set for every family that plans this shape somewhere).\n"
                "// Per family the smallest set (greedy) that stays within %.1f %% of the best measured shape on average and\n"
                "// within %.0f %% on every problem of 30 us and more.\n" % (100 * args.mean_loss, 100 * args.cell_loss)
                + stamp + "#define LINREC_BUILT_TILES(X) \\\n")
        f.write(" \\\n".join("    X(%d, 0x%02x)" % (t, sum(1 << ep for ep in shapes if t in shapes[ep])) for t in every) + "\n")
    with open(os.path.join(csrc, "linrec_plan_table.inc"), "w") as f:
        f.write("// Static plans: per entry-point family, pass and problem [2^lt rows, kPlanC[ci] columns] the fastest\n"
                "// single-pass tile shape among those whose accesses are 1, 2 or 4 columns wide, and the walk's where the\n"
                "// walk measured ahead of it (else 0), and the eighths of the single pass's last round that are cut into\n"
                "// shorter tiles (the tapered tail) where that measured ahead.  {0, ...}: not measured (too small or too\n"
                "// large a problem).\n"
                + stamp)
        f.write(f"constexpr int kPlanLtMin = {LT_MIN}, kPlanLtMax = {LT_MAX}, kPlanNc = {len(C_GRID)};\n")
        f.write("constexpr int kPlanC[kPlanNc] = {" + ", ".join(map(str, C_GRID)) + "};\n")
        f.write("struct PlanCell {\n    unsigned char lookback[3], walk[3], taper[3];\n};\n")
        f.write("// [family][backward][lt - kPlanLtMin][ci]\n")
        f.write(f"const PlanCell kPlanCells[{len(FAMILIES)}][2][kPlanLtMax - kPlanLtMin + 1][kPlanNc] = {{\n")
        for ep in sorted(names):
            f.write(f"    {{  // {names[ep]}\n")
            for bwd in (0, 1):
                f.write("        {\n")
                for lt in range(LT_MIN, LT_MAX + 1):
                    row = []
                    for ci in range(len(C_GRID)):
                        lb, walk, taper = tab.get((ep, bool(bwd), lt, ci), ([0, 0, 0], [0, 0, 0], [0, 0, 0]))
                        row.append("{{%d,%d,%d},{%d,%d,%d},{%d,%d,%d}}" % (*lb, *walk, *taper))
                    f.write("            {" + ",".join(row) + "},\n")
                f.write("        },\n")
            f.write("    },\n")
        f.write("};\n")
    print(f"wrote linrec_tile_set.inc ({len(every)} shapes) and linrec_plan_table.inc ({len(tab)} cells) to {csrc}")


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    sub = ap.add_subparsers(dest="cmd", required=True)
    m = sub.add_parser("measure")
    m.add_argument("--out", required=True)
    m.add_argument("--families", default="")
    m.add_argument("--min-columns", type=int, default=0,
                   help="only the grid cells of at least this many columns (every shape is timed on them again)")
    m.add_argument("--taper-only", nargs="+", default=[], metavar="SWEEP",
                   help="time only the tapered tails, on the fastest shapes of these earlier sweeps")
    t = sub.add_parser("table")
    t.add_argument("sweeps", nargs="+")
    t.add_argument("--out", default="", help="directory for the two generated files (default: csrc/)")
    t.add_argument("--mean-loss", type=float, default=0.005)
    t.add_argument("--cell-loss", type=float, default=0.03)
    t.add_argument("--max-shapes", type=int, default=20)
    args = ap.parse_args()
    (measure if args.cmd == "measure" else table)(args)


if __name__ == "__main__":
    main()
