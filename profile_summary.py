#!/usr/bin/env python3
"""Turns rocprofv3 output (its SQLite results) into the short text summaries kept under profiles/.

Kernel durations (one `rocprofv3 --kernel-trace --stats` run):

    cd /tmp && export TMPDIR=/tmp && cd <repository>
    rocprofv3 --kernel-trace --stats -d out/kt -o kt -- python3 bench.py --config 2 --also '' --steps 50 --warmup 5 --no-cpu-baseline
    python3 profile_summary.py kernels out/kt/kt_results.db > profiles/<name>.txt

HBM bytes per launch (two counter runs, FETCH_SIZE then WRITE_SIZE, each scaled by what the same counter
reads for the library's plain copy kernel -- 4 bytes in and 4 bytes out per element -- which bench.py runs
as the first of its streaming probes, so the unit the counter happens to use drops out):

    rocprofv3 --pmc FETCH_SIZE -d out/fetch -o fetch -- python3 bench.py --config 2 --also '' --steps 10 --warmup 2 --no-cpu-baseline
    rocprofv3 --pmc WRITE_SIZE -d out/write -o write -- python3 bench.py --config 2 --also '' --steps 10 --warmup 2 --no-cpu-baseline
    python3 profile_summary.py traffic out/fetch/fetch_results.db out/write/write_results.db \\
           --elements 67108864 --out profiles/hbm_traffic_cfg2
(for the gated layer: bench.py --gated g2 ... and --bytes-per-element 12,24; LSTM cell: --lstm l2, 24,40)

Writes <out>.json (read by bench.py for roofline.traffic) and <out>.txt.  Nothing here touches a GPU.
"""
from __future__ import annotations

import argparse
import json
import sqlite3
import sys


def kernels_main(argv):
    cur = sqlite3.connect(argv[0]).cursor()
    print("%-100s %6s %12s %12s %12s %12s %6s" % ("kernel", "calls", "total_us", "avg_us", "min_us", "max_us", "%"))
    rows = cur.execute("select name, count(*), sum(duration), avg(duration), min(duration), max(duration) from kernels "
                       "group by name order by sum(duration) desc").fetchall()
    total = sum(r[2] for r in rows) or 1
    for name, n, tot, avg, mn, mx in rows:
        print("%-100s %6d %12.1f %12.1f %12.1f %12.1f %6.2f" % (name[:100], n, tot / 1e3, avg / 1e3, mn / 1e3, mx / 1e3,
                                                                 100.0 * tot / total))


def _per_kernel(db_path, counter):
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select kernel_name, value, start from counters_collection where counter_name = ? order by start",
                       (counter,)).fetchall()
    out = {}
    for name, value, _ in rows:
        out.setdefault(name, []).append(float(value))
    return out


def _kind(name):
    if "k_stream_probe" in name:
        return "stream_probe"
    if any(k in name for k in ("k_lookback", "k_walk", "k_fixup", "k_reduce", "k_scan_summaries", "k_serial")):
        bwd = ", true" in name.split("k_", 1)[1] or "_bwd" in name
        base = name.split("linrec::", 1)[1].split("<", 1)[0].split("(", 1)[0]
        # the last template argument of the look-back kernel and of the walk is the form: 1 gated layer, 2 LSTM cell
        form = {"1": "gated:", "2": "lstm:"}.get(name.rsplit(">(", 1)[0].rsplit(",", 1)[-1].strip(), "") \
            if "k_lookback" in name or "k_walk" in name else ""
        return form + base + ("/backward" if bwd else "/forward")
    return None


def traffic_main(argv):
    ap = argparse.ArgumentParser(prog="profile_summary.py traffic")
    ap.add_argument("fetch_db")
    ap.add_argument("write_db")
    ap.add_argument("--elements", type=int, required=True, help="T*B*n of the workload (also the probe's array length)")
    ap.add_argument("--probe-launches", type=int, default=12, help="launches of each probe variant (warm-up + timed)")
    ap.add_argument("--probe-elements", type=int, default=0,
                    help="array length of the copy probe (default: min(elements, 2^28), as bench.py runs it)")
    ap.add_argument("--bytes-per-element", default="12,20",
                    help="algorithmic bytes per element forward,backward of the entry points under test "
                         "(12,20 plain; 12,24 gated layer; 24,40 LSTM cell); applied to the kernels of that form")
    ap.add_argument("--bench-args", default="",
                    help="the bench.py arguments of the two counter runs, recorded in the summary (e.g. '--gated g2')")
    ap.add_argument("--out", required=True)
    a = ap.parse_args(argv)

    E = a.elements
    Ep = a.probe_elements or min(E, 1 << 28)
    res = {"elements": E, "probe_elements": Ep, "kernels": {}}
    lines = []
    factors = {}
    for counter, db in (("FETCH_SIZE", a.fetch_db), ("WRITE_SIZE", a.write_db)):
        per = _per_kernel(db, counter)
        probe = [v for k, vs in per.items() if _kind(k) == "stream_probe" for v in vs]
        if len(probe) < a.probe_launches:
            raise SystemExit(f"{counter}: no copy-probe launches found in {db} (run bench.py with --probe)")
        copy = probe[:a.probe_launches]          # the copy variant is launched first
        copy_avg = sum(copy) / len(copy)
        factors[counter] = 4.0 * Ep / copy_avg    # bytes per counter unit
        lines.append(f"{counter}: copy kernel reads {copy_avg:.1f} per launch for {4 * Ep} bytes -> {factors[counter]:.2f} bytes per unit")
        # several kernels of one kind may have run (linrec_tune times its candidates during warm-up):
        # the one with the most launches is the plan's
        best = {}
        for name, vs in per.items():
            kind = _kind(name)
            if kind is None or kind == "stream_probe":
                continue
            if kind not in best or len(vs) > len(per[best[kind]]):
                best[kind] = name
        for kind, name in best.items():
            vs = per[name]
            d = res["kernels"].setdefault(kind, {"name": name})
            d[counter] = sum(vs) / len(vs)
            d[counter + "_launches"] = len(vs)
            d[("read" if counter == "FETCH_SIZE" else "written") + "_bytes"] = d[counter] * factors[counter]
    res["bytes_per_unit"] = factors
    for kind, d in sorted(res["kernels"].items()):
        fwd_b, bwd_b = (float(v) for v in a.bytes_per_element.split(","))
        if ":" not in kind:
            fwd_b, bwd_b = 12.0, 20.0
        alg = (bwd_b if kind.endswith("backward") else fwd_b) * E
        if "read_bytes" in d and "written_bytes" in d:
            d["hbm_bytes"] = d["read_bytes"] + d["written_bytes"]
            d["algorithmic_bytes"] = alg
            lines.append(f"{kind}: read {d['read_bytes'] / 2**20:.1f} MiB + written {d['written_bytes'] / 2**20:.1f} MiB = "
                         f"{d['hbm_bytes'] / 2**20:.1f} MiB per launch; algorithmic {alg / 2**20:.1f} MiB "
                         f"(x{d['hbm_bytes'] / alg:.3f})   [{d['name']}]")
    with open(a.out + ".json", "w") as f:
        json.dump(res, f, indent=1)
    bench = "bench.py " + (a.bench_args.strip() + " " if a.bench_args.strip() else "") + "--steps 10 --warmup 2 --no-cpu-baseline"
    head = ("HBM bytes per launch from two rocprofv3 counter runs (one MI355X), each counter scaled by what it reads for the\n"
            "library's copy kernel of known size.  Commands, from the repository root on the GPU box:\n"
            "  cd /tmp && export TMPDIR=/tmp && cd $REPO\n"
            f"  rocprofv3 --pmc FETCH_SIZE -d out/fetch -o fetch -- python3 {bench}\n"
            f"  rocprofv3 --pmc WRITE_SIZE -d out/write -o write -- python3 {bench}\n"
            f"  python3 profile_summary.py traffic out/fetch/fetch_results.db out/write/write_results.db "
            f"--elements {E} --bytes-per-element {a.bytes_per_element}"
            + (f" --bench-args '{a.bench_args.strip()}'" if a.bench_args.strip() else "") + " --out <this file>\n")
    with open(a.out + ".txt", "w") as f:
        f.write(head + "\n" + "\n".join(lines) + "\n")
    print("\n".join(lines))




if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "kernels":
        kernels_main(sys.argv[2:])
    elif len(sys.argv) >= 3 and sys.argv[1] == "traffic":
        traffic_main(sys.argv[2:])
    else:
        sys.exit("usage: profile_summary.py kernels <kt_results.db> | traffic <fetch.db> <write.db> --elements N --out PATH")
