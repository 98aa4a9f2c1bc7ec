"""The generator of the static plans (paper_1709_04057_amd/plan_sweep.py), on made-up timings: which shapes a
family is built for, what a cell of the table takes, and the files it writes.  No GPU and no library involved."""
import json
import os
import re

import pytest

from paper_1709_04057_amd import plan_sweep as ps

LB, WALK = ps.VARIANT_LOOKBACK, ps.VARIANT_WALK


def _rows(fam, T, C, p, timings, tapers=()):
    out = [dict(fam=fam, T=T, C=C, p=p, var=var, tile=tile, vec=vec, us=us) for (var, tile, vec), us in timings.items()]
    out += [dict(fam=fam, T=T, C=C, p=p, var=LB, tile=tile, vec=1, taper=2, us=us, us0=us0) for tile, us, us0 in tapers]
    return out


def _write(tmp_path, rows, name="sweep.jsonl"):
    path = tmp_path / name
    with open(path, "w") as f:
        for r in rows:
            f.write(json.dumps(r) + "\n")
    return str(path)


def test_the_smallest_set_of_shapes_within_the_targets(tmp_path):
    # shape 1 is best or nearly best everywhere; shape 2 is 1 % ahead in one cell (not worth a kernel at a 3 % cell
    # target); shape 3 is 20 % ahead in one large cell (worth one); shape 4 is never ahead
    rows = []
    for i, C in enumerate((256, 512, 1024, 2048)):
        t = {(LB, 1, 1): 100.0, (LB, 2, 1): 99.0 if i == 0 else 110.0, (LB, 3, 1): 80.0 if i == 3 else 120.0,
             (LB, 4, 1): 130.0}
        rows += _rows("gilr", 4096, C, "fwd", t)
    cells, n = ps.load([_write(tmp_path, rows)])
    assert n == 16
    shapes, (missing, mean, behind) = ps.choose_shapes(cells, ps.FAMILIES["gilr"], 0.005, 0.03, 20)
    assert shapes == [1, 3] and missing == 0 and behind == 0 and mean < 0.005
    # a looser cell target leaves shape 3 out as long as the mean allows it
    shapes, _ = ps.choose_shapes(cells, ps.FAMILIES["gilr"], 0.10, 0.50, 20)
    assert shapes == [1]
    # launch-latency differences (a fraction of a microsecond) never buy a shape
    tiny = _rows("gilr", 64, 256, "fwd", {(LB, 1, 1): 5.0, (LB, 2, 1): 4.8})
    cells, _ = ps.load([_write(tmp_path, tiny, "tiny.jsonl")])
    assert len(ps.choose_shapes(cells, ps.FAMILIES["gilr"], 0.005, 0.03, 20)[0]) == 1


def test_a_cell_takes_the_walk_and_the_tapered_tail_only_with_a_margin(tmp_path):
    fam, ep = "plain", ps.FAMILIES["plain"]
    rows = _rows(fam, 1024, 8192, "fwd", {(LB, 1, 1): 100.0, (WALK, 1, 1): 98.0})            # 2 %: not enough
    rows += _rows(fam, 1024, 16384, "fwd", {(LB, 1, 1): 100.0, (WALK, 2, 1): 80.0})          # the walk, on its own shape
    rows += _rows(fam, 65536, 1024, "bwd", {(LB, 1, 1): 100.0, (LB, 2, 2): 90.0},            # wider accesses: shape 2
                  tapers=[(1, 97.0, 100.0), (2, 89.5, 90.0)])                                # 3 % on shape 1, 0.6 % on 2
    cells, _ = ps.load([_write(tmp_path, rows)])
    tapers = ps.load_tapers([_write(tmp_path, rows)])
    tab = ps.make_table(cells, {ep: [1, 2]}, tapers)
    ci = ps.C_GRID.index
    assert tab[(ep, False, 10, ci(8192))] == ([1, 1, 1], [0, 0, 0], [0, 0, 0])
    assert tab[(ep, False, 10, ci(16384))] == ([1, 1, 1], [2, 2, 2], [0, 0, 0])
    assert tab[(ep, True, 16, ci(1024))] == ([1, 2, 2], [0, 0, 0], [2, 0, 0])
    # a later file's timing of a plan replaces an earlier one's
    again = _rows(fam, 1024, 8192, "fwd", {(WALK, 1, 1): 90.0})
    cells, n = ps.load([_write(tmp_path, rows), _write(tmp_path, again, "again.jsonl")])
    assert ps.make_table(cells, {ep: [1, 2]})[(ep, False, 10, ci(8192))][1] == [1, 1, 1]


def test_neighbours_smooth_a_cell_but_do_not_overrule_it(tmp_path):
    fam, ep = "plain", ps.FAMILIES["plain"]
    ci = ps.C_GRID.index

    def table(middle):
        rows = _rows(fam, 4096, 1024, "fwd", middle)
        for T, C in ((2048, 1024), (8192, 1024), (4096, 768), (4096, 1536)):      # the four neighbours prefer shape 1
            rows += _rows(fam, T, C, "fwd", {(LB, 1, 1): 100.0, (LB, 2, 1): 120.0})
        cells, _ = ps.load([_write(tmp_path, rows)])
        return ps.make_table(cells, {ep: [1, 2]})[(ep, False, 12, ci(1024))][0]

    assert table({(LB, 1, 1): 102.0, (LB, 2, 1): 100.0}) == [1, 1, 1]      # 2 % behind here: the neighbours decide
    assert table({(LB, 1, 1): 110.0, (LB, 2, 1): 100.0}) == [2, 2, 2]      # 10 % behind here: they do not


def test_the_written_files(tmp_path):
    rows = []
    for fam in ps.FAMILIES:
        vec = 2 if fam == "bf16" else 1
        for T in (1024, 2048):
            for p in ("fwd", "bwd"):
                rows += _rows(fam, T, 4096, p, {(LB, 7, vec): 50.0, (LB, 9, vec): 70.0, (WALK, 9, vec): 40.0 if T == 1024 else 80.0})
    sweep = _write(tmp_path, rows)

    class Args:
        sweeps, out, mean_loss, cell_loss, max_shapes = [sweep], str(tmp_path), 0.005, 0.03, 20
    ps.table(Args)
    tiles = open(tmp_path / "linrec_tile_set.inc").read()
    assert re.findall(r"X\((\d+), 0x([0-9a-f]+)\)", tiles) == [("7", "3f"), ("9", "3f")]
    table = open(tmp_path / "linrec_plan_table.inc").read()
    assert "kPlanLtMin = 6, kPlanLtMax = 20, kPlanNc = 25" in table and "unsigned char lookback[3], walk[3], taper[3];" in table
    assert table.count("{{7,7,7},{9,9,9},{0,0,0}}") == 2 * 5 and table.count("{{7,7,7},{0,0,0},{0,0,0}}") == 2 * 5
    assert table.count("{{0,7,7},{0,9,9},{0,0,0}}") == 2      # two-column shapes: nothing at one-column width


def test_grid_matches_what_the_library_looks_up():
    assert ps.C_GRID[0] == 16 and ps.C_GRID[-1] == 65536 and len(ps.C_GRID) == 25
    assert all(b / a in (1.5, 4 / 3) for a, b in zip(ps.C_GRID, ps.C_GRID[1:]))
    csrc = os.path.join(os.path.dirname(os.path.abspath(ps.__file__)), "csrc", "linrec_plan_table.inc")
    text = open(csrc).read()
    assert "{" + ", ".join(map(str, ps.C_GRID)) + "}" in text
    assert f"kPlanLtMin = {ps.LT_MIN}, kPlanLtMax = {ps.LT_MAX}" in text
