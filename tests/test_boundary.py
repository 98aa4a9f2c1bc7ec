"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, validates arguments before any HIP call, and reports its tile table."""
import ctypes

import pytest

import paper_1709_04057_amd as lr


@pytest.fixture(scope="module")
def L():
    return lr.lib()


def test_exports_every_declared_symbol(L):
    names = lr.declared_symbols()
    assert {"linrec_forward", "linrec_backward", "linrec_status_string", "linrec_version"} <= set(names)
    for name in names:
        assert hasattr(L, name), f"liblinrec.so does not export {name}"


def test_the_binding_types_every_declared_function(L):
    # without argtypes ctypes passes Python ints as 32-bit C ints: pointers and int64 sizes would be cut
    for name in lr.declared_symbols():
        fn = getattr(L, name)
        assert fn.argtypes is not None, f"binding.py sets no argument types for {name}"


def test_version_and_status_strings(L):
    assert lr.linrec_version() >= 100
    assert lr.linrec_status_string(0) == "ok"
    for code in range(-6, 0):
        assert lr.linrec_status_string(code) not in ("ok", "unknown status")
    assert lr.linrec_status_string(-99) == "unknown status"


def _p(addr):
    return ctypes.c_void_p(addr)


E = 1000 * 4 * 8  # elements of a [1000, 4, 8] tensor
A0, A1, A2, A3, A4, A5, A6 = (0x10000000 + i * 0x1000000 for i in range(7))


def test_validate_forward(L):
    v = L.linrec_validate_forward
    assert v(_p(A0), _p(A1), _p(A2), _p(A3), 1000, 4, 8) == 0
    assert v(_p(A0), _p(A1), None, _p(A3), 1000, 4, 8) == 0               # h0 optional
    assert v(_p(A0), _p(A1), None, _p(A1), 1000, 4, 8) == 0               # exact in-place on x
    assert v(None, _p(A1), None, _p(A3), 1000, 4, 8) == -1
    assert v(_p(A0), None, None, _p(A3), 1000, 4, 8) == -1
    assert v(_p(A0), _p(A1), None, None, 1000, 4, 8) == -1
    assert v(_p(A0), _p(A1), None, _p(A3), -1, 4, 8) == -2
    assert v(_p(A0), _p(A1), None, _p(A3), 1 << 30, 1 << 20, 8) == -2     # T*B*n out of range
    assert v(_p(A0), _p(A1), None, _p(A3), 1 << 62, 1 << 62, 1 << 62) == -2
    assert v(_p(A0), _p(A1), None, _p(A0), 1000, 4, 8) == -3              # h_out on lambda
    assert v(_p(A0), _p(A1), None, _p(A1 + 4), 1000, 4, 8) == -3          # partial overlap with x
    assert v(_p(A0), _p(A1), _p(A3 + 4 * (E - 1)), _p(A3), 1000, 4, 8) == -3  # h0 inside h_out
    assert v(None, None, None, None, 0, 4, 8) == 0                        # empty problems are no-ops
    assert v(None, None, None, None, 1000, 0, 8) == 0


def test_validate_backward(L):
    v = L.linrec_validate_backward
    ok = (_p(A0), _p(A1), _p(A2), _p(A3), _p(A4), _p(A5), _p(A6))
    assert v(*ok, 1000, 4, 8) == 0
    assert v(_p(A0), _p(A1), None, _p(A3), None, None, None, 1000, 4, 8) == 0   # every output optional
    assert v(_p(A0), _p(A1), None, _p(A3), _p(A3), _p(A5), None, 1000, 4, 8) == 0  # grad_x in place on grad_h
    assert v(None, _p(A1), None, _p(A3), _p(A4), None, None, 1000, 4, 8) == -1
    assert v(_p(A0), None, None, _p(A3), _p(A4), None, None, 1000, 4, 8) == -1
    assert v(_p(A0), _p(A1), None, None, _p(A4), None, None, 1000, 4, 8) == -1
    assert v(_p(A0), _p(A1), None, _p(A3), _p(A0), None, None, 1000, 4, 8) == -3   # grad_x on lambda
    assert v(_p(A0), _p(A1), None, _p(A3), _p(A4), _p(A1), None, 1000, 4, 8) == -3  # grad_lambda on h
    assert v(_p(A0), _p(A1), None, _p(A3), _p(A4), _p(A4), None, 1000, 4, 8) == -3  # two outputs share memory
    assert v(_p(A0), _p(A1), None, _p(A3), _p(A4), _p(A3), None, 1000, 4, 8) == -3  # grad_lambda on grad_h
    assert v(_p(A0), _p(A1), None, _p(A3), _p(A3 + 8), None, None, 1000, 4, 8) == -3  # shifted in-place
    assert v(*ok, 1000, 4, -8) == -2
    assert v(None, None, None, None, None, None, _p(A6), 0, 4, 8) == 0


def test_validate_bf16(L):
    # 2-byte elements: ranges are half as long as the fp32 ones
    vf, vb = L.linrec_validate_forward_bf16, L.linrec_validate_backward_bf16
    assert vf(_p(A0), _p(A1), None, _p(A3), 1000, 4, 8) == 0
    assert vf(_p(A0), _p(A1), None, _p(A1), 1000, 4, 8) == 0                  # exact in-place on x
    assert vf(_p(A0), _p(A1), None, _p(A1 + 2), 1000, 4, 8) == -3             # shifted by one element
    assert vf(_p(A0), _p(A1), None, _p(A1 + 2 * E), 1000, 4, 8) == 0          # right behind x: no overlap in bf16
    assert L.linrec_validate_forward(_p(A0), _p(A1), None, _p(A1 + 2 * E), 1000, 4, 8) == -3   # but in fp32
    assert vf(None, _p(A1), None, _p(A3), 1000, 4, 8) == -1
    assert vb(_p(A0), _p(A1), None, _p(A3), _p(A3), _p(A5), None, 1000, 4, 8) == 0
    assert vb(_p(A0), _p(A1), None, _p(A3), _p(A4), _p(A1), None, 1000, 4, 8) == -3
    assert L.linrec_forward_bf16(_p(A0), _p(A1), None, _p(A0), 10, 2, 2, None) == -3
    assert L.linrec_backward_bf16(None, None, None, None, None, None, None, 10, 0, 2, None) == 0


@pytest.mark.parametrize("suffix", ["", "_bf16"])
def test_validate_gilr(L, suffix):
    vf, vb = getattr(L, "linrec_validate_gilr_forward" + suffix), getattr(L, "linrec_validate_gilr_backward" + suffix)
    assert vf(_p(A0), _p(A1), _p(A2), _p(A3), 1, 1000, 4, 8) == 0
    assert vf(_p(A0), _p(A1), None, _p(A1), 0, 1000, 4, 8) == 0            # h_out in place on i_pre
    assert vf(_p(A0), _p(A1), None, _p(A0), 1, 1000, 4, 8) == -3           # h_out on g_pre
    assert vf(_p(A0), _p(A1), None, _p(A3), 2, 1000, 4, 8) == -5           # unknown tau
    assert vf(None, _p(A1), None, _p(A3), 1, 1000, 4, 8) == -1
    assert vf(None, None, None, None, 1, 0, 4, 8) == 0
    A7 = A6 + 0x1000000
    ok = (_p(A0), _p(A1), _p(A2), _p(A3), _p(A4), _p(A5), _p(A6), _p(A7))
    assert vb(*ok, 1, 1000, 4, 8) == 0
    assert vb(_p(A0), _p(A1), _p(A2), None, _p(A4), None, None, None, 0, 1000, 4, 8) == 0   # outputs optional
    assert vb(*ok, 7, 1000, 4, 8) == -5
    assert vb(_p(A0), None, _p(A2), None, _p(A4), _p(A5), None, None, 1, 1000, 4, 8) == -1  # i_pre required
    assert vb(_p(A0), _p(A1), _p(A2), None, _p(A4), _p(A4), None, None, 1, 1000, 4, 8) == -3  # output on grad_h
    assert vb(_p(A0), _p(A1), _p(A2), None, _p(A4), _p(A5), _p(A5), None, 1, 1000, 4, 8) == -3  # outputs share memory
    assert vb(_p(A0), _p(A1), _p(A2), None, _p(A4), _p(A5), _p(A1), None, 1, 1000, 4, 8) == -3  # output on i_pre
    assert vb(*ok, 1, 1000, -4, 8) == -2
    # an output that starts where a 1000 x 4 x 8 input ends: 2 bytes per element with bf16 storage, 4 with fp32
    end16 = _p(A0 + 1000 * 4 * 8 * 2)
    assert vf(_p(A0), _p(A1), None, end16, 1, 1000, 4, 8) == (0 if suffix else -3)
    assert getattr(L, "linrec_gilr_forward" + suffix)(_p(A0), _p(A1), None, _p(A0), 1, 10, 2, 2, None) == -3   # before any HIP call
    assert getattr(L, "linrec_gilr_backward" + suffix)(None, None, None, None, None, None, None, None, 1, 10, 0, 2, None) == 0


@pytest.mark.parametrize("suffix", ["", "_bf16"])
def test_validate_lstm_cell(L, suffix):
    vf = getattr(L, "linrec_validate_lstm_cell_forward" + suffix)
    vb = getattr(L, "linrec_validate_lstm_cell_backward" + suffix)
    B0 = [0x10000000 + i * 0x1000000 for i in range(13)]
    P = [_p(a) for a in B0]
    assert vf(P[0], P[1], P[2], P[3], P[4], P[5], P[6], 1000, 4, 8) == 0
    assert vf(P[0], P[1], P[2], None, None, P[5], None, 1000, 4, 8) == 0       # cell state only: no o_pre needed
    assert vf(P[0], P[1], P[2], P[3], None, None, P[6], 1000, 4, 8) == 0       # h only
    assert vf(P[0], P[1], P[2], None, None, P[5], P[6], 1000, 4, 8) == -1      # h wanted but no o_pre
    assert vf(P[0], P[1], P[2], P[3], None, None, None, 1000, 4, 8) == -1      # no output at all
    assert vf(P[0], P[1], None, P[3], None, P[5], P[6], 1000, 4, 8) == -1
    assert vf(P[0], P[1], P[2], P[3], None, P[1], P[6], 1000, 4, 8) == -3      # c_out on i_pre
    assert vf(P[0], P[1], P[2], P[3], None, P[5], P[5], 1000, 4, 8) == -3      # outputs share memory
    assert vf(P[0], P[1], P[2], P[3], None, P[5], P[6], 1000, -4, 8) == -2
    assert vf(None, None, None, None, None, None, None, 0, 4, 8) == 0
    ok = P[:12]
    assert vb(*ok, 1000, 4, 8) == 0
    assert vb(*P[:7], None, None, None, None, None, 1000, 4, 8) == 0           # every output optional
    assert vb(P[0], P[1], P[2], P[3], None, P[5], P[6], P[7], None, None, None, None, 1000, 4, 8) == -1  # c required
    assert vb(*P[:7], P[6], None, None, None, None, 1000, 4, 8) == -3          # output on grad_h
    assert vb(*P[:7], P[7], P[7], None, None, None, 1000, 4, 8) == -3          # outputs share memory
    assert vb(*P[:7], P[7], P[8], P[9], P[4], None, 1000, 4, 8) == -3          # output on the cell state
    end16 = _p(B0[0] + 1000 * 4 * 8 * 2)   # where a bf16 f_pre ends (an fp32 one is twice as long)
    assert vf(P[0], P[1], P[2], P[3], None, end16, P[6], 1000, 4, 8) == (0 if suffix else -3)
    assert getattr(L, "linrec_lstm_cell_forward" + suffix)(P[0], P[1], P[2], P[3], None, P[0], P[6], 10, 2, 2, None) == -3
    assert getattr(L, "linrec_lstm_cell_backward" + suffix)(*([None] * 12), 10, 0, 2, None) == 0


def test_entry_points_validate_before_touching_the_gpu(L):
    # invalid arguments must come back as error codes even on a machine without a GPU
    assert L.linrec_forward(None, _p(A1), None, _p(A3), 10, 2, 2, None) == -1
    assert L.linrec_forward(_p(A0), _p(A1), None, _p(A0), 10, 2, 2, None) == -3
    assert L.linrec_forward(_p(A0), _p(A1), None, _p(A3), -5, 2, 2, None) == -2
    assert L.linrec_forward(None, None, None, None, 0, 2, 2, None) == 0
    assert L.linrec_backward(_p(A0), None, None, _p(A3), _p(A4), None, None, 10, 2, 2, None) == -1
    assert L.linrec_backward(None, None, None, None, None, None, None, 10, 0, 2, None) == 0


def test_options_and_tile_table(L):
    assert lr.linrec_get_option(lr.OPT_VARIANT) in (0, 1, 2, 3, 4)
    old = lr.linrec_get_option(lr.OPT_VARIANT)
    lr.linrec_set_option(lr.OPT_VARIANT, lr.VARIANT_THREEPHASE)
    assert lr.linrec_get_option(lr.OPT_VARIANT) == lr.VARIANT_THREEPHASE
    lr.linrec_set_option(lr.OPT_VARIANT, old)
    with pytest.raises(lr.LinrecError):
        lr.linrec_set_option(lr.OPT_VARIANT, 17)
    with pytest.raises(lr.LinrecError):
        lr.linrec_set_option(99, 0)
    assert lr.linrec_get_option(lr.OPT_STAGGER) == 3           # documented default
    lr.linrec_set_option(lr.OPT_STAGGER, 0)
    assert lr.linrec_get_option(lr.OPT_STAGGER) == 0
    lr.linrec_set_option(lr.OPT_STAGGER, 3)
    for bad in (-1, 17):
        with pytest.raises(lr.LinrecError):
            lr.linrec_set_option(lr.OPT_STAGGER, bad)
    ids = [i for i in range(1, 129) if lr.linrec_tile_info(i) is not None]   # (ids are stable: there are gaps)
    tiles = [lr.linrec_tile_info(i) for i in ids]
    assert len(tiles) >= 4
    for t in tiles:
        assert t["cols_per_thread"] in (1, 2, 4)
        assert t["threads_cols"] * t["threads_time"] in (256, 512, 1024)
        assert t["rows"] == t["threads_time"] * t["rows_per_thread"]
    for absent in (max(ids) + 1, next(i for i in range(1, 129) if i not in ids)):
        with pytest.raises(lr.LinrecError):
            lr.linrec_set_option(lr.OPT_TILE, absent)


def test_plan_is_host_only_and_consistent(L):
    for (T, B, n) in [(1024, 2, 32), (65536, 4, 256), (1048576, 1, 128), (4096, 16, 1024), (262144, 8, 512), (7, 1, 3)]:
        for bwd in (False, True):
            for align in (4, 8, 16):
                variant, tile = lr.linrec_plan(T, B, n, backward=bwd, alignment=align)
                info = lr.linrec_tile_info(tile)
                assert variant in (lr.VARIANT_THREEPHASE, lr.VARIANT_LOOKBACK, lr.VARIANT_SERIAL, lr.VARIANT_WALK)
                assert info is not None
                assert (B * n) % info["cols_per_thread"] == 0
                assert info["cols_per_thread"] * 4 <= align
    # the other entry-point families report shapes their kernels exist for
    tiled = (lr.VARIANT_LOOKBACK, lr.VARIANT_WALK)
    for (T, B, n) in [(65536, 4, 256), (4096, 16, 1024), (300, 1, 7), (5000, 2, 33)]:
        for bwd in (False, True):
            for fam in (lr.ENTRY_GILR, lr.ENTRY_LSTM_CELL):
                v, t = lr.linrec_plan_for(fam, T, B, n, backward=bwd)
                assert v in tiled and lr.linrec_tile_has(t, fam)
                assert (B * n) % lr.linrec_tile_info(t)["cols_per_thread"] == 0
            v, t = lr.linrec_plan_for(lr.ENTRY_BF16, T, B, n, backward=bwd, alignment=4)
            assert lr.linrec_tile_has(t, lr.ENTRY_BF16)
            if (B * n) % 2:
                assert v == lr.VARIANT_SERIAL            # odd number of columns: no 4-byte rows
            else:
                assert v in tiled and lr.linrec_tile_info(t)["cols_per_thread"] == 2
            for fam in (lr.ENTRY_GILR_BF16, lr.ENTRY_LSTM_CELL_BF16):
                v, t = lr.linrec_plan_for(fam, T, B, n, backward=bwd, alignment=4)
                assert v in tiled and lr.linrec_tile_has(t, fam)
                assert lr.linrec_tile_info(t)["cols_per_thread"] in ((1,) if (B * n) % 2 else (1, 2))   # odd C: 2-byte accesses
            assert lr.linrec_plan_for(lr.ENTRY_PLAIN, T, B, n, backward=bwd) == lr.linrec_plan(T, B, n, backward=bwd)
    # short and wide: the plain fp32 recurrence walks (one workgroup per column group), the other
    # families and long sequences keep the single pass
    for bwd in (False, True):
        assert lr.linrec_plan(1024, 16, 1024, backward=bwd)[0] == lr.VARIANT_WALK
        assert lr.linrec_plan(256, 8, 1024, backward=bwd)[0] == lr.VARIANT_WALK
        assert lr.linrec_plan(65536, 16, 1024, backward=bwd)[0] == lr.VARIANT_LOOKBACK
        assert lr.linrec_plan(1024, 4, 256, backward=bwd)[0] == lr.VARIANT_LOOKBACK
        for fam in (lr.ENTRY_GILR, lr.ENTRY_LSTM_CELL, lr.ENTRY_BF16, lr.ENTRY_GILR_BF16, lr.ENTRY_LSTM_CELL_BF16):
            v, t = lr.linrec_plan_for(fam, 128, 16, 1024, backward=bwd)            # every family walks here
            assert v == lr.VARIANT_WALK and lr.linrec_tile_has(t, fam)
            assert lr.linrec_plan_for(fam, 16384, 16, 1024, backward=bwd)[0] == lr.VARIANT_LOOKBACK
    with pytest.raises(lr.LinrecError):
        lr.linrec_plan_for(9, 10, 1, 1)
    # a tile whose rows would not fit 32-bit offsets falls back to the serial kernel
    variant, _ = lr.linrec_plan(64, 1, 1 << 26, alignment=16)
    assert variant == lr.VARIANT_SERIAL


def test_generated_plan_table_names_only_shapes_its_family_is_built_for():
    """The two generated files agree: every shape a family's block of the plan table names (single pass or walk)
    carries that family's bit in the set of built shapes, and only single-pass entries have a tapered tail."""
    import os
    import re
    csrc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_1709_04057_amd", "csrc")
    with open(os.path.join(csrc, "linrec_tile_set.inc")) as f:
        built = {int(t): int(m, 16) for t, m in re.findall(r"X\((\d+), 0x([0-9a-f]+)\)", f.read())}
    with open(os.path.join(csrc, "linrec_plan_table.inc")) as f:
        blocks = f.read().split("    {  // ")[1:]
    assert len(blocks) == 6 and built
    cell = re.compile(r"\{\{(\d+),(\d+),(\d+)\},\{(\d+),(\d+),(\d+)\},\{(\d+),(\d+),(\d+)\}\}")
    for fam, block in enumerate(blocks):
        cells = [tuple(map(int, c)) for c in cell.findall(block)]
        assert len(cells) == 2 * 15 * 25
        measured = 0
        for c in cells:
            for w in range(3):
                lb, walk, taper = c[w], c[3 + w], c[6 + w]
                for t in (lb, walk):
                    assert t == 0 or built.get(t, 0) >> fam & 1, (fam, c)
                assert 0 <= taper <= 8 and (taper == 0 or (lb and not walk)), (fam, c)
                measured += lb != 0
        assert measured > 500
        # every shape the family is built for is used somewhere
        used = {c[i] for c in cells for i in range(6)} - {0}
        assert used == {t for t, m in built.items() if m >> fam & 1}, fam


def test_plan_taper_follows_the_option_then_the_plan(L):
    """LINREC_OPT_TAPER: -1 (default) takes what the static plan has for the problem, 0 switches the tapered tail
    off, 1..8 force it; only single-pass plans have one."""
    assert lr.linrec_get_option(lr.OPT_TAPER) == -1
    shapes = [(2 ** lt, 1, C) for lt in range(10, 19) for C in (96, 256, 768, 1024, 2048, 4096)]
    for fam in range(6):
        auto = {s: lr.linrec_plan_taper(fam, *s, backward=True) for s in shapes}
        assert all(0 <= t <= 8 for t in auto.values())
        old = lr.linrec_get_option(lr.OPT_TAPER)
        try:
            lr.linrec_set_option(lr.OPT_TAPER, 0)
            assert all(lr.linrec_plan_taper(fam, *s, backward=True) == 0 for s in shapes)
            lr.linrec_set_option(lr.OPT_TAPER, 3)
            for s in shapes:
                single = lr.linrec_plan_for(fam, *s, backward=True)[0] == lr.VARIANT_LOOKBACK
                assert lr.linrec_plan_taper(fam, *s, backward=True) == (3 if single else 0)
        finally:
            lr.linrec_set_option(lr.OPT_TAPER, old)
        assert {s: lr.linrec_plan_taper(fam, *s, backward=True) for s in shapes} == auto
    # the table has tapered tails for the backward passes of the gated layer and the cell on bf16 storage
    assert any(lr.linrec_plan_taper(lr.ENTRY_GILR_BF16, *s, backward=True) for s in shapes)
    assert any(lr.linrec_plan_taper(lr.ENTRY_LSTM_CELL_BF16, *s, backward=True) for s in shapes)
    with pytest.raises(lr.LinrecError):
        lr.linrec_plan_taper(9, 10, 1, 1)
    with pytest.raises(lr.LinrecError):
        lr.linrec_set_option(lr.OPT_TAPER, -2)


def test_every_plan_names_a_shape_its_family_has_kernels_for(L):
    """Each entry-point family is built for the tile shapes its static plans use.  Whatever the problem and the
    alignment -- on the measured grid, between its points, far outside it -- the automatic plan must land on a
    shape the family has, with accesses no wider than the alignment allows."""
    for fam, es in ((lr.ENTRY_PLAIN, 4), (lr.ENTRY_GILR, 4), (lr.ENTRY_LSTM_CELL, 4), (lr.ENTRY_BF16, 2),
                    (lr.ENTRY_GILR_BF16, 2), (lr.ENTRY_LSTM_CELL_BF16, 2)):
        for T in (1, 7, 30, 100, 300, 1000, 5078, 20000, 70000, 300000, 2000000, 50000000):
            for C in (1, 2, 3, 15, 16, 17, 64, 100, 128, 255, 1024, 4096, 16384, 65536, 300000):
                for bwd in (False, True):
                    for align in (2, 4, 8, 16):
                        if align < es:
                            continue
                        var, t = lr.linrec_plan_for(fam, T, 1, C, backward=bwd, alignment=align)
                        assert lr.linrec_tile_has(t, fam), (fam, T, C, bwd, align, t)
                        v = lr.linrec_tile_info(t)["cols_per_thread"]
                        if var != lr.VARIANT_SERIAL:
                            assert C % v == 0 and v * es <= align, (fam, T, C, bwd, align, t)
    # every shape some family has is described, and no family claims a shape of the wrong geometry
    for t in range(1, 129):
        fams = [f for f in range(6) if lr.linrec_tile_has(t, f)]
        info = lr.linrec_tile_info(t)
        assert (info is not None) == bool(fams)
        if info is None:
            continue
        r, v = info["rows_per_thread"], info["cols_per_thread"]
        for f in fams:
            if f != lr.ENTRY_BF16:
                assert r * v <= 64
            if f in (lr.ENTRY_GILR, lr.ENTRY_GILR_BF16, lr.ENTRY_LSTM_CELL, lr.ENTRY_LSTM_CELL_BF16):
                assert r % 8 == 0 or r < 8
            if f in (lr.ENTRY_LSTM_CELL, lr.ENTRY_LSTM_CELL_BF16):
                assert r * v <= 32
            if f == lr.ENTRY_BF16:
                assert v >= 2
    assert not lr.linrec_tile_has(1, 6) and not lr.linrec_tile_has(1, -1) and not lr.linrec_tile_has(0, 0)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asked for more (by flag or by a launcher's WORLD_SIZE) it says so and
    exits before it touches a GPU."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for argv, env in ((["--gpus", "2"], {}), ([], {"WORLD_SIZE": "2"})):
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), *argv], capture_output=True, text=True,
                           env={**os.environ, **env}, timeout=120)
        assert r.returncode != 0
        assert "ONE GPU" in r.stderr + r.stdout
        assert not any(line.startswith("{") for line in r.stdout.splitlines())


def test_a_missing_library_is_an_error_not_a_fallback(tmp_path):
    """Without liblinrec.so the binding raises on first use, and host tensors are refused outright: there is
    no CPU path behind it."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import torch, paper_1709_04057_amd as lr\n"
            "for call in (lr.lib, lr.linrec_version, lambda: lr.linrec_plan(64, 1, 64),\n"
            "             lambda: lr.linrec_forward(torch.zeros(4, 1, 2), torch.zeros(4, 1, 2), None)):\n"
            "    try:\n"
            "        call()\n"
            "    except Exception as e:\n"
            "        print('RAISED', type(e).__name__, e)\n"
            "    else:\n"
            "        print('RETURNED')\n")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=root, timeout=300,
                       env={**os.environ, "LINREC_LIB_PATH": str(tmp_path / "no_such_liblinrec.so")})
    lines = [l for l in r.stdout.splitlines() if l.startswith(("RAISED", "RETURNED"))]
    assert len(lines) == 4 and all(l.startswith("RAISED") for l in lines), r.stdout + r.stderr
    assert all("not built" in l for l in lines[:3])
    assert "CUDA tensor" in lines[3]


def test_product_and_oracle_do_not_know_each_other():
    """The oracle is test infrastructure: no file of the package (Python, HIP, C++) names it, the oracle names
    nothing of the package, and the input generators hold none of the method's arithmetic calls."""
    import os
    import re
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

    def sources(folder):
        for base, _, files in os.walk(os.path.join(root, folder)):
            if "_build" in base or "__pycache__" in base:
                continue
            for f in files:
                if f.endswith((".py", ".h", ".hip", ".cpp", ".c")):
                    yield os.path.join(base, f)

    for path in list(sources("paper_1709_04057_amd")) + [os.path.join(root, "include", "linrec.h")]:
        assert not re.search(r"\boracle\b", open(path).read()), f"{path} names the oracle"
    for path in sources("oracle"):
        text = open(path).read()
        assert not re.search(r"paper_1709_04057_amd|liblinrec\.so|hip/hip_runtime|__global__|hipLaunch|torch\.cuda", text), \
            f"{path} names the GPU path"
    gen = open(os.path.join(root, "linrec_workloads.py")).read()
    assert "import oracle" not in gen and "paper_1709_04057_amd" not in gen
    assert not re.search(r"cumsum|cumprod|linrec_forward|linrec_backward", gen)


def test_the_five_workloads_fit_the_no_allocation_scratch():
    """linrec_forward_noalloc keeps 24 bytes per tile and column (plus a 512-byte header) in a fixed array: with
    the automatic forward plans every benchmark workload has to fit it, as the header promises."""
    import linrec_workloads as wl
    cap = lr.linrec_noalloc_scratch_bytes()
    for cfg, spec in wl.CONFIGS.items():
        T, B, n = spec["T"], spec["B"], spec["n"]
        variant, tile = lr.linrec_plan(T, B, n, backward=False)
        if variant != lr.VARIANT_LOOKBACK:
            continue                                    # the walk and the serial kernel keep no words
        K = -(-T // lr.linrec_tile_info(tile)["rows"]) + 8   # (a tapered tail adds a few short tiles)
        assert 512 + 24 * K * B * n <= cap, (cfg, tile, K)


def test_rows_probe_checks_its_arguments_before_any_gpu_call():
    L = lr.lib()
    one = ctypes.c_void_p(256)                                   # any aligned non-NULL address: nothing is dereferenced
    assert L.linrec_stream_probe_rows(one, None, None, one, None, 33, 256, None) == -2       # T not a multiple of 32
    assert L.linrec_stream_probe_rows(one, None, None, one, None, 32, 100, None) == -2       # C not a multiple of 256
    assert L.linrec_stream_probe_rows(None, None, None, None, None, 32, 256, None) == -1     # no array at all
    assert L.linrec_stream_probe_rows(None, one, None, one, None, 32, 256, None) == -1       # inputs come from the front
    assert L.linrec_stream_probe_rows(one, None, None, None, one, 32, 256, None) == -1       # and so do outputs
    assert L.linrec_stream_probe_rows(ctypes.c_void_p(258), None, None, one, None, 32, 256, None) == -2
    assert L.linrec_stream_probe_rows(one, None, None, one, None, 0, 256, None) == 0         # an empty problem is a no-op
