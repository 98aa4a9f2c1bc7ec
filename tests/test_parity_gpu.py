"""GPU parity tests: liblinrec (through the C ABI) against the fp64 oracle, element by element."""
import pytest
import torch

import linrec_workloads as wl
import paper_1709_04057_amd as lr
from parity import (all_tiles, check_backward, check_forward, fwd_bwd_check, options, reruns_agree, run_backward, run_forward,
                    say)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
VARIANTS = {"threephase": lr.VARIANT_THREEPHASE, "lookback": lr.VARIANT_LOOKBACK, "serial": lr.VARIANT_SERIAL,
            "walk": lr.VARIANT_WALK}


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    lr.lib()  # fails loudly if liblinrec.so is not built
    yield
    torch.cuda.synchronize()
    lr.linrec_release_workspace()


# ------------------------------------------------------------------------------------------------
# edge shapes: T and C around tile / wavefront boundaries, every tile shape, every variant
# ------------------------------------------------------------------------------------------------
EDGE_T = [1, 2, 63, 64, 65, 127, 129, 257, 600, 1031]
EDGE_BN = [(1, 1), (1, 3), (1, 63), (1, 64), (1, 65), (1, 100), (3, 100), (2, 32), (1, 128), (4, 68)]


@pytest.mark.parametrize("variant", ["threephase", "lookback", "walk"])
def test_edge_shapes_all_tiles(variant):
    tiles = all_tiles(lr.ENTRY_PLAIN)
    seed = 0
    for tile_id, info in tiles:
        for (B, n) in EDGE_BN:
            if (B * n) % info["cols_per_thread"]:
                continue  # the library would replace the tile; covered by the narrower tiles
            for T in EDGE_T:
                seed += 1
                if seed % 3 and T not in (1, 65, 1031):   # thin the grid, keep the corners
                    continue
                inp = wl.make_generic(T, B, n, seed, device=DEV, lam_kind=("mixed", "signed", "sigmoid")[seed % 3],
                                      with_h0=bool(seed % 2))
                with options(variant=VARIANTS[variant], tile=tile_id, chunk_tiles=(seed % 4)):
                    fwd_bwd_check(inp, f"edge {variant} tile={tile_id} seed={seed}")


def test_edge_shapes_serial():
    seed = 1000
    for (B, n) in EDGE_BN:
        for T in (1, 2, 65, 600):
            seed += 1
            inp = wl.make_generic(T, B, n, seed, device=DEV, lam_kind="signed", with_h0=bool(seed % 2))
            with options(variant=lr.VARIANT_SERIAL):
                fwd_bwd_check(inp, f"edge serial seed={seed}")


def test_auto_plan_edge_shapes():
    seed = 2000
    for (B, n) in EDGE_BN:
        for T in (1, 129, 1031, 5000):
            seed += 1
            inp = wl.make_generic(T, B, n, seed, device=DEV, lam_kind="mixed")
            fwd_bwd_check(inp, f"edge auto seed={seed}")


# ------------------------------------------------------------------------------------------------
# the five workloads
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("variant", ["threephase", "lookback", "walk"])
def test_config1_full(variant):
    inp = wl.make_inputs(1, device=DEV)
    with options(variant=VARIANTS[variant]):
        fwd_bwd_check(inp, f"cfg1 {variant}")


@pytest.mark.parametrize("cfg,shape", [(2, (8192, 4, 256)), (3, (65536, 1, 128)), (4, (1024, 16, 1024)),
                                       (5, (16384, 8, 512))])
@pytest.mark.parametrize("variant", ["threephase", "lookback", "walk"])
def test_configs_reduced_T_every_vector_tile(cfg, shape, variant):
    """Same widths and value distributions as the full workloads, shorter T; every multi-column tile shape."""
    T, B, n = shape
    inp = wl.make_inputs(cfg, T=T, B=B, n=n, device=DEV)
    for tile_id, info in all_tiles(lr.ENTRY_PLAIN):
        if info["cols_per_thread"] == 1 and info["rows_per_thread"] < 32:
            continue
        with options(variant=VARIANTS[variant], tile=tile_id):
            fwd_bwd_check(inp, f"cfg{cfg} reduced {variant} tile={tile_id}")


@pytest.mark.parametrize("cfg", [2, 3, 4])
@pytest.mark.parametrize("variant", ["threephase", "lookback"])
def test_configs_full_size(cfg, variant):
    """Full-size workloads in the launch configuration the benchmark times (automatic plan)."""
    inp = wl.make_inputs(cfg, device=DEV)
    with options(variant=VARIANTS[variant]):
        fwd_bwd_check(inp, f"cfg{cfg} full {variant}")


def test_config4_full_size_walk():
    """Workload 4 (the widest one) at full size through the walk, which the plan would not take at this length."""
    inp = wl.make_inputs(4, device=DEV)
    with options(variant=lr.VARIANT_WALK):
        fwd_bwd_check(inp, "cfg4 full walk")


@pytest.mark.parametrize("shape", [(1024, 16, 1024), (512, 8, 1024), (200, 3, 5000), (2048, 2, 4096), (1024, 16, 4096),
                                   (64, 16, 4096)])
def test_short_wide_shapes_take_the_walk(shape):
    """Automatic plan on short, wide problems: one workgroup per column group walks the sequence (no
    look-back) -- in the forward pass of every one of these shapes, and in the backward pass wherever it
    measured ahead of the single pass; ragged numbers of columns and rows included."""
    T, B, n = shape
    assert lr.linrec_plan(T, B, n, backward=False)[0] == lr.VARIANT_WALK
    assert lr.linrec_plan(T, B, n, backward=True)[0] in (lr.VARIANT_WALK, lr.VARIANT_LOOKBACK)
    fwd_bwd_check(wl.make_inputs(2, T=T, B=B, n=n, device=DEV), f"short wide {shape} auto")


def test_config5_full_size_lookback():
    inp = wl.make_inputs(5, device=DEV)
    fwd_bwd_check(inp, "cfg5 full auto")


@pytest.mark.parametrize("variant", ["lookback", "threephase"])
def test_tensors_beyond_4_gib(variant):
    """6 GiB per tensor (workload 5's recipe, 1.5 times its length): element offsets pass 2^32 bytes, which
    the tiles' 32-bit offsets must never see (each tile addresses from its own 64-bit origin)."""
    inp = wl.make_inputs(5, T=393216, device=DEV)
    assert inp["lam"].numel() * 4 > 2**32
    with options(variant=VARIANTS[variant]):
        fwd_bwd_check(inp, f"cfg5 x1.5 (6 GiB tensors) {variant}")


@pytest.mark.parametrize("cfg,shape", [(3, (262144, 1, 128)), (5, (65536, 2, 128))])
def test_per_channel_lambda_accuracy_stress(cfg, shape):
    """lambda (or its mixture class) held constant along T per column: true long memory."""
    T, B, n = shape
    inp = wl.make_inputs(cfg, T=T, B=B, n=n, device=DEV, per_channel=True)
    for variant in ("threephase", "lookback"):
        with options(variant=VARIANTS[variant]):
            fwd_bwd_check(inp, f"cfg{cfg}b per-channel {variant}")


# ------------------------------------------------------------------------------------------------
# invariants the mathematics fixes, checked on the GPU result itself
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("variant", ["threephase", "lookback", "serial", "walk"])
def test_lambda_zero_is_bit_exact(variant):
    inp = wl.make_generic(3000, 2, 96, 31, device=DEV)
    inp["lam"].zero_()
    with options(variant=VARIANTS[variant]):
        h = run_forward(inp)
        gx, gl, gh0 = run_backward(inp, h)
    torch.cuda.synchronize()
    assert torch.equal(h, inp["x"])
    assert torch.equal(gx, inp["grad_h"])
    assert torch.equal(gl[1:], inp["grad_h"][1:] * inp["x"][:-1])
    assert torch.equal(gl[0], inp["grad_h"][0] * inp["h0"])
    assert torch.equal(gh0, torch.zeros_like(gh0))


@pytest.mark.parametrize("variant", ["threephase", "lookback", "walk"])
def test_lambda_one_is_prefix_sum(variant):
    inp = wl.make_generic(20000, 1, 64, 32, device=DEV)
    inp["lam"].fill_(1.0)
    with options(variant=VARIANTS[variant]):
        h = run_forward(inp)
    torch.cuda.synchronize()
    ref = inp["h0"].double()[None] + torch.cumsum(inp["x"].double(), dim=0)
    err = (h.double() - ref).abs().max().item()
    assert err <= 1e-5 * (1 + ref.abs().max().item())


@pytest.mark.parametrize("variant", ["threephase", "lookback", "walk"])
def test_split_resume_matches_one_shot(variant):
    """Forward on [0,T1) then [T1,T) seeded with h[T1-1] equals the one-shot run (C_{-1} = h_0)."""
    inp = wl.make_inputs(2, T=6000, B=2, n=128, device=DEV)
    with options(variant=VARIANTS[variant]):
        h = run_forward(inp)
        T1 = 2500
        a = lr.linrec_forward(inp["lam"][:T1].contiguous(), inp["x"][:T1].contiguous(), inp["h0"])
        b = lr.linrec_forward(inp["lam"][T1:].contiguous(), inp["x"][T1:].contiguous(), a[T1 - 1].contiguous())
    torch.cuda.synchronize()
    two = torch.cat([a, b])
    scale = 1 + h.abs().max().item()
    assert (two - h).abs().max().item() <= 2e-5 * scale
    check_forward(inp, two, "split resume")


# ------------------------------------------------------------------------------------------------
# boundary behaviour on the device
# ------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("variant", ["threephase", "lookback", "serial", "walk"])
def test_in_place_and_optional_outputs(variant):
    inp = wl.make_inputs(2, T=3000, B=2, n=64, device=DEV)
    with options(variant=VARIANTS[variant]):
        h_ref = run_forward(inp)
        xbuf = inp["x"].clone()
        h_inplace = lr.linrec_forward(inp["lam"], xbuf, inp["h0"], h_out=xbuf)
        assert h_inplace.data_ptr() == xbuf.data_ptr()
        gx_ref, gl_ref, gh0_ref = run_backward(inp, h_ref)
        ebuf = inp["grad_h"].clone()
        gx_in, gl2, gh02 = lr.linrec_backward(inp["lam"], h_ref, inp["h0"], ebuf, grad_x=ebuf)
        only_x = lr.linrec_backward(inp["lam"], h_ref, inp["h0"], inp["grad_h"], want_grad_lambda=False,
                                    want_grad_h0=False)
        only_l = lr.linrec_backward(inp["lam"], h_ref, inp["h0"], inp["grad_h"], want_grad_x=False, want_grad_h0=False)
        only_0 = lr.linrec_backward(inp["lam"], h_ref, inp["h0"], inp["grad_h"], want_grad_x=False,
                                    want_grad_lambda=False)
        no_h0 = lr.linrec_backward(inp["lam"], h_ref, None, inp["grad_h"])
    torch.cuda.synchronize()
    ex = variant != "lookback"   # (repeats of the single pass agree to rounding, the others bit for bit)
    assert reruns_agree(h_inplace, h_ref, ex)
    assert reruns_agree(gx_in, gx_ref, ex) and reruns_agree(gl2, gl_ref, ex) and reruns_agree(gh02, gh0_ref, ex)
    assert reruns_agree(only_x[0], gx_ref, ex) and only_x[1] is None and only_x[2] is None
    assert reruns_agree(only_l[1], gl_ref, ex) and only_l[0] is None
    assert reruns_agree(only_0[2], gh0_ref, ex)
    assert reruns_agree(no_h0[1][1:], gl_ref[1:], ex) and torch.equal(no_h0[1][0], torch.zeros_like(gl_ref[0]))
    check_forward(inp, h_ref, f"in-place {variant}")
    check_backward(inp, h_ref, gx_ref, gl_ref, gh0_ref, f"in-place {variant}")


def test_unaligned_pointers_take_the_scalar_path():
    T, B, n = 2000, 2, 64
    big = wl.make_generic(T, B, n + 1, 41, device=DEV)            # odd row length => views below are 4-byte aligned only
    flat = {k: big[k].reshape(-1) for k in ("lam", "x", "grad_h")}
    E = T * B * n
    inp = dict(T=T, B=B, n=n, h0=None)
    for k in flat:
        inp[k] = flat[k][1:1 + E].view(T, B, n)
        assert inp[k].data_ptr() % 16 != 0
    h = run_forward(inp)
    torch.cuda.synchronize()
    check_forward(inp, h, "unaligned")
    gx, gl, gh0 = run_backward(inp, h)
    torch.cuda.synchronize()
    check_backward(inp, h, gx, gl, gh0, "unaligned")


def test_empty_problems_are_no_ops():
    z = torch.empty((0, 2, 8), device=DEV)
    h0 = torch.randn((2, 8), device=DEV)
    assert lr.linrec_forward(z, z, h0).shape == (0, 2, 8)
    gx, gl, gh0 = lr.linrec_backward(z, z, h0, z, grad_h0=torch.ones((2, 8), device=DEV))
    torch.cuda.synchronize()
    assert torch.equal(gh0, torch.zeros_like(gh0))
    z2 = torch.empty((5, 0, 8), device=DEV)
    assert lr.linrec_forward(z2, z2, None).shape == (5, 0, 8)


def test_invalid_arguments_raise_on_device_pointers():
    a = torch.randn((10, 2, 4), device=DEV)
    with pytest.raises(lr.LinrecError) as ei:
        lr.linrec_forward(a, a.clone(), None, h_out=a)            # h_out on lambda
    assert ei.value.status == -3


@pytest.mark.parametrize("variant", ["threephase", "lookback", "walk"])
def test_deterministic_and_stream_safe(variant):
    inp = wl.make_inputs(5, T=20000, B=2, n=256, device=DEV)
    with options(variant=VARIANTS[variant]):
        h1 = run_forward(inp)
        h2 = run_forward(inp)
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            h3 = lr.linrec_forward(inp["lam"], inp["x"], inp["h0"])
            g3 = lr.linrec_backward(inp["lam"], h3, inp["h0"], inp["grad_h"])
        g1 = run_backward(inp, h1)
        s.synchronize()
        lr.linrec_check(s)
    torch.cuda.synchronize()
    ex = VARIANTS[variant] != lr.VARIANT_LOOKBACK   # (repeats of the single pass agree to rounding only)
    assert reruns_agree(h1, h2, ex) and reruns_agree(h1, h3, ex)
    for a, b in zip(g1, g3):
        assert reruns_agree(a, b, ex)


def test_lookback_repeated_calls_and_shape_changes():
    """The look-back workspace is reused across calls (epochs) and regrown; many calls, changing shapes."""
    shapes = [(4096, 1, 128), (700, 3, 100), (20000, 2, 64), (4096, 1, 128), (33, 1, 8), (50000, 1, 32)]
    with options(variant=lr.VARIANT_LOOKBACK):
        for rep in range(3):
            for i, (T, B, n) in enumerate(shapes):
                inp = wl.make_generic(T, B, n, 500 + 10 * rep + i, device=DEV, lam_kind="mixed")
                for _ in range(3):
                    h = run_forward(inp)
                fwd_bwd_check(inp, f"repeat rep={rep} shape={T}x{B}x{n}")
                check_forward(inp, h, "repeat")


def test_lookback_wait_limit_is_reported_and_recovered():
    """A spin limit of one poll makes some look-back waits give up; the kernel must still finish, the
    failure must be reported by linrec_check, and the next healthy call must be correct."""
    inp = wl.make_inputs(2, T=65536, B=1, n=128, device=DEV)
    with options(variant=lr.VARIANT_LOOKBACK, spin_limit=1):
        say("spin-limit: launching with a limit of one poll")
        run_forward(inp)
        torch.cuda.synchronize()
        try:
            lr.linrec_check()
            gave_up = False
        except lr.LinrecError as e:
            assert e.status == -6
            gave_up = True
        say(f"spin-limit: gave_up={gave_up}")
    lr.linrec_check()                                             # the flag was cleared
    with options(variant=lr.VARIANT_LOOKBACK):
        fwd_bwd_check(inp, "after spin-limit")


def test_hip_graph_replay_matches_eager():
    """The look-back kernels keep their call state (ticket, epoch) on the device, so a captured launch
    can be replayed.  Replays are interleaved with eager calls and synchronisations, and every replay
    is compared with the eager result."""
    inp = wl.make_inputs(2, T=16384, B=2, n=128, device=DEV)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with options(variant=lr.VARIANT_LOOKBACK):
        with torch.cuda.stream(s):
            h = torch.empty_like(inp["x"])
            gx, gl = torch.empty_like(h), torch.empty_like(h)
            gh0 = torch.empty_like(inp["h0"])
            for _ in range(2):                                    # allocates the stream's workspace: not capturable
                lr.linrec_forward(inp["lam"], inp["x"], inp["h0"], h_out=h)
                lr.linrec_backward(inp["lam"], h, inp["h0"], inp["grad_h"], grad_x=gx, grad_lambda=gl, grad_h0=gh0)
            s.synchronize()
            ref = [t.clone() for t in (h, gx, gl, gh0)]
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s):
                lr.linrec_forward(inp["lam"], inp["x"], inp["h0"], h_out=h)
                lr.linrec_backward(inp["lam"], h, inp["h0"], inp["grad_h"], grad_x=gx, grad_lambda=gl, grad_h0=gh0)
            for rep in range(4):
                say(f"graph replay {rep}")
                for t in (h, gx, gl, gh0):
                    t.fill_(float("nan"))
                g.replay()
                s.synchronize()
                for got, want in zip((h, gx, gl, gh0), ref):
                    assert reruns_agree(got, want), f"replay {rep} differs from the eager result"
                # eager work of the library on the same stream between replays
                other = wl.make_generic(3000 + 500 * rep, 1, 96, 900 + rep, device=DEV)
                fwd_bwd_check(other, f"eager between replays {rep}")
            lr.linrec_check(s)
    check_forward(inp, ref[0], "graph reference")


def test_tuned_plan_is_used_and_correct():
    """linrec_tune() times the candidate plans on scratch tensors and later calls with that shape use
    the winner; results must stay correct whatever it picked."""
    T, B, n = 20000, 2, 96
    inp = wl.make_inputs(2, T=T, B=B, n=n, device=DEV)
    lr.linrec_tune(T, B, n, backward=False)
    lr.linrec_tune(T, B, n, backward=True)
    vf, tf = lr.linrec_plan(T, B, n, backward=False)
    vb, tb = lr.linrec_plan(T, B, n, backward=True)
    say(f"tuned plan: forward tile {tf}, backward tile {tb}")
    assert vf == lr.VARIANT_LOOKBACK and vb == lr.VARIANT_LOOKBACK
    assert lr.linrec_tile_info(tf) is not None and lr.linrec_tile_info(tb) is not None
    fwd_bwd_check(inp, "tuned plan")
    with pytest.raises(lr.LinrecError):
        lr.linrec_tune(0, 2, 3)
    # a short, wide shape: the walk is among the candidates, and whatever wins is used and is right
    T, B, n = 700, 8, 1536
    for bwd in (False, True):
        lr.linrec_tune(T, B, n, backward=bwd)
        v, t = lr.linrec_plan(T, B, n, backward=bwd)
        say(f"tuned plan, short and wide, {'backward' if bwd else 'forward'}: variant {v} tile {t}")
        assert v in (lr.VARIANT_WALK, lr.VARIANT_LOOKBACK) and lr.linrec_tile_info(t) is not None
        with options(variant=lr.VARIANT_LOOKBACK):                      # an explicit variant is not overridden
            assert lr.linrec_plan(T, B, n, backward=bwd)[0] == lr.VARIANT_LOOKBACK
    fwd_bwd_check(wl.make_inputs(2, T=T, B=B, n=n, device=DEV), "tuned plan, short and wide")


@pytest.mark.parametrize("cfg", [2, 3])
def test_configs_full_size_with_tuned_plan(cfg):
    """What bench.py times: the plan linrec_tune() picks for the full-size workload."""
    inp = wl.make_inputs(cfg, device=DEV)
    lr.linrec_tune(inp["T"], inp["B"], inp["n"], backward=False)
    lr.linrec_tune(inp["T"], inp["B"], inp["n"], backward=True)
    say(f"cfg{cfg} tuned: fwd {lr.linrec_plan(inp['T'], inp['B'], inp['n'], backward=False)}, "
        f"bwd {lr.linrec_plan(inp['T'], inp['B'], inp['n'], backward=True)}")
    fwd_bwd_check(inp, f"cfg{cfg} full tuned")


@pytest.mark.parametrize("variant", ["threephase", "lookback", "walk"])
def test_non_finite_values_stay_in_their_column(variant):
    """NaN / Inf in one column must not leak into other columns, and must not hang the look-back."""
    inp = wl.make_inputs(2, T=9000, B=1, n=96, device=DEV)
    clean = {k: (v.clone() if torch.is_tensor(v) else v) for k, v in inp.items()}
    inp["x"][1234, 0, 5] = float("nan")
    inp["x"][4321, 0, 17] = float("inf")
    inp["lam"][100, 0, 40] = float("nan")
    bad = [5, 17, 40]
    good = [c for c in range(96) if c not in bad]
    with options(variant=VARIANTS[variant]):
        h = run_forward(inp)
        h_clean = run_forward(clean)
        gx, gl, gh0 = run_backward(inp, h_clean)       # backward on finite h: only lambda's NaN column is affected
        gx_c, gl_c, gh0_c = run_backward(clean, h_clean)
    torch.cuda.synchronize()
    lr.linrec_check()
    ex = variant != "lookback"
    assert reruns_agree(h[:, :, good], h_clean[:, :, good], ex)
    assert torch.isnan(h[1234:, 0, 5]).all() and torch.isfinite(h[:1234, 0, 5]).all()
    assert not torch.isfinite(h[4321:, 0, 17]).any() and torch.isfinite(h[:4321, 0, 17]).all()
    assert torch.isnan(h[100:, 0, 40]).all()
    ok = [c for c in range(96) if c != 40]
    assert reruns_agree(gx[:, :, ok], gx_c[:, :, ok], ex) and reruns_agree(gl[:, :, ok], gl_c[:, :, ok], ex)
    assert torch.isnan(gx[:99, 0, 40]).all() and torch.isfinite(gx[100:, 0, 40]).all()


@pytest.mark.parametrize("variant", ["threephase", "lookback", "serial", "walk"])
def test_growing_recurrence_within_the_documented_domain(variant):
    """|lambda| > 1 is supported while the partial products stay finite."""
    T, B, n = 700, 1, 64
    inp = wl.make_generic(T, B, n, 77, device=DEV, lam_kind="signed")
    inp["lam"] = (1.0 + 0.02 * inp["lam"]).contiguous()          # in [0.98, 1.02]: products up to ~1e6
    with options(variant=VARIANTS[variant]):
        fwd_bwd_check(inp, f"growing {variant}")


WIDE_TILES = [i for i, info in all_tiles(lr.ENTRY_PLAIN) if info["threads_cols"] > 64]


@pytest.mark.parametrize("variant", ["threephase", "lookback", "walk"])
def test_tiles_wider_than_a_wavefront_on_problems_narrower_than_the_tile(variant):
    """Shapes with 128 or 256 threads side by side: two or four wavefronts share a row of the tile, and on a narrow or
    ragged problem whole wavefronts hold no column at all (they still take part in the scan's barriers and in the
    look-back's vote)."""
    assert WIDE_TILES, "the build has no tile wider than a wavefront"
    for tile in WIDE_TILES:
        for C in (1, 37, 65, 129, 257):
            for T in (1, 700, 2100):
                inp = wl.make_generic(T, 1, C, seed=tile * 1000 + C + T, device=DEV, lam_kind="mixed", with_h0=bool((C + T) & 1))
                with options(variant=getattr(lr, "VARIANT_" + variant.upper()), tile=tile):
                    fwd_bwd_check(inp, f"tile {tile} T={T} C={C} {variant}")
