"""The cached look-back workspace across calls: stale words, the epoch's wrap, growth and retirement,
reservation ahead of a HIP-graph capture, pinned plans.  Every kernel here exits normally: the reuse paths
are driven from the host through the library's test options (a fill pattern for newly allocated words, a
planted stored epoch), never by breaking a kernel."""
import pytest
import torch

import linrec_workloads as wl
import paper_1709_04057_amd as lr
from parity import (check_backward, check_forward, fwd_bwd_check, one_column_tiles, options, reruns_agree, run_backward,
                    run_forward, say)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
WRAP = 2 ** 31 - 2          # largest stored epoch; the call that runs on it wraps the counter to 0


class test_options:
    def __init__(self, **kw):
        self.kw = kw
        self.ids = dict(fill=lr.OPT_TEST_FILL, epoch=lr.OPT_TEST_EPOCH)

    def __enter__(self):
        for k, v in self.kw.items():
            lr.linrec_set_option(self.ids[k], v)

    def __exit__(self, *exc):
        lr.linrec_set_option(lr.OPT_TEST_FILL, 0)
        lr.linrec_set_option(lr.OPT_TEST_EPOCH, -1)
        return False


@pytest.mark.parametrize("fill", [0xDEADBEEF, 0x80000000, 0xFFFFFFFF])
def test_stale_words_with_foreign_tags_are_ignored(fill):
    """A newly allocated workspace whose words all carry a non-zero pattern (as memory that an earlier,
    unrelated epoch wrote would): no tag of a running call matches it, so results are unchanged."""
    s = torch.cuda.Stream()                      # a stream of its own: its workspace is allocated here
    inp = wl.make_inputs(2, T=30000, B=2, n=96, device=DEV)
    with test_options(fill=fill), options(variant=lr.VARIANT_LOOKBACK), torch.cuda.stream(s):
        for rep in range(3):
            say(f"fill {fill:#x}: call {rep}")
            fwd_bwd_check(inp, f"poisoned workspace {fill:#x} call {rep}")
        bigger = wl.make_inputs(5, T=70000, B=2, n=128, device=DEV)   # grows: the new block is poisoned too
        fwd_bwd_check(bigger, f"poisoned workspace {fill:#x}, grown")
        lr.linrec_check(s)


@pytest.mark.parametrize("start", [WRAP - 5, WRAP - 2, WRAP - 1])
def test_epoch_wrap(start):
    """Calls across the wrap of the 31-bit epoch.  The workspace is first used from its true start, so
    words tagged with the small epochs the counter returns to after the wrap are lying in it; the stored
    epoch is then planted just below the wrap, the periodic clearing of stale words comes two calls later
    (before the first call that runs on a small epoch again), and eight calls run through the wrap --
    each checked against the oracle."""
    s = torch.cuda.Stream()
    shapes = [(9000, 2, 64), (20000, 1, 160), (9000, 2, 64)]
    with options(variant=lr.VARIANT_LOOKBACK), torch.cuda.stream(s):
        for i, (T, B, n) in enumerate(shapes):            # epochs 1, 2, ... leave their words behind
            fwd_bwd_check(wl.make_generic(T, B, n, 40 + i, device=DEV, lam_kind="mixed"), f"before planting {i}")
        with test_options(epoch=start):
            for call in range(8):
                T, B, n = shapes[call % len(shapes)]
                inp = wl.make_generic(T, B, n, 60 + call, device=DEV, lam_kind="mixed")
                say(f"epoch planted at {start}: call {call}")
                h = run_forward(inp)
                s.synchronize()
                check_forward(inp, h, f"wrap from {start} call {call}")
                if call % 2:
                    gx, gl, gh0 = run_backward(inp, h)
                    s.synchronize()
                    check_backward(inp, h, gx, gl, gh0, f"wrap from {start} call {call}")
        assert lr.linrec_get_option(lr.OPT_TEST_EPOCH) == -1      # consumed by the first call
        lr.linrec_check(s)


def test_growth_retires_the_old_block_and_a_recorded_graph_stays_valid():
    """A launch recorded in a HIP graph keeps the pointers of the workspace block it was recorded with.
    A larger eager call on the same stream makes the workspace grow; the old block is retired, not
    freed, so replays before and after give the eager result."""
    inp = wl.make_inputs(2, T=12000, B=2, n=64, device=DEV)
    big = wl.make_inputs(2, T=60000, B=4, n=128, device=DEV)
    s = torch.cuda.Stream()
    with options(variant=lr.VARIANT_LOOKBACK), torch.cuda.stream(s):
        h = torch.empty_like(inp["x"])
        lr.linrec_forward(inp["lam"], inp["x"], inp["h0"], h_out=h)          # allocates the small block
        s.synchronize()
        ref = h.clone()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            lr.linrec_forward(inp["lam"], inp["x"], inp["h0"], h_out=h)
        for rep in range(3):
            say(f"replay {rep}, then a larger eager call")
            h.fill_(float("nan"))
            g.replay()
            s.synchronize()
            assert reruns_agree(h, ref), f"replay {rep} differs"
            fwd_bwd_check(big if rep == 0 else inp, f"eager between replays {rep}")   # rep 0 grows the workspace
        lr.linrec_check(s)
    check_forward(inp, ref, "graph reference")


def test_reserve_then_capture_without_an_eager_call():
    """linrec_reserve_workspace sizes the workspace ahead of time, so the first call of a shape on a stream
    can be captured; without it the call refuses to grow the workspace under capture (LINREC_ERR_CAPTURE),
    enqueues nothing and leaves the capture intact."""
    inp = wl.make_inputs(2, T=40000, B=2, n=128, device=DEV)
    T, B, n = inp["T"], inp["B"], inp["n"]
    with options(variant=lr.VARIANT_LOOKBACK, tile=one_column_tiles(lr.ENTRY_PLAIN)[-1]):
        # (the kernels' code object is loaded by a first, eager launch of the same tile shape on another stream)
        fwd_bwd_check(wl.make_inputs(2, T=600, B=1, n=64, device=DEV), "loads the kernels")
        # (1) no reservation: the captured call is refused, the capture survives and can still record work
        s1 = torch.cuda.Stream()
        with torch.cuda.stream(s1):
            h = torch.empty_like(inp["x"])
            probe = torch.zeros(8, device=DEV)
            s1.synchronize()
            g1 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g1, stream=s1):
                with pytest.raises(lr.LinrecError) as err:
                    lr.linrec_forward(inp["lam"], inp["x"], inp["h0"], h_out=h)
                probe.add_(1.0)
            assert err.value.status == lr.ERR_CAPTURE
            g1.replay()
            s1.synchronize()
            assert float(probe[0]) == 1.0
        # (2) reserved: the very first forward and backward calls on the stream are captured and replayed
        s2 = torch.cuda.Stream()
        with torch.cuda.stream(s2):
            lr.linrec_reserve_workspace(lr.ENTRY_PLAIN, T, B, n, backward=False, stream=s2)
            lr.linrec_reserve_workspace(lr.ENTRY_PLAIN, T, B, n, backward=True, stream=s2)
            h = torch.empty_like(inp["x"])
            gx, gl = torch.empty_like(h), torch.empty_like(h)
            gh0 = torch.empty_like(inp["h0"])
            g2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g2, stream=s2):
                lr.linrec_forward(inp["lam"], inp["x"], inp["h0"], h_out=h)
                lr.linrec_backward(inp["lam"], h, inp["h0"], inp["grad_h"], grad_x=gx, grad_lambda=gl, grad_h0=gh0)
            for rep in range(3):
                for t in (h, gx, gl, gh0):
                    t.fill_(float("nan"))
                g2.replay()
                s2.synchronize()
                check_forward(inp, h, f"reserved, replay {rep}")
                check_backward(inp, h, gx, gl, gh0, f"reserved, replay {rep}")
            lr.linrec_check(s2)


def test_pinned_plan_is_reported_used_and_forgotten():
    T, B, n = 21000, 2, 96
    inp = wl.make_inputs(2, T=T, B=B, n=n, device=DEV)
    auto, auto_bwd = lr.linrec_plan(T, B, n, backward=False), lr.linrec_plan(T, B, n, backward=True)
    other, third = [t for t in one_column_tiles(lr.ENTRY_PLAIN) if t != auto[1]][:2]
    lr.linrec_pin_plan(lr.ENTRY_PLAIN, T, B, n, False, lr.VARIANT_LOOKBACK, other, persistent=1, taper=2)
    try:
        assert lr.linrec_plan(T, B, n, backward=False) == (lr.VARIANT_LOOKBACK, other)
        assert lr.linrec_plan(T, B, n, backward=True) == auto_bwd                 # the other pass is untouched
        assert lr.linrec_plan_for(lr.ENTRY_GILR, T, B, n, backward=False) == \
            lr.linrec_plan_for(lr.ENTRY_GILR, T + 1, B, n, backward=False)       # and so are the other families
        fwd_bwd_check(inp, "pinned plan")
        # a thread's own tile option still wins
        with options(tile=third):
            assert lr.linrec_plan(T, B, n, backward=False)[1] == third
    finally:
        lr.linrec_pin_plan(lr.ENTRY_PLAIN, T, B, n, False, lr.VARIANT_LOOKBACK, 0)
    assert lr.linrec_plan(T, B, n, backward=False) == auto
    with pytest.raises(lr.LinrecError):
        lr.linrec_pin_plan(lr.ENTRY_PLAIN, T, B, n, False, lr.VARIANT_THREEPHASE, other)
    with pytest.raises(lr.LinrecError):
        lr.linrec_pin_plan(lr.ENTRY_PLAIN, T, B, n, False, lr.VARIANT_LOOKBACK, 999)


def test_options_belong_to_the_calling_thread():
    """A thread that changes its options does not change the plan other threads' calls get."""
    import threading
    T, B, n = 20000, 2, 96
    seen = {}

    def worker():
        torch.cuda.set_device(0)
        seen["variant"] = lr.linrec_get_option(lr.OPT_VARIANT)
        seen["plan"] = lr.linrec_plan(T, B, n, backward=False)

    with options(variant=lr.VARIANT_SERIAL, tile=one_column_tiles(lr.ENTRY_PLAIN)[0]):
        t = threading.Thread(target=worker)
        t.start()
        t.join()
        assert lr.linrec_plan(T, B, n, backward=False)[0] == lr.VARIANT_SERIAL
    assert seen["variant"] == lr.VARIANT_AUTO and seen["plan"][0] != lr.VARIANT_SERIAL
