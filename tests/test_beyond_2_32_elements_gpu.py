"""Tensors of more than 2^32 elements (17 GB in fp32): the largest sizes a single MI355X still holds for
a forward+backward pass.  Element indices no longer fit 32 bits, so every index the kernels form from
T, C, a tile number or a column must be 64-bit, and the 32-bit offsets inside a tile must stay relative
to the tile's own origin.  The oracle evaluates whole columns (columns are independent recurrences,
Section 2): the first, a middle band and the last, which hold the lowest and the highest addresses.
"""
import numpy as np
import pytest
import torch

import linrec_workloads as wl
import paper_1709_04057_amd as lr
from parity import check_backward, check_forward, options, run_backward, run_forward, say
from test_bf16_parity_gpu import bf16_check
from test_bf16_parity_gpu import to_bf16 as plain_to_bf16
from test_forms_bf16_parity_gpu import cell16_check, gated16_check
from test_forms_bf16_parity_gpu import to_bf16 as forms_to_bf16
from test_gilr_parity_gpu import gated_check

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

# a ragged number of rows; only the last 8 thousand of them lie beyond element 2^32
T, B, n = 1_056_801, 8, 512
C = B * n
COLS = np.concatenate([np.arange(0, 32), np.arange(2040, 2056), np.arange(C - 32, C)])
VARIANTS = dict(lookback=lr.VARIANT_LOOKBACK, threephase=lr.VARIANT_THREEPHASE, walk=lr.VARIANT_WALK,
                serial=lr.VARIANT_SERIAL)


NEEDS_BYTES = 150 << 30  # the largest case holds 7 fp32 tensors of 17 GB, plus what the generators use meanwhile


@pytest.fixture(autouse=True)
def _device_memory():
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < NEEDS_BYTES:
        pytest.skip(f"needs {NEEDS_BYTES >> 30} GiB of free device memory, {free >> 30} GiB are free")
    yield
    torch.cuda.empty_cache()


def test_plain_recurrence_every_variant():
    inp = wl.make_inputs(5, T=T, B=B, n=n, device=DEV)
    assert inp["lam"].numel() > 2**32
    sel = torch.as_tensor(COLS, device=DEV)

    def pick(t, rows=True):  # the sampled columns as a problem of its own, [T, 1, len(COLS)]
        if t is None:
            return None
        return (t.reshape(T, C)[:, sel].reshape(T, 1, -1) if rows else t.reshape(C)[sel].reshape(1, -1)).contiguous()

    sub = dict(T=T, B=1, n=len(COLS), lam=pick(inp["lam"]), x=pick(inp["x"]), h0=pick(inp["h0"], rows=False),
               grad_h=pick(inp["grad_h"]))
    for name, variant in VARIANTS.items():
        with options(variant=variant):
            say(f"2^32+ elements, {name}: forward")
            h = run_forward(inp)
            torch.cuda.synchronize()
            hs = pick(h)
            check_forward(sub, hs, f"2^32+ elements {name}")
            say(f"2^32+ elements, {name}: backward")
            gx, gl, gh0 = run_backward(inp, h)
            torch.cuda.synchronize()
            check_backward(sub, hs, pick(gx), pick(gl), pick(gh0, rows=False), f"2^32+ elements {name}")
            lr.linrec_check()
            del h, gx, gl, gh0


def test_plain_recurrence_bf16_storage():
    inp = plain_to_bf16(wl.make_inputs(5, T=T, B=B, n=n, device=DEV))
    torch.cuda.empty_cache()
    r = bf16_check(inp, "2^32+ elements bf16", cols=COLS)
    say(f"2^32+ elements bf16: {r}")


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_gated_layer(storage):
    inp = wl.make_gated(T, B, n, seed=91, device=DEV, gate_mean=2.0)
    if storage == "bf16":
        inp = forms_to_bf16(inp)
        torch.cuda.empty_cache()
        r = gated16_check(inp, lr.TAU_TANH, "2^32+ elements gated bf16", cols=COLS)
    else:
        r = gated_check(inp, lr.TAU_TANH, "2^32+ elements gated", cols=COLS)
    say(f"2^32+ elements gated {storage}: {r}")


def test_lstm_cell_bf16_storage():
    # (eleven tensors: with fp32 storage they would not fit the GPU's memory at this size)
    inp = forms_to_bf16(wl.make_lstm(T, B, n, seed=92, device=DEV, forget_mean=2.0))
    torch.cuda.empty_cache()
    r = cell16_check(inp, "2^32+ elements cell bf16", cols=COLS)
    say(f"2^32+ elements cell bf16: {r}")
