"""Seeded random sweep over shapes and launch options for every entry point, each case compared
element by element with the fp64 oracle (arXiv 1709.04057: Sections 2, 2.2, 3.1, 3.2).  Complements the
hand-picked edge shapes: ragged tiles, partial column groups, short sequences, option combinations; a
second set has thousands of columns, a third tens to hundreds of thousands of steps on few columns."""
import numpy as np
import pytest
import torch

import linrec_workloads as wl
import paper_1709_04057_amd as lr
from parity import all_tiles, fwd_bwd_check, options, say
from test_bf16_parity_gpu import bf16_check, to_bf16
from test_gilr_parity_gpu import gated_check
from test_lstm_parity_gpu import cell_check
from test_forms_bf16_parity_gpu import cell16_check, gated16_check
from test_forms_bf16_parity_gpu import to_bf16 as forms_to_bf16

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TILE_CHOICES = [0] + [i for i, _ in all_tiles()]     # 0 = the library's own choice


def _cases(seed, n):
    rng = np.random.default_rng(seed)
    for i in range(n):
        T = int(rng.choice([rng.integers(1, 40), rng.integers(40, 1200), rng.integers(1200, 9000)]))
        C = int(rng.choice([rng.integers(1, 20), rng.integers(20, 140), rng.integers(140, 600)]))
        B = int(rng.choice([1, 1, 2, 3]))
        n_ = max(1, C // B)
        opts = dict(variant=int(rng.choice([lr.VARIANT_AUTO, lr.VARIANT_LOOKBACK, lr.VARIANT_LOOKBACK, lr.VARIANT_THREEPHASE,
                                            lr.VARIANT_SERIAL, lr.VARIANT_WALK])),
                    tile=int(rng.choice(TILE_CHOICES)), persistent=int(rng.integers(-1, 2)),
                    taper=int(rng.choice([-1, 0, 2, 8])), hprev_late=int(rng.integers(-1, 2)))
        yield i, T, B, n_, opts, int(rng.integers(1 << 30))


def _wide_cases(seed, n):
    """Thousands of columns (many column groups, the multi-column shapes, the walk) on short sequences."""
    rng = np.random.default_rng(seed)
    for i in range(n):
        T, C, B = int(rng.integers(50, 2000)), int(rng.integers(1000, 12000)), int(rng.choice([1, 2, 4]))
        opts = dict(variant=int(rng.choice([lr.VARIANT_AUTO, lr.VARIANT_LOOKBACK, lr.VARIANT_WALK])),
                    tile=int(rng.choice(TILE_CHOICES)), persistent=int(rng.integers(-1, 2)),
                    taper=int(rng.choice([-1, 0, 2])), hprev_late=int(rng.integers(-1, 2)))
        yield i, T, B, max(1, C // B), opts, int(rng.integers(1 << 30))


def _long_cases(seed, n):
    """Long sequences on few columns: hundreds of tiles along T, look-back windows over many predecessors,
    the short tiles that end a sequence."""
    rng = np.random.default_rng(seed)
    for i in range(n):
        C = int(rng.choice([rng.integers(1, 9), rng.integers(9, 70), rng.integers(70, 300)]))
        T = int(rng.integers(20000, min(400000, 12_000_000 // C)))
        B = int(rng.choice([1, 1, 2]))
        opts = dict(variant=int(rng.choice([lr.VARIANT_AUTO, lr.VARIANT_LOOKBACK, lr.VARIANT_LOOKBACK, lr.VARIANT_THREEPHASE])),
                    tile=int(rng.choice(TILE_CHOICES)), persistent=int(rng.integers(-1, 2)),
                    taper=int(rng.choice([-1, 0, 2, 8])), hprev_late=int(rng.integers(-1, 2)))
        yield i, T, B, max(1, C // B), opts, int(rng.integers(1 << 30))


ENTRIES = {"plain": 1, "gated": 2, "lstm": 3, "bf16": 4, "gated_bf16": 5, "lstm_bf16": 6}


@pytest.mark.parametrize("shapes", ["mixed", "wide", "long"])
@pytest.mark.parametrize("entry", list(ENTRIES))
def test_random_shapes_and_options(entry, shapes):
    cases = {"mixed": lambda: _cases(ENTRIES[entry], 40), "wide": lambda: _wide_cases(100 + ENTRIES[entry], 12),
             "long": lambda: _long_cases(200 + ENTRIES[entry], 10)}[shapes]()
    for i, T, B, n, opts, seed in cases:
        label = f"{entry} #{i} T={T} B={B} n={n} {opts}"
        say(label)
        with options(**opts):
            if entry == "plain":
                kind = ["sigmoid", "signed", "mixed"][seed % 3]
                fwd_bwd_check(wl.make_generic(T, B, n, seed=seed, device=DEV, lam_kind=kind, with_h0=bool(seed & 8)), label)
            elif entry == "gated":
                gated_check(wl.make_gated(T, B, n, seed=seed, device=DEV, gate_mean=float(seed % 5) - 1.0, gate_std=2.0,
                                          with_h0=bool(seed & 8)), lr.TAU_TANH if seed & 16 else lr.TAU_IDENTITY, label)
            elif entry == "lstm":
                cell_check(wl.make_lstm(T, B, n, seed=seed, device=DEV, forget_mean=float(seed % 4), with_c0=bool(seed & 8)),
                           label)
            elif entry == "gated_bf16":
                gated16_check(forms_to_bf16(wl.make_gated(T, B, n, seed=seed, device=DEV, gate_mean=float(seed % 5) - 1.0,
                                                          gate_std=2.0, with_h0=bool(seed & 8))),
                              lr.TAU_TANH if seed & 16 else lr.TAU_IDENTITY, label)
            elif entry == "lstm_bf16":
                cell16_check(forms_to_bf16(wl.make_lstm(T, B, n, seed=seed, device=DEV, forget_mean=float(seed % 4),
                                                        with_c0=bool(seed & 8))), label)
            else:
                bf16_check(to_bf16(wl.make_generic(T, B, n, seed=seed, device=DEV, with_h0=bool(seed & 8))), label)
    torch.cuda.synchronize()
    lr.linrec_check()
