"""Thin Python binding of liblinrec (AMD MI355X / gfx950).

The functions here only marshal arguments (device pointers, shapes, the current HIP stream) into the
C ABI declared in ``include/linrec.h``; every step of the recurrence runs in the library's HIP
kernels.  There is no CPU fallback: if ``liblinrec.so`` has not been built the first call raises.
PyTorch is used for device memory and streams only.
"""
from .autograd import gilr, linear_recurrence, lstm_cell  # noqa: F401
from .binding import (  # noqa: F401
    ENTRY_BF16,
    ENTRY_GILR,
    ENTRY_GILR_BF16,
    ENTRY_LSTM_CELL,
    ENTRY_LSTM_CELL_BF16,
    ENTRY_PLAIN,
    LinrecError,
    OPT_CHUNK_TILES,
    OPT_GRID_CAP,
    OPT_HPREV_LATE,
    OPT_PERSISTENT,
    OPT_SPIN_LIMIT,
    OPT_STAGGER,
    OPT_TAPER,
    OPT_TILE,
    OPT_VARIANT,
    TAU_IDENTITY,
    TAU_TANH,
    VARIANT_AUTO,
    VARIANT_LOOKBACK,
    VARIANT_SERIAL,
    VARIANT_THREEPHASE,
    VARIANT_WALK,
    declared_symbols,
    lib,
    lib_path,
    linrec_backward,
    linrec_check,
    linrec_forward,
    linrec_get_option,
    linrec_gilr_backward,
    linrec_gilr_forward,
    linrec_lstm_cell_backward,
    linrec_lstm_cell_forward,
    linrec_plan,
    linrec_plan_for,
    linrec_release_workspace,
    linrec_set_option,
    linrec_status_string,
    linrec_stream_probe,
    linrec_tile_info,
    linrec_tune,
    linrec_tune_for,
    linrec_version,
)
