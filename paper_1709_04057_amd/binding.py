"""ctypes binding of the liblinrec C ABI (argument marshalling only)."""
from __future__ import annotations

import ctypes
import os
import re

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("LINREC_LIB_PATH", os.path.join(_HERE, "liblinrec.so"))
_HEADER = os.path.join(os.path.dirname(_HERE), "include", "linrec.h")
_lib = None

VARIANT_AUTO, VARIANT_THREEPHASE, VARIANT_LOOKBACK, VARIANT_SERIAL, VARIANT_WALK = 0, 1, 2, 3, 4
TAU_IDENTITY, TAU_TANH = 0, 1
OPT_VARIANT, OPT_TILE, OPT_CHUNK_TILES, OPT_SPIN_LIMIT, OPT_HPREV_LATE, OPT_TAPER, OPT_PERSISTENT, OPT_GRID_CAP = 1, 2, 3, 4, 5, 6, 7, 8
OPT_STAGGER = 9
OPT_TEST_FILL, OPT_TEST_EPOCH = 10, 11
ERR_CAPTURE, ERR_SCRATCH = -7, -8


class LinrecError(RuntimeError):
    def __init__(self, status, detail=""):
        self.status = status
        msg = "liblinrec error %d: %s" % (status, linrec_status_string(status))
        if detail:
            msg += " (" + detail + ")"
        super().__init__(msg)


def lib_path() -> str:
    return _LIB_PATH


def lib():
    """Loads liblinrec.so (built in-tree by ``paper_1709_04057_amd/build.py``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                "liblinrec.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                "(there is no CPU fallback)")
        L = ctypes.CDLL(_LIB_PATH)
        i64, p, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        pi = ctypes.POINTER(ctypes.c_int)
        L.linrec_forward.argtypes = [p, p, p, p, i64, i64, i64, p]
        L.linrec_forward.restype = ci
        L.linrec_backward.argtypes = [p, p, p, p, p, p, p, i64, i64, i64, p]
        L.linrec_backward.restype = ci
        L.linrec_forward_noalloc.argtypes = [p, p, p, p, i64, i64, i64, p]
        L.linrec_forward_noalloc.restype = ci
        L.linrec_noalloc_scratch_bytes.argtypes = []
        L.linrec_noalloc_scratch_bytes.restype = i64
        L.linrec_pin_plan.argtypes = [ci, i64, i64, i64, ci, ci, ci, ci, ci]
        L.linrec_pin_plan.restype = ci
        L.linrec_reserve_workspace.argtypes = [ci, i64, i64, i64, ci, p]
        L.linrec_reserve_workspace.restype = ci
        for fn in (L.linrec_forward_bf16,):
            fn.argtypes = [p, p, p, p, i64, i64, i64, p]
            fn.restype = ci
        L.linrec_backward_bf16.argtypes = [p, p, p, p, p, p, p, i64, i64, i64, p]
        L.linrec_backward_bf16.restype = ci
        L.linrec_validate_forward_bf16.argtypes = [p, p, p, p, i64, i64, i64]
        L.linrec_validate_forward_bf16.restype = ci
        L.linrec_validate_backward_bf16.argtypes = [p, p, p, p, p, p, p, i64, i64, i64]
        L.linrec_validate_backward_bf16.restype = ci
        L.linrec_validate_forward.argtypes = [p, p, p, p, i64, i64, i64]
        L.linrec_validate_forward.restype = ci
        L.linrec_validate_backward.argtypes = [p, p, p, p, p, p, p, i64, i64, i64]
        L.linrec_validate_backward.restype = ci
        L.linrec_gilr_forward.argtypes = [p, p, p, p, ci, i64, i64, i64, p]
        L.linrec_gilr_forward.restype = ci
        L.linrec_gilr_backward.argtypes = [p, p, p, p, p, p, p, p, ci, i64, i64, i64, p]
        L.linrec_gilr_backward.restype = ci
        L.linrec_validate_gilr_forward.argtypes = [p, p, p, p, ci, i64, i64, i64]
        L.linrec_validate_gilr_forward.restype = ci
        L.linrec_validate_gilr_backward.argtypes = [p, p, p, p, p, p, p, p, ci, i64, i64, i64]
        L.linrec_validate_gilr_backward.restype = ci
        L.linrec_lstm_cell_forward.argtypes = [p] * 7 + [i64, i64, i64, p]
        L.linrec_lstm_cell_forward.restype = ci
        L.linrec_lstm_cell_backward.argtypes = [p] * 12 + [i64, i64, i64, p]
        L.linrec_lstm_cell_backward.restype = ci
        L.linrec_validate_lstm_cell_forward.argtypes = [p] * 7 + [i64, i64, i64]
        L.linrec_validate_lstm_cell_forward.restype = ci
        L.linrec_validate_lstm_cell_backward.argtypes = [p] * 12 + [i64, i64, i64]
        L.linrec_validate_lstm_cell_backward.restype = ci
        for name in ("gilr_forward", "gilr_backward", "lstm_cell_forward", "lstm_cell_backward"):
            getattr(L, "linrec_%s_bf16" % name).argtypes = getattr(L, "linrec_" + name).argtypes
            getattr(L, "linrec_%s_bf16" % name).restype = ci
            getattr(L, "linrec_validate_%s_bf16" % name).argtypes = getattr(L, "linrec_validate_" + name).argtypes
            getattr(L, "linrec_validate_%s_bf16" % name).restype = ci
        L.linrec_set_option.argtypes = [ci, i64]
        L.linrec_set_option.restype = ci
        L.linrec_get_option.argtypes = [ci]
        L.linrec_get_option.restype = i64
        L.linrec_tile_info.argtypes = [ci, pi, pi, pi, pi]
        L.linrec_tile_info.restype = ci
        L.linrec_plan_taper.argtypes = [ci, i64, i64, i64, ci, ci]
        L.linrec_plan_taper.restype = ci
        L.linrec_tile_has.argtypes = [ci, ci]
        L.linrec_tile_has.restype = ci
        L.linrec_plan.argtypes = [i64, i64, i64, ci, ci, pi, pi]
        L.linrec_plan.restype = ci
        L.linrec_plan_for.argtypes = [ci, i64, i64, i64, ci, ci, pi, pi]
        L.linrec_plan_for.restype = ci
        L.linrec_stream_probe.argtypes = [p, p, p, p, p, i64, p]
        L.linrec_stream_probe.restype = ci
        L.linrec_stream_probe_rows.argtypes = [p, p, p, p, p, i64, i64, p]
        L.linrec_stream_probe_rows.restype = ci
        L.linrec_tune.argtypes = [i64, i64, i64, ci, p]
        L.linrec_tune.restype = ci
        L.linrec_tune_for.argtypes = [ci, i64, i64, i64, ci, p]
        L.linrec_tune_for.restype = ci
        L.linrec_check.argtypes = [p]
        L.linrec_check.restype = ci
        L.linrec_release_workspace.argtypes = []
        L.linrec_release_workspace.restype = ci
        L.linrec_status_string.argtypes = [ci]
        L.linrec_status_string.restype = ctypes.c_char_p
        L.linrec_last_hip_error.argtypes = []
        L.linrec_last_hip_error.restype = ctypes.c_char_p
        L.linrec_version.argtypes = []
        L.linrec_version.restype = ci
        _lib = L
    return _lib


def declared_symbols():
    """Names of the functions declared in include/linrec.h."""
    with open(_HEADER) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    return sorted(set(re.findall(r"\b(linrec_[a-z0-9_]+)\s*\(", text)))


def linrec_status_string(status: int) -> str:
    return lib().linrec_status_string(int(status)).decode()


def linrec_version() -> int:
    return lib().linrec_version()


def _check(rc):
    if rc != 0:
        detail = lib().linrec_last_hip_error().decode() if rc == -4 else ""
        raise LinrecError(rc, detail)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _tbn(t, name, dtype=None):
    import torch
    dtype = dtype or torch.float32
    if t.dtype != dtype or not t.is_cuda or not t.is_contiguous() or t.dim() != 3:
        raise ValueError(f"{name} must be a contiguous {dtype} CUDA tensor of shape [T, B, n]")
    return t.shape


def _bn(t, name, B, n, dtype=None):
    import torch
    dtype = dtype or torch.float32
    if t is None:
        return
    if t.dtype != dtype or not t.is_cuda or not t.is_contiguous() or tuple(t.shape) != (B, n):
        raise ValueError(f"{name} must be a contiguous {dtype} CUDA tensor of shape [B, n] = [{B}, {n}]")


def linrec_forward(lam, x, h0=None, h_out=None, stream=None):
    """h_out[t] = lam[t] * h_out[t-1] + x[t], h_out[-1] = h0.  Enqueues on ``stream`` and returns h_out.

    float32 tensors go to linrec_forward, bfloat16 tensors (all of them) to linrec_forward_bf16."""
    import torch
    dt = lam.dtype if lam.dtype == torch.bfloat16 else torch.float32
    T, B, n = _tbn(lam, "lambda", dt)
    if tuple(x.shape) != (T, B, n):
        raise ValueError("x must have lambda's shape")
    _tbn(x, "x", dt)
    _bn(h0, "h0", B, n, dt)
    if h_out is None:
        h_out = torch.empty_like(x)
    elif tuple(_tbn(h_out, "h_out", dt)) != (T, B, n):
        raise ValueError("h_out must have lambda's shape")
    fn = lib().linrec_forward_bf16 if dt == torch.bfloat16 else lib().linrec_forward
    _check(fn(_ptr(lam), _ptr(x), _ptr(h0), _ptr(h_out), T, B, n, _stream_ptr(stream)))
    return h_out


def linrec_forward_noalloc(lam, x, h0, h_out, stream=None):
    """linrec_forward through the entry point that allocates nothing; ``h_out`` must be given (float32 only)."""
    T, B, n = _tbn(lam, "lambda")
    if tuple(_tbn(x, "x")) != (T, B, n) or tuple(_tbn(h_out, "h_out")) != (T, B, n):
        raise ValueError("x and h_out must have lambda's shape")
    _bn(h0, "h0", B, n)
    _check(lib().linrec_forward_noalloc(_ptr(lam), _ptr(x), _ptr(h0), _ptr(h_out), T, B, n, _stream_ptr(stream)))
    return h_out


def linrec_noalloc_scratch_bytes() -> int:
    return int(lib().linrec_noalloc_scratch_bytes())


def linrec_backward(lam, h, h0, grad_h, grad_x=None, grad_lambda=None, grad_h0=None, stream=None,
                    want_grad_x=True, want_grad_lambda=True, want_grad_h0=True):
    """Gradients of the recurrence for upstream ``grad_h``; returns (grad_x, grad_lambda, grad_h0).

    Output tensors are allocated unless given; pass ``want_*=False`` to skip an output (returned as None).
    float32 tensors go to linrec_backward, bfloat16 tensors (all of them) to linrec_backward_bf16.
    """
    import torch
    dt = lam.dtype if lam.dtype == torch.bfloat16 else torch.float32
    T, B, n = _tbn(lam, "lambda", dt)
    for name, t in (("h", h), ("grad_h", grad_h)):
        if tuple(_tbn(t, name, dt)) != (T, B, n):
            raise ValueError(f"{name} must have lambda's shape")
    _bn(h0, "h0", B, n, dt)
    if grad_x is None and want_grad_x:
        grad_x = torch.empty_like(grad_h)
    if grad_lambda is None and want_grad_lambda:
        grad_lambda = torch.empty_like(grad_h)
    if grad_h0 is None and want_grad_h0:
        grad_h0 = torch.empty((B, n), dtype=dt, device=lam.device)
    for name, t in (("grad_x", grad_x), ("grad_lambda", grad_lambda)):
        if t is not None and tuple(_tbn(t, name, dt)) != (T, B, n):
            raise ValueError(f"{name} must have lambda's shape")
    _bn(grad_h0, "grad_h0", B, n, dt)
    fn = lib().linrec_backward_bf16 if dt == torch.bfloat16 else lib().linrec_backward
    _check(fn(_ptr(lam), _ptr(h), _ptr(h0), _ptr(grad_h), _ptr(grad_x), _ptr(grad_lambda), _ptr(grad_h0), T, B, n,
              _stream_ptr(stream)))
    return grad_x, grad_lambda, grad_h0


def linrec_gilr_forward(g_pre, i_pre, h0=None, h_out=None, tau=TAU_TANH, stream=None):
    """h[t] = g*h[t-1] + (1-g)*tau(i_pre[t]) with g = sigmoid(g_pre[t]); returns h_out.

    float32 tensors go to linrec_gilr_forward, bfloat16 tensors (all of them) to linrec_gilr_forward_bf16."""
    import torch
    dt = g_pre.dtype if g_pre.dtype == torch.bfloat16 else torch.float32
    T, B, n = _tbn(g_pre, "g_pre", dt)
    if tuple(_tbn(i_pre, "i_pre", dt)) != (T, B, n):
        raise ValueError("i_pre must have g_pre's shape")
    _bn(h0, "h0", B, n, dt)
    if h_out is None:
        h_out = torch.empty_like(i_pre)
    elif tuple(_tbn(h_out, "h_out", dt)) != (T, B, n):
        raise ValueError("h_out must have g_pre's shape")
    fn = lib().linrec_gilr_forward_bf16 if dt == torch.bfloat16 else lib().linrec_gilr_forward
    _check(fn(_ptr(g_pre), _ptr(i_pre), _ptr(h0), _ptr(h_out), int(tau), T, B, n,
                                     _stream_ptr(stream)))
    return h_out


def linrec_gilr_backward(g_pre, i_pre, h, h0, grad_h, grad_g_pre=None, grad_i_pre=None, grad_h0=None, tau=TAU_TANH,
                         stream=None, want_grad_g_pre=True, want_grad_i_pre=True, want_grad_h0=True):
    """Gradients of the gated layer w.r.t. its pre-activations; returns (grad_g_pre, grad_i_pre, grad_h0)."""
    import torch
    dt = g_pre.dtype if g_pre.dtype == torch.bfloat16 else torch.float32
    T, B, n = _tbn(g_pre, "g_pre", dt)
    for name, t in (("i_pre", i_pre), ("h", h), ("grad_h", grad_h)):
        if tuple(_tbn(t, name, dt)) != (T, B, n):
            raise ValueError(f"{name} must have g_pre's shape")
    _bn(h0, "h0", B, n, dt)
    if grad_g_pre is None and want_grad_g_pre:
        grad_g_pre = torch.empty_like(grad_h)
    if grad_i_pre is None and want_grad_i_pre:
        grad_i_pre = torch.empty_like(grad_h)
    if grad_h0 is None and want_grad_h0:
        grad_h0 = torch.empty((B, n), dtype=dt, device=g_pre.device)
    for name, t in (("grad_g_pre", grad_g_pre), ("grad_i_pre", grad_i_pre)):
        if t is not None and tuple(_tbn(t, name, dt)) != (T, B, n):
            raise ValueError(f"{name} must have g_pre's shape")
    _bn(grad_h0, "grad_h0", B, n, dt)
    fn = lib().linrec_gilr_backward_bf16 if dt == torch.bfloat16 else lib().linrec_gilr_backward
    _check(fn(_ptr(g_pre), _ptr(i_pre), _ptr(h), _ptr(h0), _ptr(grad_h), _ptr(grad_g_pre),
                                      _ptr(grad_i_pre), _ptr(grad_h0), int(tau), T, B, n, _stream_ptr(stream)))
    return grad_g_pre, grad_i_pre, grad_h0


def linrec_lstm_cell_forward(f_pre, i_pre, z_pre, o_pre, c0=None, c_out=None, h_out=None, stream=None,
                             want_c=True, want_h=True):
    """c[t] = f*c[t-1] + i*z, h[t] = o*c[t] with f, i, o = sigmoid(pre-activations), z = tanh(z_pre); returns (c, h)."""
    import torch
    dt = f_pre.dtype if f_pre.dtype == torch.bfloat16 else torch.float32
    T, B, n = _tbn(f_pre, "f_pre", dt)
    for name, t in (("i_pre", i_pre), ("z_pre", z_pre)) + ((("o_pre", o_pre),) if o_pre is not None else ()):
        if tuple(_tbn(t, name, dt)) != (T, B, n):
            raise ValueError(f"{name} must have f_pre's shape")
    _bn(c0, "c0", B, n, dt)
    if c_out is None and want_c:
        c_out = torch.empty_like(f_pre)
    if h_out is None and want_h:
        h_out = torch.empty_like(f_pre)
    for name, t in (("c_out", c_out), ("h_out", h_out)):
        if t is not None and tuple(_tbn(t, name, dt)) != (T, B, n):
            raise ValueError(f"{name} must have f_pre's shape")
    fn = lib().linrec_lstm_cell_forward_bf16 if dt == torch.bfloat16 else lib().linrec_lstm_cell_forward
    _check(fn(_ptr(f_pre), _ptr(i_pre), _ptr(z_pre), _ptr(o_pre), _ptr(c0), _ptr(c_out),
                                          _ptr(h_out), T, B, n, _stream_ptr(stream)))
    return c_out, h_out


def linrec_lstm_cell_backward(f_pre, i_pre, z_pre, o_pre, c, c0, grad_h, grads=None, grad_c0=None, stream=None,
                              want=(True, True, True, True), want_grad_c0=True):
    """Gradients of the cell; returns (grad_f_pre, grad_i_pre, grad_z_pre, grad_o_pre, grad_c0).

    ``grads`` may hold four preallocated tensors (or None entries); ``want[k] = False`` skips output k."""
    import torch
    dt = f_pre.dtype if f_pre.dtype == torch.bfloat16 else torch.float32
    T, B, n = _tbn(f_pre, "f_pre", dt)
    for name, t in (("i_pre", i_pre), ("z_pre", z_pre), ("o_pre", o_pre), ("c", c), ("grad_h", grad_h)):
        if tuple(_tbn(t, name, dt)) != (T, B, n):
            raise ValueError(f"{name} must have f_pre's shape")
    _bn(c0, "c0", B, n, dt)
    outs = list(grads) if grads is not None else [None] * 4
    for k in range(4):
        if outs[k] is None and want[k]:
            outs[k] = torch.empty_like(grad_h)
        if outs[k] is not None and tuple(_tbn(outs[k], "grads[%d]" % k, dt)) != (T, B, n):
            raise ValueError("gradient outputs must have f_pre's shape")
    if grad_c0 is None and want_grad_c0:
        grad_c0 = torch.empty((B, n), dtype=dt, device=f_pre.device)
    _bn(grad_c0, "grad_c0", B, n, dt)
    fn = lib().linrec_lstm_cell_backward_bf16 if dt == torch.bfloat16 else lib().linrec_lstm_cell_backward
    _check(fn(_ptr(f_pre), _ptr(i_pre), _ptr(z_pre), _ptr(o_pre), _ptr(c), _ptr(c0),
              _ptr(grad_h), _ptr(outs[0]), _ptr(outs[1]), _ptr(outs[2]), _ptr(outs[3]),
              _ptr(grad_c0), T, B, n, _stream_ptr(stream)))
    return outs[0], outs[1], outs[2], outs[3], grad_c0


def linrec_set_option(option: int, value: int) -> None:
    _check(lib().linrec_set_option(int(option), int(value)))


def linrec_get_option(option: int) -> int:
    return int(lib().linrec_get_option(int(option)))


def linrec_tile_info(tile_id: int):
    """Returns dict(threads_cols, threads_time, rows_per_thread, cols_per_thread, rows, cols), or None for an id
    the library has no kernel of."""
    a, b, c, d = (ctypes.c_int() for _ in range(4))
    rc = lib().linrec_tile_info(int(tile_id), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(d))
    if rc != 0:
        return None
    return dict(threads_cols=a.value, threads_time=b.value, rows_per_thread=c.value, cols_per_thread=d.value,
                rows=b.value * c.value, cols=a.value * d.value)


def linrec_plan_taper(entry_point, T, B, n, backward=False, alignment=16) -> int:
    """Eighths of the last round of tiles the plan of this problem cuts into shorter tiles (0: none)."""
    rc = lib().linrec_plan_taper(int(entry_point), int(T), int(B), int(n), int(bool(backward)), int(alignment))
    if rc < 0:
        _check(rc)
    return rc


def linrec_tile_has(tile_id: int, entry_point: int) -> bool:
    """Whether the library has kernels of this tile shape for entry-point family ``entry_point`` (ENTRY_*)."""
    return bool(lib().linrec_tile_has(int(tile_id), int(entry_point)))


def linrec_plan(T, B, n, backward=False, alignment=16):
    """(variant, tile id) the library would pick for tensors aligned to ``alignment`` bytes."""
    v, t = ctypes.c_int(), ctypes.c_int()
    _check(lib().linrec_plan(int(T), int(B), int(n), int(bool(backward)), int(alignment), ctypes.byref(v), ctypes.byref(t)))
    return v.value, t.value


ENTRY_PLAIN, ENTRY_GILR, ENTRY_LSTM_CELL, ENTRY_BF16, ENTRY_GILR_BF16, ENTRY_LSTM_CELL_BF16 = 0, 1, 2, 3, 4, 5


def linrec_plan_for(entry_point, T, B, n, backward=False, alignment=16):
    """(variant, tile id) for one of the entry-point families ENTRY_*."""
    v, t = ctypes.c_int(), ctypes.c_int()
    _check(lib().linrec_plan_for(int(entry_point), int(T), int(B), int(n), int(bool(backward)), int(alignment),
                                 ctypes.byref(v), ctypes.byref(t)))
    return v.value, t.value


def linrec_pin_plan(entry_point, T, B, n, backward, variant, tile_id, persistent=-1, taper=0) -> None:
    """Fixes the plan of one shape for all threads (``tile_id = 0`` forgets it); see include/linrec.h."""
    _check(lib().linrec_pin_plan(int(entry_point), int(T), int(B), int(n), int(bool(backward)), int(variant),
                                 int(tile_id), int(persistent), int(taper)))


def linrec_reserve_workspace(entry_point, T, B, n, backward=False, stream=None) -> None:
    """Sizes the stream's cached workspace for a later call of this shape, so that the call allocates nothing."""
    _check(lib().linrec_reserve_workspace(int(entry_point), int(T), int(B), int(n), int(bool(backward)),
                                          _stream_ptr(stream)))


def linrec_stream_probe(in0, in1, in2, out0, out1, stream=None) -> None:
    """Pure streaming kernel over flat float32 CUDA tensors (None = absent); see include/linrec.h."""
    n = next(t for t in (out0, out1, in0, in1, in2) if t is not None).numel()
    _check(lib().linrec_stream_probe(_ptr(in0), _ptr(in1), _ptr(in2), _ptr(out0), _ptr(out1), n, _stream_ptr(stream)))


def linrec_stream_probe_rows(in0, in1, in2, out0, out1, T, C, stream=None) -> None:
    """The streaming kernel in the geometry of a tile, over [T, C] float32 CUDA tensors (None = absent, given from
    the front); see include/linrec.h."""
    import torch
    for t in (in0, in1, in2, out0, out1):
        if t is not None and (not t.is_cuda or t.dtype != torch.float32 or not t.is_contiguous() or t.numel() != T * C):
            raise ValueError("linrec_stream_probe_rows: contiguous float32 CUDA tensors of T*C elements")
    _check(lib().linrec_stream_probe_rows(_ptr(in0), _ptr(in1), _ptr(in2), _ptr(out0), _ptr(out1), int(T), int(C),
                                          _stream_ptr(stream)))


def linrec_tune_for(entry_point, T, B, n, backward=False, stream=None) -> None:
    """linrec_tune for one of the entry-point families ENTRY_*."""
    _check(lib().linrec_tune_for(int(entry_point), int(T), int(B), int(n), int(bool(backward)), _stream_ptr(stream)))


def linrec_tune(T, B, n, backward=False, stream=None) -> None:
    """Times the candidate plans for this shape on the GPU and remembers the fastest (see include/linrec.h)."""
    _check(lib().linrec_tune(int(T), int(B), int(n), int(bool(backward)), _stream_ptr(stream)))


def linrec_check(stream=None) -> None:
    """Synchronises the stream and raises if a look-back kernel gave up waiting."""
    _check(lib().linrec_check(_stream_ptr(stream)))


def linrec_release_workspace() -> None:
    _check(lib().linrec_release_workspace())
