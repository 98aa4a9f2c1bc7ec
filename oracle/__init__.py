"""fp64 CPU oracle for the diagonal linear recurrence of arXiv 1709.04057.

TEST INFRASTRUCTURE.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the GPU library never does, and
this package never imports the GPU library.

The arithmetic lives in ``linrec_oracle.c`` (plain sequential C loops); this
module compiles it with gcc, loads it through ctypes and offers numpy-level
wrappers:

* :func:`forward`, :func:`backward` -- one-shot evaluation, fp64 outputs;
* :func:`forward_compare`, :func:`backward_compare` -- stream a big problem
  through the same C loops in row slabs and fold the error norms against a
  candidate result, so that no full-size fp64 tensor is ever materialised.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "linrec_oracle.c")
_LIB = os.path.join(_HERE, "liblinrec_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile linrec_oracle.c into liblinrec_oracle.so next to it (gcc, -O2, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64 = ctypes.c_int64
        p = ctypes.c_void_p
        lib.linrec_oracle_forward.argtypes = [p, p, p, p, i64, i64, i64, i64, i64, i64]
        lib.linrec_oracle_forward.restype = None
        lib.linrec_oracle_backward.argtypes = [p, p, p, p, p, p, p, p, i64, i64, i64, i64, i64, i64]
        lib.linrec_oracle_backward.restype = None
        lib.linrec_oracle_gilr_forward.argtypes = [p, p, ctypes.c_int, p, p, i64, i64, i64, i64, i64, i64]
        lib.linrec_oracle_gilr_forward.restype = None
        lib.linrec_oracle_gilr_backward.argtypes = [p, p, ctypes.c_int, p, p, p, p, p, p, p,
                                                    i64, i64, i64, i64, i64, i64]
        lib.linrec_oracle_gilr_backward.restype = None
        lib.linrec_oracle_lstm_forward.argtypes = [p, p, p, p, p, p, p, i64, i64, i64, i64, i64, i64]
        lib.linrec_oracle_lstm_forward.restype = None
        lib.linrec_oracle_lstm_backward.argtypes = [p] * 13 + [i64] * 6
        lib.linrec_oracle_lstm_backward.restype = None
        _lib = lib
    return _lib


def _f32_2d(a, name):
    a = np.asarray(a)
    if a.dtype != np.float32:
        raise TypeError(f"{name} must be float32 (the oracle widens the same fp32 bits the GPU reads)")
    if a.ndim < 1:
        raise ValueError(f"{name} must have a leading time axis")
    T = a.shape[0]
    a2 = np.ascontiguousarray(a).reshape(T, -1) if T > 0 else np.zeros((0, int(np.prod(a.shape[1:], dtype=np.int64))), np.float32)
    return a2


def _f32_1d(a, C, name):
    if a is None:
        return None
    a = np.ascontiguousarray(np.asarray(a))
    if a.dtype != np.float32:
        raise TypeError(f"{name} must be float32")
    a = a.reshape(-1)
    if a.shape[0] != C:
        raise ValueError(f"{name} must have B*n = {C} elements")
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _col_ranges(C, threads):
    threads = max(1, min(int(threads), C if C > 0 else 1))
    edges = [(C * i) // threads for i in range(threads + 1)]
    return [(edges[i], edges[i + 1]) for i in range(threads) if edges[i + 1] > edges[i]]


def _run_over_columns(fn, C, threads):
    ranges = _col_ranges(C, threads)
    if len(ranges) <= 1:
        for c0, c1 in ranges:
            fn(c0, c1)
        return
    with ThreadPoolExecutor(max_workers=len(ranges)) as ex:
        for f in [ex.submit(fn, c0, c1) for c0, c1 in ranges]:
            f.result()


def forward_slab(lam2, x2, state, href, t0, t1, threads=1):
    """Advance ``state`` (fp64 [C]) over rows [t0, t1) and write those rows of ``href`` (fp64 [T, C])."""
    lib = _load()
    T, C = lam2.shape

    def work(c0, c1):
        lib.linrec_oracle_forward(_ptr(lam2), _ptr(x2), _ptr(state), _ptr(href), T, C, t0, t1, c0, c1)

    _run_over_columns(work, C, threads)


def forward(lam, x, h0=None, threads=1):
    """h[t] = lam[t]*h[t-1] + x[t], h[-1] = h0 (zeros when None).  Returns fp64 with lam's shape."""
    lam2 = _f32_2d(lam, "lambda")
    x2 = _f32_2d(x, "x")
    if lam2.shape != x2.shape:
        raise ValueError("lambda and x must have the same shape")
    T, C = lam2.shape
    h0v = _f32_1d(h0, C, "h0")
    state = np.zeros(C, np.float64) if h0v is None else h0v.astype(np.float64)
    href = np.empty((T, C), np.float64)
    if T > 0 and C > 0:
        forward_slab(lam2, x2, state, href, 0, T, threads)
    return href.reshape(np.asarray(lam).shape)


def backward_slab(lam2, h2, h0v, e2, gstate, gx, glam, gh0, t0, t1, threads=1):
    """Walk rows t1-1 .. t0; ``gstate`` carries g[t1] in and g[t0] out; gx/glam are fp64 [T, C]."""
    lib = _load()
    T, C = lam2.shape

    def work(c0, c1):
        lib.linrec_oracle_backward(_ptr(lam2), _ptr(h2), _ptr(h0v), _ptr(e2), _ptr(gstate),
                                   _ptr(gx), _ptr(glam), _ptr(gh0), T, C, t0, t1, c0, c1)

    _run_over_columns(work, C, threads)


def backward(lam, h, h0, grad_h, threads=1):
    """Returns (grad_x, grad_lambda, grad_h0) in fp64 for upstream ``grad_h`` = dL/dh.

    ``h`` is the fp32 forward output that the backward pass is given; ``h0`` may be None (zero state).
    """
    lam2 = _f32_2d(lam, "lambda")
    h2 = _f32_2d(h, "h")
    e2 = _f32_2d(grad_h, "grad_h")
    if not (lam2.shape == h2.shape == e2.shape):
        raise ValueError("lambda, h and grad_h must have the same shape")
    T, C = lam2.shape
    h0v = _f32_1d(h0, C, "h0")
    gstate = np.zeros(C, np.float64)
    gx = np.empty((T, C), np.float64)
    glam = np.empty((T, C), np.float64)
    gh0 = np.zeros(C, np.float64)
    if T > 0 and C > 0:
        backward_slab(lam2, h2, h0v, e2, gstate, gx, glam, gh0, 0, T, threads)
    shp = np.asarray(lam).shape
    return gx.reshape(shp), glam.reshape(shp), gh0.reshape(shp[1:])


def _slab_rows(T, C, slab_elems):
    return max(1, min(T, slab_elems // max(C, 1)))


def forward_compare(lam, x, h0, h_cand, threads=1, slab_elems=1 << 24, rel=0.0):
    """Stream the forward oracle in row slabs and fold error norms against the candidate ``h_cand``.

    Returns ``{"max_abs_err", "max_abs_ref", "worst_index"}``; never holds more than one fp64 slab.
    With ``rel > 0`` the folded error is ``max(|cand - ref| - rel*|ref|)``: what is left of each element's
    error after an allowance proportional to its own reference value (the rounding of a result that is
    stored in a narrower type), so that a per-element bound ``rel*|ref| + tol`` can be checked at any size.
    """
    lam2 = _f32_2d(lam, "lambda")
    x2 = _f32_2d(x, "x")
    hc = np.asarray(h_cand)
    T, C = lam2.shape
    hc2 = hc.reshape(T, C)
    h0v = _f32_1d(h0, C, "h0")
    state = np.zeros(C, np.float64) if h0v is None else h0v.astype(np.float64)
    rows = _slab_rows(T, C, slab_elems)
    max_err, max_ref, worst = 0.0, 0.0, (-1, -1)
    lib = _load()
    for t0 in range(0, T, rows):
        t1 = min(T, t0 + rows)
        # the C loop indexes full-size arrays; hand it a slab-relative view of the output
        slab = np.empty((t1 - t0, C), np.float64)

        def work(c0, c1, t0=t0, t1=t1, slab=slab):
            lib.linrec_oracle_forward(_ptr(lam2[t0:t1]), _ptr(x2[t0:t1]), _ptr(state), _ptr(slab),
                                      t1 - t0, C, 0, t1 - t0, c0, c1)

        _run_over_columns(work, C, threads)
        err = np.abs(hc2[t0:t1].astype(np.float64) - slab)
        if rel:
            err -= rel * np.abs(slab)
        # NaN in either side must fail the comparison, not vanish in a max()
        if not np.all(np.isfinite(err)):
            bad = np.argwhere(~np.isfinite(err))[0]
            return {"max_abs_err": float("inf"), "max_abs_ref": float(np.nanmax(np.abs(slab))),
                    "worst_index": (int(t0 + bad[0]), int(bad[1]))}
        i = int(np.argmax(err))
        if err.flat[i] > max_err:
            max_err = float(err.flat[i])
            worst = (t0 + i // C, i % C)
        max_ref = max(max_ref, float(np.max(np.abs(slab))))
    return {"max_abs_err": max_err, "max_abs_ref": max_ref, "worst_index": worst}


def backward_compare(lam, h, h0, grad_h, gx_cand, glam_cand, gh0_cand, threads=1, slab_elems=1 << 24, rel=0.0):
    """Stream the backward oracle (last rows first) and fold error norms against candidates.

    Returns a dict ``{name: {"max_abs_err", "max_abs_ref"}}`` for grad_x, grad_lambda, grad_h0
    (``rel`` as in :func:`forward_compare`).
    """
    lam2 = _f32_2d(lam, "lambda")
    h2 = _f32_2d(h, "h")
    e2 = _f32_2d(grad_h, "grad_h")
    T, C = lam2.shape
    h0v = _f32_1d(h0, C, "h0")
    gxc = np.asarray(gx_cand).reshape(T, C)
    glc = np.asarray(glam_cand).reshape(T, C)
    gstate = np.zeros(C, np.float64)
    gh0 = np.zeros(C, np.float64)
    rows = _slab_rows(T, C, slab_elems)
    out = {k: {"max_abs_err": 0.0, "max_abs_ref": 0.0} for k in ("grad_x", "grad_lambda", "grad_h0")}

    def fold(name, cand, ref):
        err = np.abs(cand.astype(np.float64) - ref)
        if rel:
            err -= rel * np.abs(ref)
        m = float(np.max(err)) if err.size else 0.0
        if not np.all(np.isfinite(err)):
            m = float("inf")
        out[name]["max_abs_err"] = max(out[name]["max_abs_err"], m)
        out[name]["max_abs_ref"] = max(out[name]["max_abs_ref"], float(np.max(np.abs(ref))) if ref.size else 0.0)

    lib = _load()
    t1 = T
    while t1 > 0:
        t0 = max(0, t1 - rows)
        # Views that start at row max(t0-1, 0) keep the neighbours the loop reads
        # (lambda[t+1], h[t-1]) inside the arrays handed to C.
        base = max(t0 - 1, 0)
        top = min(t1 + 1, T)
        lam_v, h_v, e_v = lam2[base:top], h2[base:top], e2[base:top]
        n_v = top - base
        gx_s = np.empty((n_v, C), np.float64)
        gl_s = np.empty((n_v, C), np.float64)
        # Inside the view the slab is rows [t0-base, t1-base).  The view ends at row t1
        # (so lambda[t1] is readable) unless t1 == T, and then the view's own length
        # tells the C loop that the last row has no successor.
        T_v = n_v
        h0_arg = h0v if t0 == 0 else None

        def work(c0, c1, lam_v=lam_v, h_v=h_v, e_v=e_v, gx_s=gx_s, gl_s=gl_s, T_v=T_v,
                 lo=t0 - base, hi=t1 - base, h0_arg=h0_arg):
            lib.linrec_oracle_backward(_ptr(lam_v), _ptr(h_v), _ptr(h0_arg), _ptr(e_v), _ptr(gstate),
                                       _ptr(gx_s), _ptr(gl_s), _ptr(gh0), T_v, C, lo, hi, c0, c1)

        _run_over_columns(work, C, threads)
        lo, hi = t0 - base, t1 - base
        fold("grad_x", gxc[t0:t1], gx_s[lo:hi])
        fold("grad_lambda", glc[t0:t1], gl_s[lo:hi])
        t1 = t0
    if gh0_cand is not None:
        fold("grad_h0", np.asarray(gh0_cand).reshape(C), gh0)
    return out


# ---------------------------------------------------------------------------------------------
# Gated (GILR) form: h_t = g_t*h_{t-1} + (1-g_t)*i_t with g = sigmoid(g_pre), i = tau(i_pre)
# ---------------------------------------------------------------------------------------------
TAU_IDENTITY, TAU_TANH = 0, 1


def gilr_forward(g_pre, i_pre, h0=None, tau=TAU_TANH, threads=1):
    """fp64 h of the gated form from the fp32 pre-activations; same shape as ``g_pre``."""
    g2 = _f32_2d(g_pre, "g_pre")
    i2 = _f32_2d(i_pre, "i_pre")
    if g2.shape != i2.shape:
        raise ValueError("g_pre and i_pre must have the same shape")
    T, C = g2.shape
    h0v = _f32_1d(h0, C, "h0")
    state = np.zeros(C, np.float64) if h0v is None else h0v.astype(np.float64)
    href = np.empty((T, C), np.float64)
    lib = _load()
    if T > 0 and C > 0:
        _run_over_columns(lambda c0, c1: lib.linrec_oracle_gilr_forward(
            _ptr(g2), _ptr(i2), int(tau), _ptr(state), _ptr(href), T, C, 0, T, c0, c1), C, threads)
    return href.reshape(np.asarray(g_pre).shape)


def gilr_backward(g_pre, i_pre, h, h0, grad_h, tau=TAU_TANH, threads=1):
    """Returns (grad_g_pre, grad_i_pre, grad_h0) in fp64 for upstream ``grad_h`` = dL/dh."""
    g2 = _f32_2d(g_pre, "g_pre")
    i2 = _f32_2d(i_pre, "i_pre")
    h2 = _f32_2d(h, "h")
    e2 = _f32_2d(grad_h, "grad_h")
    if not (g2.shape == i2.shape == h2.shape == e2.shape):
        raise ValueError("g_pre, i_pre, h and grad_h must have the same shape")
    T, C = g2.shape
    h0v = _f32_1d(h0, C, "h0")
    dstate = np.zeros(C, np.float64)
    gg = np.empty((T, C), np.float64)
    gi = np.empty((T, C), np.float64)
    gh0 = np.zeros(C, np.float64)
    lib = _load()
    if T > 0 and C > 0:
        _run_over_columns(lambda c0, c1: lib.linrec_oracle_gilr_backward(
            _ptr(g2), _ptr(i2), int(tau), _ptr(h2), _ptr(h0v), _ptr(e2), _ptr(dstate),
            _ptr(gg), _ptr(gi), _ptr(gh0), T, C, 0, T, c0, c1), C, threads)
    shp = np.asarray(g_pre).shape
    return gg.reshape(shp), gi.reshape(shp), gh0.reshape(shp[1:])


# ---------------------------------------------------------------------------------------------
# LSTM-cell form: c_t = f_t*c_{t-1} + i_t*z_t, h_t = o_t*c_t, gates from their pre-activations
# ---------------------------------------------------------------------------------------------
def lstm_forward(f_pre, i_pre, z_pre, o_pre, c0=None, threads=1):
    """Returns (c, h) in fp64, both with ``f_pre``'s shape."""
    a = [_f32_2d(v, n) for v, n in ((f_pre, "f_pre"), (i_pre, "i_pre"), (z_pre, "z_pre"), (o_pre, "o_pre"))]
    if not all(v.shape == a[0].shape for v in a):
        raise ValueError("the four pre-activation tensors must have the same shape")
    T, C = a[0].shape
    c0v = _f32_1d(c0, C, "c0")
    state = np.zeros(C, np.float64) if c0v is None else c0v.astype(np.float64)
    cref = np.empty((T, C), np.float64)
    href = np.empty((T, C), np.float64)
    lib = _load()
    if T > 0 and C > 0:
        _run_over_columns(lambda x0, x1: lib.linrec_oracle_lstm_forward(
            _ptr(a[0]), _ptr(a[1]), _ptr(a[2]), _ptr(a[3]), _ptr(state), _ptr(cref), _ptr(href), T, C, 0, T, x0, x1),
            C, threads)
    shp = np.asarray(f_pre).shape
    return cref.reshape(shp), href.reshape(shp)


def lstm_backward(f_pre, i_pre, z_pre, o_pre, c, c0, grad_h, threads=1):
    """Returns (grad_f_pre, grad_i_pre, grad_z_pre, grad_o_pre, grad_c0) in fp64; ``c`` is the fp32 cell state."""
    a = [_f32_2d(v, n) for v, n in ((f_pre, "f_pre"), (i_pre, "i_pre"), (z_pre, "z_pre"), (o_pre, "o_pre"),
                                    (c, "c"), (grad_h, "grad_h"))]
    if not all(v.shape == a[0].shape for v in a):
        raise ValueError("all [T, C] tensors must have the same shape")
    T, C = a[0].shape
    c0v = _f32_1d(c0, C, "c0")
    dstate = np.zeros(C, np.float64)
    outs = [np.empty((T, C), np.float64) for _ in range(4)]
    gc0 = np.zeros(C, np.float64)
    lib = _load()
    if T > 0 and C > 0:
        _run_over_columns(lambda x0, x1: lib.linrec_oracle_lstm_backward(
            _ptr(a[0]), _ptr(a[1]), _ptr(a[2]), _ptr(a[3]), _ptr(a[4]), _ptr(c0v), _ptr(a[5]), _ptr(dstate),
            _ptr(outs[0]), _ptr(outs[1]), _ptr(outs[2]), _ptr(outs[3]), _ptr(gc0), T, C, 0, T, x0, x1), C, threads)
    shp = np.asarray(f_pre).shape
    return tuple(o.reshape(shp) for o in outs) + (gc0.reshape(shp[1:]),)


# ---------------------------------------------------------------------------------------------
# Element-complete comparison of the gated layer and the cell at sizes whose fp64 tensors would not
# fit: the columns are independent recurrences, so the one-shot functions above are run on blocks of
# whole columns (all T rows of each) and the error norms are folded block by block.
# ---------------------------------------------------------------------------------------------
def _fold(out, name, cand, ref, rel=0.0):
    err = np.abs(np.asarray(cand, dtype=np.float64) - ref)
    if rel:
        err -= rel * np.abs(ref)
    m = float(np.max(err)) if err.size else 0.0
    if err.size and not np.all(np.isfinite(err)):   # NaN / Inf on either side fails the comparison
        m = float("inf")
    rec = out.setdefault(name, {"max_abs_err": 0.0, "max_abs_ref": 0.0})
    rec["max_abs_err"] = max(rec["max_abs_err"], m)
    rec["max_abs_ref"] = max(rec["max_abs_ref"], float(np.max(np.abs(ref))) if ref.size else 0.0)


def _col_blocks(T, C, block_elems):
    w = max(1, min(C, block_elems // max(T, 1)))
    return [(c0, min(C, c0 + w)) for c0 in range(0, C, w)]


def _cols(a, c0, c1):
    return None if a is None else np.ascontiguousarray(a[..., c0:c1])


def gilr_compare(g_pre, i_pre, h0, grad_h, h_cand, gg_cand, gi_cand, gh0_cand, tau=TAU_TANH, threads=1,
                 block_elems=1 << 23, rel=0.0):
    """Every element of a gated-layer result against :func:`gilr_forward` / :func:`gilr_backward`.

    ``h_cand`` (fp32 values, [T, C]) is compared with the forward oracle and is also the ``h`` the
    backward oracle is given, as the GPU backward pass is.  Gradient candidates may be None (skipped).
    Returns ``{name: {"max_abs_err", "max_abs_ref"}}`` for h and the gradients that were given
    (``rel`` as in :func:`forward_compare`)."""
    g2, i2, hc, e2 = _f32_2d(g_pre, "g_pre"), _f32_2d(i_pre, "i_pre"), _f32_2d(h_cand, "h_cand"), None
    T, C = g2.shape
    h0v = _f32_1d(h0, C, "h0")
    backward = grad_h is not None and any(c is not None for c in (gg_cand, gi_cand, gh0_cand))
    if backward:
        e2 = _f32_2d(grad_h, "grad_h")
    out = {}
    for c0, c1 in _col_blocks(T, C, block_elems):
        gb, ib, hb, h0b = _cols(g2, c0, c1), _cols(i2, c0, c1), _cols(hc, c0, c1), _cols(h0v, c0, c1)
        _fold(out, "h", hb, gilr_forward(gb, ib, h0b, tau, threads=threads), rel)
        if backward:
            refs = gilr_backward(gb, ib, hb, h0b, _cols(e2, c0, c1), tau, threads=threads)
            for name, cand, ref in zip(("grad_g_pre", "grad_i_pre"), (gg_cand, gi_cand), refs[:2]):
                if cand is not None:
                    _fold(out, name, np.asarray(cand).reshape(T, C)[:, c0:c1], ref, rel)
            if gh0_cand is not None:
                _fold(out, "grad_h0", np.asarray(gh0_cand).reshape(C)[c0:c1], refs[2], rel)
    return out


def lstm_compare(f_pre, i_pre, z_pre, o_pre, c0, grad_h, c_cand, h_cand, grad_cands, gc0_cand, threads=1,
                 block_elems=1 << 22, rel=0.0):
    """Every element of an LSTM-cell result against :func:`lstm_forward` / :func:`lstm_backward`.

    ``c_cand`` is compared with the forward oracle and is the cell state the backward oracle is given;
    ``grad_cands`` holds the four pre-activation gradients (None entries are skipped)."""
    pre = [_f32_2d(v, n) for v, n in ((f_pre, "f_pre"), (i_pre, "i_pre"), (z_pre, "z_pre"), (o_pre, "o_pre"))]
    T, C = pre[0].shape
    cc = _f32_2d(c_cand, "c_cand")
    hc = None if h_cand is None else np.asarray(h_cand).reshape(T, C)
    c0v = _f32_1d(c0, C, "c0")
    grad_cands = [None] * 4 if grad_cands is None else list(grad_cands)
    backward = grad_h is not None and (any(g is not None for g in grad_cands) or gc0_cand is not None)
    e2 = _f32_2d(grad_h, "grad_h") if backward else None
    out = {}
    names = ("grad_f_pre", "grad_i_pre", "grad_z_pre", "grad_o_pre")
    for a, b in _col_blocks(T, C, block_elems):
        pb = [_cols(p, a, b) for p in pre]
        cb, c0b = _cols(cc, a, b), _cols(c0v, a, b)
        cref, href = lstm_forward(*pb, c0b, threads=threads)
        _fold(out, "c", cb, cref, rel)
        if hc is not None:
            _fold(out, "h", hc[:, a:b], href, rel)
        if backward:
            refs = lstm_backward(*pb, cb, c0b, _cols(e2, a, b), threads=threads)
            for name, cand, ref in zip(names, grad_cands, refs[:4]):
                if cand is not None:
                    _fold(out, name, np.asarray(cand).reshape(T, C)[:, a:b], ref, rel)
            if gc0_cand is not None:
                _fold(out, "grad_c0", np.asarray(gc0_cand).reshape(C)[a:b], refs[4], rel)
    return out
