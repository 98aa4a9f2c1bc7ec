"""Pins for the LSTM-cell form of the fp64 CPU oracle.

arXiv 1709.04057, Section 3.2 (the GILR-LSTM's cell): with f, i, o = sigmoid of their pre-activations
and z = tanh(z_pre),
    c_t = f_t*c_{t-1} + i_t*z_t,     h_t = o_t*c_t
and the gradients with respect to the four pre-activations and c_0 for an upstream dL/dh.

Each pin is a function of ``fwd(f_pre, i_pre, z_pre, o_pre, c0) -> (c, h)`` and
``bwd(f_pre, i_pre, z_pre, o_pre, c, c0, grad_h) -> (gf, gi, gz, go, gc0)`` on float32 numpy arrays
[T, C].  The oracle must pass all of them; planted mistakes must each fail at least one.
"""
from fractions import Fraction

import numpy as np
import pytest
import scipy.special


def _rng(seed):
    return np.random.default_rng(seed)


def _f32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _grid(rng, shape, q=2.0 ** -8, scale=1.0):
    return _f32(np.round(rng.normal(scale=scale, size=shape) / q) * q)


def _acts(f_pre, i_pre, z_pre, o_pre):
    e = scipy.special.expit
    return (e(f_pre.astype(np.float64)), e(i_pre.astype(np.float64)), np.tanh(z_pre.astype(np.float64)),
            e(o_pre.astype(np.float64)))


# --------------------------------------------------------------------------- pins
def pin_half_gates_exact(fwd, bwd):
    # all gate pre-activations 0: f = i = o = 1/2 exactly; z_pre in {-40, 0, 40}: tanh = -1, 0, 1
    # exactly in fp64.  Every value is then a dyadic rational that fp64 (and fp32 for c) holds exactly.
    rng = _rng(51)
    T, C = 14, 4
    zero = np.zeros((T, C), np.float32)
    zsel = rng.integers(-1, 2, size=(T, C))
    z_pre = _f32(40.0 * zsel)
    c0 = _grid(rng, C)
    e = _grid(rng, (T, C), q=2.0 ** -4)
    c, h = fwd(zero, zero, z_pre, zero, c0)
    half = Fraction(1, 2)
    Cx = [[None] * C for _ in range(T)]
    for k in range(C):
        s = Fraction(float(c0[k]))
        for t in range(T):
            s = half * s + half * int(zsel[t, k])
            Cx[t][k] = s
            assert Fraction(float(c[t, k])) == s and Fraction(float(h[t, k])) == half * s, (t, k)
    c32 = _f32(c)
    assert np.array_equal(c32.astype(np.float64), c)
    gf, gi, gz, go, gc0 = bwd(zero, zero, z_pre, zero, c32, c0, e)
    for k in range(C):
        d = Fraction(0)
        for t in range(T - 1, -1, -1):
            et = Fraction(float(e[t, k]))
            d = et * half + (half * d if t + 1 < T else 0)
            cp = Cx[t - 1][k] if t > 0 else Fraction(float(c0[k]))
            z = int(zsel[t, k])
            assert Fraction(float(go[t, k])) == et * Cx[t][k] * Fraction(1, 4), (t, k)
            assert Fraction(float(gf[t, k])) == d * cp * Fraction(1, 4), (t, k)
            assert Fraction(float(gi[t, k])) == d * z * Fraction(1, 4), (t, k)
            assert Fraction(float(gz[t, k])) == d * half * (1 - z * z), (t, k)
        assert Fraction(float(gc0[k])) == half * d


def pin_constant_gates_closed_form(fwd, bwd):
    # gates and candidate constant along T: c_t = i*z*(1 - f^(t+1))/(1 - f) + f^(t+1)*c0, h_t = o*c_t
    rng = _rng(52)
    T, C = 150, 6
    pre = [_f32(rng.normal(m, 1.0, C)) for m in (0.5, 0.0, 0.0, 0.3)]
    c0 = _f32(rng.normal(size=C))
    f, i, z, o = _acts(*pre)
    full = [np.broadcast_to(p, (T, C)).copy() for p in pre]
    c, h = fwd(*full, c0)
    p = f[None, :] ** np.arange(1, T + 1)[:, None]
    ref = (i * z)[None, :] * (1 - p) / (1 - f)[None, :] + p * c0.astype(np.float64)[None, :]
    np.testing.assert_allclose(c, ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(h, o[None, :] * ref, rtol=1e-12, atol=1e-13)
    c_none, _ = fwd(*full, None)
    np.testing.assert_allclose(c_none, (i * z)[None, :] * (1 - p) / (1 - f)[None, :], rtol=1e-12, atol=1e-13)


def pin_cumprod_closed_form(fwd, bwd):
    rng = _rng(53)
    T, C = 40, 8
    pre = [_f32(rng.normal(m, 1.0, (T, C))) for m in (0.5, 0.0, 0.0, 0.0)]
    c0 = _f32(rng.normal(size=C))
    f, i, z, o = _acts(*pre)
    cp = np.cumprod(f, axis=0)
    ref = cp * (c0.astype(np.float64)[None, :] + np.cumsum(i * z / cp, axis=0))
    c, h = fwd(*pre, c0)
    np.testing.assert_allclose(c, ref, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(h, o * ref, rtol=1e-10, atol=1e-12)


def pin_saturated_gates(fwd, bwd):
    # forget closed, input and output open: h_t = c_t = tanh(z_pre_t); forget open, input closed: c_t = c0
    rng = _rng(54)
    T, C = 30, 5
    z_pre = _f32(rng.normal(size=(T, C)))
    c0 = _f32(rng.normal(size=C))
    big = np.full((T, C), 40.0, np.float32)
    c, h = fwd(-big, big, z_pre, big, c0)
    np.testing.assert_allclose(c, np.tanh(z_pre.astype(np.float64)), rtol=0, atol=1e-14)
    np.testing.assert_allclose(h, c, rtol=0, atol=1e-14)
    c, h = fwd(big, -big, z_pre, np.zeros((T, C), np.float32), c0)
    np.testing.assert_allclose(c, np.broadcast_to(c0.astype(np.float64), (T, C)), rtol=0, atol=1e-14)
    np.testing.assert_allclose(h, 0.5 * c, rtol=0, atol=1e-14)


def pin_finite_differences(fwd, bwd):
    # L = sum(e * h); central differences with one Richardson step in every single input element
    rng = _rng(55)
    T, C = 9, 3
    pre = [_grid(rng, (T, C)) for _ in range(4)]
    c0 = _grid(rng, C)
    e = _grid(rng, (T, C))
    e64 = e.astype(np.float64)
    s1, s2 = 2.0 ** -5, 2.0 ** -6

    def loss(p, cc0):
        return np.sum(e64 * fwd(*p, cc0)[1], axis=0)

    def deriv(make):
        d1 = (loss(*make(+s1)) - loss(*make(-s1))) / (2 * s1)
        d2 = (loss(*make(+s2)) - loss(*make(-s2))) / (2 * s2)
        return (4 * d2 - d1) / 3

    c, h = fwd(*pre, c0)
    grads = bwd(*pre, _f32(c), c0, e)
    for which in range(4):
        scale = np.abs(grads[which]).max()
        assert scale > 1e-2
        for t in range(T):
            def make(s, t=t, which=which):
                p = [a.copy() for a in pre]
                p[which][t] += np.float32(s)
                return p, c0

            np.testing.assert_allclose(grads[which][t], deriv(make), rtol=0, atol=2e-6 * scale)
    np.testing.assert_allclose(grads[4], deriv(lambda s: (pre, c0 + np.float32(s))), rtol=0,
                               atol=1e-9 * (1 + np.abs(grads[4]).max()))


def pin_reduction_to_the_plain_recurrence(fwd, bwd):
    # c is the plain recurrence with lambda = f, x = i*z; the cell gradients follow from its (separately
    # pinned) backward pass with upstream e*o:  d = grad_x,  d*c_{t-1} = grad_lambda
    import oracle as plain

    rng = _rng(56)
    T, C = 300, 5
    pre = [_f32(rng.normal(m, 1.0, (T, C))) for m in (1.0, 0.0, 0.0, 0.0)]
    c0 = _f32(rng.normal(size=C))
    e = _f32(rng.normal(size=(T, C)))
    f, i, z, o = _acts(*pre)
    c, h = fwd(*pre, c0)
    cref = plain.forward(_f32(f), _f32(i * z), c0)               # fp32 lambda and x: ~1e-7 relative off
    np.testing.assert_allclose(c, cref, rtol=0, atol=3e-6 * np.abs(cref).max())
    np.testing.assert_allclose(h, o * c, rtol=1e-13, atol=0)
    c32 = _f32(c)
    gf, gi, gz, go, gc0 = bwd(*pre, c32, c0, e)
    gx, gl, gh0 = plain.backward(_f32(f), c32, c0, _f32(e.astype(np.float64) * o))
    tol = lambda a: 1e-5 * np.abs(a).max()
    np.testing.assert_allclose(gf, gl * f * (1 - f), rtol=0, atol=tol(gf))
    np.testing.assert_allclose(gi, gx * z * i * (1 - i), rtol=0, atol=tol(gi))
    np.testing.assert_allclose(gz, gx * i * (1 - z * z), rtol=0, atol=tol(gz))
    np.testing.assert_allclose(go, e.astype(np.float64) * c32.astype(np.float64) * o * (1 - o), rtol=1e-12, atol=0)
    np.testing.assert_allclose(gc0, gh0, rtol=0, atol=tol(gc0))


ALL_PINS = [pin_half_gates_exact, pin_constant_gates_closed_form, pin_cumprod_closed_form, pin_saturated_gates,
            pin_finite_differences, pin_reduction_to_the_plain_recurrence]


@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda p: p.__name__)
@pytest.mark.parametrize("threads", [1, 3])
def test_lstm_oracle_passes_pin(oracle, pin, threads):
    pin(lambda *a: oracle.lstm_forward(*a, threads=threads), lambda *a: oracle.lstm_backward(*a, threads=threads))


# --------------------------------------------------------------------------- planted mistakes
def _sig(v):
    return 1.0 / (1.0 + np.exp(-v))


def _mut_fwd(f_pre, i_pre, z_pre, o_pre, c0, mode=""):
    T, C = f_pre.shape
    s = np.zeros(C) if (c0 is None or mode == "drop_c0") else c0.astype(np.float64)
    cs = np.empty((T, C)); hs = np.empty((T, C))
    for t in range(T):
        f = _sig(f_pre[t].astype(np.float64)); i = _sig(i_pre[t].astype(np.float64))
        o = _sig(o_pre[t].astype(np.float64)); z = np.tanh(z_pre[t].astype(np.float64))
        if mode == "z_sigmoid":
            z = _sig(z_pre[t].astype(np.float64))
        if mode == "i_tanh":
            i = np.tanh(i_pre[t].astype(np.float64))
        if mode == "f_next" and t + 1 < T:
            f = _sig(f_pre[t + 1].astype(np.float64))
        prev = s
        if mode == "gilr_style":
            s = f * s + (1 - f) * z
        elif mode == "sign":
            s = f * s - i * z
        elif mode == "drop_i":
            s = f * s + z
        else:
            s = f * s + i * z
        cs[t] = s
        hs[t] = {"no_o": s, "o_on_prev": o * prev, "tanh_c": o * np.tanh(s)}.get(mode, o * s)
    return cs, hs


def _mut_bwd(f_pre, i_pre, z_pre, o_pre, c, c0, e, mode=""):
    T, C = f_pre.shape
    d = np.zeros(C)
    gf, gi, gz, go = (np.empty((T, C)) for _ in range(4))
    for t in range(T - 1, -1, -1):
        f = _sig(f_pre[t].astype(np.float64)); i = _sig(i_pre[t].astype(np.float64))
        o = _sig(o_pre[t].astype(np.float64)); z = np.tanh(z_pre[t].astype(np.float64))
        et = e[t].astype(np.float64)
        direct = et if mode == "d_no_o" else et * o
        if mode == "f_t":
            d = direct + f * d
        elif t + 1 < T:
            d = direct + _sig(f_pre[t + 1].astype(np.float64)) * d
        else:
            d = direct
        ct = c[t].astype(np.float64)
        if mode == "gf_c_t":
            cp = ct
        elif t > 0:
            cp = c[t - 1].astype(np.float64)
        else:
            cp = np.zeros(C) if (c0 is None or mode == "drop_c0") else c0.astype(np.float64)
        go[t] = (d if mode == "go_uses_d" else et) * (cp if mode == "go_c_prev" else ct) * o * (1 - o)
        gf[t] = d * cp * (1.0 if mode == "gf_no_prime" else f * (1 - f))
        gi[t] = d * z * (1.0 if mode == "gi_no_prime" else i * (1 - i))
        gz[t] = d * (1.0 if mode == "gz_drop_i" else i) * (1.0 if mode == "gz_no_prime" else 1 - z * z)
    f0 = _sig(f_pre[0].astype(np.float64))
    gc0 = {"gc0_no_f": d, "gc0_one_minus_f": (1 - f0) * d}.get(mode, f0 * d)
    return gf, gi, gz, go, gc0


FWD_MUTANTS = ["drop_c0", "z_sigmoid", "i_tanh", "f_next", "gilr_style", "sign", "drop_i", "no_o", "o_on_prev", "tanh_c"]
BWD_MUTANTS = ["d_no_o", "f_t", "gf_c_t", "drop_c0", "go_uses_d", "go_c_prev", "gf_no_prime", "gi_no_prime",
               "gz_drop_i", "gz_no_prime", "gc0_no_f", "gc0_one_minus_f"]


@pytest.mark.parametrize("name", ["none"] + ["fwd:" + m for m in FWD_MUTANTS] + ["bwd:" + m for m in BWD_MUTANTS])
def test_lstm_pins_catch_planted_mistakes(name):
    side, _, mode = name.partition(":")
    fwd = (lambda *a: _mut_fwd(*a, mode=mode)) if side == "fwd" else (lambda *a: _mut_fwd(*a))
    bwd = (lambda *a: _mut_bwd(*a, mode=mode)) if side == "bwd" else (lambda *a: _mut_bwd(*a))
    failed = []
    for pin in ALL_PINS:
        try:
            pin(fwd, bwd)
        except AssertionError:
            failed.append(pin.__name__)
    if name == "none":
        assert not failed, f"the unmutated replica fails {failed}: the pins are wrong"
    else:
        assert failed, f"no pin notices the planted mistake {name}"


# --------------------------------------------------------------------------- the column-block comparison
def test_lstm_compare_agrees_with_one_shot(oracle):
    """lstm_compare reports exactly what the one-shot functions give, block by block."""
    rng = np.random.default_rng(78)
    f32 = lambda a: np.ascontiguousarray(np.asarray(a, dtype=np.float32))
    T, C = 250, 9
    pre = [f32(rng.normal(m, 1.0, (T, C))) for m in (1.0, 0.0, 0.0, 0.0)]
    c0, e = f32(rng.normal(size=C)), f32(rng.normal(size=(T, C)))
    c, h = oracle.lstm_forward(*pre, c0)
    cc, hc = f32(c), f32(h)
    grads = oracle.lstm_backward(*pre, cc, c0, e)
    gc = [f32(g) for g in grads]
    r = oracle.lstm_compare(*pre, c0, e, cc, hc, gc[:4], gc[4], threads=2, block_elems=2 * T)
    assert r["c"]["max_abs_err"] == np.abs(cc.astype(np.float64) - c).max()
    assert r["h"]["max_abs_err"] == np.abs(hc.astype(np.float64) - h).max()
    for k, name in enumerate(("grad_f_pre", "grad_i_pre", "grad_z_pre", "grad_o_pre", "grad_c0")):
        assert r[name]["max_abs_err"] == np.abs(gc[k].astype(np.float64) - grads[k]).max(), name
        assert r[name]["max_abs_ref"] == np.abs(grads[k]).max(), name
    for col in (0, 4, C - 1):
        bad = gc[2].copy()
        bad[3, col] -= np.float32(0.25)
        rb = oracle.lstm_compare(*pre, c0, e, cc, hc, [gc[0], gc[1], bad, gc[3]], gc[4], block_elems=2 * T)
        assert abs(rb["grad_z_pre"]["max_abs_err"] - abs(float(bad[3, col]) - grads[2][3, col])) < 1e-12
    hb = hc.copy()
    hb[0, 0] = np.inf
    assert oracle.lstm_compare(*pre, c0, None, cc, hb, None, None)["h"]["max_abs_err"] == float("inf")
    # outputs that were skipped are skipped here too
    r = oracle.lstm_compare(*pre, None, e, f32(oracle.lstm_forward(*pre, None)[0]), None, [None, gc[1], None, None], None)
    assert "h" not in r and "grad_f_pre" not in r and "grad_c0" not in r and "grad_i_pre" in r
