"""Pins for the gated (GILR) form of the fp64 CPU oracle.

arXiv 1709.04057, Section 3.1 ("Gated impulse linear recurrent layer"):
    g_t = sigmoid(g_pre_t),  i_t = tau(i_pre_t),  h_t = g_t*h_{t-1} + (1 - g_t)*i_t
and the gradients with respect to g_pre, i_pre and h0 that follow from Section 2.2's backward
recurrence by the chain rule.

Each pin is a function of ``gfwd(g_pre, i_pre, h0, tau) -> h`` and
``gbwd(g_pre, i_pre, h, h0, grad_h, tau) -> (grad_g_pre, grad_i_pre, grad_h0)`` on float32 numpy
arrays [T, C].  The oracle must pass all of them; planted mistakes must each fail at least one.
"""
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

IDENT, TANH = 0, 1


def _rng(seed):
    return np.random.default_rng(seed)


def _f32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _grid(rng, shape, q=2.0 ** -8, scale=1.0):
    return _f32(np.round(rng.normal(scale=scale, size=shape) / q) * q)


# --------------------------------------------------------------------------- pins
def pin_half_gate_exact(gfwd, gbwd):
    # g_pre == 0 gives g = 1/2 exactly; with tau = identity and dyadic inputs every value of the
    # recurrence and of its gradients is a dyadic rational that fp64 holds exactly.
    rng = _rng(41)
    T, C = 14, 3
    i = _grid(rng, (T, C))
    h0 = _grid(rng, C)
    e = _grid(rng, (T, C), q=2.0 ** -4)
    g_pre = np.zeros((T, C), np.float32)
    h = gfwd(g_pre, i, h0, IDENT)
    half = Fraction(1, 2)
    H = [[None] * C for _ in range(T)]
    for c in range(C):
        s = Fraction(float(h0[c]))
        for t in range(T):
            s = half * s + half * Fraction(float(i[t, c]))
            H[t][c] = s
            assert Fraction(float(h[t, c])) == s, (t, c)
    h32 = _f32(h)
    assert np.array_equal(h32.astype(np.float64), h)          # 8 + 14 fractional bits: exact in fp32
    gg, gi, gh0 = gbwd(g_pre, i, h32, h0, e, IDENT)
    for c in range(C):
        d = Fraction(0)
        for t in range(T - 1, -1, -1):
            d = Fraction(float(e[t, c])) + (half * d if t + 1 < T else 0)
            hp = H[t - 1][c] if t > 0 else Fraction(float(h0[c]))
            assert Fraction(float(gi[t, c])) == d * half, (t, c)
            assert Fraction(float(gg[t, c])) == d * (hp - Fraction(float(i[t, c]))) * Fraction(1, 4), (t, c)
        assert Fraction(float(gh0[c])) == half * d


def pin_moving_average_closed_form(gfwd, gbwd):
    # constant gate and constant impulse along T: h_t = i*(1 - g^(t+1)) + g^(t+1)*h0
    rng = _rng(42)
    T, C = 200, 7
    z = _f32(rng.normal(1.0, 1.5, C))
    y = _f32(rng.normal(size=C))
    h0 = _f32(rng.normal(size=C))
    g_pre = np.broadcast_to(z, (T, C)).copy()
    i_pre = np.broadcast_to(y, (T, C)).copy()
    g = scipy.special.expit(z.astype(np.float64))
    for tau, imp in ((TANH, np.tanh(y.astype(np.float64))), (IDENT, y.astype(np.float64))):
        h = gfwd(g_pre, i_pre, h0, tau)
        p = g[None, :] ** np.arange(1, T + 1)[:, None]
        ref = imp[None, :] * (1.0 - p) + p * h0.astype(np.float64)[None, :]
        np.testing.assert_allclose(h, ref, rtol=0, atol=1e-13)
    # no initial state: h0 = None is a zero state
    h = gfwd(g_pre, i_pre, None, TANH)
    np.testing.assert_allclose(h, np.tanh(y.astype(np.float64))[None, :] * (1.0 - p), rtol=0, atol=1e-13)


def pin_convex_hull(gfwd, gbwd):
    # every h_t is a convex combination of h0 and the impulses seen so far
    rng = _rng(43)
    T, C = 400, 16
    g_pre = _f32(rng.normal(0.0, 3.0, (T, C)))
    i_pre = _f32(rng.normal(0.0, 2.0, (T, C)))
    h0 = _f32(rng.normal(size=C))
    for tau in (TANH, IDENT):
        imp = np.tanh(i_pre.astype(np.float64)) if tau == TANH else i_pre.astype(np.float64)
        h = gfwd(g_pre, i_pre, h0, tau)
        hi = np.maximum.accumulate(np.vstack([h0[None, :].astype(np.float64), imp]), axis=0)[1:]
        lo = np.minimum.accumulate(np.vstack([h0[None, :].astype(np.float64), imp]), axis=0)[1:]
        assert np.all(h <= hi + 1e-12) and np.all(h >= lo - 1e-12)
        # and not degenerate: the state does move with the impulses
        assert np.abs(np.diff(h, axis=0)).max() > 0.1


def pin_cumprod_closed_form(gfwd, gbwd):
    # time-varying gates, short T: h_t = cp_t * (h0 + sum_{s<=t} x_s / cp_s), cp = cumprod(g),
    # x = (1-g)*tau(i_pre); evaluated with numpy's cumprod / cumsum and scipy's expit
    rng = _rng(44)
    T, C = 40, 9
    g_pre = _f32(rng.normal(0.5, 1.0, (T, C)))
    i_pre = _f32(rng.normal(size=(T, C)))
    h0 = _f32(rng.normal(size=C))
    g = scipy.special.expit(g_pre.astype(np.float64))
    for tau in (TANH, IDENT):
        imp = np.tanh(i_pre.astype(np.float64)) if tau == TANH else i_pre.astype(np.float64)
        x = scipy.special.expit(-g_pre.astype(np.float64)) * imp          # 1 - sigmoid(z) = sigmoid(-z)
        cp = np.cumprod(g, axis=0)
        ref = cp * (h0.astype(np.float64)[None, :] + np.cumsum(x / cp, axis=0))
        np.testing.assert_allclose(gfwd(g_pre, i_pre, h0, tau), ref, rtol=1e-10, atol=1e-12)


def pin_saturated_gates(gfwd, gbwd):
    # gate fully open (g -> 1): the state is frozen at h0; fully closed (g -> 0): h_t = tau(i_pre_t)
    rng = _rng(45)
    T, C = 50, 4
    i_pre = _f32(rng.normal(size=(T, C)))
    h0 = _f32(rng.normal(size=C))
    e = _f32(rng.normal(size=(T, C)))
    hold = gfwd(np.full((T, C), 40.0, np.float32), i_pre, h0, TANH)
    np.testing.assert_allclose(hold, np.broadcast_to(h0.astype(np.float64), (T, C)), rtol=0, atol=1e-14)
    g_pre = np.full((T, C), -40.0, np.float32)
    follow = gfwd(g_pre, i_pre, h0, TANH)
    np.testing.assert_allclose(follow, np.tanh(i_pre.astype(np.float64)), rtol=0, atol=1e-14)
    # closed gate: nothing flows back in time, grad_i_pre = e * tanh', grad_g_pre ~ 0, grad_h0 ~ 0
    gg, gi, gh0 = gbwd(g_pre, i_pre, _f32(follow), h0, e, TANH)
    np.testing.assert_allclose(gi, e.astype(np.float64) * (1 - np.tanh(i_pre.astype(np.float64)) ** 2),
                               rtol=1e-12, atol=1e-15)
    assert np.abs(gg).max() < 1e-15 and np.abs(gh0).max() < 1e-15


def pin_gilr_finite_differences(gfwd, gbwd):
    # L = sum(e * h); central differences with one Richardson step (error O(step^4)) in every
    # single input element; inputs on a dyadic grid so that perturbed values are exact in fp32
    rng = _rng(46)
    T, C = 10, 3
    g_pre = _grid(rng, (T, C))
    i_pre = _grid(rng, (T, C))
    h0 = _grid(rng, C)
    e = _grid(rng, (T, C))
    e64 = e.astype(np.float64)
    s1, s2 = 2.0 ** -5, 2.0 ** -6

    for tau in (TANH, IDENT):
        def loss(gp, ip, hh0):
            return np.sum(e64 * gfwd(gp, ip, hh0, tau), axis=0)

        def deriv(make):
            d1 = (loss(*make(+s1)) - loss(*make(-s1))) / (2 * s1)
            d2 = (loss(*make(+s2)) - loss(*make(-s2))) / (2 * s2)
            return (4 * d2 - d1) / 3

        h = gfwd(g_pre, i_pre, h0, tau)
        gg, gi, gh0 = gbwd(g_pre, i_pre, _f32(h), h0, e, tau)
        sg, si = np.abs(gg).max(), np.abs(gi).max()
        assert sg > 1e-2 and si > 1e-2
        for t in range(T):
            def mg(s, t=t):
                p = g_pre.copy(); p[t] += np.float32(s); return p, i_pre, h0

            def mi(s, t=t):
                p = i_pre.copy(); p[t] += np.float32(s); return g_pre, p, h0

            np.testing.assert_allclose(gg[t], deriv(mg), rtol=0, atol=2e-6 * sg)
            np.testing.assert_allclose(gi[t], deriv(mi), rtol=0, atol=2e-6 * si)
        np.testing.assert_allclose(gh0, deriv(lambda s: (g_pre, i_pre, h0 + np.float32(s))), rtol=0,
                                   atol=1e-9 * (1 + np.abs(gh0).max()))


def pin_chain_rule_through_plain_backward(gfwd, gbwd):
    # the gated gradients follow from the plain recurrence's grad_lambda and grad_x (pinned
    # separately) with lambda = g, x = (1-g)*i:  dL/dg = grad_lambda - grad_x*i,  dL/di = grad_x*(1-g)
    import oracle as plain

    rng = _rng(47)
    T, C = 300, 5
    g_pre = _f32(rng.normal(1.0, 1.0, (T, C)))
    i_pre = _f32(rng.normal(size=(T, C)))
    h0 = _f32(rng.normal(size=C))
    e = _f32(rng.normal(size=(T, C)))
    h32 = _f32(gfwd(g_pre, i_pre, h0, TANH))
    gg, gi, gh0 = gbwd(g_pre, i_pre, h32, h0, e, TANH)
    g64 = scipy.special.expit(g_pre.astype(np.float64))
    imp = np.tanh(i_pre.astype(np.float64))
    gx, gl, gh0_plain = plain.backward(_f32(g64), h32, h0, e)     # fp32 lambda: 6e-8 relative off
    np.testing.assert_allclose(gg, (gl - gx * imp) * g64 * (1 - g64), rtol=0, atol=1e-5 * np.abs(gg).max())
    np.testing.assert_allclose(gi, gx * (1 - g64) * (1 - imp ** 2), rtol=0, atol=1e-5 * np.abs(gi).max())
    np.testing.assert_allclose(gh0, gh0_plain, rtol=0, atol=1e-5 * np.abs(gh0).max())


ALL_PINS = [pin_half_gate_exact, pin_moving_average_closed_form, pin_convex_hull, pin_cumprod_closed_form,
            pin_saturated_gates, pin_gilr_finite_differences, pin_chain_rule_through_plain_backward]


# --------------------------------------------------------------------------- the oracle under test
@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda p: p.__name__)
@pytest.mark.parametrize("threads", [1, 3])
def test_gilr_oracle_passes_pin(oracle, pin, threads):
    pin(lambda gp, ip, h0, tau: oracle.gilr_forward(gp, ip, h0, tau, threads=threads),
        lambda gp, ip, h, h0, e, tau: oracle.gilr_backward(gp, ip, h, h0, e, tau, threads=threads))


# --------------------------------------------------------------------------- planted mistakes
def _sig(z):
    return 1.0 / (1.0 + np.exp(-z))


def _mut_fwd(g_pre, i_pre, h0, tau, mode=""):
    T, C = g_pre.shape
    s = np.zeros(C) if (h0 is None or mode == "drop_h0") else h0.astype(np.float64)
    out = np.empty((T, C))
    for t in range(T):
        z = g_pre[t].astype(np.float64)
        g = _sig(-z) if mode == "sigmoid_neg" else _sig(z)
        y = i_pre[t].astype(np.float64)
        use_tanh = (tau == TANH)
        if mode == "tau_ignored":
            use_tanh = True
        if mode == "no_tanh":
            use_tanh = False
        i = np.tanh(y) if use_tanh else y
        if mode == "drop_one_minus_g":
            s = g * s + i
        elif mode == "gate_swapped":
            s = (1 - g) * s + g * i
        elif mode == "gate_next" and t + 1 < T:
            gn = _sig(g_pre[t + 1].astype(np.float64))
            s = gn * s + (1 - gn) * i
        else:
            s = g * s + (1 - g) * i
        out[t] = s
    return out


def _mut_bwd(g_pre, i_pre, h, h0, e, tau, mode=""):
    T, C = g_pre.shape
    d = np.zeros(C)
    gg = np.empty((T, C)); gi = np.empty((T, C))
    for t in range(T - 1, -1, -1):
        g = _sig(g_pre[t].astype(np.float64))
        y = i_pre[t].astype(np.float64)
        i = np.tanh(y) if tau == TANH else y
        if mode == "gate_t":
            d = e[t].astype(np.float64) + g * d
        elif t + 1 < T:
            d = e[t].astype(np.float64) + _sig(g_pre[t + 1].astype(np.float64)) * d
        else:
            d = e[t].astype(np.float64)
        if mode == "h_t":
            hp = h[t].astype(np.float64)
        elif t > 0:
            hp = h[t - 1].astype(np.float64)
        else:
            hp = np.zeros(C) if (h0 is None or mode == "drop_h0") else h0.astype(np.float64)
        dg = d * (hp - i)
        if mode == "dg_no_impulse":
            dg = d * hp
        if mode == "dg_sign":
            dg = d * (i - hp)
        di = d * (1 - g)
        if mode == "di_no_gate":
            di = d
        if mode == "di_gate":
            di = d * g
        gg[t] = dg if mode == "no_sigmoid_prime" else dg * g * (1 - g)
        tp = (1 - i * i) if tau == TANH else 1.0
        if mode == "no_tanh_prime":
            tp = 1.0
        if mode == "tanh_prime_always":
            tp = 1 - np.tanh(y) ** 2
        gi[t] = di * tp
    g0 = _sig(g_pre[0].astype(np.float64))
    gh0 = {"gh0_no_gate": d, "gh0_one_minus_g": (1 - g0) * d}.get(mode, g0 * d)
    return gg, gi, gh0


FWD_MUTANTS = ["drop_h0", "sigmoid_neg", "tau_ignored", "no_tanh", "drop_one_minus_g", "gate_swapped", "gate_next"]
BWD_MUTANTS = ["gate_t", "h_t", "drop_h0", "dg_no_impulse", "dg_sign", "di_no_gate", "di_gate", "no_sigmoid_prime",
               "no_tanh_prime", "tanh_prime_always", "gh0_no_gate", "gh0_one_minus_g"]


@pytest.mark.parametrize("name", ["none"] + ["fwd:" + m for m in FWD_MUTANTS] + ["bwd:" + m for m in BWD_MUTANTS])
def test_gilr_pins_catch_planted_mistakes(name):
    side, _, mode = name.partition(":")
    gfwd = (lambda *a: _mut_fwd(*a, mode=mode)) if side == "fwd" else (lambda *a: _mut_fwd(*a))
    gbwd = (lambda *a: _mut_bwd(*a, mode=mode)) if side == "bwd" else (lambda *a: _mut_bwd(*a))
    failed = []
    for pin in ALL_PINS:
        try:
            pin(gfwd, gbwd)
        except AssertionError:
            failed.append(pin.__name__)
    if name == "none":
        assert not failed, f"the unmutated replica fails {failed}: the pins are wrong"
    else:
        assert failed, f"no pin notices the planted mistake {name}"


# --------------------------------------------------------------------------- the column-block comparison
def test_gilr_compare_agrees_with_one_shot(oracle):
    """gilr_compare (whole-column blocks, folded error norms) reports exactly what the one-shot functions
    give, finds a planted error in any block, and fails on a NaN instead of swallowing it."""
    rng = _rng(77)
    T, C = 300, 11
    gp, ip = _f32(rng.normal(1.0, 1.5, (T, C))), _f32(rng.normal(size=(T, C)))
    h0, e = _f32(rng.normal(size=C)), _f32(rng.normal(size=(T, C)))
    for tau in (IDENT, TANH):
        h = oracle.gilr_forward(gp, ip, h0, tau)
        hc = _f32(h)
        gg, gi, gh0 = oracle.gilr_backward(gp, ip, hc, h0, e, tau)
        ggc, gic, gh0c = _f32(gg), _f32(gi), _f32(gh0)
        hc2 = hc.copy()
        # (the backward reference is evaluated on the candidate h, so plant the forward error in a copy)
        r = oracle.gilr_compare(gp, ip, h0, e, hc, ggc, gic, gh0c, tau, threads=2, block_elems=3 * T)
        assert r["h"]["max_abs_err"] == np.abs(hc.astype(np.float64) - h).max()
        assert r["h"]["max_abs_ref"] == np.abs(h).max()
        assert r["grad_g_pre"]["max_abs_err"] == np.abs(ggc.astype(np.float64) - gg).max()
        assert r["grad_i_pre"]["max_abs_err"] == np.abs(gic.astype(np.float64) - gi).max()
        assert r["grad_h0"]["max_abs_err"] == np.abs(gh0c.astype(np.float64) - gh0).max()
        assert r["grad_g_pre"]["max_abs_ref"] == np.abs(gg).max()
        for col in (0, 5, C - 1):                       # a planted error in the first, a middle and the last block
            bad = ggc.copy()
            bad[17, col] += np.float32(0.5)
            rb = oracle.gilr_compare(gp, ip, h0, e, hc, bad, gic, gh0c, tau, block_elems=3 * T)
            assert abs(rb["grad_g_pre"]["max_abs_err"] - abs(float(bad[17, col]) - gg[17, col])) < 1e-12
        hc2[T - 1, C - 1] = np.nan
        assert oracle.gilr_compare(gp, ip, h0, None, hc2, None, None, None, tau)["h"]["max_abs_err"] == float("inf")
    # no initial state, forward only
    h = oracle.gilr_forward(gp, ip, None, TANH)
    r = oracle.gilr_compare(gp, ip, None, None, _f32(h), None, None, None, TANH, block_elems=T)
    assert set(r) == {"h"} and r["h"]["max_abs_err"] < 1e-6
