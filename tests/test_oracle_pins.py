"""Pins for the fp64 CPU oracle: it is checked against things other than itself.

Each pin is a function of two callables ``fwd(lam, x, h0) -> h`` and
``bwd(lam, h, h0, grad_h) -> (grad_x, grad_lambda, grad_h0)`` working on float32 numpy arrays of
shape [T, C] (h0: [C] or None).  The real oracle must pass every pin; deliberately broken variants
(a dropped term, a shifted index, a swapped operand, a wrong sign) must each fail at least one pin,
which shows that the pins would catch such a mistake in the oracle itself.

Equations: arXiv 1709.04057 Section 2 (recurrence; Algorithm 1 gives C_{-1} = h_0), Section 1 (SCAN
returns n outputs for n inputs), Section 2.2 (backpropagation).
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.signal

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_example_T4.txt")


# --------------------------------------------------------------------------- helpers
def _rng(seed):
    return np.random.default_rng(seed)


def _f32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _adversarial_lambda(rng, T, C):
    """lambda with exact 0, 1, -1, tiny and ordinary values mixed per element."""
    lam = rng.uniform(-1.0, 1.0, size=(T, C))
    cls = rng.integers(0, 6, size=(T, C))
    lam = np.where(cls == 0, 0.0, lam)
    lam = np.where(cls == 1, 1.0, lam)
    lam = np.where(cls == 2, -1.0, lam)
    lam = np.where(cls == 3, 1e-20, lam)
    return _f32(lam)


def exact_forward(lam, x, h0):
    """Closed form h_t = sum_{s<=t} (prod_{r=s+1..t} lam_r) x_s + (prod_{r<=t} lam_r) h0, term by term,
    in exact rational arithmetic (O(T^2) per column; tiny shapes only)."""
    T, C = lam.shape
    out = [[None] * C for _ in range(T)]
    mag = np.zeros((T, C))
    for c in range(C):
        L = [Fraction(float(v)) for v in lam[:, c]]
        X = [Fraction(float(v)) for v in x[:, c]]
        H0 = Fraction(float(h0[c])) if h0 is not None else Fraction(0)
        for t in range(T):
            total = Fraction(0)
            absum = Fraction(0)
            for s in range(t + 1):
                prod = Fraction(1)
                for r in range(s + 1, t + 1):
                    prod *= L[r]
                total += prod * X[s]
                absum += abs(prod * X[s])
            prod = Fraction(1)
            for r in range(0, t + 1):
                prod *= L[r]
            total += prod * H0
            absum += abs(prod * H0)
            out[t][c] = total
            mag[t, c] = float(absum)
    return out, mag


def exact_backward(lam, h, h0, e):
    """Closed form g_t = sum_{s>=t} (prod_{r=t+1..s} lam_r) e_s in exact rationals, then
    grad_lambda_t = h_{t-1} g_t (h_{-1} = h0) and grad_h0 = lam_0 g_0."""
    T, C = lam.shape
    g = [[None] * C for _ in range(T)]
    gl = [[None] * C for _ in range(T)]
    gh0 = [None] * C
    mag = np.zeros((T, C))
    for c in range(C):
        L = [Fraction(float(v)) for v in lam[:, c]]
        E = [Fraction(float(v)) for v in e[:, c]]
        for t in range(T):
            total = Fraction(0)
            absum = Fraction(0)
            for s in range(t, T):
                prod = Fraction(1)
                for r in range(t + 1, s + 1):
                    prod *= L[r]
                total += prod * E[s]
                absum += abs(prod * E[s])
            g[t][c] = total
            mag[t, c] = float(absum)
            hprev = Fraction(float(h[t - 1, c])) if t > 0 else (Fraction(float(h0[c])) if h0 is not None else Fraction(0))
            gl[t][c] = total * hprev
        gh0[c] = L[0] * g[0][c]
    return g, gl, gh0, mag


def _assert_close_exact(got, exact, mag, what, ulps=256):
    """|got - exact| must stay within a few fp64 roundings of the sum of absolute terms."""
    T = len(exact)
    C = len(exact[0])
    for t in range(T):
        for c in range(C):
            err = abs(Fraction(float(got[t, c])) - exact[t][c])
            bound = Fraction(ulps * 2.0 ** -52) * Fraction(float(mag[t, c])) + Fraction(1, 10 ** 300)
            assert err <= bound, f"{what}[{t},{c}]: got {got[t, c]!r}, exact {float(exact[t][c])!r}"


# --------------------------------------------------------------------------- the pins
def pin_golden_worked_example(fwd, bwd):
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, *nums = line.split()
            vals[name] = np.array([float(v) for v in nums])
    T, C = 4, 2
    lam = _f32(vals["lambda"].reshape(T, C))
    x = _f32(vals["x"].reshape(T, C))
    e = _f32(vals["grad_h"].reshape(T, C))
    h0 = _f32(vals["h0"])
    h = fwd(lam, x, h0)
    assert np.array_equal(h, vals["h"].reshape(T, C))
    gx, gl, gh0 = bwd(lam, _f32(h), h0, e)
    assert np.array_equal(gx, vals["grad_x"].reshape(T, C))
    assert np.array_equal(gl, vals["grad_lambda"].reshape(T, C))
    assert np.array_equal(gh0, vals["grad_h0"])


def pin_forward_closed_form(fwd, bwd):
    for seed, (T, C), with_h0 in [(1, (1, 3), True), (2, (2, 2), False), (3, (17, 3), True), (4, (64, 2), True)]:
        rng = _rng(seed)
        lam = _adversarial_lambda(rng, T, C) if seed % 2 else _f32(rng.uniform(0, 1, (T, C)))
        x = _f32(rng.normal(size=(T, C)))
        h0 = _f32(rng.normal(size=C)) if with_h0 else None
        exact, mag = exact_forward(lam, x, h0)
        _assert_close_exact(fwd(lam, x, h0), exact, mag, "h")


def pin_backward_closed_form(fwd, bwd):
    for seed, (T, C), with_h0 in [(11, (1, 2), True), (12, (2, 3), False), (13, (23, 2), True), (14, (64, 2), True)]:
        rng = _rng(seed)
        lam = _adversarial_lambda(rng, T, C) if seed % 2 else _f32(rng.uniform(0, 1, (T, C)))
        h = _f32(rng.normal(size=(T, C)))          # any fp32 tensor: the contract is on the inputs
        e = _f32(rng.normal(size=(T, C)))
        h0 = _f32(rng.normal(size=C)) if with_h0 else None
        g, gl, gh0, mag = exact_backward(lam, h, h0, e)
        gx_o, gl_o, gh0_o = bwd(lam, h, h0, e)
        _assert_close_exact(gx_o, g, mag, "grad_x")
        habs = np.abs(np.vstack([(h0 if h0 is not None else np.zeros(C))[None, :], h[:-1]])).astype(np.float64)
        _assert_close_exact(gl_o, gl, mag * habs, "grad_lambda")
        _assert_close_exact(gh0_o[None, :], [gh0], (mag[0] * np.abs(lam[0]))[None, :], "grad_h0")


def pin_lambda_zero(fwd, bwd):
    rng = _rng(21)
    T, C = 37, 5
    lam = np.zeros((T, C), np.float32)
    x = _f32(rng.normal(size=(T, C)))
    h0 = _f32(rng.normal(size=C))
    e = _f32(rng.normal(size=(T, C)))
    h = fwd(lam, x, h0)
    assert np.array_equal(h, x.astype(np.float64))
    gx, gl, gh0 = bwd(lam, _f32(h), h0, e)
    assert np.array_equal(gx, e.astype(np.float64))
    assert np.array_equal(gl[1:], e[1:].astype(np.float64) * x[:-1].astype(np.float64))
    assert np.array_equal(gl[0], e[0].astype(np.float64) * h0.astype(np.float64))
    assert np.array_equal(gh0, np.zeros(C))


def pin_lambda_one(fwd, bwd):
    rng = _rng(22)
    T, C = 300, 4
    lam = np.ones((T, C), np.float32)
    x = _f32(rng.normal(size=(T, C)))
    h0 = _f32(rng.normal(size=C))
    e = _f32(rng.normal(size=(T, C)))
    h = fwd(lam, x, h0)
    ref = h0.astype(np.float64)[None, :] + np.cumsum(x.astype(np.float64), axis=0)
    np.testing.assert_allclose(h, ref, rtol=0, atol=1e-12)
    gx, gl, gh0 = bwd(lam, _f32(h), h0, e)
    rev = np.cumsum(e.astype(np.float64)[::-1], axis=0)[::-1]
    np.testing.assert_allclose(gx, rev, rtol=0, atol=1e-12)
    np.testing.assert_allclose(gh0, rev[0], rtol=0, atol=1e-12)


def pin_geometric_series(fwd, bwd):
    # lambda = c, x = 1, h0 = 0  =>  h_t = (1 - c^(t+1)) / (1 - c)   (0-based t)
    T = 5000
    cs = np.array([0.5, 0.9, 0.999, -0.75], np.float32)
    lam = np.broadcast_to(cs, (T, cs.size)).copy()
    x = np.ones((T, cs.size), np.float32)
    h = fwd(lam, x, None)
    c64 = cs.astype(np.float64)
    t = np.arange(1, T + 1, dtype=np.float64)[:, None]
    ref = (1.0 - c64[None, :] ** t) / (1.0 - c64[None, :])
    np.testing.assert_allclose(h, ref, rtol=1e-12, atol=0)


def pin_lfilter(fwd, bwd):
    # constant lambda per column is the one-pole IIR filter y[t] = c*y[t-1] + x[t]
    rng = _rng(23)
    T, C = 2000, 3
    cs = _f32([0.3, 0.95, -0.6])
    lam = np.broadcast_to(cs, (T, C)).copy()
    x = _f32(rng.normal(size=(T, C)))
    h = fwd(lam, x, None)
    for c in range(C):
        ref = scipy.signal.lfilter([1.0], [1.0, -float(cs[c])], x[:, c].astype(np.float64))
        np.testing.assert_allclose(h[:, c], ref, rtol=1e-10, atol=1e-12)


def pin_single_impulse_gradient(fwd, bwd):
    # upstream gradient only in the last row  =>  g_t = e_{T-1} * prod_{r=t+1..T-1} lam_r
    rng = _rng(24)
    T, C = 4096, 3
    lam = _f32(1.0 - 10.0 ** rng.uniform(-4, -1, size=(T, C)))
    h = _f32(rng.normal(size=(T, C)))
    e = np.zeros((T, C), np.float32)
    e[-1] = rng.normal(size=C)
    gx, gl, gh0 = bwd(lam, h, None, e)
    l64 = lam.astype(np.float64)
    shifted = np.vstack([l64[1:], np.ones((1, C))])          # row t holds lam[t+1]; last row 1
    ref = e[-1].astype(np.float64)[None, :] * np.cumprod(shifted[::-1], axis=0)[::-1]
    np.testing.assert_allclose(gx, ref, rtol=1e-11, atol=0)
    np.testing.assert_allclose(gh0, l64[0] * ref[0], rtol=1e-11, atol=0)
    assert np.array_equal(gl[0], np.zeros(C))                # h0 = None => h_{-1} = 0


def pin_finite_differences(fwd, bwd):
    # L = sum(grad_h * h).  h is affine in each single lambda[t,c], x[t,c] and h0[c] (multilinear), so a
    # one-sided difference quotient with any step is exact up to fp64 rounding: no truncation error.
    # Inputs are kept on a coarse dyadic grid so that the perturbed values are exact in fp32.
    rng = _rng(25)
    T, C = 24, 3
    q = 2.0 ** -8
    lam = _f32(np.round(rng.uniform(-1, 1, (T, C)) / q) * q)
    x = _f32(np.round(rng.normal(size=(T, C)) / q) * q)
    h0 = _f32(np.round(rng.normal(size=C) / q) * q)
    e = _f32(np.round(rng.normal(size=(T, C)) / q) * q)
    e64 = e.astype(np.float64)

    def loss(l, xx, hh0):
        return np.sum(e64 * fwd(l, xx, hh0), axis=0)            # per column

    h = fwd(lam, x, h0)
    # backward is handed fp32 h; make it exact by checking representability first
    h32 = _f32(h)
    gx, gl, gh0 = bwd(lam, h32, h0, e)
    gl_true_scale = np.abs(h).max() * np.abs(gx).max()
    base = loss(lam, x, h0)
    step = 0.125
    for t in range(T):
        lp = lam.copy(); lp[t] += step
        fd = (loss(lp, x, h0) - base) / step
        # bwd used fp32-rounded h for grad_lambda; allow that rounding (2^-24 relative on h)
        np.testing.assert_allclose(gl[t], fd, rtol=0, atol=2e-7 * gl_true_scale + 1e-9)
        xp = x.copy(); xp[t] += step
        fd = (loss(lam, xp, h0) - base) / step
        np.testing.assert_allclose(gx[t], fd, rtol=0, atol=1e-10 * (1 + np.abs(gx).max()))
    hp = h0 + np.float32(step)
    fd = (loss(lam, x, hp) - base) / step
    np.testing.assert_allclose(gh0, fd, rtol=0, atol=1e-10 * (1 + np.abs(gh0).max()))


def pin_adjoint_identity(fwd, bwd):
    # for fixed lambda, h is linear in (x, h0):  <grad_h, h> = <grad_x, x> + <grad_h0, h0>
    rng = _rng(26)
    T, C = 3000, 8
    lam = _f32(1.0 / (1.0 + np.exp(-rng.normal(2.0, 1.0, (T, C)))))
    x = _f32(rng.normal(size=(T, C)))
    h0 = _f32(rng.normal(size=C))
    e = _f32(rng.normal(size=(T, C)))
    h = fwd(lam, x, h0)
    gx, gl, gh0 = bwd(lam, _f32(h), h0, e)
    lhs = np.sum(e.astype(np.float64) * h, axis=0)
    rhs = np.sum(gx * x.astype(np.float64), axis=0) + gh0 * h0.astype(np.float64)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-10, atol=1e-9)


def pin_row_perturbation(fwd, bwd):
    # perturb a whole row lambda[t,:] += d: per column dL_c = d_c * grad_lambda[t,c] exactly (affinity)
    rng = _rng(27)
    T, C = 1500, 6
    lam = _f32(rng.uniform(0.0, 1.0, (T, C)))
    x = _f32(rng.normal(size=(T, C)))
    h0 = _f32(rng.normal(size=C))
    e = _f32(rng.normal(size=(T, C)))
    e64 = e.astype(np.float64)
    h = fwd(lam, x, h0)
    gx, gl, gh0 = bwd(lam, _f32(h), h0, e)
    base = np.sum(e64 * h, axis=0)
    scale = np.abs(gl).max()
    for t in (0, 1, 777, T - 2, T - 1):
        d = _f32(rng.choice([-0.25, 0.125, 0.0625], size=C))
        lp = lam.copy(); lp[t] += d
        dL = np.sum(e64 * fwd(lp, x, h0), axis=0) - base
        lam_step = (lp[t].astype(np.float64) - lam[t].astype(np.float64))
        np.testing.assert_allclose(dL, lam_step * gl[t], rtol=0, atol=3e-7 * scale)


def pin_no_h0_row_and_shapes(fwd, bwd):
    # T outputs for T inputs; row 0 already contains the first update (no copy of h0 in the output)
    lam = _f32([[0.5], [0.5]])
    x = _f32([[1.0], [1.0]])
    h = fwd(lam, x, _f32([4.0]))
    assert h.shape == (2, 1)
    assert np.array_equal(h[:, 0], [3.0, 2.5])
    # operand order: the pair operator is not commutative; (lam, x) = (2, 1) then (3, 10) from h0 = 1
    h = fwd(_f32([[2.0], [3.0]]), _f32([[1.0], [10.0]]), _f32([1.0]))
    assert np.array_equal(h[:, 0], [3.0, 19.0])


ALL_PINS = [pin_golden_worked_example, pin_forward_closed_form, pin_backward_closed_form, pin_lambda_zero,
            pin_lambda_one, pin_geometric_series, pin_lfilter, pin_single_impulse_gradient,
            pin_finite_differences, pin_adjoint_identity, pin_row_perturbation, pin_no_h0_row_and_shapes]


# --------------------------------------------------------------------------- the oracle under test
def _oracle_fns(oracle, threads=1):
    def fwd(lam, x, h0):
        return oracle.forward(lam, x, h0, threads=threads)

    def bwd(lam, h, h0, e):
        return oracle.backward(lam, h, h0, e, threads=threads)

    return fwd, bwd


@pytest.mark.parametrize("pin", ALL_PINS, ids=lambda p: p.__name__)
def test_oracle_passes_pin(oracle, pin):
    fwd, bwd = _oracle_fns(oracle)
    pin(fwd, bwd)


@pytest.mark.parametrize("pin", [pin_forward_closed_form, pin_backward_closed_form, pin_adjoint_identity],
                         ids=lambda p: p.__name__)
def test_oracle_passes_pin_threaded(oracle, pin):
    fwd, bwd = _oracle_fns(oracle, threads=3)
    pin(fwd, bwd)


# --------------------------------------------------------------------------- planted mistakes
def _mutants():
    """Plausible wrong implementations (plain fp64 numpy loops), each differing from the definition
    in one place.  They are never used as a reference for anything."""

    def good_fwd(lam, x, h0, *, mode=""):
        T, C = lam.shape
        s = np.zeros(C) if h0 is None else h0.astype(np.float64)
        if mode == "drop_h0":
            s = np.zeros(C)
        out = np.empty((T, C))
        for t in range(T):
            l = lam[t].astype(np.float64)
            xx = x[t].astype(np.float64)
            if mode == "lam_shift" and t + 1 < T:
                l = lam[t + 1].astype(np.float64)
            if mode == "swap":
                s = xx * s + l
            elif mode == "sign":
                s = l * s - xx
            elif mode == "h0_row":
                out[t] = s
                s = l * s + xx
                continue
            else:
                s = l * s + xx
            out[t] = s
        return out

    def good_bwd(lam, h, h0, e, *, mode=""):
        T, C = lam.shape
        g = np.zeros(C)
        gx = np.empty((T, C)); gl = np.empty((T, C))
        for t in range(T - 1, -1, -1):
            if mode == "lam_t":                                   # lambda_t instead of lambda_{t+1}
                g = e[t].astype(np.float64) + lam[t].astype(np.float64) * g
            elif t + 1 < T:
                g = e[t].astype(np.float64) + lam[t + 1].astype(np.float64) * g
            else:
                g = e[t].astype(np.float64)
            gx[t] = g
            if mode == "h_t":                                     # h_t instead of h_{t-1}
                hp = h[t].astype(np.float64)
            elif t > 0:
                hp = h[t - 1].astype(np.float64)
            else:
                hp = np.zeros(C) if (h0 is None or mode == "gl_drop_h0") else h0.astype(np.float64)
            gl[t] = g * hp
        if mode == "gh0_no_lam":
            gh0 = g.copy()
        elif mode == "gh0_zero":
            gh0 = np.zeros(C)
        else:
            gh0 = lam[0].astype(np.float64) * g
        if mode == "gx_is_e":
            gx = e.astype(np.float64)
        return gx, gl, gh0

    muts = {}
    for m in ("drop_h0", "lam_shift", "swap", "sign", "h0_row"):
        muts["fwd:" + m] = (lambda lam, x, h0, m=m: good_fwd(lam, x, h0, mode=m), lambda *a: good_bwd(*a))
    for m in ("lam_t", "h_t", "gl_drop_h0", "gh0_no_lam", "gh0_zero", "gx_is_e"):
        muts["bwd:" + m] = (lambda *a: good_fwd(*a), lambda lam, h, h0, e, m=m: good_bwd(lam, h, h0, e, mode=m))
    muts["none"] = (lambda *a: good_fwd(*a), lambda *a: good_bwd(*a))
    return muts


@pytest.mark.parametrize("name", sorted(_mutants().keys()))
def test_pins_catch_planted_mistakes(name):
    fwd, bwd = _mutants()[name]
    failed = []
    for pin in ALL_PINS:
        try:
            pin(fwd, bwd)
        except AssertionError:
            failed.append(pin.__name__)
    if name == "none":
        assert failed == [], f"the unmodified loops must pass every pin, failed: {failed}"
    else:
        assert failed, f"planted mistake {name!r} slipped through every pin"


# --------------------------------------------------------------------------- streaming interface
def test_slab_and_column_split_invariance(oracle):
    """Running rows [0,T1) then [T1,T) with the carried state is bit-identical to one shot
    (chunk invariance of Algorithm 1), for forward and backward, and so is splitting columns."""
    rng = _rng(31)
    T, C = 513, 7
    lam = _f32(rng.uniform(-1, 1, (T, C)))
    x = _f32(rng.normal(size=(T, C)))
    h0 = _f32(rng.normal(size=C))
    e = _f32(rng.normal(size=(T, C)))
    h = oracle.forward(lam, x, h0)
    state = h0.astype(np.float64)
    h2 = np.empty((T, C))
    for a, b in [(0, 1), (1, 200), (200, 512), (512, 513)]:
        oracle.forward_slab(lam, x, state, h2, a, b, threads=2)
    assert np.array_equal(h, h2)
    h32 = _f32(h)
    gx, gl, gh0 = oracle.backward(lam, h32, h0, e)
    gstate = np.zeros(C); gx2 = np.empty((T, C)); gl2 = np.empty((T, C)); gh02 = np.zeros(C)
    for a, b in [(400, 513), (399, 400), (1, 399), (0, 1)]:
        oracle.backward_slab(lam, h32, h0, e, gstate, gx2, gl2, gh02, a, b, threads=3)
    assert np.array_equal(gx, gx2) and np.array_equal(gl, gl2) and np.array_equal(gh0, gh02)


def test_compare_helpers_agree_with_one_shot(oracle):
    rng = _rng(32)
    T, C = 1000, 5
    lam = _f32(rng.uniform(0, 1, (T, C)))
    x = _f32(rng.normal(size=(T, C)))
    h0 = _f32(rng.normal(size=C))
    e = _f32(rng.normal(size=(T, C)))
    h = oracle.forward(lam, x, h0)
    cand = _f32(h)
    cand[123, 2] += np.float32(0.5)
    r = oracle.forward_compare(lam, x, h0, cand, threads=2, slab_elems=64 * C)
    assert r["worst_index"] == (123, 2)
    assert abs(r["max_abs_err"] - abs(float(cand[123, 2]) - h[123, 2])) < 1e-12
    assert r["max_abs_ref"] == np.abs(h).max()
    h32 = _f32(h)
    gx, gl, gh0 = oracle.backward(lam, h32, h0, e)
    gxc, glc, gh0c = _f32(gx), _f32(gl), _f32(gh0)
    glc[0, 1] += np.float32(0.25)
    for h0_arg in (h0,):
        r = oracle.backward_compare(lam, h32, h0_arg, e, gxc, glc, gh0c, threads=2, slab_elems=37 * C)
        assert r["grad_x"]["max_abs_err"] == np.abs(gxc.astype(np.float64) - gx).max()
        assert r["grad_lambda"]["max_abs_err"] == np.abs(glc.astype(np.float64) - gl).max()
        assert r["grad_h0"]["max_abs_err"] == np.abs(gh0c.astype(np.float64) - gh0).max()
        assert r["grad_x"]["max_abs_ref"] == np.abs(gx).max()
    # NaN in the candidate must be reported as a failure, not swallowed
    cand2 = _f32(h); cand2[5, 0] = np.nan
    assert oracle.forward_compare(lam, x, h0, cand2)["max_abs_err"] == float("inf")
    # the per-element allowance: an error of exactly rel*|ref| everywhere leaves nothing; one element
    # pushed further leaves exactly its excess
    scaled = h * (1 + 2.0 ** -8)
    r = oracle.forward_compare(lam, x, h0, scaled, slab_elems=64 * C, rel=2.0 ** -8)
    assert r["max_abs_err"] <= 1e-12 * np.abs(h).max()
    scaled[77, 3] += np.copysign(0.125, h[77, 3])
    r = oracle.forward_compare(lam, x, h0, scaled, slab_elems=64 * C, rel=2.0 ** -8)
    assert r["worst_index"] == (77, 3) and abs(r["max_abs_err"] - 0.125) < 1e-9
    rb = oracle.backward_compare(lam, h32, h0, e, gx * (1 - 2.0 ** -8), gl, gh0, slab_elems=37 * C, rel=2.0 ** -8)
    assert rb["grad_x"]["max_abs_err"] <= 1e-12 * np.abs(gx).max() and rb["grad_lambda"]["max_abs_err"] == 0.0


def test_empty_shapes(oracle):
    z = np.zeros((0, 3), np.float32)
    assert oracle.forward(z, z, None).shape == (0, 3)
    gx, gl, gh0 = oracle.backward(z, z, None, z)
    assert gx.shape == (0, 3) and np.array_equal(gh0, np.zeros(3))
