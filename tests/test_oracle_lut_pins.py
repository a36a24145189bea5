"""Pins for the table-interpolated oracle (paper Sec. 4.2); CPU only.

Checked against things other than the oracle itself: the trigonometric closed form of the samples,
a hand-worked table, the classical linear-interpolation error bound, the mean-value property of a
difference quotient, numerical differentiation of the interpolated forward pass, the adjoint
identity, exactness where interpolation is exact, and convergence to the exact layer.
"""
import os

import numpy as np
import pytest

import oracle


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def _layer(seed, B, I, O, d):
    x = _rand(seed, B, I)
    C = _rand(seed + 1, I, O, d + 1) / np.sqrt(I * (d + 1))
    dy = _rand(seed + 2, B, O)
    return x, C, dy


# ------------------------------------------------------------------- table

@pytest.mark.parametrize("n", [2, 3, 17, 1025])
def test_table_matches_trigonometric_form(n):
    d = 9
    lut = oracle.lut_build(d, n)
    xs = np.linspace(-1.0, 1.0, n)
    want = np.cos(np.arange(d + 1)[:, None] * np.arccos(xs)[None, :])
    assert lut.shape == (d + 1, n)
    assert np.max(np.abs(lut - want)) < 5e-13
    # end points exactly: T_k(1) = 1, T_k(-1) = (-1)^k
    assert np.all(lut[:, -1] == 1.0)
    assert np.all(lut[:, 0] == (-1.0) ** np.arange(d + 1))


def _read_golden(golden_dir):
    rows, example = [], None
    with open(os.path.join(golden_dir, "lut_n5_degree3.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if "|" in line:
                parts = [p.split() for p in line.split("|")]
                example = (float(parts[0][0]), int(parts[1][0]), float(parts[2][0]),
                           np.array(parts[3], dtype=float), np.array(parts[4], dtype=float))
            else:
                rows.append([float(t) for t in line.split()])
    return np.array(rows), example


def test_hand_worked_table_and_interpolation(golden_dir):
    table, (u, cell, frac, T, dT) = _read_golden(golden_dir)
    lut = oracle.lut_build(3, 5)
    assert np.array_equal(lut, table)
    gT, gdT, gcell, gfrac = oracle.lut_eval(lut, u)
    assert gcell == cell and abs(gfrac - frac) < 1e-15
    assert np.allclose(gT, T, atol=1e-15) and np.allclose(gdT, dT, atol=1e-15)


def test_cell_choice_and_clamping_at_the_ends():
    lut = oracle.lut_build(5, 9)                      # step 1/4
    T, dT, cell, frac = oracle.lut_eval(lut, 1.0)
    assert cell == 7 and frac == 1.0 and np.array_equal(T, lut[:, 8])
    T, dT, cell, frac = oracle.lut_eval(lut, -1.0)
    assert cell == 0 and frac == 0.0 and np.array_equal(T, lut[:, 0])
    # a grid point belongs to the cell that starts there
    T, dT, cell, frac = oracle.lut_eval(lut, 0.25)
    assert cell == 5 and frac == 0.0 and np.array_equal(T, lut[:, 5])
    # just below it: previous cell, fraction close to one
    _, _, cell, frac = oracle.lut_eval(lut, 0.25 - 1e-9)
    assert cell == 4 and 0.999999 < frac < 1.0


def test_shift_selects_the_neighbouring_line():
    lut = oracle.lut_build(6, 33)
    u = -1.0 + 2.0 / 32 * 11                          # grid point 11
    T0, dT0, cell, frac = oracle.lut_eval(lut, u)
    Tm, dTm, _, _ = oracle.lut_eval(lut, u, shift=-1)
    assert cell == 11
    assert np.allclose(T0, Tm, atol=1e-14)            # the interpolant is continuous at the knot
    _, dT_left, cell_left, _ = oracle.lut_eval(lut, u - 1e-9)
    assert cell_left == 10 and np.allclose(dTm, dT_left, atol=1e-12)
    assert np.max(np.abs(dTm - dT0)) > 1e-2           # the difference quotient is not


# ----------------------------------------------------------- approximation

@pytest.mark.parametrize("n", [65, 257, 1025])
def test_interpolation_error_within_the_classical_bound(n):
    """|p(u) - f(u)| <= h^2/8 max|f''| for linear interpolation; max|T_k''| = k^2(k^2-1)/3 (at u = +-1)."""
    d = 8
    lut = oracle.lut_build(d, n)
    h = 2.0 / (n - 1)
    us = np.linspace(-1, 1, 20011)
    worst = np.zeros(d + 1)
    for u in us:
        T, _, _, _ = oracle.lut_eval(lut, u)
        worst = np.maximum(worst, np.abs(T - oracle.cheb_T(u, d)))
    k = np.arange(d + 1)
    bound = h * h / 8.0 * k * k * (k * k - 1) / 3.0
    assert np.all(worst <= bound * (1 + 1e-9) + 1e-14)
    assert np.all(worst[:2] < 1e-14)                  # degree 0 and 1 are reproduced exactly
    assert np.all(worst[2:] >= 0.5 * bound[2:])       # and the bound is nearly attained near the ends


def test_interpolation_error_falls_fourfold_when_the_step_halves():
    d = 6
    us = np.linspace(-0.999, 0.999, 4001)
    errs = []
    for n in (129, 257, 513):
        lut = oracle.lut_build(d, n)
        errs.append(max(np.max(np.abs(oracle.lut_eval(lut, u)[0] - oracle.cheb_T(u, d))) for u in us))
    assert 3.5 < errs[0] / errs[1] < 4.5 and 3.5 < errs[1] / errs[2] < 4.5


def test_difference_quotient_is_the_derivative_somewhere_in_the_cell():
    """Mean-value theorem: (T(b)-T(a))/(b-a) = T'(xi) for some xi in [a,b]; also first-order accurate."""
    d, n = 7, 129
    lut = oracle.lut_build(d, n)
    h = 2.0 / (n - 1)
    k = np.arange(d + 1)
    max_second = k * k * (k * k - 1) / 3.0
    for u in np.linspace(-0.9999, 0.9999, 777):
        _, dT, cell, _ = oracle.lut_eval(lut, u)
        a = -1.0 + cell * h
        inside = np.array([oracle.cheb_dT(a + t * h, d) for t in np.linspace(0, 1, 41)])
        assert np.all(dT >= inside.min(axis=0) - 1e-9) and np.all(dT <= inside.max(axis=0) + 1e-9)
        assert np.all(np.abs(dT - oracle.cheb_dT(u, d)) <= h * max_second + 1e-9)
    assert dT[0] == 0.0 and abs(dT[1] - 1.0) < 1e-12


# ------------------------------------------------------------------ layer

def test_exact_where_interpolation_is_exact():
    # degree <= 1: every basis function is linear, the table reproduces it
    x, C, dy = _layer(3, 40, 6, 5, 1)
    lut = oracle.lut_build(1, 33)
    assert np.allclose(oracle.forward_lut(x, C, lut), oracle.forward(x, C), atol=1e-13)
    dx, dC = oracle.backward_lut(x, C, dy, lut)
    ex, eC = oracle.backward(x, C, dy)
    assert np.allclose(dx, ex, atol=1e-12) and np.allclose(dC, eC, atol=1e-12)
    # any degree: inputs whose tanh is a grid point
    d, n = 5, 17
    lut = oracle.lut_build(d, n)
    grid = np.linspace(-1, 1, n)[1:-1]
    x = np.arctanh(np.random.default_rng(0).choice(grid, size=(30, 4)))
    C = _rand(1, 4, 3, d + 1)
    assert np.allclose(oracle.forward_lut(x, C, lut), oracle.forward(x, C), atol=1e-11)


def test_dx_is_the_derivative_of_the_interpolated_forward():
    B, I, O, d, n = 12, 5, 4, 6, 65
    x, C, dy = _layer(11, B, I, O, d)
    lut = oracle.lut_build(d, n)
    dx, _, frac = oracle.backward_lut(x, C, dy, lut, want_frac=True)
    h = 1e-6
    checked = 0
    for b in range(B):
        for i in range(I):
            if not 0.05 < frac[b, i] < 0.95:          # stay inside one cell for x +- h
                continue
            xp, xm = x.copy(), x.copy()
            xp[b, i] += h
            xm[b, i] -= h
            num = np.sum((oracle.forward_lut(xp, C, lut) - oracle.forward_lut(xm, C, lut)) * dy) / (2 * h)
            assert abs(num - dx[b, i]) <= 1e-7 * max(1.0, abs(dx[b, i]))
            checked += 1
    assert checked > 40


def test_adjoint_identity_and_linearity():
    x, C, dy = _layer(21, 50, 7, 6, 5)
    lut = oracle.lut_build(5, 129)
    y = oracle.forward_lut(x, C, lut)
    _, dC = oracle.backward_lut(x, C, dy, lut, need_dx=False)
    assert abs(np.sum(dy * y) - np.sum(C * dC)) <= 1e-11 * np.sum(np.abs(dy * y))
    assert np.allclose(oracle.forward_lut(x, 2.5 * C, lut), 2.5 * y, rtol=1e-13)


def test_layout_of_coefficients_and_table_rows():
    """One-hot coefficient C[i,o,k] = 1 makes y[:,o] the interpolated T_k of input i alone."""
    B, I, O, d, n = 9, 3, 4, 4, 33
    x = _rand(5, B, I)
    lut = oracle.lut_build(d, n)
    for (i, o, k) in [(0, 0, 0), (2, 1, 3), (1, 3, 4), (0, 2, 2)]:
        C = np.zeros((I, O, d + 1))
        C[i, o, k] = 1.0
        y = oracle.forward_lut(x, C, lut)
        want = np.array([oracle.lut_eval(lut, np.tanh(x[b, i]))[0][k] for b in range(B)])
        assert np.allclose(y[:, o], want, atol=1e-14)
        assert np.all(np.delete(y, o, axis=1) == 0.0)


def test_converges_to_the_exact_layer():
    x, C, dy = _layer(31, 64, 16, 12, 6)
    y_ref = oracle.forward(x, C)
    dx_ref, dC_ref = oracle.backward(x, C, dy)
    prev = None
    for n in (257, 1025, 4097):
        lut = oracle.lut_build(6, n)
        ey = oracle.rel_err(oracle.forward_lut(x, C, lut), y_ref)
        dx, dC = oracle.backward_lut(x, C, dy, lut)
        edx, edC = oracle.rel_err(dx, dx_ref), oracle.rel_err(dC, dC_ref)
        if prev is not None:
            assert 10 < prev[0] / ey < 22 and 10 < prev[2] / edC < 22      # second order: 16x per 4x samples
            assert 3 < prev[1] / edx < 5.5                                  # first order: 4x per 4x samples
        prev = (ey, edx, edC)
    assert prev[0] < 2e-5 and prev[2] < 2e-5 and prev[1] < 5e-3


def test_sampled_dC_matches_the_full_computation():
    x, C, dy = _layer(41, 70, 6, 5, 4)
    lut = oracle.lut_build(4, 65)
    _, dC = oracle.backward_lut(x, C, dy, lut, need_dx=False)
    is_, os_, ks = [0, 5, 3, 2], [4, 0, 2, 2], [0, 4, 1, 3]
    got = oracle.dC_lut_at(x, dy, lut, is_, os_, ks)
    assert np.allclose(got, dC[is_, os_, ks], rtol=1e-13, atol=1e-13)


# ------------------------------------------- auxiliary derivative table (second-order dx)

def _d3_bound(k):
    """max |T_k'''| on [-1, 1], attained at the ends: k^2 (k^2-1)(k^2-4) / 15."""
    return k * k * (k * k - 1) * (k * k - 4) / 15.0


@pytest.mark.parametrize("n", [2, 3, 17, 1025])
def test_derivative_table_matches_closed_forms(n):
    d = 9
    dlut = oracle.lut_build_derivative(d, n)
    assert dlut.shape == (d + 1, n)
    xs = np.linspace(-1.0, 1.0, n)
    k = np.arange(d + 1)
    # ends: T_k'(+-1) = (+-1)^(k+1) k^2, exactly
    assert np.array_equal(dlut[:, -1], (k * k).astype(float))
    assert np.array_equal(dlut[:, 0], ((-1.0) ** (k + 1)) * k * k)
    # interior: k sin(k t) / sin t at x = cos t
    inner = slice(1, n - 1)
    if n > 2:
        t = np.arccos(xs[inner])
        want = k[:, None] * np.sin(k[:, None] * t[None, :]) / np.sin(t)[None, :]
        assert np.max(np.abs(dlut[:, inner] - want)) < 2e-10
    # numpy's Chebyshev derivative as an independent generator
    for kk in range(d + 1):
        c = np.zeros(kk + 1)
        c[kk] = 1.0
        der = np.polynomial.chebyshev.chebder(c) if kk >= 1 else np.zeros(1)
        assert np.max(np.abs(dlut[kk] - np.polynomial.chebyshev.chebval(xs, der))) < 1e-10


def test_hand_worked_derivative_table(golden_dir):
    rows, example = [], None
    with open(os.path.join(golden_dir, "dlut_n5_degree3.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if "|" in line:
                u, vals = line.split("|")
                example = (float(u), np.array(vals.split(), dtype=float))
            else:
                rows.append([float(t) for t in line.split()])
    dlut = oracle.lut_build_derivative(3, 5)
    assert np.array_equal(dlut, np.array(rows))
    assert np.allclose(oracle.lut_eval_derivative(dlut, example[0]), example[1], atol=1e-15)


def test_interpolated_derivative_is_exact_where_it_must_be():
    n, d = 33, 7
    dlut = oracle.lut_build_derivative(d, n)
    xs = np.linspace(-1.0, 1.0, n)
    for i in (0, 1, 7, 16, 31, 32):                       # at grid points (both ends: the clamped last cell)
        assert np.allclose(oracle.lut_eval_derivative(dlut, xs[i]), dlut[:, i], rtol=0, atol=1e-12)
    for u in (-0.93, -0.2, 0.031, 0.77):                  # T_0' = 0, T_1' = 1, T_2' = 4u are linear: no error
        got = oracle.lut_eval_derivative(dlut, u)
        assert np.allclose(got[:3], [0.0, 1.0, 4.0 * u], atol=1e-13)


@pytest.mark.parametrize("n", [17, 129, 1025])
def test_interpolated_derivative_error_bound_and_order(n):
    """Linear interpolation of T_k' errs by at most Delta^2/8 max|T_k'''|; near the ends (where T_k''' is
    largest) a cell midpoint comes close to the bound; halving the step divides the error by about four."""
    d = 8
    def worst(nn):
        dlut = oracle.lut_build_derivative(d, nn)
        us = np.linspace(-1.0, 1.0, 40 * (nn - 1) + 1)
        got = np.array([oracle.lut_eval_derivative(dlut, u) for u in us])
        want = np.array([oracle.cheb_dT(u, d) for u in us])
        return np.max(np.abs(got - want), axis=0)
    delta = 2.0 / (n - 1)
    err = worst(n)
    for k in range(d + 1):
        bound = delta * delta / 8.0 * _d3_bound(k)
        assert err[k] <= bound * (1 + 1e-9) + 1e-12, (k, err[k], bound)
        if k >= 3 and n >= 129:
            assert err[k] >= 0.8 * bound, (k, err[k], bound)     # nearly attained in the end cells
    if n >= 129:                                              # 17 samples are too coarse for the asymptotic order
        err2 = worst(2 * (n - 1) + 1)
        for k in range(3, d + 1):
            assert 3.5 <= err[k] / err2[k] <= 4.5, (k, err[k] / err2[k])


def test_dx_with_derivative_table_against_a_written_out_sum():
    """The layer formula around the table: dx[b,i] = (1-u^2) sum_o dy[b,o] sum_{k>=1} C[i,o,k] dT_k(u), with dT
    taken from numpy's own piecewise-linear interpolation of the table rows."""
    B, I, O, d, n = 3, 4, 2, 5, 21
    x, C, dy = _layer(71, B, I, O, d)
    dlut = oracle.lut_build_derivative(d, n)
    grid = np.linspace(-1.0, 1.0, n)
    want = np.zeros((B, I))
    for b in range(B):
        for i in range(I):
            u = np.tanh(x[b, i])
            dT = np.array([np.interp(u, grid, dlut[k]) for k in range(d + 1)])
            want[b, i] = (1.0 - u * u) * sum(dy[b, o] * sum(C[i, o, k] * dT[k] for k in range(1, d + 1)) for o in range(O))
    assert np.allclose(oracle.dx_lut2(x, C, dy, dlut), want, rtol=1e-12, atol=1e-13)
    # coefficients of T_0 never reach dx
    C2 = C.copy()
    C2[:, :, 0] += 5.0
    assert np.allclose(oracle.dx_lut2(x, C2, dy, dlut), want, rtol=1e-12, atol=1e-13)


def test_dx_with_derivative_table_converges_to_the_exact_layer_at_second_order():
    x, C, dy = _layer(81, 300, 20, 12, 8)
    exact, _ = oracle.backward(x, C, dy, need_dC=False)
    errs = [oracle.rel_err(oracle.dx_lut2(x, C, dy, oracle.lut_build_derivative(8, n)), exact) for n in (129, 257, 513, 1025)]
    for a, b in zip(errs, errs[1:]):
        assert 3.0 <= a / b <= 5.0, errs
    assert errs[-1] <= 1e-3                                # the bound stated for any table variant, at 1025 samples
    # the first-order difference quotient of the plain table is far outside it at the same size
    lut = oracle.lut_build(8, 1025)
    first_order, _ = oracle.backward_lut(x, C, dy, lut, need_dC=False)
    assert oracle.rel_err(first_order, exact) > 1e-2
