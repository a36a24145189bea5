"""Pins for the fp64 CPU oracle: everything here runs without a GPU.

The oracle is checked against things other than itself: closed forms of the
Chebyshev polynomials (paper Eq. 1 against Eq. 2), explicit low-degree
polynomials, numpy's own Chebyshev basis, a brute-force evaluation that uses
the trigonometric form, the adjoint identity between forward and dC, central
finite differences for dx and dC, degenerate cases and a hand-worked example.
"""
import json
import math
import os

import numpy as np
import pytest
from numpy.polynomial import chebyshev as npcheb

import oracle
from paper_2511_14852_amd import workloads as wl


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------- basis pins

def _parse_num(tok):
    r2 = math.sqrt(2.0) / 2.0
    val = 1.0
    for f in tok.split("*"):
        f = f.strip()
        if f == "r2":
            val *= r2
        elif f == "-r2":
            val *= -r2
        else:
            val *= float(f)
    return val


def test_basis_special_angles_golden(golden_dir):
    """Eq. 1 closed form at textbook angles, values and derivatives."""
    rows = 0
    with open(os.path.join(golden_dir, "chebyshev_special_angles.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            u_s, t_s, dt_s = [p.strip() for p in line.split("|")]
            u = _parse_num(u_s)
            want_T = np.array([_parse_num(t) for t in t_s.split()])
            want_dT = np.array([_parse_num(t) for t in dt_s.split()])
            d = len(want_T) - 1
            np.testing.assert_allclose(oracle.cheb_T(u, d), want_T, atol=1e-14)
            np.testing.assert_allclose(oracle.cheb_dT(u, d), want_dT, atol=2e-13)
            rows += 1
    assert rows == 6


def test_recurrence_equals_trig_form_on_theta_grid():
    """T_k(cos t) = cos(k t): Eq. 2 against Eq. 1, degrees up to 24."""
    d = 24
    for theta in np.linspace(0.0, math.pi, 257):
        u = math.cos(theta)
        want = np.cos(np.arange(d + 1) * theta)
        np.testing.assert_allclose(oracle.cheb_T(u, d), want, atol=5e-12)
        np.testing.assert_allclose(oracle.cheb_T_trig(u, d), want, atol=5e-12)


def test_explicit_low_degree_polynomials_and_symmetry():
    for u in np.linspace(-1, 1, 41):
        T = oracle.cheb_T(u, 6)
        assert T[0] == 1.0 and T[1] == u
        assert T[2] == pytest.approx(2 * u * u - 1, abs=1e-13)
        assert T[3] == pytest.approx(4 * u ** 3 - 3 * u, abs=1e-13)
        assert T[4] == pytest.approx(8 * u ** 4 - 8 * u ** 2 + 1, abs=1e-13)
        assert T[5] == pytest.approx(16 * u ** 5 - 20 * u ** 3 + 5 * u, abs=1e-13)
        assert np.all(np.abs(T) <= 1 + 1e-14)
        Tm = oracle.cheb_T(-u, 6)
        np.testing.assert_allclose(Tm, T * (-1.0) ** np.arange(7), atol=1e-13)
        dT = oracle.cheb_dT(u, 5)
        assert dT[0] == 0.0 and dT[1] == 1.0
        assert dT[2] == pytest.approx(4 * u, abs=1e-13)
        assert dT[3] == pytest.approx(12 * u * u - 3, abs=1e-13)
        assert dT[4] == pytest.approx(32 * u ** 3 - 16 * u, abs=1e-13)
        assert dT[5] == pytest.approx(80 * u ** 4 - 60 * u ** 2 + 5, abs=1e-13)


def test_derivative_closed_form_and_endpoints():
    d = 12
    k = np.arange(d + 1)
    for theta in np.linspace(0.05, math.pi - 0.05, 101):
        want = k * np.sin(k * theta) / math.sin(theta)
        np.testing.assert_allclose(oracle.cheb_dT(math.cos(theta), d), want, rtol=0, atol=1e-10)
    np.testing.assert_allclose(oracle.cheb_dT(1.0, d), k ** 2.0, atol=0)
    np.testing.assert_allclose(oracle.cheb_dT(-1.0, d), (-1.0) ** (k + 1) * k ** 2.0, atol=0)


def test_derivative_matches_numpy_chebder():
    d = 9
    for u in np.linspace(-0.99, 0.99, 37):
        for kk in range(d + 1):
            coef = np.zeros(kk + 1)
            coef[kk] = 1.0
            want = npcheb.chebval(u, npcheb.chebder(coef)) if kk > 0 else 0.0
            assert oracle.cheb_dT(u, d)[kk] == pytest.approx(want, abs=1e-11)


# ------------------------------------------------------------- forward pins

def test_forward_matches_numpy_chebvander_einsum():
    """Independent basis generator (numpy) + einsum contraction."""
    for (B, I, O, d, seed) in [(7, 5, 3, 4, 1), (16, 9, 11, 8, 2), (3, 1, 1, 1, 3), (5, 4, 6, 0, 4)]:
        x = _rand(seed, B, I) * 1.5
        C = _rand(seed + 100, I, O, d + 1)
        V = npcheb.chebvander(np.tanh(x), d)            # [B, I, d+1]
        want = np.einsum("bik,iok->bo", V, C)
        np.testing.assert_allclose(oracle.forward(x, C), want, rtol=0, atol=1e-12)


def test_forward_brute_force_trig_form_tiny():
    """Triple loop written out, basis from cos(k acos u): independent of the recurrence code."""
    B, I, O, d = 2, 3, 2, 3
    x = _rand(11, B, I)
    C = _rand(12, I, O, d + 1)
    want = np.zeros((B, O))
    for b in range(B):
        for o in range(O):
            s = 0.0
            for i in range(I):
                theta = math.acos(math.tanh(x[b, i]))
                for k in range(d + 1):
                    s += C[i, o, k] * math.cos(k * theta)
            want[b, o] = s
    np.testing.assert_allclose(oracle.forward(x, C), want, atol=1e-13)


def test_forward_degree_one_is_a_matmul():
    B, I, O = 9, 6, 4
    x = _rand(21, B, I)
    C = _rand(22, I, O, 2)
    want = np.tanh(x) @ C[:, :, 1] + C[:, :, 0].sum(axis=0)[None, :]
    np.testing.assert_allclose(oracle.forward(x, C), want, atol=1e-13)


def test_forward_one_hot_coefficient_selects_basis_function():
    B, I, O, d = 4, 3, 2, 5
    x = _rand(31, B, I)
    for (i, o, k) in [(0, 0, 0), (2, 1, 5), (1, 0, 3)]:
        C = np.zeros((I, O, d + 1))
        C[i, o, k] = 1.0
        y = oracle.forward(x, C)
        want = np.zeros((B, O))
        want[:, o] = np.cos(k * np.arccos(np.tanh(x[:, i])))
        np.testing.assert_allclose(y, want, atol=1e-13)


def test_forward_coefficient_layout_is_in_out_degree():
    """A transposed operand (reading C as [out,in,k] or [in,k,out]) must fail this."""
    B, I, O, d = 3, 2, 4, 2
    x = _rand(41, B, I)
    C = _rand(42, I, O, d + 1)
    y = oracle.forward(x, C)
    V = npcheb.chebvander(np.tanh(x), d)
    wrong1 = np.einsum("bik,oik->bo", V, C.reshape(O, I, d + 1))
    wrong2 = np.einsum("bik,iko->bo", V, C.reshape(I, d + 1, O))
    assert np.max(np.abs(y - wrong1)) > 1e-3
    assert np.max(np.abs(y - wrong2)) > 1e-3


# ------------------------------------------------------------ backward pins

def test_adjoint_identity_pins_dC_to_forward():
    """y is linear in C, so <dy, y> = <C, dC> exactly."""
    for (B, I, O, d, seed) in [(13, 7, 5, 6, 1), (4, 2, 9, 3, 2), (64, 3, 2, 8, 3)]:
        x = _rand(seed, B, I)
        C = _rand(seed + 1, I, O, d + 1)
        dy = _rand(seed + 2, B, O)
        y = oracle.forward(x, C)
        _, dC = oracle.backward(x, C, dy, need_dx=False)
        lhs = float(np.sum(dy * y))
        rhs = float(np.sum(C * dC))
        assert lhs == pytest.approx(rhs, rel=1e-12, abs=1e-12)


def test_dC_equals_einsum_of_numpy_basis():
    B, I, O, d = 10, 4, 3, 5
    x = _rand(51, B, I)
    C = _rand(52, I, O, d + 1)
    dy = _rand(53, B, O)
    V = npcheb.chebvander(np.tanh(x), d)
    want = np.einsum("bik,bo->iok", V, dy)
    _, dC = oracle.backward(x, C, dy, need_dx=False)
    np.testing.assert_allclose(dC, want, atol=1e-12)


def test_dx_central_finite_differences_every_element():
    """Pins dx, including the tanh derivative factor (1 - u^2)."""
    B, I, O, d = 3, 4, 5, 6
    x = _rand(61, B, I)
    C = _rand(62, I, O, d + 1)
    dy = _rand(63, B, O)
    dx, _ = oracle.backward(x, C, dy, need_dC=False)
    h = 1e-6
    for b in range(B):
        for i in range(I):
            xp, xm = x.copy(), x.copy()
            xp[b, i] += h
            xm[b, i] -= h
            fd = (np.sum(dy * oracle.forward(xp, C)) - np.sum(dy * oracle.forward(xm, C))) / (2 * h)
            assert dx[b, i] == pytest.approx(fd, rel=2e-7, abs=2e-8)
    # without the tanh factor the result would differ visibly
    u = np.tanh(x)
    assert np.max(np.abs(dx - dx / np.maximum(1 - u * u, 1e-3))) > 1e-3


def test_dx_directional_finite_difference():
    B, I, O, d = 6, 7, 3, 8
    x = _rand(71, B, I) * 0.8
    C = _rand(72, I, O, d + 1) / math.sqrt(I * (d + 1))
    dy = _rand(73, B, O)
    dx, _ = oracle.backward(x, C, dy, need_dC=False)
    for s in range(4):
        v = _rand(80 + s, B, I)
        h = 1e-6
        fd = (np.sum(dy * oracle.forward(x + h * v, C)) - np.sum(dy * oracle.forward(x - h * v, C))) / (2 * h)
        assert float(np.sum(dx * v)) == pytest.approx(fd, rel=1e-6, abs=1e-8)


def test_dC_finite_differences():
    B, I, O, d = 5, 3, 2, 4
    x = _rand(91, B, I)
    C = _rand(92, I, O, d + 1)
    dy = _rand(93, B, O)
    _, dC = oracle.backward(x, C, dy, need_dx=False)
    base = np.sum(dy * oracle.forward(x, C))
    for (i, o, k) in [(0, 0, 0), (2, 1, 4), (1, 0, 2), (2, 0, 1)]:
        Cp = C.copy()
        Cp[i, o, k] += 0.5                       # exact: the loss is linear in C
        fd = (np.sum(dy * oracle.forward(x, Cp)) - base) / 0.5
        assert dC[i, o, k] == pytest.approx(fd, rel=1e-11, abs=1e-11)


def test_dx_brute_force_trig_derivative_tiny():
    B, I, O, d = 2, 2, 3, 4
    x = _rand(101, B, I) * 0.7
    C = _rand(102, I, O, d + 1)
    dy = _rand(103, B, O)
    want = np.zeros((B, I))
    for b in range(B):
        for i in range(I):
            u = math.tanh(x[b, i])
            th = math.acos(u)
            s = 0.0
            for o in range(O):
                for k in range(1, d + 1):
                    s += dy[b, o] * C[i, o, k] * k * math.sin(k * th) / math.sin(th)
            want[b, i] = (1 - u * u) * s
    dx, _ = oracle.backward(x, C, dy, need_dC=False)
    np.testing.assert_allclose(dx, want, atol=1e-12)


def test_degenerate_cases():
    B, I, O = 6, 3, 4
    x = _rand(111, B, I)
    dy = _rand(112, B, O)
    # degree 0: y independent of x, dx = 0, dC[i,o,0] = sum_b dy[b,o]
    C0 = _rand(113, I, O, 1)
    y = oracle.forward(x, C0)
    np.testing.assert_allclose(y, np.broadcast_to(C0[:, :, 0].sum(axis=0), (B, O)), atol=1e-14)
    dx, dC = oracle.backward(x, C0, dy)
    assert np.all(dx == 0.0)
    np.testing.assert_allclose(dC[:, :, 0], np.broadcast_to(dy.sum(axis=0), (I, O)), atol=1e-13)
    # zero coefficients
    Cz = np.zeros((I, O, 5))
    assert np.all(oracle.forward(x, Cz) == 0.0)
    dx, _ = oracle.backward(x, Cz, dy)
    assert np.all(dx == 0.0)
    # one-hot dy picks one row/column
    dyh = np.zeros((B, O))
    dyh[2, 1] = 1.0
    C = _rand(114, I, O, 4)
    dx, dC = oracle.backward(x, C, dyh)
    assert np.all(dx[[0, 1, 3, 4, 5]] == 0.0)
    assert np.all(dC[:, [0, 2, 3], :] == 0.0)
    V = npcheb.chebvander(np.tanh(x[2]), 3)
    np.testing.assert_allclose(dC[:, 1, :], V, atol=1e-14)
    # empty batch
    assert oracle.forward(np.zeros((0, I)), C).shape == (0, O)
    dx, dC = oracle.backward(np.zeros((0, I)), C, np.zeros((0, O)))
    assert dx.shape == (0, I) and np.all(dC == 0.0)
    # saturated tanh: u = +-1, derivative factor vanishes
    xs = np.array([[40.0, -40.0, 0.0]])
    dx, _ = oracle.backward(xs, C, np.ones((1, O)))
    assert dx[0, 0] == 0.0 and dx[0, 1] == 0.0 and dx[0, 2] != 0.0


def test_hand_worked_layer_golden(golden_dir):
    with open(os.path.join(golden_dir, "hand_worked_layer.json")) as f:
        g = json.load(f)
    u = np.array(g["u"], dtype=np.float64)
    x = np.arctanh(u)
    C = np.array(g["C"], dtype=np.float64)
    dy = np.array(g["dy"], dtype=np.float64)
    assert C.shape[2] == g["degree"] + 1
    np.testing.assert_allclose(oracle.forward(x, C), np.array(g["y"]), atol=1e-14)
    dx, dC = oracle.backward(x, C, dy)
    np.testing.assert_allclose(dC, np.array(g["dC"]), atol=1e-14)
    np.testing.assert_allclose(dx, np.array(g["dx"]), atol=1e-13)


# ------------------------------------------------- sampled-output functions

def test_sampled_functions_agree_with_full_ones_and_numpy():
    B, I, O, d = 20, 6, 7, 5
    x = _rand(121, B, I)
    C = _rand(122, I, O, d + 1)
    dy = _rand(123, B, O)
    V = npcheb.chebvander(np.tanh(x), d)
    y = np.einsum("bik,iok->bo", V, C)
    dC = np.einsum("bik,bo->iok", V, dy)
    dx_full, _ = oracle.backward(x, C, dy, need_dC=False)
    rng = np.random.default_rng(5)
    bs = rng.integers(0, B, 50)
    os_ = rng.integers(0, O, 50)
    is_ = rng.integers(0, I, 50)
    ks = rng.integers(0, d + 1, 50)
    np.testing.assert_allclose(oracle.forward_at(x, C, bs, os_), y[bs, os_], atol=1e-12)
    np.testing.assert_allclose(oracle.dC_at(x, dy, d, is_, os_, ks), dC[is_, os_, ks], atol=1e-12)
    np.testing.assert_allclose(oracle.dx_at(x, C, dy, bs, is_), dx_full[bs, is_], atol=1e-12)


def test_fp32_inputs_are_promoted_exactly():
    B, I, O, d = 8, 4, 3, 4
    x = wl.make_x(B, I, 7)
    C = wl.make_coeff(I, O, d, 8)
    assert x.dtype == np.float32 and C.dtype == np.float32
    np.testing.assert_array_equal(oracle.forward(x, C), oracle.forward(x.astype(np.float64), C.astype(np.float64)))


# ------------------------------------------------------ workload generators

def test_workload_generators_are_seeded_and_shaped():
    w = wl.WORKLOADS["c2"]
    assert w.layers == [(8, 64), (64, 64), (64, 1)] and w.batch == 65536 and w.degree == 6
    x0, Cs, dy = wl.workload_inputs(w, batch=512)
    x0b, Csb, dyb = wl.workload_inputs(w, batch=512)
    np.testing.assert_array_equal(x0, x0b)
    np.testing.assert_array_equal(Cs[1], Csb[1])
    assert x0.shape == (512, 8) and Cs[2].shape == (64, 1, 7) and dy.shape == (512, 1)
    assert x0.dtype == np.float32
    big = wl.make_coeff(64, 64, 6, 3)
    assert np.std(big) == pytest.approx(1 / math.sqrt(64 * 7), rel=0.05)
    w4 = wl.WORKLOADS["c4"]
    x4, _, _ = wl.workload_inputs(w4, batch=4000)
    assert np.mean(x4) == pytest.approx(-2.0, abs=0.05) and np.std(x4) == pytest.approx(1.5, rel=0.05)
    assert wl.layer_flops(16384, 1024, 1024, 8) == 2 * 16384 * 1024 * 1024 * 26
