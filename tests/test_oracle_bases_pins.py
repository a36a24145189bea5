"""Pins for the Legendre / Hermite / Fourier layer oracle (paper Sec. 2.3, Sec. 6.3); CPU only."""
import numpy as np
import pytest
from numpy.polynomial import hermite as nph
from numpy.polynomial import legendre as npl

import oracle

CHEB, LEG, HERM, FOUR = oracle.BASIS_CHEBYSHEV, oracle.BASIS_LEGENDRE, oracle.BASIS_HERMITE, oracle.BASIS_FOURIER


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def _layer(seed, B, I, O, d):
    return _rand(seed, B, I), _rand(seed + 1, I, O, d + 1) / np.sqrt(I * (d + 1)), _rand(seed + 2, B, O)


@pytest.mark.parametrize("kind,mod", [(LEG, npl), (HERM, nph)])
def test_polynomial_families_match_numpy(kind, mod):
    d = 9
    vander = {LEG: npl.legvander, HERM: nph.hermvander}[kind]
    der = {LEG: npl.legder, HERM: nph.hermder}[kind]
    val = {LEG: npl.legval, HERM: nph.hermval}[kind]
    for x in np.linspace(-3, 3, 41):
        u = np.tanh(x)
        Bv, dB = oracle.basis_eval(kind, x, d)
        assert np.allclose(Bv, vander(np.array([u]), d)[0], rtol=1e-12, atol=1e-12)
        for k in range(d + 1):
            e = np.zeros(d + 1)
            e[k] = 1.0
            want = val(u, der(e)) * (1.0 - u * u) if k > 0 else 0.0
            assert abs(dB[k] - want) <= 1e-10 * max(1.0, abs(want))


def test_explicit_low_degrees_and_end_points():
    x = 0.37
    u = np.tanh(x)
    P, _ = oracle.basis_eval(LEG, x, 3)
    assert np.allclose(P, [1, u, (3 * u * u - 1) / 2, (5 * u ** 3 - 3 * u) / 2], atol=1e-15)
    H, _ = oracle.basis_eval(HERM, x, 3)
    assert np.allclose(H, [1, 2 * u, 4 * u * u - 2, 8 * u ** 3 - 12 * u], atol=1e-14)
    # P_k(1) = 1 and H_k(0) = 0 for odd k, (-1)^{k/2} k!/(k/2)! for even k
    P, _ = oracle.basis_eval(LEG, 40.0, 7)           # tanh(40) = 1 in fp64
    assert np.allclose(P, 1.0, atol=1e-12)
    H, _ = oracle.basis_eval(HERM, 0.0, 8)
    assert np.allclose(H, [1, 0, -2, 0, 12, 0, -120, 0, 1680], atol=1e-12)


def test_fourier_is_cos_and_sin_of_multiples():
    for x in (-2.5, -0.3, 0.0, 1.1, 7.0):
        Bv, dB = oracle.basis_eval(FOUR, x, 8)
        m = np.arange(1, 5)
        assert Bv[0] == 1.0 and dB[0] == 0.0
        assert np.allclose(Bv[1::2], np.cos(m * x), atol=1e-15) and np.allclose(Bv[2::2], np.sin(m * x), atol=1e-15)
        assert np.allclose(Bv[1::2] ** 2 + Bv[2::2] ** 2, 1.0, atol=1e-14)
    # textbook angle: x = pi/3
    Bv, _ = oracle.basis_eval(FOUR, np.pi / 3, 4)
    assert np.allclose(Bv, [1, 0.5, np.sqrt(3) / 2, -0.5, np.sqrt(3) / 2], atol=1e-15)
    with pytest.raises(ValueError):
        oracle.basis_eval(FOUR, 0.1, 5)               # odd "degree" has no cos/sin pairing


@pytest.mark.parametrize("kind,d", [(LEG, 5), (HERM, 5), (FOUR, 6), (CHEB, 5)])
def test_derivative_by_central_differences(kind, d):
    h = 1e-6
    for x in (-1.7, -0.2, 0.4, 2.3):
        _, dB = oracle.basis_eval(kind, x, d)
        num = (oracle.basis_eval(kind, x + h, d)[0] - oracle.basis_eval(kind, x - h, d)[0]) / (2 * h)
        assert np.allclose(dB, num, rtol=1e-7, atol=1e-7)


def test_chebyshev_kind_equals_the_chebyshev_oracle():
    x, C, dy = _layer(3, 40, 7, 5, 6)
    assert np.allclose(oracle.forward_basis(CHEB, x, C), oracle.forward(x, C), rtol=1e-13, atol=1e-13)
    dx, dC = oracle.backward_basis(CHEB, x, C, dy)
    ex, eC = oracle.backward(x, C, dy)
    assert np.allclose(dx, ex, rtol=1e-12, atol=1e-13) and np.allclose(dC, eC, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("kind,d", [(LEG, 6), (HERM, 4), (FOUR, 6)])
def test_layer_against_brute_force_adjoint_and_finite_differences(kind, d):
    B, I, O = 9, 4, 3
    x, C, dy = _layer(50 + kind, B, I, O, d)
    y = oracle.forward_basis(kind, x, C)
    brute = np.zeros((B, O))
    for b in range(B):
        for i in range(I):
            Bv, _ = oracle.basis_eval(kind, x[b, i], d)
            brute[b] += C[i] @ Bv
    assert np.allclose(y, brute, rtol=1e-13, atol=1e-13)
    dx, dC = oracle.backward_basis(kind, x, C, dy)
    assert abs(np.sum(dy * y) - np.sum(C * dC)) <= 1e-11 * np.sum(np.abs(dy * y))
    h = 1e-6
    for b in range(B):
        for i in range(I):
            xp, xm = x.copy(), x.copy()
            xp[b, i] += h
            xm[b, i] -= h
            num = np.sum((oracle.forward_basis(kind, xp, C) - oracle.forward_basis(kind, xm, C)) * dy) / (2 * h)
            assert abs(num - dx[b, i]) <= 1e-6 * max(1.0, abs(dx[b, i]))
    # layout: a one-hot coefficient picks one basis function of one input for one output
    Ch = np.zeros_like(C)
    Ch[2, 1, d - 1] = 1.0
    yh = oracle.forward_basis(kind, x, Ch)
    want = np.array([oracle.basis_eval(kind, x[b, 2], d)[0][d - 1] for b in range(B)])
    assert np.allclose(yh[:, 1], want, atol=1e-14) and np.all(np.delete(yh, 1, axis=1) == 0.0)
