"""Pins of the oracle's backward pass (gradient of <g, S(x)> with respect to x).

The paper states that the transform is differentiable and used inside gradient-based
reconstruction (section 3); it prints no gradient formula, so the oracle's chain of
adjoints is pinned to what mathematics fixes: central finite differences of the oracle's
own forward cascade (a wrong sign, a missing conjugate, a dropped normalisation or a
mis-ordered channel anywhere in the chain changes the directional derivative), the closed
form of the order-0 term, and linearity in g.
"""
import numpy as np
import pytest

import oracle
from oracle import scattering as osc


def _fd(x, g, d, J, L, mo, bank, eps=1e-6):
    f = lambda z: float(np.sum(g * oracle.scattering2d(z, J, L, mo, bank=bank)))
    return (f(x + eps * d) - f(x - eps * d)) / (2 * eps)


@pytest.mark.parametrize("shape,J,L,mo", [((16, 16), 2, 3, 2), ((32, 16), 3, 2, 2),
                                          ((16, 32), 2, 4, 1), ((32, 32), 2, 8, 2),
                                          ((8, 8), 1, 2, 2)])
def test_directional_derivative_matches_finite_differences(shape, J, L, mo):
    rng = np.random.default_rng(sum(shape) + 17 * J + L)
    bank = oracle.bank_2d(shape[0], shape[1], J, L)
    x = rng.standard_normal((2,) + shape)
    S = oracle.scattering2d(x, J, L, mo, bank=bank)
    g = rng.standard_normal(S.shape)
    gx = oracle.scattering2d_backward(x, g, J, L, mo, bank=bank)
    assert gx.shape == x.shape
    for _ in range(3):
        d = rng.standard_normal(x.shape)
        fd = _fd(x, g, d, J, L, mo, bank)
        an = float(np.sum(gx * d))
        assert abs(fd - an) <= 1e-6 * max(abs(fd), 1e-3), (fd, an)


def test_each_channel_group_contributes():
    """g restricted to one order at a time: each restricted gradient still matches finite
    differences, and they add up to the full gradient (catches channel mis-ordering)."""
    rng = np.random.default_rng(3)
    J, L, shape = 2, 3, (16, 16)
    bank = oracle.bank_2d(16, 16, J, L)
    x = rng.standard_normal(shape)
    rows = osc.coeff_index_2d(J, L)
    order = np.array([r[0] for r in rows])
    S = oracle.scattering2d(x, J, L, bank=bank)
    g = rng.standard_normal(S.shape)
    total = oracle.scattering2d_backward(x, g, J, L, bank=bank)
    parts = np.zeros_like(total)
    d = rng.standard_normal(shape)
    for o in (0, 1, 2):
        go = g * (order == o)[:, None, None]
        part = oracle.scattering2d_backward(x, go, J, L, bank=bank)
        fd = _fd(x, go, d, J, L, 2, bank)
        assert abs(fd - np.sum(part * d)) <= 1e-6 * max(abs(fd), 1e-3)
        parts += part
    assert np.allclose(parts, total, rtol=1e-12, atol=1e-12)


def test_order0_gradient_is_upsampled_correlation_with_phi():
    """S0 = (x conv phi)[2^J n] is linear; its transpose applied to g is
    sum_m g[m] phi[2^J m - n] (periodic), written out with the spatial filter."""
    J, L, n = 2, 2, 16
    bank = oracle.bank_2d(n, n, J, L)
    phi = bank['phi']
    rng = np.random.default_rng(9)
    x = rng.standard_normal((n, n))
    K = 1 + J * L + L * L * J * (J - 1) // 2
    m = n >> J
    g = np.zeros((K, m, m))
    g[0] = rng.standard_normal((m, m))
    got = oracle.scattering2d_backward(x, g, J, L, bank=bank)
    want = np.zeros((n, n))
    for a in range(m):
        for b in range(m):
            want += g[0, a, b] * np.roll(np.roll(phi[::-1, ::-1], 1 + (a << J), axis=0),
                                         1 + (b << J), axis=1)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)


def test_linear_in_g_and_zero():
    rng = np.random.default_rng(4)
    J, L, shape = 2, 2, (16, 16)
    bank = oracle.bank_2d(16, 16, J, L)
    x = rng.standard_normal(shape)
    S = oracle.scattering2d(x, J, L, bank=bank)
    g1, g2 = rng.standard_normal(S.shape), rng.standard_normal(S.shape)
    b = lambda g: oracle.scattering2d_backward(x, g, J, L, bank=bank)
    assert np.allclose(b(2.5 * g1 - g2), 2.5 * b(g1) - b(g2), rtol=1e-11, atol=1e-12)
    assert np.all(b(np.zeros_like(g1)) == 0)


def test_zero_input_leaves_only_the_order0_term():
    """y = 0 exactly for x = 0, and the convention g_y = 0 at y = 0 leaves only the linear
    order-0 term of the gradient."""
    J, L, n = 2, 2, 16
    bank = oracle.bank_2d(n, n, J, L)
    x = np.zeros((n, n))
    K = 1 + J * L + L * L * J * (J - 1) // 2
    rng = np.random.default_rng(6)
    g = rng.standard_normal((K, n >> J, n >> J))
    g0 = np.zeros_like(g)
    g0[0] = g[0]
    full = oracle.scattering2d_backward(x, g, J, L, bank=bank)
    only0 = oracle.scattering2d_backward(x, g0, J, L, bank=bank)
    assert np.array_equal(full, only0)
    assert np.abs(full).max() > 0


@pytest.mark.parametrize("n,J,Q,mo,o", [(64, 3, 2, 2, 0), (256, 4, 1, 2, 0), (128, 3, 3, 1, 0),
                                        (64, 3, 2, 2, 1)])
def test_1d_directional_derivative_matches_finite_differences(n, J, Q, mo, o):
    rng = np.random.default_rng(n + J + Q + o)
    bank = oracle.bank_1d(n, J, Q)
    x = rng.standard_normal((2, n))
    S = oracle.scattering1d(x, J, Q, mo, bank=bank, oversampling=o)
    g = rng.standard_normal(S.shape)
    gx = oracle.scattering1d_backward(x, g, J, Q, mo, bank=bank, oversampling=o)
    f = lambda z: float(np.sum(g * oracle.scattering1d(z, J, Q, mo, bank=bank, oversampling=o)))
    for _ in range(3):
        d = rng.standard_normal(x.shape)
        eps = 1e-6
        fd = (f(x + eps * d) - f(x - eps * d)) / (2 * eps)
        assert abs(fd - np.sum(gx * d)) <= 1e-6 * max(abs(fd), 1e-3)
