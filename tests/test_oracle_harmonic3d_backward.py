"""Pins of the 3-D oracle's backward pass (CPU): finite differences of the forward oracle,
the closed form of the order-0 term, linearity in the output gradient, zero input."""
import numpy as np
import pytest

from oracle import harmonic3d as o3


def _case(shape, J, L, max_order, seed, batch=2):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch,) + shape) + 0.3
    bank = o3.bank_3d(shape, J, L)
    y = o3.harmonic_scattering3d(x, J, L, max_order, bank=bank)
    g = rng.standard_normal(y.shape)
    return x, g, bank


@pytest.mark.parametrize("shape,J,L,mo", [((8, 8, 8), 1, 1, 2), ((8, 8, 8), 2, 2, 2),
                                          ((4, 8, 16), 2, 1, 2), ((8, 8, 8), 2, 1, 1)])
def test_directional_derivatives_match_finite_differences(shape, J, L, mo):
    x, g, bank = _case(shape, J, L, mo, seed=sum(shape) + J + L)
    gx = o3.harmonic_scattering3d_backward(x, g, J, L, mo, bank=bank)
    rng = np.random.default_rng(5)
    for _ in range(3):
        d = rng.standard_normal(x.shape)
        eps = 1e-6
        fp = o3.harmonic_scattering3d(x + eps * d, J, L, mo, bank=bank)
        fm = o3.harmonic_scattering3d(x - eps * d, J, L, mo, bank=bank)
        fd = (g * (fp - fm)).sum() / (2 * eps)
        an = (gx * d).sum()
        assert abs(fd - an) <= 1e-6 * max(abs(fd), abs(an), 1e-3), (fd, an)


def test_order0_gradient_is_the_lowpass_correlation():
    shape, J, L = (8, 8, 8), 1, 1
    x, g, bank = _case(shape, J, L, 2, seed=3, batch=1)
    g0 = np.zeros_like(g)
    g0[:, 0] = g[:, 0]
    gx = o3.harmonic_scattering3d_backward(x, g0, J, L, 2, bank=bank)
    # brute force: d/dx[u] sum_n g[n] (x conv phi)[2n] = sum_n g[n] phi[2n - u]
    phi = bank['phi']
    want = np.zeros(shape)
    for u in np.ndindex(*shape):
        acc = 0.0
        for n in np.ndindex(*[s // 2 for s in shape]):
            idx = tuple((2 * n[d] - u[d]) % shape[d] for d in range(3))
            acc += g[0, 0][n] * phi[idx]
        want[u] = acc
    assert np.abs(gx[0] - want).max() <= 1e-12


def test_linear_in_the_output_gradient_and_zero_input():
    shape, J, L = (8, 8, 8), 2, 1
    x, g, bank = _case(shape, J, L, 2, seed=11)
    g2 = np.random.default_rng(12).standard_normal(g.shape)
    a = o3.harmonic_scattering3d_backward(x, g, J, L, 2, bank=bank)
    b = o3.harmonic_scattering3d_backward(x, g2, J, L, 2, bank=bank)
    c = o3.harmonic_scattering3d_backward(x, 2.0 * g - 3.0 * g2, J, L, 2, bank=bank)
    assert np.abs(c - (2.0 * a - 3.0 * b)).max() <= 1e-11 * np.abs(c).max()
    # x = 0: every modulus signal is zero and passes no gradient; only S0's term is left
    z = o3.harmonic_scattering3d_backward(np.zeros_like(x), g, J, L, 2, bank=bank)
    g0 = np.zeros_like(g)
    g0[:, 0] = g[:, 0]
    z0 = o3.harmonic_scattering3d_backward(np.zeros_like(x), g0, J, L, 2, bank=bank)
    assert np.array_equal(z, z0)


def test_gradient_does_not_depend_on_batch_neighbours():
    shape, J, L = (8, 8, 8), 1, 2
    x, g, bank = _case(shape, J, L, 2, seed=21, batch=3)
    whole = o3.harmonic_scattering3d_backward(x, g, J, L, 2, bank=bank)
    one = o3.harmonic_scattering3d_backward(x[1:2], g[1:2], J, L, 2, bank=bank)
    assert np.abs(whole[1:2] - one).max() <= 1e-13
