"""Pins for the oracle's filter banks (CPU only).

Each test checks the spatially built, numpy-transformed oracle filters against
something fixed by mathematics rather than by the oracle's own code: the analytic
Fourier transform of a (periodised) Gabor function, symmetry identities, and the
Littlewood-Paley / Parseval energy relations of a wavelet frame.
"""
import math

import numpy as np
import pytest

from oracle import filters


# ---- closed form (Poisson summation): the DFT of a sampled, N-periodised function is
# its continuous Fourier transform sampled at 2 pi k / N and summed over 2 pi aliases.

def _gauss_hat_2d(w_r, w_c, sigma, theta, slant):
    ct, st = math.cos(theta), math.sin(theta)
    along = w_r * ct + w_c * st
    across = -w_r * st + w_c * ct
    return np.exp(-0.5 * sigma * sigma * (along ** 2 + (across / slant) ** 2))


def _morlet_hat_2d_closed(n_r, n_c, sigma, xi, theta, slant, aliases=6):
    wr = 2 * math.pi * np.arange(n_r)[:, None] / n_r
    wc = 2 * math.pi * np.arange(n_c)[None, :] / n_c
    gab = np.zeros((n_r, n_c))
    env = np.zeros((n_r, n_c))
    gab0 = 0.0
    env0 = 0.0
    xr, xc = xi * math.cos(theta), xi * math.sin(theta)
    for a in range(-aliases, aliases + 1):
        for b in range(-aliases, aliases + 1):
            sr, sc = 2 * math.pi * a, 2 * math.pi * b
            gab += _gauss_hat_2d(wr + sr - xr, wc + sc - xc, sigma, theta, slant)
            env += _gauss_hat_2d(wr + sr, wc + sc, sigma, theta, slant)
            gab0 += float(_gauss_hat_2d(sr - xr, sc - xc, sigma, theta, slant))
            env0 += float(_gauss_hat_2d(sr, sc, sigma, theta, slant))
    return gab - (gab0 / env0) * env


@pytest.mark.parametrize("n_r,n_c,J,L", [(32, 32, 2, 8), (64, 32, 3, 4), (16, 16, 2, 6)])
def test_morlet_2d_matches_analytic_fourier_transform(n_r, n_c, J, L):
    bank = filters.bank_2d(n_r, n_c, J, L)
    for j in range(J):
        for l in range(L):
            closed = _morlet_hat_2d_closed(n_r, n_c, 0.8 * 2 ** j, 0.75 * math.pi / 2 ** j,
                                           math.pi * l / L, 4.0 / L)
            assert np.abs(bank['psi_hat'][j, l] - closed).max() < 1e-13


def test_gaussian_2d_matches_analytic_fourier_transform():
    n, J = 64, 3
    sigma = 0.8 * 2 ** J
    got = np.fft.fft2(filters.gaussian_2d(n, n, sigma))
    w = 2 * math.pi * np.arange(n) / n
    one = sum(np.exp(-0.5 * sigma ** 2 * (w + 2 * math.pi * a) ** 2) for a in range(-4, 5))
    assert np.abs(got - one[:, None] * one[None, :]).max() < 1e-14


@pytest.mark.parametrize("n,J,Q", [(256, 4, 1), (1024, 5, 8), (512, 3, 4)])
def test_morlet_1d_matches_analytic_fourier_transform(n, J, Q):
    bank = filters.bank_1d(n, J, Q)
    w = 2 * math.pi * np.arange(n) / n
    shifts = [2 * math.pi * a for a in range(-6, 7)]

    def closed(sigma, xi):
        gab = sum(np.exp(-0.5 * sigma ** 2 * (w + s - xi) ** 2) for s in shifts)
        env = sum(np.exp(-0.5 * sigma ** 2 * (w + s) ** 2) for s in shifts)
        gab0 = sum(math.exp(-0.5 * sigma ** 2 * (s - xi) ** 2) for s in shifts)
        env0 = sum(math.exp(-0.5 * sigma ** 2 * s ** 2) for s in shifts)
        return gab - gab0 / env0 * env

    for k in range(J * Q):
        xi = 0.75 * math.pi * 2 ** (-k / Q)
        sigma = 0.8 * 2 ** k if Q == 1 else 0.3 * math.pi / (xi * (1 - 2 ** (-1 / Q)))
        assert np.abs(bank['psi1_hat'][k] - closed(sigma, xi)).max() < 1e-12
    for j in range(J):
        assert np.abs(bank['psi2_hat'][j]
                      - closed(0.8 * 2 ** j, 0.75 * math.pi / 2 ** j)).max() < 1e-12
    assert bank['j1'] == [k // Q for k in range(J * Q)]


def test_q1_first_order_bank_equals_second_order_bank():
    bank = filters.bank_1d(512, 4, 1)
    assert np.abs(bank['psi1_hat'] - bank['psi2_hat']).max() < 1e-14


# ---- identities

def test_filter_identities_2d():
    n, J, L = 32, 2, 8
    bank = filters.bank_2d(n, n, J, L)
    ph, ps = bank['phi_hat'], bank['psi_hat']
    assert np.abs(ps[:, :, 0, 0]).max() < 1e-15           # zero mean
    assert abs(ph[0, 0] - 1.0) < 1e-14                    # unit mass
    assert np.abs(ps.imag).max() < 1e-14                  # psi(-u) = conj psi(u)
    assert np.abs(ph.imag).max() < 1e-14
    assert abs(bank['psi'].sum(axis=(-2, -1))).max() < 1e-15
    # rotating by 90 degrees: psi_hat_{theta+pi/2}[k_r, k_c] = psi_hat_theta[k_c, -k_r]
    k = np.arange(n)
    for j in range(J):
        for l in range(L // 2):
            a = ps[j, l + L // 2]
            b = ps[j, l][np.ix_(k, (-k) % n)].T   # b[k_r, k_c] = ps[k_c, -k_r]
            assert np.abs(a - b).max() < 1e-14
    # close to analytic: the response at the mirrored frequency is small next to the
    # peak (for j = 0 the 2 pi alias of the wide Gaussian reaches it, so j >= 1 only)
    for j in range(J):
        pk = np.unravel_index(np.argmax(ps[j, 0].real), (n, n))
        assert pk[1] == 0 and 0 < pk[0] < n // 2          # theta=0 oscillates along rows
        if j >= 1:
            assert abs(ps[j, 0][(-pk[0]) % n, 0]) < 5e-2 * ps[j, 0].real.max()


def test_orientation_convention():
    """theta = 0 responds to a wave varying along the first (row) axis only."""
    n = 32
    bank = filters.bank_2d(n, n, 1, 4)
    r = np.arange(n)[:, None] + 0 * np.arange(n)[None, :]
    wave = np.exp(2j * math.pi * 12 * r / n)             # frequency index (12, 0) ~ 3pi/4
    resp = [abs((np.fft.fft2(wave) * bank['psi_hat'][0, l]).sum()) for l in range(4)]
    assert np.argmax(resp) == 0
    resp_t = [abs((np.fft.fft2(wave.T) * bank['psi_hat'][0, l]).sum()) for l in range(4)]
    assert np.argmax(resp_t) == 2


@pytest.mark.parametrize("J", [2, 3])
def test_littlewood_paley_2d(J):
    n, L = 64, 8
    bank = filters.bank_2d(n, n, J, L)
    k = np.arange(n)
    neg = np.ix_((-k) % n, (-k) % n)
    p2 = (np.abs(bank['psi_hat']) ** 2).sum(axis=(0, 1))
    A = np.abs(bank['phi_hat']) ** 2 + 0.5 * (p2 + p2[neg])
    assert abs(A[0, 0] - 1.0) < 1e-12
    assert A.max() < 1.0 + 1e-2
    assert A.min() > 0.05


def test_littlewood_paley_1d():
    n, J, Q = 2048, 6, 8
    bank = filters.bank_1d(n, J, Q)
    p2 = (np.abs(bank['psi1_hat']) ** 2).sum(axis=0)
    A = np.abs(bank['phi_hat']) ** 2 + 0.5 * (p2 + p2[(-np.arange(n)) % n])
    assert abs(A[0] - 1.0) < 1e-12
    assert A.max() < 1.0 + 1e-2
    # the band between the lowest and highest centre frequency is covered
    lo = int(0.75 * math.pi * 2 ** (-(J * Q - 1) / Q) / (2 * math.pi) * n) + 1
    hi = int(0.75 * math.pi / (2 * math.pi) * n)
    assert A[lo:hi].min() > 0.5


def test_parseval_of_first_layer():
    """sum of energies of x*phi and x*psi equals the spectrum-weighted energy of x, and
    is bounded by max A * ||x||^2 (real x)."""
    rng = np.random.default_rng(3)
    n, J, L = 32, 2, 8
    bank = filters.bank_2d(n, n, J, L)
    x = rng.standard_normal((n, n))
    X = np.fft.fft2(x)
    spatial = (np.abs(np.fft.ifft2(X * bank['phi_hat'])) ** 2).sum()
    spatial += sum((np.abs(np.fft.ifft2(X * bank['psi_hat'][j, l])) ** 2).sum()
                   for j in range(J) for l in range(L))
    w = np.abs(bank['phi_hat']) ** 2 + (np.abs(bank['psi_hat']) ** 2).sum(axis=(0, 1))
    spectral = (np.abs(X) ** 2 * w).sum() / (n * n)
    assert abs(spatial - spectral) < 1e-10 * spectral
    k = np.arange(n)
    A = 0.5 * (w + w[np.ix_((-k) % n, (-k) % n)])
    assert spatial <= A.max() * (x * x).sum() * (1 + 1e-12)
