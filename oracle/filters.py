"""Oracle filter banks (fp64, numpy) -- TEST INFRASTRUCTURE, not the product path.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package.  It shares no code with the HIP library: filters are built here in the
*spatial* domain (sampled, periodised, then transformed with numpy's FFT), while
the library evaluates the analytic Fourier transform directly.

What the paper fixes (section 2, "Definition" and "Implementation"): signals live
on a periodic grid, first and second order use Morlet wavelet banks that are
close to analytic, and a lowpass phi_J averages at scale 2^J.  The paper prints no
formula or constant for the filters; the readings used here are

* 2-D Morlet: Gaussian envelope with unit L1 mass, standard deviation sigma along
  the oscillation direction e_theta = (cos theta, sin theta) in (row, col) axes and
  sigma/slant across it, modulated by exp(i xi <u, e_theta>), minus K times the
  envelope with K chosen on the periodised samples so that the wavelet sums to 0.
* constants: sigma_j = 0.8 * 2^j, xi_j = (3 pi / 4) * 2^-j, slant = 4 / L,
  theta_l = pi * l / L, phi_J an isotropic Gaussian of sigma = 0.8 * 2^J, unit mass.
* 1-D first order (Q wavelets per octave): xi_k = (3 pi / 4) 2^(-k/Q),
  sigma_k = 0.3 pi / (xi_k (1 - 2^(-1/Q))) for Q > 1 and 0.8 * 2^k for Q = 1,
  octave j1(k) = floor(k / Q), k = 0 .. J*Q-1; second order is the Q = 1 bank.
* periodisation: the continuous filter is sampled at the integers and summed over
  all shifts by multiples of the grid size (enough wraps that the dropped tail is
  below 1e-40 of the peak).

parity unpinned by the paper: the 1-D Q > 1 construction above is this build's
reading (the paper never mentions Q); it is pinned only to its own closed form.
"""
import math

import numpy as np


def _wrapped_axis(n, reach):
    """Integer coordinates covering `wraps` periods on both sides of [0, n).

    Returns (coords, wraps): coords has length (2*wraps+1)*n and starts at -wraps*n.
    """
    wraps = int(math.ceil(reach / n))
    return np.arange(-wraps * n, (wraps + 1) * n, dtype=np.float64), wraps


def _periodise_1d(values, n):
    """Sum samples taken on a (2W+1)*n long axis over all shifts by n."""
    return values.reshape(-1, n).sum(axis=0)


def _periodise_2d(values, n_r, n_c):
    """Sum samples over all shifts by (n_r, n_c) multiples."""
    a = values.shape[0] // n_r
    b = values.shape[1] // n_c
    return values.reshape(a, n_r, b, n_c).sum(axis=(0, 2))


# ----------------------------------------------------------------------------- 2-D

def gaussian_2d(n_r, n_c, sigma):
    """Periodised isotropic Gaussian with unit continuous mass on an n_r x n_c grid."""
    reach = 14.0 * sigma
    ur, _ = _wrapped_axis(n_r, reach)
    uc, _ = _wrapped_axis(n_c, reach)
    g = np.exp(-(ur[:, None] ** 2 + uc[None, :] ** 2) / (2.0 * sigma * sigma))
    g /= 2.0 * math.pi * sigma * sigma
    return _periodise_2d(g, n_r, n_c)


def morlet_2d(n_r, n_c, sigma, xi, theta, slant):
    """Periodised 2-D Morlet wavelet (complex, spatial domain), zero sum."""
    reach = 14.0 * sigma / min(slant, 1.0)
    ur, _ = _wrapped_axis(n_r, reach)
    uc, _ = _wrapped_axis(n_c, reach)
    ct, st = math.cos(theta), math.sin(theta)
    along = ur[:, None] * ct + uc[None, :] * st
    across = -ur[:, None] * st + uc[None, :] * ct
    env = np.exp(-(along ** 2 + (slant * across) ** 2) / (2.0 * sigma * sigma))
    env *= slant / (2.0 * math.pi * sigma * sigma)
    gabor = env * np.exp(1j * xi * along)
    env_p = _periodise_2d(env, n_r, n_c)
    gabor_p = _periodise_2d(gabor, n_r, n_c)
    k = gabor_p.sum() / env_p.sum()
    return gabor_p - k * env_p


def bank_2d(n_r, n_c, J, L):
    """Spatial and Fourier 2-D filters.

    Returns dict with
      'psi'     : complex array (J, L, n_r, n_c), spatial wavelets
      'phi'     : real array (n_r, n_c), spatial lowpass
      'psi_hat' : complex array (J, L, n_r, n_c) = FFT2(psi)
      'phi_hat' : complex array (n_r, n_c) = FFT2(phi)
    """
    slant = 4.0 / L
    psi = np.empty((J, L, n_r, n_c), dtype=np.complex128)
    for j in range(J):
        for l in range(L):
            psi[j, l] = morlet_2d(n_r, n_c, 0.8 * 2.0 ** j,
                                  0.75 * math.pi * 2.0 ** (-j),
                                  math.pi * l / L, slant)
    phi = gaussian_2d(n_r, n_c, 0.8 * 2.0 ** J)
    return {'psi': psi, 'phi': phi,
            'psi_hat': np.fft.fft2(psi), 'phi_hat': np.fft.fft2(phi)}


# ----------------------------------------------------------------------------- 1-D

def gaussian_1d(n, sigma):
    """Periodised Gaussian with unit continuous mass on n samples."""
    t, _ = _wrapped_axis(n, 14.0 * sigma)
    g = np.exp(-t * t / (2.0 * sigma * sigma)) / (math.sqrt(2.0 * math.pi) * sigma)
    return _periodise_1d(g, n)


def morlet_1d(n, sigma, xi):
    """Periodised 1-D Morlet wavelet (complex), zero sum."""
    t, _ = _wrapped_axis(n, 14.0 * sigma)
    env = np.exp(-t * t / (2.0 * sigma * sigma)) / (math.sqrt(2.0 * math.pi) * sigma)
    gabor = env * np.exp(1j * xi * t)
    env_p = _periodise_1d(env, n)
    gabor_p = _periodise_1d(gabor, n)
    k = gabor_p.sum() / env_p.sum()
    return gabor_p - k * env_p


def params_1d(J, Q):
    """(sigma, xi, octave) lists for the first-order (Q per octave) and second-order
    (one per octave) 1-D banks."""
    first = []
    for k in range(J * Q):
        xi = 0.75 * math.pi * 2.0 ** (-k / Q)
        if Q == 1:
            sigma = 0.8 * 2.0 ** k
        else:
            sigma = 0.3 * math.pi / (xi * (1.0 - 2.0 ** (-1.0 / Q)))
        first.append((sigma, xi, k // Q))
    second = [(0.8 * 2.0 ** j, 0.75 * math.pi * 2.0 ** (-j), j) for j in range(J)]
    return first, second


def bank_1d(n, J, Q):
    """Spatial and Fourier 1-D filters.

    Returns dict with 'psi1' (J*Q, n), 'psi2' (J, n), 'phi' (n,), their FFTs
    'psi1_hat', 'psi2_hat', 'phi_hat', and 'j1' (octave of each first-order
    wavelet), 'j2' (octave of each second-order wavelet).
    """
    first, second = params_1d(J, Q)
    psi1 = np.stack([morlet_1d(n, s, x) for (s, x, _) in first])
    psi2 = np.stack([morlet_1d(n, s, x) for (s, x, _) in second])
    phi = gaussian_1d(n, 0.8 * 2.0 ** J)
    return {'psi1': psi1, 'psi2': psi2, 'phi': phi,
            'psi1_hat': np.fft.fft(psi1), 'psi2_hat': np.fft.fft(psi2),
            'phi_hat': np.fft.fft(phi),
            'j1': [o for (_, _, o) in first], 'j2': [o for (_, _, o) in second]}
