"""Pins of the 3-D solid harmonic scattering oracle.

The paper gives the non-linearity rho = sqrt(sum_m |x conv psi_{j,l,m}|^2) and names solid
harmonic wavelets (section 2, "Implementation") but prints no formula, so the pins are
what mathematics fixes for the reading taken in oracle/harmonic3d.py: the closed-form
Fourier transform of a solid harmonic times a Gaussian (Hecke-Bochner), the addition
theorem of spherical harmonics, covariance with the symmetries of the cubic grid (which
only holds if the sum over m runs over a complete basis of degree l), the l = 0 case
(plain Gaussian filtering), brute-force periodic convolution, and translation covariance.
"""
import numpy as np
import pytest
from scipy import special

from oracle import harmonic3d as h3


def _omega(shape):
    ax = [2 * np.pi * np.fft.fftfreq(n) for n in shape]
    return np.stack(np.meshgrid(*ax, indexing='ij'))


def _analytic_hat(shape, j, l, m, aliases=2):
    """(-i)^l (2^j |w|)^l exp(-(2^j |w|)^2 / 2) Y_l^m(w / |w|), summed over 2 pi aliases."""
    base = _omega(shape)
    out = np.zeros(shape, dtype=np.complex128)
    rng = range(-aliases, aliases + 1)
    for a0 in rng:
        for a1 in rng:
            for a2 in rng:
                w = (base + 2 * np.pi * np.array([a0, a1, a2])[:, None, None, None]) * 2.0 ** j
                r = np.sqrt((w ** 2).sum(axis=0))
                safe = np.where(r > 0, r, 1.0)
                Y = special.sph_harm_y(l, m, np.arccos(np.clip(w[2] / safe, -1, 1)),
                                       np.arctan2(w[1], w[0]))
                if l > 0:
                    Y = np.where(r > 0, Y, 0.0)
                out += (-1j) ** l * r ** l * np.exp(-0.5 * r ** 2) * Y
    return out


@pytest.mark.parametrize("j,l,m", [(0, 0, 0), (0, 1, -1), (0, 2, 1), (1, 1, 0), (1, 2, -2), (1, 3, 3)])
def test_wavelet_spectrum_is_the_hecke_bochner_closed_form(j, l, m):
    shape = (16, 16, 16)
    got = np.fft.fftn(h3.solid_harmonic_wavelet(shape, j, l, m, shifts=3))
    want = _analytic_hat(shape, j, l, m, aliases=3)
    assert np.abs(got - want).max() <= 1e-9 * max(np.abs(want).max(), 1e-3)


def test_sum_over_m_follows_the_addition_theorem():
    shape, j = (16, 16, 16), 1
    w = _omega(shape) * 2.0 ** j
    r2 = (w ** 2).sum(axis=0)
    for l in (0, 1, 2, 3):
        tot = sum(np.abs(np.fft.fftn(h3.solid_harmonic_wavelet(shape, j, l, m))) ** 2
                  for m in range(-l, l + 1))
        want = (2 * l + 1) / (4 * np.pi) * r2 ** l * np.exp(-r2)
        assert np.abs(tot - want).max() <= 2e-3 * want.max()   # aliases at j = 1 are below this


def test_lowpass_has_unit_mass_and_gaussian_spectrum():
    shape, J = (16, 16, 16), 2
    phi = h3.gaussian_lowpass(shape, J, shifts=4)
    assert abs(phi.sum() - 1.0) < 1e-9
    w2 = (_omega(shape) ** 2).sum(axis=0)
    assert np.abs(np.fft.fftn(phi).real - np.exp(-0.5 * w2 * 16.0)).max() < 1e-9


def test_counts_and_shapes():
    x = np.zeros((2, 8, 8, 16))
    S = h3.harmonic_scattering3d(x, 2, 2)
    assert S.shape == (2, 1 + 2 * 3 + 3 * 1, 2, 2, 4)
    assert len(h3.coeff_index_3d(2, 2)) == S.shape[1]
    assert h3.harmonic_scattering3d(x, 2, 2, max_order=1).shape[1] == 7
    assert len(h3.coeff_index_3d(3, 1)) == 1 + 3 * 2 + 2 * 3


def test_covariance_with_grid_rotations_and_reflections():
    """rho sums over a complete basis of degree l, so it commutes with every symmetry of
    the cubic grid; so do the isotropic lowpass and the sampling grid (phase 0)."""
    rng = np.random.default_rng(0)
    n, J, L = 8, 1, 2
    x = rng.standard_normal((n, n, n))
    bank = h3.bank_3d((n, n, n), J, L)
    S = h3.harmonic_scattering3d(x, J, L, bank=bank)
    # quarter turn about the last axis: (a, b, c) -> (-b, a, c) on the periodic grid
    xr = np.roll(np.rot90(x, 1, axes=(0, 1)), 1, axis=0)
    Sr = h3.harmonic_scattering3d(xr, J, L, bank=bank)
    m = n >> J
    want = np.stack([np.roll(np.rot90(S[k], 1, axes=(0, 1)), 1, axis=0) for k in range(S.shape[0])])
    # rotating the samples 2 n maps them to -2 n' = 2 (m - n') mod 2 m: same subgrid
    assert Sr.shape == want.shape and m == 4
    assert np.abs(Sr - want).max() <= 1e-10 * np.abs(S).max()
    # reflection of the first axis
    xf = np.roll(x[::-1], 1, axis=0)
    Sf = h3.harmonic_scattering3d(xf, J, L, bank=bank)
    wantf = np.stack([np.roll(S[k][::-1], 1, axis=0) for k in range(S.shape[0])])
    assert np.abs(Sf - wantf).max() <= 1e-10 * np.abs(S).max()


def test_degree_zero_is_gaussian_filtering():
    rng = np.random.default_rng(1)
    n, J = 8, 2
    x = rng.standard_normal((n, n, n))
    bank = h3.bank_3d((n, n, n), J, 0)
    S = h3.harmonic_scattering3d(x, J, 0, bank=bank)
    # psi_{j,0,0} = Gaussian(std 2^j) / sqrt(4 pi), written out independently
    u = np.stack(np.meshgrid(*[np.fft.fftfreq(n, 1.0 / n)] * 3, indexing='ij'))
    for j in range(J):
        g = np.zeros((n, n, n))
        for s in np.ndindex(7, 7, 7):
            d2 = sum((u[a] + (s[a] - 3) * n) ** 2 for a in range(3))
            g += np.exp(-0.5 * d2 / 4.0 ** j)
        g /= (2 * np.pi) ** 1.5 * 8.0 ** j * np.sqrt(4 * np.pi)
        U = np.abs(np.fft.ifftn(np.fft.fftn(x) * np.fft.fftn(g)))
        want = np.fft.ifftn(np.fft.fftn(U) * bank['phi_hat']).real[::4, ::4, ::4]
        assert np.abs(S[1 + j] - want).max() <= 1e-9 * np.abs(want).max()


def test_first_order_against_brute_force_convolution():
    rng = np.random.default_rng(2)
    n, J, L = 4, 1, 1
    x = rng.standard_normal((n, n, n))
    bank = h3.bank_3d((n, n, n), J, L)
    S = h3.harmonic_scattering3d(x, J, L, bank=bank)
    psi, phi = bank['psi'][0][1], bank['phi']           # j = 0, l = 1: three wavelets

    def pconv(a, b):
        out = np.zeros(a.shape, dtype=np.result_type(a, b))
        for i in np.ndindex(*a.shape):
            for k in np.ndindex(*a.shape):
                out[i] += a[k] * b[tuple((np.array(i) - np.array(k)) % n)]
        return out

    U = np.sqrt(sum(np.abs(pconv(x, psi[m])) ** 2 for m in range(3)))
    want = pconv(U, phi).real[::2, ::2, ::2]
    assert np.abs(S[2] - want).max() <= 1e-10 * np.abs(want).max()


def test_translation_by_the_sampling_step():
    rng = np.random.default_rng(3)
    n, J, L = 8, 1, 1
    x = rng.standard_normal((n, n, n))
    bank = h3.bank_3d((n, n, n), J, L)
    a = h3.harmonic_scattering3d(x, J, L, bank=bank)
    b = h3.harmonic_scattering3d(np.roll(x, 2, axis=1), J, L, bank=bank)
    assert np.abs(b - np.roll(a, 1, axis=2)).max() <= 1e-12 * np.abs(a).max()


def test_oversampled_output_contains_the_default_one():
    """With oversampling o the outputs are read on a grid 2^o times finer; every 2^o-th
    sample of it is the default output, and o >= J gives the lowpassed signals in full."""
    rng = np.random.default_rng(8)
    shape, J, L = (8, 16, 8), 2, 1
    x = rng.standard_normal((2,) + shape)
    bank = h3.bank_3d(shape, J, L)
    base = h3.harmonic_scattering3d(x, J, L, bank=bank)
    for o in (1, 2, 5):
        y = h3.harmonic_scattering3d(x, J, L, bank=bank, oversampling=o)
        st = 1 << min(o, J)
        assert y.shape[-3:] == tuple(s >> (J - min(o, J)) for s in shape)
        assert np.array_equal(y[..., ::st, ::st, ::st], base)


def test_padded_volume_extension_sizes_and_constant():
    from oracle.scattering import padded_size
    rng = np.random.default_rng(9)
    x = rng.standard_normal((1, 5, 7, 6))
    J, L = 1, 1
    y = h3.harmonic_scattering3d_padded(x, J, L)
    assert y.shape == (1, 1 + J * (L + 1), 3, 4, 3)
    # same as transforming numpy's symmetric pad rolled so that the volume starts at 0
    P = [padded_size(k, J) for k in (5, 7, 6)]
    xp = x
    for axis, (k, Pk) in enumerate(zip((5, 7, 6), P)):
        h = (Pk - k + 1) // 2
        xp = np.roll(np.pad(xp, [(0, 0)] * (axis + 1) + [(Pk - k - h, h)] + [(0, 0)] * (2 - axis),
                            mode='symmetric'), -(Pk - k - h), axis=axis + 1)
    want = h3.harmonic_scattering3d(xp, J, L)[..., :3, :4, :3]
    assert np.abs(y - want).max() <= 1e-13
    # a constant volume stays constant under the symmetric extension: S0 equals it
    c = h3.harmonic_scattering3d_padded(np.full((1, 5, 7, 6), 1.5), J, L)
    assert np.abs(c[:, 0] - 1.5).max() <= 1e-12
