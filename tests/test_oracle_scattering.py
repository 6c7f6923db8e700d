"""Pins for the oracle's scattering cascade (CPU only).

The oracle's FFT-domain cascade is compared against computations that do not use
it: a direct O(N^2) DFT, direct spatial circular convolutions (brute force) of the
spatial filters -- at full resolution for the paper's three defining equations, and
on the subsampled grids with strided filter samples for the subsampled cascade --
plus invariants (shift covariance, transposition symmetry, homogeneity), special
inputs and the closed-form channel count.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import filters, scattering

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ brute force helpers

def _dft_matrix(n):
    k = np.arange(n)
    return np.exp(-2j * np.pi * np.outer(k, k) / n)


def _circ_conv_2d(x, h):
    """(x conv h)[n] = sum_m x[m] h[n - m], indices modulo the grid, by direct summation."""
    out = np.zeros(x.shape, dtype=np.result_type(x, h))
    for mr in range(x.shape[0]):
        for mc in range(x.shape[1]):
            out += x[mr, mc] * np.roll(h, (mr, mc), axis=(0, 1))
    return out


def _circ_conv_1d(x, h):
    out = np.zeros(x.shape, dtype=np.result_type(x, h))
    for m in range(x.shape[0]):
        out += x[m] * np.roll(h, m)
    return out


def test_numpy_fft_is_the_stated_dft():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((8, 16)) + 1j * rng.standard_normal((8, 16))
    ref = _dft_matrix(8) @ x @ _dft_matrix(16).T
    assert np.abs(np.fft.fft2(x) - ref).max() < 1e-12
    back = np.conj(_dft_matrix(8)) @ ref @ np.conj(_dft_matrix(16)).T / (8 * 16)
    assert np.abs(np.fft.ifft2(ref) - back).max() < 1e-13
    assert np.abs(back - x).max() < 1e-13


def test_fold_is_subsampling():
    """sub(F, r) is the spectrum of the signal sampled at multiples of 2^r."""
    rng = np.random.default_rng(1)
    y = rng.standard_normal((16, 32)) + 1j * rng.standard_normal((16, 32))
    got = np.fft.ifft2(scattering.sub(np.fft.fft2(y), 2, (-2, -1)))
    assert np.abs(got - y[::4, ::4]).max() < 1e-13
    z = rng.standard_normal(64)
    got = np.fft.ifft(scattering.sub(np.fft.fft(z), 3, (-1,)))
    assert np.abs(got - z[::8]).max() < 1e-13


# ------------------------------------------------------------------ definition (plain)

@pytest.mark.parametrize("n,J,L", [(8, 1, 4), (16, 2, 2)])
def test_plain_2d_equals_direct_convolution(n, J, L):
    rng = np.random.default_rng(10 + n)
    x = rng.standard_normal((n, n))
    bank = filters.bank_2d(n, n, J, L)
    got = oracle.scattering2d_plain(x, J, L, bank=bank)
    s = 1 << J
    want = [_circ_conv_2d(x, bank['phi'])[::s, ::s]]
    second = []
    for j1 in range(J):
        for t1 in range(L):
            u1 = np.abs(_circ_conv_2d(x, bank['psi'][j1, t1]))
            want.append(_circ_conv_2d(u1, bank['phi'])[::s, ::s])
            for j2 in range(j1 + 1, J):
                for t2 in range(L):
                    v = np.abs(_circ_conv_2d(u1, bank['psi'][j2, t2]))
                    second.append(_circ_conv_2d(v, bank['phi'])[::s, ::s])
    want = np.stack(want + second)
    assert got.shape == want.shape
    assert np.abs(got - want).max() < 1e-12


def test_plain_1d_equals_direct_convolution():
    n, J, Q = 64, 3, 2
    rng = np.random.default_rng(5)
    x = rng.standard_normal(n)
    bank = filters.bank_1d(n, J, Q)
    got = oracle.scattering1d_plain(x, J, Q, bank=bank)
    s = 1 << J
    want = [_circ_conv_1d(x, bank['phi'])[::s]]
    second = []
    for k in range(J * Q):
        u1 = np.abs(_circ_conv_1d(x, bank['psi1'][k]))
        want.append(_circ_conv_1d(u1, bank['phi'])[::s])
        for j2 in range(k // Q + 1, J):
            v = np.abs(_circ_conv_1d(u1, bank['psi2'][j2]))
            second.append(_circ_conv_1d(v, bank['phi'])[::s])
    want = np.stack(want + second)
    assert got.shape == want.shape
    assert np.abs(got - want).max() < 1e-12


# ------------------------------------------------------------------ subsampled cascade

@pytest.mark.parametrize("n_r,n_c,J,L", [(16, 16, 2, 4), (16, 32, 2, 2), (32, 32, 3, 2)])
def test_cascade_2d_equals_spatial_cascade_on_subsampled_grids(n_r, n_c, J, L):
    """Brute force in the spatial domain: each stage convolves on its own (subsampled)
    grid with the spatial filter sampled at that grid's stride and scaled by the
    stride^2 (a Riemann sum of the same continuous convolution), then subsamples."""
    rng = np.random.default_rng(20 + n_r + n_c)
    x = rng.standard_normal((n_r, n_c))
    bank = filters.bank_2d(n_r, n_c, J, L)
    got = oracle.scattering2d(x, J, L, bank=bank)

    def at_res(h, r):
        return h[::1 << r, ::1 << r] * float(4 ** r)

    s = 1 << J
    want = [_circ_conv_2d(x, bank['phi'])[::s, ::s]]
    second = []
    for j1 in range(J):
        for t1 in range(L):
            d1 = 1 << j1
            u1 = np.abs(_circ_conv_2d(x, bank['psi'][j1, t1]))[::d1, ::d1]
            d = 1 << (J - j1)
            want.append(_circ_conv_2d(u1, at_res(bank['phi'], j1))[::d, ::d])
            for j2 in range(j1 + 1, J):
                for t2 in range(L):
                    d = 1 << (j2 - j1)
                    v = np.abs(_circ_conv_2d(u1, at_res(bank['psi'][j2, t2], j1)))[::d, ::d]
                    d = 1 << (J - j2)
                    second.append(_circ_conv_2d(v, at_res(bank['phi'], j2))[::d, ::d])
    want = np.stack(want + second)
    assert got.shape == want.shape == (1 + J * L + L * L * J * (J - 1) // 2, n_r >> J, n_c >> J)
    assert np.abs(got - want).max() < 1e-12


@pytest.mark.parametrize("n,J,Q", [(64, 3, 2), (128, 3, 1)])
def test_cascade_1d_equals_spatial_cascade_on_subsampled_grids(n, J, Q):
    rng = np.random.default_rng(30 + n)
    x = rng.standard_normal(n)
    bank = filters.bank_1d(n, J, Q)
    got = oracle.scattering1d(x, J, Q, bank=bank)

    def at_res(h, r):
        return h[::1 << r] * float(2 ** r)

    want = [_circ_conv_1d(x, bank['phi'])[::1 << J]]
    second = []
    for k in range(J * Q):
        j1 = k // Q
        u1 = np.abs(_circ_conv_1d(x, bank['psi1'][k]))[::1 << j1]
        want.append(_circ_conv_1d(u1, at_res(bank['phi'], j1))[::1 << (J - j1)])
        for j2 in range(j1 + 1, J):
            v = np.abs(_circ_conv_1d(u1, at_res(bank['psi2'][j2], j1)))[::1 << (j2 - j1)]
            second.append(_circ_conv_1d(v, at_res(bank['phi'], j2))[::1 << (J - j2)])
    want = np.stack(want + second)
    assert got.shape == want.shape
    assert np.abs(got - want).max() < 1e-12


def test_first_layer_is_exact():
    """|x conv psi| on the subsampled grid is exact (no approximation before the modulus)."""
    n, J, L = 16, 2, 4
    rng = np.random.default_rng(2)
    x = rng.standard_normal((n, n))
    bank = filters.bank_2d(n, n, J, L)
    u = scattering.first_layer_2d(x, J, L, bank=bank)
    for j1 in range(J):
        for t in range(L):
            full = np.abs(_circ_conv_2d(x, bank['psi'][j1, t]))
            assert np.abs(u[j1][t] - full[::1 << j1, ::1 << j1]).max() < 1e-13


def test_cascade_approximates_the_definition():
    """S0 identical; S1, S2 within a few percent of the per-order maximum."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 64, 64))
    J, L = 3, 8
    bank = filters.bank_2d(64, 64, J, L)
    a = oracle.scattering2d(x, J, L, bank=bank)
    b = oracle.scattering2d_plain(x, J, L, bank=bank)
    order = np.array([r[0] for r in oracle.coeff_index_2d(J, L)])
    assert np.abs(a - b)[:, order == 0].max() < 1e-13
    for o, band in ((1, 0.03), (2, 0.08)):
        rel = np.abs(a - b)[:, order == o].max() / np.abs(b)[:, order == o].max()
        assert 1e-6 < rel < band


# ------------------------------------------------------------------ invariants

def test_shift_covariance_2d():
    """Circular shifts by multiples of 2^J shift the output by whole samples, exactly."""
    rng = np.random.default_rng(11)
    J, L, n = 2, 4, 32
    x = rng.standard_normal((n, n))
    bank = filters.bank_2d(n, n, J, L)
    base = oracle.scattering2d(x, J, L, bank=bank)
    moved = oracle.scattering2d(np.roll(x, (4 * 3, 4 * 5), axis=(0, 1)), J, L, bank=bank)
    assert np.abs(moved - np.roll(base, (3, 5), axis=(-2, -1))).max() < 1e-13
    # a shift that is not a multiple of 2^J is NOT a pure relabelling
    odd = oracle.scattering2d(np.roll(x, 1, axis=0), J, L, bank=bank)
    assert np.abs(odd - base).max() > 1e-3


def test_shift_covariance_1d():
    rng = np.random.default_rng(12)
    J, Q, n = 4, 4, 512
    x = rng.standard_normal(n)
    bank = filters.bank_1d(n, J, Q)
    base = oracle.scattering1d(x, J, Q, bank=bank)
    moved = oracle.scattering1d(np.roll(x, 16 * 7), J, Q, bank=bank)
    assert np.abs(moved - np.roll(base, 7, axis=-1)).max() < 1e-13


def test_transpose_symmetry():
    """S(x^T) is S(x) transposed with every angle index l replaced by (L/2 - l) mod L."""
    rng = np.random.default_rng(13)
    J, L, n = 2, 8, 32
    x = rng.standard_normal((n, n))
    bank = filters.bank_2d(n, n, J, L)
    a = oracle.scattering2d(x, J, L, bank=bank)
    b = oracle.scattering2d(x.T, J, L, bank=bank)
    rows = oracle.coeff_index_2d(J, L)
    pos = {r: i for i, r in enumerate(rows)}

    def mirror(t):
        return (L // 2 - t) % L if t >= 0 else -1

    for i, (o, j1, t1, j2, t2) in enumerate(rows):
        k = pos[(o, j1, mirror(t1), j2, mirror(t2))]
        assert np.abs(b[i] - a[k].T).max() < 1e-13


def test_special_inputs():
    J, L, n = 2, 4, 16
    bank = filters.bank_2d(n, n, J, L)
    order = np.array([r[0] for r in oracle.coeff_index_2d(J, L)])
    const = oracle.scattering2d(np.full((n, n), 2.5), J, L, bank=bank)
    assert np.abs(const[order == 0] - 2.5).max() < 1e-13
    assert np.abs(const[order > 0]).max() < 1e-13
    # unit impulse: S0 samples the periodised lowpass itself
    imp = np.zeros((n, n))
    imp[0, 0] = 1.0
    s = oracle.scattering2d(imp, J, L, bank=bank)
    assert np.abs(s[0] - bank['phi'][::4, ::4]).max() < 1e-14
    u = scattering.first_layer_2d(imp, J, L, bank=bank)
    assert np.abs(u[1][2] - np.abs(bank['psi'][1, 2])[::2, ::2]).max() < 1e-14
    # homogeneity of degree one under real scaling
    rng = np.random.default_rng(14)
    x = rng.standard_normal((n, n))
    a = oracle.scattering2d(x, J, L, bank=bank)
    b = oracle.scattering2d(-3.0 * x, J, L, bank=bank)
    assert np.abs(b[order > 0] - 3.0 * a[order > 0]).max() < 1e-12
    assert np.abs(b[order == 0] + 3.0 * a[order == 0]).max() < 1e-12
    # S1, S2 are averages of non-negative signals by a positive filter
    assert a[order > 0].min() > 0.0


def test_batch_axes_are_independent_planes():
    rng = np.random.default_rng(15)
    x = rng.standard_normal((2, 3, 16, 16))
    bank = filters.bank_2d(16, 16, 2, 4)
    full = oracle.scattering2d(x, 2, 4, bank=bank)
    assert full.shape == (2, 3, 1 + 8 + 16, 4, 4)
    one = oracle.scattering2d(x[1, 2], 2, 4, bank=bank)
    assert np.abs(full[1, 2] - one).max() < 1e-14


# ------------------------------------------------------------------ channel count / order

def _golden_counts():
    rows = []
    with open(os.path.join(GOLDEN, "coeff_counts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(tuple(int(v) for v in line.split()))
    return rows


@pytest.mark.parametrize("dims,J,LQ,max_order,K", _golden_counts())
def test_channel_count(dims, J, LQ, max_order, K):
    if dims == 2:
        rows = oracle.coeff_index_2d(J, LQ, max_order)
    else:
        rows = oracle.coeff_index_1d(J, LQ, max_order)
    assert len(rows) == K == len(set(rows))
    orders = [r[0] for r in rows]
    assert orders == sorted(orders) and orders[0] == 0 and orders.count(0) == 1
    for (o, j1, t1, j2, t2) in rows:
        if o == 2:
            assert j2 > j1


def test_max_order_1_is_a_prefix():
    rng = np.random.default_rng(16)
    x = rng.standard_normal((16, 16))
    bank = filters.bank_2d(16, 16, 2, 4)
    a = oracle.scattering2d(x, 2, 4, max_order=1, bank=bank)
    b = oracle.scattering2d(x, 2, 4, max_order=2, bank=bank)
    assert a.shape[0] == 9 and np.array_equal(a, b[:9])
    y = rng.standard_normal(256)
    b1 = filters.bank_1d(256, 3, 2)
    a = oracle.scattering1d(y, 3, 2, max_order=1, bank=b1)
    b = oracle.scattering1d(y, 3, 2, max_order=2, bank=b1)
    assert a.shape[0] == 7 and np.array_equal(a, b[:7])
