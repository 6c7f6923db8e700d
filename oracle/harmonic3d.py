"""Oracle for the 3-D solid harmonic scattering transform (fp64, numpy + scipy) -- TEST
INFRASTRUCTURE, not the product; it shares no code with the HIP library.

Section 2 of the paper: the 3-D transform uses solid harmonic wavelets psi_{j,l,m} (j the
scale, l and m the azimuthal and magnetic quantum numbers) and the non-linearity
rho(x conv psi_{j,l}) = sqrt(sum_m |x conv psi_{j,l,m}|^2); with a lowpass phi_J the three
defining equations are S0 = x conv phi_J, S1 = rho(x conv psi_l1) conv phi_J,
S2 = rho(rho(x conv psi_l1) conv psi_l2) conv phi_J, all convolutions periodic.

The paper prints no wavelet formula, constants, index set or sampling for 3-D -- readings
taken here ("parity unpinned by the paper"; the pins are mathematical identities):

* wavelet: psi_{l,m}(u) = (2 pi)^(-3/2) exp(-|u|^2 / 2) |u|^l Y_l^m(u / |u|) (the solid
  harmonic wavelet of the work the paper cites for it), dilated as
  psi_{j,l,m}(u) = 2^(-3j) psi_{l,m}(2^-j u), j = 0 .. J-1, l = 0 .. L, m = -l .. l;
* lowpass: phi_J a Gaussian of standard deviation 2^J and unit mass;
* both sampled at the integers and periodised (summed over all grid shifts);
* second order: same l, scales j2 > j1 (the "typical" |lambda_2| > |lambda_1| read on
  the scale index); K = 1 + J (L+1) + (L+1) J (J-1) / 2 channels ordered S0, S1 by (j, l),
  S2 by (j1, l, j2);
* everything is evaluated at full resolution and the outputs are read at the samples
  2^J n (the definition taken literally; no intermediate subsampling).
"""
import numpy as np
from scipy import special


def _grid(shape):
    """Signed integer coordinates of the periodic grid, shape (3, N0, N1, N2)."""
    ax = [np.fft.fftfreq(n, d=1.0 / n) for n in shape]
    return np.stack(np.meshgrid(*ax, indexing='ij'))


def _shifts(shape, sigma):
    """Per axis, the number s of grid shifts on each side such that the summed copies cover 10
    standard deviations, (s + 1/2) n >= 10 sigma (beyond that the Gaussian factor is below
    2e-22 of its peak, whatever the polynomial factor here)."""
    return tuple(max(0, int(np.ceil(10.0 * sigma / n - 0.5))) for n in shape)


def _shift_ranges(shifts, shape):
    if np.isscalar(shifts):
        shifts = (int(shifts),) * len(shape)
    return [range(-s, s + 1) for s in shifts]


def solid_harmonic_wavelet(shape, j, l, m, shifts=None):
    """psi_{j,l,m} sampled on the grid and periodised: sum over grid shifts of
    2^(-3j) (2 pi)^(-3/2) exp(-|v|^2 / 2) |v|^l Y_l^m(v / |v|), v = 2^-j u."""
    if shifts is None:
        shifts = _shifts(shape, float(2 ** j))
    base = _grid(shape).astype(np.float64)
    out = np.zeros(shape, dtype=np.complex128)
    r0, r1, r2 = _shift_ranges(shifts, shape)
    for s0 in r0:
        for s1 in r1:
            for s2 in r2:
                u = base + np.array([s0 * shape[0], s1 * shape[1], s2 * shape[2]],
                                    dtype=np.float64)[:, None, None, None]
                v = u / float(2 ** j)
                r = np.sqrt((v ** 2).sum(axis=0))
                safe = np.where(r > 0, r, 1.0)
                polar = np.arccos(np.clip(v[2] / safe, -1.0, 1.0))   # angle from the last axis
                azim = np.arctan2(v[1], v[0])
                Y = special.sph_harm_y(l, m, polar, azim)
                if l > 0:
                    Y = np.where(r > 0, Y, 0.0)      # |v|^l vanishes at the origin anyway
                out += np.exp(-0.5 * r ** 2) * r ** l * Y
    return out * (2.0 * np.pi) ** -1.5 / float(8 ** j)


def gaussian_lowpass(shape, J, shifts=None):
    sigma = float(2 ** J)
    if shifts is None:
        shifts = _shifts(shape, sigma)
    base = _grid(shape).astype(np.float64)
    out = np.zeros(shape)
    r0, r1, r2 = _shift_ranges(shifts, shape)
    for s0 in r0:
        for s1 in r1:
            for s2 in r2:
                u = base + np.array([s0 * shape[0], s1 * shape[1], s2 * shape[2]],
                                    dtype=np.float64)[:, None, None, None]
                out += np.exp(-0.5 * (u ** 2).sum(axis=0) / sigma ** 2)
    return out / ((2.0 * np.pi) ** 1.5 * sigma ** 3)


def bank_3d(shape, J, L):
    """Spatial filters and their DFTs: psi[j][l] has shape (2l+1, N0, N1, N2)."""
    psi = [[np.stack([solid_harmonic_wavelet(shape, j, l, m) for m in range(-l, l + 1)])
            for l in range(L + 1)] for j in range(J)]
    phi = gaussian_lowpass(shape, J)
    return {'psi': psi, 'phi': phi,
            'psi_hat': [[np.fft.fftn(p, axes=(-3, -2, -1)) for p in row] for row in psi],
            'phi_hat': np.fft.fftn(phi)}


def coeff_index_3d(J, L, max_order=2):
    """Rows (order, j1, l, j2); unused fields are -1."""
    rows = [(0, -1, -1, -1)]
    for j in range(J):
        for l in range(L + 1):
            rows.append((1, j, l, -1))
    if max_order >= 2:
        for j1 in range(J):
            for l in range(L + 1):
                for j2 in range(j1 + 1, J):
                    rows.append((2, j1, l, j2))
    return rows


def harmonic_scattering3d(x, J, L, max_order=2, bank=None, oversampling=0):
    """x: (..., N0, N1, N2) real, sides multiples of 2^J.
    Returns (..., K, N0 >> J, N1 >> J, N2 >> J).  oversampling = o: the outputs are read at
    the samples 2^max(J-o, 0) n instead (nothing else is subsampled in this transform)."""
    x = np.asarray(x, dtype=np.float64)
    shape = x.shape[-3:]
    if bank is None:
        bank = bank_3d(shape, J, L)
    psi_hat, phi_hat = bank['psi_hat'], bank['phi_hat']
    ax = (-3, -2, -1)
    s = 1 << max(J - oversampling, 0)
    lead = x.shape[:-3]

    def rho(Fh, wav_hat):
        # sqrt of the sum over m of |F conv psi_m|^2, F given by its DFT
        y = np.fft.ifftn(Fh[..., None, :, :, :] * wav_hat, axes=ax)
        return np.sqrt((np.abs(y) ** 2).sum(axis=-4))

    def lowpass(F):
        return np.fft.ifftn(np.fft.fftn(F, axes=ax) * phi_hat, axes=ax).real[..., ::s, ::s, ::s]

    X = np.fft.fftn(x, axes=ax)
    out = [lowpass(x)]
    s2 = []
    for j1 in range(J):
        for l in range(L + 1):
            U1 = rho(X, psi_hat[j1][l])
            out.append(lowpass(U1))
            if max_order < 2:
                continue
            U1h = np.fft.fftn(U1, axes=ax)
            for j2 in range(j1 + 1, J):
                s2.append(lowpass(rho(U1h, psi_hat[j2][l])))
    out.extend(s2)
    return np.stack(out, axis=len(lead))


def harmonic_scattering3d_padded(x, J, L, max_order=2, oversampling=0):
    """Volumes of any size (the reading taken for signals that are not periodic powers of
    two, as for the 2-D transform): symmetric extension to the periodic grid of
    ``padded_size`` per axis, the periodic transform there, and the output samples that lie
    inside the volume, ceil(N / 2^max(J-o,0)) per axis."""
    from .scattering import pad_index, padded_size
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[-3:]
    P = [padded_size(k, J) for k in n]
    xp = x[..., pad_index(n[0], P[0]), :, :][..., :, pad_index(n[1], P[1]), :][..., pad_index(n[2], P[2])]
    y = harmonic_scattering3d(xp, J, L, max_order, oversampling=oversampling)
    st = 1 << max(J - oversampling, 0)
    o = [-(-k // st) for k in n]
    return y[..., :o[0], :o[1], :o[2]]


def harmonic_scattering3d_backward(x, g, J, L, max_order=2, bank=None, oversampling=0):
    """Gradient of sum(g * harmonic_scattering3d(x)) with respect to x (the paper lists
    differentiability as a feature, section 3, and prints no gradient): the adjoint chain of
    the transform above.  x: (..., N0, N1, N2) real; g: the shape of the transform's output.

    With F real, y_m = F conv psi_m and U = sqrt(sum_m |y_m|^2):
        dU = sum_m Re(conj(y_m) dy_m) / U            (no gradient where U = 0)
        g_F = Re sum_m corr(g_U y_m / U, psi_m)       (corr = adjoint of conv)
    and for S = (F conv phi)[2^J n]: g_F = corr(upsample_zero(g_S), phi)."""
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    shape = x.shape[-3:]
    if bank is None:
        bank = bank_3d(shape, J, L)
    psi_hat, phi_hat = bank['psi_hat'], bank['phi_hat']
    ax = (-3, -2, -1)
    s = 1 << max(J - oversampling, 0)
    lead = x.shape[:-3]
    nl = len(lead)

    def chan(c):
        return g[(slice(None),) * nl + (c,)]

    def lowpass_adj(gs):
        up = np.zeros(lead + shape)
        up[..., ::s, ::s, ::s] = gs
        return np.fft.ifftn(np.fft.fftn(up, axes=ax) * np.conj(phi_hat), axes=ax).real

    def filtered(Fh, wav_hat):
        y = np.fft.ifftn(Fh[..., None, :, :, :] * wav_hat, axes=ax)
        return y, np.sqrt((np.abs(y) ** 2).sum(axis=-4))

    def rho_adj(gU, y, U, wav_hat):
        safe = np.where(U > 0, U, 1.0)
        h = np.where(U > 0, gU / safe, 0.0)[..., None, :, :, :] * y
        return np.fft.ifftn((np.fft.fftn(h, axes=ax) * np.conj(wav_hat)).sum(axis=-4), axes=ax).real

    X = np.fft.fftn(x, axes=ax)
    gx = lowpass_adj(chan(0))
    c1, c2 = 1, 1 + J * (L + 1)
    for j1 in range(J):
        for l in range(L + 1):
            y1, U1 = filtered(X, psi_hat[j1][l])
            gU1 = lowpass_adj(chan(c1))
            c1 += 1
            if max_order >= 2:
                U1h = np.fft.fftn(U1, axes=ax)
                for j2 in range(j1 + 1, J):
                    y2, U2 = filtered(U1h, psi_hat[j2][l])
                    gU1 = gU1 + rho_adj(lowpass_adj(chan(c2)), y2, U2, psi_hat[j2][l])
                    c2 += 1
            gx = gx + rho_adj(gU1, y1, U1, psi_hat[j1][l])
    return gx


def harmonic_scattering3d_padded_backward(x, g, J, L, max_order=2, oversampling=0):
    """Gradient of sum(g * harmonic_scattering3d_padded(x)) with respect to x: zero-extend g
    to the periodic grid's output (adjoint of the crop), run the periodic backward pass on
    the extended volume, and add every extended sample's gradient to the voxel it mirrors
    (adjoint of the symmetric extension)."""
    from .scattering import pad_index, padded_size
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    n = x.shape[-3:]
    P = [padded_size(k, J) for k in n]
    idx = [pad_index(k, Pk) for k, Pk in zip(n, P)]
    xp = x[..., idx[0], :, :][..., :, idx[1], :][..., idx[2]]
    st = max(J - oversampling, 0)
    gp = np.zeros(g.shape[:-3] + tuple(Pk >> st for Pk in P))
    gp[..., :g.shape[-3], :g.shape[-2], :g.shape[-1]] = g
    gxp = harmonic_scattering3d_backward(xp, gp, J, L, max_order, oversampling=oversampling)
    a = np.zeros(x.shape[:-3] + (n[0], P[1], P[2]))
    np.add.at(a, (Ellipsis, idx[0], slice(None), slice(None)), gxp)
    b = np.zeros(x.shape[:-3] + (n[0], n[1], P[2]))
    np.add.at(b, (Ellipsis, idx[1], slice(None)), a)
    out = np.zeros(x.shape)
    np.add.at(out, (Ellipsis, idx[2]), b)
    return out
