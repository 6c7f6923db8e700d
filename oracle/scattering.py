"""Oracle scattering transforms (fp64, numpy) -- TEST INFRASTRUCTURE, not the product.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
package; it shares no code with the HIP library.

Two families of functions:

* ``scattering2d`` / ``scattering1d`` -- the cascade as the paper's section 2
  ("Implementation") describes it: every periodic convolution is a product in the
  Fourier domain, every signal produced by filtering (and modulus) is downsampled.
  The paper gives no schedule; the reading taken is: after a wavelet of octave j the
  signal lives on the grid subsampled by 2^j (sample phase 0), after phi_J on the
  grid subsampled by 2^J.  A filter applied to a signal that already lives at
  resolution r is the full-resolution filter with its Fourier blocks summed
  (``fold``), i.e. the spatial filter sampled at stride 2^r and rescaled.
  This is an approximation of the definition for S1 and S2 (the modulus aliases a
  little when subsampled) and exact for S0 and for the first wavelet-modulus layer.

* ``scattering2d_plain`` / ``scattering1d_plain`` -- the paper's three equations of
  section 2 ("Definition") taken literally: every convolution at full resolution,
  the result sampled at multiples of 2^J.  Used as a loose cross-check only.

Second-order index set: the "typical" choice of section 2, |lambda_2| > |lambda_1|,
read as octave j2 strictly greater than octave j1, all orientations.

Output channel order: S0; then S1 ordered by (j1, theta1) -- in 1-D by wavelet
index k; then S2 ordered by (j1, theta1, j2, theta2) -- in 1-D by (k, j2).
FFT convention: forward sum x[n] exp(-2 pi i k n / N), inverse carries 1/N per axis.
"""
import numpy as np

from . import filters


# ------------------------------------------------------------------ index tables

def coeff_index_2d(J, L, max_order=2):
    """Rows (order, j1, theta1, j2, theta2); unused fields are -1."""
    rows = [(0, -1, -1, -1, -1)]
    for j1 in range(J):
        for t1 in range(L):
            rows.append((1, j1, t1, -1, -1))
    if max_order >= 2:
        for j1 in range(J):
            for t1 in range(L):
                for j2 in range(j1 + 1, J):
                    for t2 in range(L):
                        rows.append((2, j1, t1, j2, t2))
    return rows


def coeff_index_1d(J, Q, max_order=2):
    """Rows (order, j1, k1, j2, k2): k1 = first-order wavelet index (octave j1 =
    k1 // Q), k2 = second-order wavelet index (= its octave j2).  Unused = -1."""
    rows = [(0, -1, -1, -1, -1)]
    for k in range(J * Q):
        rows.append((1, k // Q, k, -1, -1))
    if max_order >= 2:
        for k in range(J * Q):
            for j2 in range(k // Q + 1, J):
                rows.append((2, k // Q, k, j2, j2))
    return rows


# ------------------------------------------------------------------ fold / sub

def fold(F, r, axes):
    """Sum the 2^r Fourier blocks along each of `axes` (the last len(axes) axes).

    fold(F)[k] = sum_a F[k + a*M], M = N / 2^r.  No normalisation.
    """
    out = F
    for ax in axes:
        ax = ax % out.ndim
        n = out.shape[ax]
        shp = out.shape[:ax] + (1 << r, n >> r) + out.shape[ax + 1:]
        out = out.reshape(shp).sum(axis=ax)
    return out


def sub(F, r, axes):
    """Fourier transform of the signal subsampled by 2^r at phase 0 along `axes`."""
    return fold(F, r, axes) / float(1 << (r * len(axes)))


# ------------------------------------------------------------------ 2-D cascade

def scattering2d(x, J, L, max_order=2, bank=None, oversampling=0):
    """Order-<=2 scattering of real images, Fourier-domain cascade with subsampling.

    x: array (..., N_r, N_c), N_r and N_c multiples of 2^J.
    Returns float64 array (..., K, N_r >> rJ, N_c >> rJ), rJ = max(J - oversampling, 0).

    oversampling = o keeps every signal 2^o times finer than the default schedule: after
    a wavelet of octave j the grid is subsampled by 2^max(j - o, 0), the output by
    2^max(J - o, 0).  With o >= J nothing is subsampled and the result, read at the
    samples 2^J n, is the paper's definition itself (``scattering2d_plain``).
    """
    x = np.asarray(x, dtype=np.float64)
    n_r, n_c = x.shape[-2:]
    if bank is None:
        bank = filters.bank_2d(n_r, n_c, J, L)
    psi_hat, phi_hat = bank['psi_hat'], bank['phi_hat']
    ax = (-2, -1)
    lead = x.shape[:-2]
    res = lambda j: max(j - oversampling, 0)   # log2 of the subsampling after octave j
    rJ = res(J)
    X = np.fft.fft2(x)
    out = []
    # S0 = (x conv phi_J) sampled at 2^rJ n
    out.append(np.fft.ifft2(sub(X * phi_hat, rJ, ax)).real)
    s2 = []
    for j1 in range(J):
        r1 = res(j1)
        phi_r1 = fold(phi_hat, r1, ax)
        for t1 in range(L):
            U1 = np.abs(np.fft.ifft2(sub(X * psi_hat[j1, t1], r1, ax)))
            U1h = np.fft.fft2(U1)
            out.append(np.fft.ifft2(sub(U1h * phi_r1, rJ - r1, ax)).real)
            if max_order < 2:
                continue
            for j2 in range(j1 + 1, J):
                r2 = res(j2)
                phi_r2 = fold(phi_hat, r2, ax)
                for t2 in range(L):
                    psi_r = fold(psi_hat[j2, t2], r1, ax)
                    V = np.abs(np.fft.ifft2(sub(U1h * psi_r, r2 - r1, ax)))
                    Vh = np.fft.fft2(V)
                    s2.append(np.fft.ifft2(sub(Vh * phi_r2, rJ - r2, ax)).real)
    out.extend(s2)
    return np.stack(out, axis=len(lead))


def tile(G, r, axes):
    """Adjoint of ``fold``: repeat G 2^r times along each of `axes` (periodic extension of
    a spectrum of M points to N = 2^r M points)."""
    reps = [1] * G.ndim
    for ax in axes:
        reps[ax % G.ndim] = 1 << r
    return np.tile(G, reps)


def scattering2d_backward(x, g, J, L, max_order=2, bank=None, oversampling=0):
    """Gradient of sum(g * scattering2d(x)) with respect to x (vector-Jacobian product).

    The cascade is a chain of real-linear maps and complex moduli, so its transpose is the
    chain of adjoints in reverse order (section 3 of the paper relies on this chain being
    differentiable; it gives no formulas).  With the real inner product Re<a, b>:
    adjoint of fft2 = n * ifft2, of ifft2 = fft2 / n (n = number of grid points), of
    ``fold`` = ``tile``, of the product with a real filter = the same product, of taking
    the real part = inclusion, and d|y| = Re(conj(y) dy) / |y|, hence g_y = g_U * y / |y|
    (taken as 0 where y = 0).

    x: (..., N_r, N_c) real; g: (..., K, N_r >> rJ, N_c >> rJ) real with rJ = max(J -
    oversampling, 0) as in ``scattering2d``.  Returns (..., N_r, N_c).
    """
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    n_r, n_c = x.shape[-2:]
    if bank is None:
        bank = filters.bank_2d(n_r, n_c, J, L)
    psi_hat, phi_hat = bank['psi_hat'], bank['phi_hat']
    ax = (-2, -1)
    res = lambda j: max(j - oversampling, 0)
    rJ = res(J)
    m_pts = float((n_r >> rJ) * (n_c >> rJ))

    def unit(y):
        a = np.abs(y)
        return np.where(a > 0, y / np.where(a > 0, a, 1.0), 0.0)

    def lowpass_adjoint(gs, phi_r, r):
        # S = Re ifft2(sub(Z^ * phi, r)):  g_Z^ = tile(fft2(g_S) / m) / 4^r * phi
        return tile(np.fft.fft2(gs) / m_pts, r, ax) / float(4 ** r) * phi_r

    X = np.fft.fft2(x)
    gX = lowpass_adjoint(g[..., 0, :, :], phi_hat, rJ)
    c1 = 1
    c2 = 1 + J * L
    for j1 in range(J):
        r1 = res(j1)
        phi_j1 = fold(phi_hat, r1, ax)
        n1 = float((n_r >> r1) * (n_c >> r1))
        for t1 in range(L):
            y1 = np.fft.ifft2(sub(X * psi_hat[j1, t1], r1, ax))
            U1h = np.fft.fft2(np.abs(y1))
            gU1h = lowpass_adjoint(g[..., c1, :, :], phi_j1, rJ - r1)
            c1 += 1
            if max_order >= 2:
                for j2 in range(j1 + 1, J):
                    r2 = res(j2)
                    phi_j2 = fold(phi_hat, r2, ax)
                    n2 = float((n_r >> r2) * (n_c >> r2))
                    for t2 in range(L):
                        psi_r = fold(psi_hat[j2, t2], r1, ax)
                        y2 = np.fft.ifft2(sub(U1h * psi_r, r2 - r1, ax))
                        gVh = lowpass_adjoint(g[..., c2, :, :], phi_j2, rJ - r2)
                        c2 += 1
                        gV = (np.fft.ifft2(gVh) * n2).real
                        gY2 = np.fft.fft2(gV * unit(y2)) / n2
                        gU1h = gU1h + tile(gY2, r2 - r1, ax) / float(4 ** (r2 - r1)) * psi_r
            gU1 = (np.fft.ifft2(gU1h) * n1).real
            gY1 = np.fft.fft2(gU1 * unit(y1)) / n1
            gX = gX + tile(gY1, r1, ax) / float(4 ** r1) * psi_hat[j1, t1]
    return (np.fft.ifft2(gX) * float(n_r * n_c)).real


# ------------------------------------------------------------------ signals of any size

def padded_size(n, J):
    """Smallest power of two >= n + 2^J: the periodic grid a signal of n samples is
    extended to (at least 2^J samples of margin in total)."""
    p = 1
    while p < n + (1 << J):
        p *= 2
    return p


def pad_index(n, P):
    """Source index of every sample of the period-P symmetric extension of n samples.

    The signal sits at 0..n-1.  The margin n..P-1 is filled by half-sample-symmetric
    reflection: its first ceil((P-n)/2) samples continue past the right edge
    (x[n-1], x[n-2], ...), the rest lead up to the left edge of the next period
    (..., x[1], x[0]), so the periodic signal has no jump at either edge.  Reflection
    repeats with period 2n when the margin is longer than the signal."""
    h = (P - n + 1) // 2
    i = np.arange(P)
    v = np.where(i < n + h, i, i - P)          # virtual position on the infinite extension
    v = np.mod(v, 2 * n)
    return np.where(v < n, v, 2 * n - 1 - v)


def scattering2d_padded(x, J, L, max_order=2):
    """Scattering of images of any size (the paper's usage example applies the transform
    to a 28 x 28 array and does not say how; reading taken): extend symmetrically to the
    periodic grid of ``padded_size`` per axis, run the periodic cascade there, keep the
    output samples 2^J n that lie inside the image, n < ceil(N / 2^J) per axis."""
    x = np.asarray(x, dtype=np.float64)
    n_r, n_c = x.shape[-2:]
    P_r, P_c = padded_size(n_r, J), padded_size(n_c, J)
    xp = x[..., pad_index(n_r, P_r), :][..., :, pad_index(n_c, P_c)]
    S = scattering2d(xp, J, L, max_order)
    return S[..., :-(-n_r >> J), :-(-n_c >> J)]


def scattering2d_padded_backward(x, g, J, L, max_order=2):
    """Gradient of sum(g * scattering2d_padded(x)) with respect to x: zero-extend g to the
    periodic grid's output (adjoint of the crop), run the periodic backward pass on the
    extended image, and add every extended sample's gradient to the pixel it mirrors
    (adjoint of the symmetric extension)."""
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    n_r, n_c = x.shape[-2:]
    P_r, P_c = padded_size(n_r, J), padded_size(n_c, J)
    ir, ic = pad_index(n_r, P_r), pad_index(n_c, P_c)
    xp = x[..., ir, :][..., :, ic]
    gp = np.zeros(g.shape[:-2] + (P_r >> J, P_c >> J))
    gp[..., :g.shape[-2], :g.shape[-1]] = g
    gxp = scattering2d_backward(xp, gp, J, L, max_order)
    rows = np.zeros(x.shape[:-2] + (n_r, P_c))
    np.add.at(rows, (Ellipsis, ir, slice(None)), gxp)
    out = np.zeros(x.shape)
    np.add.at(out, (Ellipsis, ic), rows)
    return out


def scattering1d_padded(x, J, Q, max_order=2):
    """1-D counterpart of ``scattering2d_padded``."""
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[-1]
    P = padded_size(n, J)
    S = scattering1d(x[..., pad_index(n, P)], J, Q, max_order)
    return S[..., :-(-n >> J)]


def scattering1d_padded_backward(x, g, J, Q, max_order=2):
    """1-D counterpart of ``scattering2d_padded_backward``."""
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    n = x.shape[-1]
    P = padded_size(n, J)
    idx = pad_index(n, P)
    gp = np.zeros(g.shape[:-1] + (P >> J,))
    gp[..., :g.shape[-1]] = g
    gxp = scattering1d_backward(x[..., idx], gp, J, Q, max_order)
    out = np.zeros(x.shape)
    np.add.at(out, (Ellipsis, idx), gxp)
    return out


def scattering2d_plain(x, J, L, max_order=2, bank=None):
    """The three defining equations at full resolution, sampled at 2^J n."""
    x = np.asarray(x, dtype=np.float64)
    n_r, n_c = x.shape[-2:]
    if bank is None:
        bank = filters.bank_2d(n_r, n_c, J, L)
    psi_hat, phi_hat = bank['psi_hat'], bank['phi_hat']
    lead = x.shape[:-2]
    s = 1 << J
    X = np.fft.fft2(x)
    out = [np.fft.ifft2(X * phi_hat).real[..., ::s, ::s]]
    s2 = []
    for j1 in range(J):
        for t1 in range(L):
            U1 = np.abs(np.fft.ifft2(X * psi_hat[j1, t1]))
            U1h = np.fft.fft2(U1)
            out.append(np.fft.ifft2(U1h * phi_hat).real[..., ::s, ::s])
            if max_order < 2:
                continue
            for j2 in range(j1 + 1, J):
                for t2 in range(L):
                    V = np.abs(np.fft.ifft2(U1h * psi_hat[j2, t2]))
                    s2.append(np.fft.ifft2(np.fft.fft2(V) * phi_hat).real[..., ::s, ::s])
    out.extend(s2)
    return np.stack(out, axis=len(lead))


# ------------------------------------------------------------------ 1-D cascade

def scattering1d(x, J, Q, max_order=2, bank=None, oversampling=0):
    """Order-<=2 scattering of real 1-D signals, Fourier-domain cascade.

    x: array (..., N), N a multiple of 2^J.  Returns float64 (..., K, N >> rJ) with
    rJ = max(J - oversampling, 0); see ``scattering2d`` for `oversampling`.
    """
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[-1]
    if bank is None:
        bank = filters.bank_1d(n, J, Q)
    psi1_hat, psi2_hat, phi_hat = bank['psi1_hat'], bank['psi2_hat'], bank['phi_hat']
    ax = (-1,)
    lead = x.shape[:-1]
    res = lambda j: max(j - oversampling, 0)
    rJ = res(J)
    X = np.fft.fft(x)
    out = [np.fft.ifft(sub(X * phi_hat, rJ, ax)).real]
    s2 = []
    for k in range(J * Q):
        j1 = bank['j1'][k]
        r1 = res(j1)
        U1 = np.abs(np.fft.ifft(sub(X * psi1_hat[k], r1, ax)))
        U1h = np.fft.fft(U1)
        out.append(np.fft.ifft(sub(U1h * fold(phi_hat, r1, ax), rJ - r1, ax)).real)
        if max_order < 2:
            continue
        for j2 in range(j1 + 1, J):
            r2 = res(j2)
            psi_r = fold(psi2_hat[j2], r1, ax)
            V = np.abs(np.fft.ifft(sub(U1h * psi_r, r2 - r1, ax)))
            Vh = np.fft.fft(V)
            s2.append(np.fft.ifft(sub(Vh * fold(phi_hat, r2, ax), rJ - r2, ax)).real)
    out.extend(s2)
    return np.stack(out, axis=len(lead))


def scattering1d_backward(x, g, J, Q, max_order=2, bank=None, oversampling=0):
    """Gradient of sum(g * scattering1d(x)) with respect to x; the 1-D counterpart of
    ``scattering2d_backward`` (same adjoints, one axis).

    x: (..., N) real; g: (..., K, N >> rJ) real.  Returns (..., N)."""
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    n = x.shape[-1]
    if bank is None:
        bank = filters.bank_1d(n, J, Q)
    psi1_hat, psi2_hat, phi_hat = bank['psi1_hat'], bank['psi2_hat'], bank['phi_hat']
    ax = (-1,)
    res = lambda j: max(j - oversampling, 0)
    rJ = res(J)
    m_pts = float(n >> rJ)

    def unit(y):
        a = np.abs(y)
        return np.where(a > 0, y / np.where(a > 0, a, 1.0), 0.0)

    def lowpass_adjoint(gs, phi_r, r):
        return tile(np.fft.fft(gs) / m_pts, r, ax) / float(2 ** r) * phi_r

    X = np.fft.fft(x)
    gX = lowpass_adjoint(g[..., 0, :], phi_hat, rJ)
    c1 = 1
    c2 = 1 + J * Q
    for k in range(J * Q):
        j1 = bank['j1'][k]
        r1 = res(j1)
        n1 = float(n >> r1)
        y1 = np.fft.ifft(sub(X * psi1_hat[k], r1, ax))
        U1h = np.fft.fft(np.abs(y1))
        gU1h = lowpass_adjoint(g[..., c1, :], fold(phi_hat, r1, ax), rJ - r1)
        c1 += 1
        if max_order >= 2:
            for j2 in range(j1 + 1, J):
                r2 = res(j2)
                n2 = float(n >> r2)
                psi_r = fold(psi2_hat[j2], r1, ax)
                y2 = np.fft.ifft(sub(U1h * psi_r, r2 - r1, ax))
                gVh = lowpass_adjoint(g[..., c2, :], fold(phi_hat, r2, ax), rJ - r2)
                c2 += 1
                gV = (np.fft.ifft(gVh) * n2).real
                gY2 = np.fft.fft(gV * unit(y2)) / n2
                gU1h = gU1h + tile(gY2, r2 - r1, ax) / float(2 ** (r2 - r1)) * psi_r
        gU1 = (np.fft.ifft(gU1h) * n1).real
        gY1 = np.fft.fft(gU1 * unit(y1)) / n1
        gX = gX + tile(gY1, r1, ax) / float(2 ** r1) * psi1_hat[k]
    return (np.fft.ifft(gX) * float(n)).real


def scattering1d_plain(x, J, Q, max_order=2, bank=None):
    """The three defining equations at full resolution, sampled at 2^J n (1-D)."""
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[-1]
    if bank is None:
        bank = filters.bank_1d(n, J, Q)
    psi1_hat, psi2_hat, phi_hat = bank['psi1_hat'], bank['psi2_hat'], bank['phi_hat']
    lead = x.shape[:-1]
    s = 1 << J
    X = np.fft.fft(x)
    out = [np.fft.ifft(X * phi_hat).real[..., ::s]]
    s2 = []
    for k in range(J * Q):
        j1 = bank['j1'][k]
        U1 = np.abs(np.fft.ifft(X * psi1_hat[k]))
        U1h = np.fft.fft(U1)
        out.append(np.fft.ifft(U1h * phi_hat).real[..., ::s])
        if max_order < 2:
            continue
        for j2 in range(j1 + 1, J):
            V = np.abs(np.fft.ifft(U1h * psi2_hat[j2]))
            s2.append(np.fft.ifft(np.fft.fft(V) * phi_hat).real[..., ::s])
    out.extend(s2)
    return np.stack(out, axis=len(lead))


def first_layer_2d(x, J, L, bank=None):
    """U1[j1, theta1] = |x conv psi| on the grid subsampled by 2^j1 (exact, no
    approximation involved).  Returns a list over j1 of arrays (..., L, M, M)."""
    x = np.asarray(x, dtype=np.float64)
    n_r, n_c = x.shape[-2:]
    if bank is None:
        bank = filters.bank_2d(n_r, n_c, J, L)
    X = np.fft.fft2(x)
    res = []
    for j1 in range(J):
        res.append(np.stack(
            [np.abs(np.fft.ifft2(sub(X * bank['psi_hat'][j1, t], j1, (-2, -1))))
             for t in range(L)], axis=x.ndim - 2))
    return res
