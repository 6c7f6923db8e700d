"""Seeded synthetic inputs for the five benchmark configurations.

This module holds none of the scattering arithmetic: it only draws test signals.
Both the CPU oracle's tests and the GPU harness take their inputs from here, so the
two sides see identical float32 arrays.

The paper runs its examples on natural images (32x32 colour thumbnails, digit
images), larger textures and spoken-digit audio (section 4, "Documentation and
examples"); none of those datasets is available, so each configuration draws a
synthetic stand-in with the same shape and rough statistics:

  0: 2-D J=2 L=8, 4 x 1 x 32 x 32, i.i.d. N(0, 1) pixels
  1: 2-D J=2 L=8, 1024 x 3 x 32 x 32, 8 Gaussian blobs + N(0, 0.1) noise, clipped to [0, 1]
  2: 2-D J=3 L=8, 128 x 3 x 256 x 256, 1/f^2-power Gaussian field, zero mean, unit variance
  3: 2-D J=4 L=8, 32 x 1 x 512 x 512, 4 sinusoidal gratings + 3 step edges + N(0, 0.05) noise
  4: 1-D J=6 Q=8, 64 x 65536, 16 decaying chirps/tones + white noise at 20 dB SNR

Every plane (one image channel or one 1-D signal) has its own random stream, keyed
by (configuration seed, plane number), so the first P planes of a configuration are
the same arrays whatever P is asked for.
"""
import math

import numpy as np

BASE_SEED = 181211214

CONFIGS = (
    dict(name="2d_J2_L8_32x32_b4", dims=2, shape=(32, 32), J=2, LQ=8, batch=4, channels=1),
    dict(name="2d_J2_L8_32x32_b1024x3", dims=2, shape=(32, 32), J=2, LQ=8, batch=1024, channels=3),
    dict(name="2d_J3_L8_256x256_b128x3", dims=2, shape=(256, 256), J=3, LQ=8, batch=128, channels=3),
    dict(name="2d_J4_L8_512x512_b32", dims=2, shape=(512, 512), J=4, LQ=8, batch=32, channels=1),
    dict(name="1d_J6_Q8_65536_b64", dims=1, shape=(65536,), J=6, LQ=8, batch=64, channels=1),
)


def _rng(config, plane):
    return np.random.Generator(np.random.PCG64([BASE_SEED + config, plane]))


def _white(rng, shape):
    return rng.standard_normal(shape)


def _blobs(rng, shape):
    n_r, n_c = shape
    r = np.arange(n_r)[:, None]
    c = np.arange(n_c)[None, :]
    img = np.zeros(shape)
    for _ in range(8):
        cr, cc = rng.uniform(0, n_r), rng.uniform(0, n_c)
        s = rng.uniform(1.5, 5.0)
        a = rng.uniform(0.2, 1.0)
        img += a * np.exp(-((r - cr) ** 2 + (c - cc) ** 2) / (2 * s * s))
    img += 0.1 * rng.standard_normal(shape)
    return np.clip(img, 0.0, 1.0)


def _pink_field(rng, shape):
    n_r, n_c = shape
    w = np.fft.fft2(rng.standard_normal(shape))
    fr = np.fft.fftfreq(n_r)[:, None]
    fc = np.fft.fftfreq(n_c)[None, :]
    rad = np.sqrt(fr * fr + fc * fc)
    rad[0, 0] = 1.0
    w /= rad                      # amplitude 1/f, power 1/f^2
    w[0, 0] = 0.0
    img = np.fft.ifft2(w).real
    img -= img.mean()
    return img / img.std()


def _gratings_edges(rng, shape):
    n_r, n_c = shape
    r = np.arange(n_r)[:, None] * 1.0
    c = np.arange(n_c)[None, :] * 1.0
    img = np.zeros(shape)
    for _ in range(4):
        th = rng.uniform(0, math.pi)
        f = rng.uniform(1 / 64, 1 / 4)
        a = rng.uniform(0.25, 1.0)
        ph = rng.uniform(0, 2 * math.pi)
        img += a * np.sin(2 * math.pi * f * (r * math.cos(th) + c * math.sin(th)) + ph)
    for _ in range(3):
        th = rng.uniform(0, 2 * math.pi)
        off = rng.uniform(0.25, 0.75)
        h = rng.uniform(-1.0, 1.0)
        d = (r - off * n_r) * math.cos(th) + (c - off * n_c) * math.sin(th)
        img += h * (d > 0)
    img += 0.05 * rng.standard_normal(shape)
    return img


def _chirps(rng, shape):
    (n,) = shape
    t = np.arange(n, dtype=np.float64)
    sig = np.zeros(n)
    for i in range(16):
        f0 = math.exp(rng.uniform(math.log(1e-3), math.log(0.3)))
        t0 = rng.uniform(0, 0.8 * n)
        tau = rng.uniform(n / 64, n / 4)
        a = rng.uniform(0.2, 1.0)
        if i % 2 == 0:
            c = 0.0               # pure tone
        else:
            # linear sweep ending within one octave above or below f0, below Nyquist
            f1 = min(f0 * 2.0 ** rng.uniform(-1.0, 1.0), 0.45)
            c = (f1 - f0) / n
        tt = t - t0
        on = tt >= 0
        env = np.where(on, np.exp(-np.where(on, tt, 0.0) / tau), 0.0)
        sig += a * env * np.sin(2 * math.pi * (f0 * tt + 0.5 * c * tt * tt))
    p_sig = np.mean(sig * sig)
    noise = rng.standard_normal(n)
    noise *= math.sqrt(p_sig / 100.0) / noise.std()     # 20 dB SNR
    return sig + noise


_GENERATORS = (_white, _blobs, _pink_field, _gratings_edges, _chirps)


def config(i):
    """The dictionary describing configuration i (0-based); 5 is the 3-D volume case."""
    return dict(VOLUME_CONFIG if i == len(CONFIGS) else CONFIGS[i])


def num_planes(i):
    c = config(i)
    return c["batch"] * c["channels"]


def planes(i, count=None, start=0):
    """float32 array (count, *shape): planes start .. start+count-1 of configuration i.

    Planes are numbered batch-major (plane = image * channels + channel).
    """
    c = config(i)
    if count is None:
        count = num_planes(i) - start
    if c["dims"] == 3:
        return volumes(c["shape"], count, start)
    out = np.empty((count,) + tuple(c["shape"]), dtype=np.float32)
    gen = _GENERATORS[i]
    for p in range(count):
        out[p] = gen(_rng(i, start + p), c["shape"]).astype(np.float32)
    return out


# 3-D stand-in (the paper applies the solid harmonic transform to electronic densities of
# small molecules, section 2 and its 3-D example; no such data set is available): a sum of
# 6 to 20 isotropic Gaussian "atoms" with integer weights 1 .. 8 and widths of 1 to 2.5
# voxels, placed in the central half of a periodic box.
VOLUME_CONFIG = dict(name="3d_J2_L3_64x64x64_b16", dims=3, shape=(64, 64, 64), J=2, LQ=3, batch=16,
                     channels=1)
_VOLUME_STREAM = 5


def _atoms(rng, shape):
    ax = [np.arange(n, dtype=np.float64) for n in shape]
    vol = np.zeros(shape)
    for _ in range(int(rng.integers(6, 21))):
        pos = [rng.uniform(0.25 * n, 0.75 * n) for n in shape]
        w = float(rng.integers(1, 9))
        s = rng.uniform(1.0, 2.5)
        g = []
        for a, p, n in zip(ax, pos, shape):
            d = np.abs(a - p)
            d = np.minimum(d, n - d)                       # periodic distance
            g.append(np.exp(-0.5 * (d / s) ** 2))
        vol += w * g[0][:, None, None] * g[1][None, :, None] * g[2][None, None, :]
    return vol


def volumes(shape, count, start=0):
    """float32 array (count, *shape) of synthetic densities, one random stream per volume."""
    out = np.empty((count,) + tuple(shape), dtype=np.float32)
    for p in range(count):
        out[p] = _atoms(_rng(_VOLUME_STREAM, start + p), tuple(shape)).astype(np.float32)
    return out
