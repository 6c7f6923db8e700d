"""The seeded input generators: shapes, dtype, determinism, stated statistics."""
import numpy as np

from paper_1812_11214_amd import workloads


def test_shapes_and_determinism():
    for i in range(5):
        c = workloads.config(i)
        a = workloads.planes(i, 3)
        b = workloads.planes(i, 2, start=1)
        assert a.dtype == np.float32 and a.shape == (3,) + tuple(c["shape"])
        assert np.array_equal(a[1:], b)            # plane p does not depend on the count
        assert np.isfinite(a).all()
        assert not np.array_equal(a[0], a[1])
    assert [workloads.num_planes(i) for i in range(5)] == [4, 3072, 384, 32, 64]


def test_stated_statistics():
    x = workloads.planes(0, 4)
    assert abs(x.mean()) < 0.1 and abs(x.std() - 1.0) < 0.1
    x = workloads.planes(1, 6)
    assert x.min() >= 0.0 and x.max() <= 1.0 and x.std() > 0.05
    x = workloads.planes(2, 2).astype(np.float64)
    assert np.abs(x.mean(axis=(1, 2))).max() < 1e-6
    assert np.abs(x.std(axis=(1, 2)) - 1.0).max() < 1e-5
    # power falls roughly as 1/f^2: low band holds far more energy than high band
    P = np.abs(np.fft.fft2(x[0])) ** 2
    assert P[1:4, 1:4].mean() > 100 * P[60:120, 60:120].mean()
    x = workloads.planes(4, 1).astype(np.float64)
    assert x.shape == (1, 65536) and x.std() > 0.01
