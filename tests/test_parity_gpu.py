"""Parity of the HIP library against the fp64 oracle, element by element (needs a GPU)."""
import numpy as np
import pytest

import oracle
import paper_1812_11214_amd as scat
from paper_1812_11214_amd import workloads

from parity import TOL, gpu_forward, order_of_channels, per_order_errors

pytestmark = pytest.mark.gpu


def _check_2d(x, J, L, max_order=2, bank=None):
    shape = x.shape[-2:]
    plan = scat.Scattering(shape, J, L, max_order)
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    assert rows == oracle.coeff_index_2d(J, L, max_order)
    want = oracle.scattering2d(x, J, L, max_order, bank=bank)
    errs = per_order_errors(got, want, order_of_channels(rows), x)
    print("2d", shape, J, L, max_order, errs, flush=True)
    assert max(errs.values()) <= TOL, errs
    return got, want


def _check_1d(x, J, Q, max_order=2):
    plan = scat.Scattering(x.shape[-1:], J, Q, max_order)
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    assert rows == oracle.coeff_index_1d(J, Q, max_order)
    want = oracle.scattering1d(x, J, Q, max_order)
    errs = per_order_errors(got, want, order_of_channels(rows), x)
    print("1d", x.shape, J, Q, max_order, errs, flush=True)
    assert max(errs.values()) <= TOL, errs
    return got, want


def test_config0_white_noise_32x32():
    c = workloads.config(0)
    _check_2d(workloads.planes(0), c["J"], c["LQ"])


def test_config1_blobs_prefix():
    c = workloads.config(1)
    _check_2d(workloads.planes(1, 96), c["J"], c["LQ"])


@pytest.mark.parametrize("shape,J,L,max_order", [
    ((8, 8), 1, 4, 2), ((16, 16), 2, 3, 2), ((64, 64), 3, 8, 2), ((64, 64), 3, 8, 1),
    ((32, 128), 3, 4, 2), ((128, 32), 2, 6, 2), ((16, 16), 4, 2, 2), ((4, 4), 2, 1, 2),
    ((128, 128), 4, 2, 2),
])
def test_2d_shapes(shape, J, L, max_order):
    rng = np.random.default_rng(hash((shape, J, L)) % 2**32)
    x = rng.standard_normal((5,) + shape).astype(np.float32)
    _check_2d(x, J, L, max_order)


def test_2d_edge_inputs():
    rng = np.random.default_rng(5)
    x = np.zeros((4, 32, 32), dtype=np.float32)
    x[0] = 3.25                       # constant: S1 = S2 = 0
    x[1, 0, 0] = 1.0                  # impulse
    x[2] = rng.standard_normal((32, 32)) * 1e4
    x[3] = rng.standard_normal((32, 32)) * 1e-4
    _check_2d(x, 2, 8)


def test_config2_256x256_sample():
    c = workloads.config(2)
    x = workloads.planes(2, 3)
    _check_2d(x, c["J"], c["LQ"])


def test_config3_512x512_sample():
    c = workloads.config(3)
    x = workloads.planes(3, 1)
    _check_2d(x, c["J"], c["LQ"])


@pytest.mark.parametrize("n,J,Q,max_order", [
    (64, 3, 2, 2), (256, 4, 1, 2), (1024, 5, 8, 2), (4096, 6, 8, 1), (8, 3, 1, 2), (2048, 2, 3, 2),
])
def test_1d_shapes(n, J, Q, max_order):
    rng = np.random.default_rng(n + J + Q)
    x = rng.standard_normal((3, n)).astype(np.float32)
    _check_1d(x, J, Q, max_order)


def test_config4_1d_sample():
    c = workloads.config(4)
    x = workloads.planes(4, 2)
    _check_1d(x, c["J"], c["LQ"])


def test_batch_and_repeatability():
    """Results do not depend on batch size or call order; leading dims are planes."""
    import torch
    x = workloads.planes(0, 4)
    plan = scat.Scattering((32, 32), 2, 8)
    try:
        a = gpu_forward(plan, x)
        b = gpu_forward(plan, x[1:2])
        c = gpu_forward(plan, x)
        assert np.array_equal(a, c)
        assert np.array_equal(a[1:2], b)
        y = plan.forward(torch.from_numpy(x.reshape(2, 2, 32, 32)).cuda())
        assert tuple(y.shape) == (2, 2, 81, 8, 8)
        assert np.array_equal(y.cpu().numpy().reshape(4, 81, 8, 8), a)
        empty = plan.forward(torch.empty((0, 32, 32), dtype=torch.float32, device="cuda"))
        assert tuple(empty.shape) == (0, 81, 8, 8)
    finally:
        plan.close()
