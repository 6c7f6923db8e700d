"""Seeded random plan configurations against the oracle (needs a GPU): shapes, depths,
filter counts, orders and oversampling drawn at random within what the constructors
accept, so that schedule decisions taken from the shape (which kernels a plan uses) are
exercised off the beaten sizes.  Every case must either run and match, or be refused at
plan creation with a shape / argument status -- never fail at run time."""
import numpy as np
import pytest

import oracle
import paper_1812_11214_amd as scat
from oracle import harmonic3d as o3

from parity import TOL, gpu_forward, order_of_channels, per_order_errors

pytestmark = pytest.mark.gpu


def _run(shape, J, LQ, mo, o, x, want_fn):
    try:
        plan = scat.Scattering(shape, J, LQ, mo, oversampling=o)
    except scat.ScatError as e:
        assert e.status in (1, 2), e
        return None
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    errs = per_order_errors(got, want_fn(), order_of_channels(rows), x)
    assert max(errs.values()) <= TOL, (shape, J, LQ, mo, o, errs)
    return errs


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_2d(seed):
    rng = np.random.default_rng(1000 + seed)
    accepted = 0
    for _ in range(10):
        lr, lc = int(rng.integers(2, 9)), int(rng.integers(2, 9))
        J = int(rng.integers(1, min(lr, lc, 5) + 1))
        L = int(rng.integers(1, 9))
        mo = int(rng.integers(1, 3))
        o = int(rng.choice([0, 0, 0, 1]))
        shape = (1 << lr, 1 << lc)
        x = rng.standard_normal((2,) + shape).astype(np.float32)
        accepted += _run(shape, J, L, mo, o, x,
                         lambda: oracle.scattering2d(x, J, L, mo, oversampling=o)) is not None
    # every drawn plan is within the documented limits: a sweep that refuses them tests nothing
    assert accepted >= 8, accepted


@pytest.mark.parametrize("seed", [1, 2])
def test_random_1d(seed):
    rng = np.random.default_rng(2000 + seed)
    accepted = 0
    for _ in range(10):
        lg = int(rng.integers(4, 16))
        n = 1 << lg
        J = int(rng.integers(1, min(lg, 8) + 1))
        Q = int(rng.integers(1, 9))
        mo = int(rng.integers(1, 3))
        o = int(rng.choice([0, 0, 1, 2]))
        x = rng.standard_normal((3, n)).astype(np.float32)
        accepted += _run((n,), J, Q, mo, o, x,
                         lambda: oracle.scattering1d(x, J, Q, mo, oversampling=o)) is not None
    assert accepted >= 8, accepted


@pytest.mark.parametrize("seed", [1, 2])
def test_random_3d(seed):
    rng = np.random.default_rng(3000 + seed)
    accepted = tried = 0
    for _ in range(6):
        l = [int(rng.integers(2, 7)) for _ in range(3)]
        if sum(l) > 16:
            continue
        tried += 1
        J = int(rng.integers(1, min(min(l), 3) + 1))
        L = int(rng.integers(0, 4))
        mo = int(rng.integers(1, 3))
        o = int(rng.choice([0, 0, 1]))
        shape = tuple(1 << v for v in l)
        x = rng.standard_normal((2,) + shape).astype(np.float32)
        accepted += _run(shape, J, L, mo, o, x,
                         lambda: o3.harmonic_scattering3d(x, J, L, mo, oversampling=o)) is not None
    assert tried >= 2 and accepted >= tried - 1, (tried, accepted)
