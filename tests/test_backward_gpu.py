"""Parity of the HIP backward pass with the fp64 oracle's chain of adjoints.

Tolerance.  The gradient passes through y / |y| at every modulus; where |y| is within
fp32 rounding of zero the phase of the fp32 y is noise, so isolated samples of g_y can
differ from fp64 by O(|g_U|).  Their effect on the final gradient is damped by the
filters that follow: measured errors are 1e-7 ... 8e-6 of the gradient's largest entry.
The bar is the forward pass's: 1e-4 of max |grad| per plane (and 1e-5 in relative L2
norm); any structural mistake (wrong channel, missing term, wrong sign or scale) gives
errors of order 1.
"""
import numpy as np
import pytest

import oracle
import paper_1812_11214_amd as scat
from paper_1812_11214_amd import workloads

pytestmark = pytest.mark.gpu

TOL_MAX = 1e-4
TOL_L2 = 1e-5


def _backward(shape, J, L, max_order, x, g):
    import torch
    plan = scat.Scattering(shape, J, L, max_order)
    try:
        gi = plan.backward(torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda())
        torch.cuda.synchronize()
        return gi.cpu().numpy()
    finally:
        plan.close()


def _check(shape, J, L, max_order, x, g):
    got = _backward(shape, J, L, max_order, x, g)
    bank = oracle.bank_2d(shape[0], shape[1], J, L)
    want = oracle.scattering2d_backward(x.astype(np.float64), g.astype(np.float64), J, L,
                                        max_order, bank=bank)
    worst_max, worst_l2 = 0.0, 0.0
    for p in range(x.shape[0]):
        d = got[p].astype(np.float64) - want[p]
        worst_max = max(worst_max, np.abs(d).max() / np.abs(want[p]).max())
        worst_l2 = max(worst_l2, np.linalg.norm(d) / np.linalg.norm(want[p]))
    print("backward", shape, J, L, max_order, "max-rel %.2e l2-rel %.2e" % (worst_max, worst_l2),
          flush=True)
    assert worst_max <= TOL_MAX and worst_l2 <= TOL_L2, (worst_max, worst_l2)
    return got, want


@pytest.mark.parametrize("shape,J,L,max_order,batch", [
    ((32, 32), 2, 8, 2, 5), ((16, 16), 2, 3, 2, 3), ((64, 64), 3, 4, 2, 3),
    ((32, 64), 2, 3, 1, 2), ((64, 32), 3, 2, 2, 2), ((128, 128), 3, 2, 2, 2),
    ((8, 8), 1, 4, 2, 3), ((128, 128), 4, 3, 2, 1),
    # coarse octaves too small for the fused row pass of the recomputed forward cascade
    ((32, 128), 4, 2, 2, 2), ((64, 128), 4, 2, 2, 2), ((16, 128), 3, 2, 2, 2),
    # 2 : 1 nodes held by one workgroup (both orientations), with and without children
    ((64, 128), 2, 3, 2, 2), ((128, 64), 2, 2, 2, 2), ((128, 256), 3, 2, 2, 1),
    # more children than one launch of the row-adjoint kernel takes (33 for x), nodes down to 8 x 8
    ((64, 64), 4, 8, 2, 1),
    # first order only at 256 x 256: leaves of 256 (column and row passes) and 128 (node kernel)
    ((256, 256), 2, 2, 1, 1),
    # 512-wide rows: the per-level schedule, with the node kernel where nodes fit
    ((64, 512), 3, 2, 2, 1),
])
def test_backward_shapes(shape, J, L, max_order, batch):
    rng = np.random.default_rng(hash((shape, J, L, max_order)) % 2**32)
    x = rng.standard_normal((batch,) + shape).astype(np.float32)
    K = 1 + J * L + (L * L * J * (J - 1) // 2 if max_order == 2 else 0)
    g = rng.standard_normal((batch, K, shape[0] >> J, shape[1] >> J)).astype(np.float32)
    _check(shape, J, L, max_order, x, g)


def test_backward_headline_shape():
    """256 x 256, J = 3, L = 8 on two planes of the headline workload."""
    c = workloads.config(2)
    x = workloads.planes(2, 2)
    rng = np.random.default_rng(21)
    g = rng.standard_normal((2, 217, 32, 32)).astype(np.float32)
    _check(tuple(c["shape"]), c["J"], c["LQ"], 2, x, g)


def test_backward_order0_only_is_linear_and_exact():
    """With g on channel 0 only the gradient does not depend on x and equals the
    transposed lowpass; fp32 reproduces it to rounding."""
    rng = np.random.default_rng(8)
    shape, J, L = (64, 64), 2, 4
    K = 1 + J * L + L * L
    g = np.zeros((2, K, 16, 16), dtype=np.float32)
    g[:, 0] = rng.standard_normal((2, 16, 16))
    x1 = rng.standard_normal((2,) + shape).astype(np.float32)
    x2 = rng.standard_normal((2,) + shape).astype(np.float32)
    a = _backward(shape, J, L, 2, x1, g)
    b = _backward(shape, J, L, 2, x2, g)
    assert np.array_equal(a, b)
    want = oracle.scattering2d_backward(x1.astype(np.float64), g.astype(np.float64), J, L)
    assert np.abs(a - want).max() <= 1e-5 * np.abs(want).max()


def test_backward_chunked_and_repeatable():
    """Same gradient whether the batch runs in one chunk or several, and on a second call;
    a forward call in between (shared scratch) does not disturb it."""
    import torch
    rng = np.random.default_rng(12)
    shape, J, L = (64, 64), 3, 4
    K = 1 + J * L + L * L * 3
    x = torch.from_numpy(rng.standard_normal((9,) + shape).astype(np.float32)).cuda()
    g = torch.from_numpy(rng.standard_normal((9, K, 8, 8)).astype(np.float32)).cuda()
    plan = scat.Scattering(shape, J, L)
    try:
        a = plan.backward(x, g).clone()
        plan.forward(x)
        b = plan.backward(x, g).clone()
        parts = torch.cat([plan.backward(x[:4].contiguous(), g[:4].contiguous()),
                           plan.backward(x[4:].contiguous(), g[4:].contiguous())])
        torch.cuda.synchronize()
        assert torch.equal(a, b) and torch.equal(a, parts)
        assert plan.backward_workspace_bytes(9) > plan.workspace_bytes(9)
    finally:
        plan.close()


def test_backward_zero_input_and_zero_gradient():
    import torch
    shape, J, L = (32, 32), 2, 8
    K = 1 + J * L + L * L
    rng = np.random.default_rng(2)
    g = rng.standard_normal((2, K, 8, 8)).astype(np.float32)
    x0 = np.zeros((2,) + shape, dtype=np.float32)
    got = _backward(shape, J, L, 2, x0, g)
    g0 = np.zeros_like(g)
    g0[:, 0] = g[:, 0]
    only0 = _backward(shape, J, L, 2, x0, g0)
    assert np.array_equal(got, only0) and np.abs(got).max() > 0
    x = rng.standard_normal((2,) + shape).astype(np.float32)
    assert np.all(_backward(shape, J, L, 2, x, np.zeros_like(g)) == 0)


def test_backward_tiny_input_gives_finite_gradient():
    """Inputs so small that |y|^2 is a denormal (or underflows) before the modulus: the
    gradient must stay finite and bounded by what the unit factors y/|y| allow."""
    shape, J, L = (32, 32), 2, 8
    K = 1 + J * L + L * L
    rng = np.random.default_rng(4)
    g = rng.standard_normal((3, K, 8, 8)).astype(np.float32)
    x = rng.standard_normal((3,) + shape).astype(np.float32)
    ref = _backward(shape, J, L, 2, x, g)
    for scale in (1e-18, 1e-20, 1e-23):
        got = _backward(shape, J, L, 2, (x * np.float32(scale)).astype(np.float32), g)
        assert np.isfinite(got).all(), scale
        assert np.abs(got).max() <= 10 * np.abs(ref).max(), scale


@pytest.mark.parametrize("n,J,Q,max_order,o,batch", [
    (64, 3, 2, 2, 0, 3), (256, 4, 1, 2, 0, 2), (1024, 5, 8, 2, 0, 2), (4096, 6, 8, 1, 0, 2),
    (2048, 2, 3, 2, 0, 2), (1024, 5, 2, 2, 2, 3), (65536, 6, 8, 2, 0, 1),
    (32768, 7, 4, 2, 0, 1), (8192, 4, 12, 2, 1, 2),
    # 512-point rows of the four-step matrix: the per-level schedule
    (262144, 3, 1, 2, 0, 1),
])
def test_backward_1d(n, J, Q, max_order, o, batch):
    import torch
    rng = np.random.default_rng(n + 3 * J + Q + o)
    x = rng.standard_normal((batch, n)).astype(np.float32)
    plan = scat.Scattering((n,), J, Q, max_order, oversampling=o)
    try:
        g = rng.standard_normal((batch, plan.K) + plan.out_shape).astype(np.float32)
        gi = plan.backward(torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda())
        torch.cuda.synchronize()
        got = gi.cpu().numpy().astype(np.float64)
    finally:
        plan.close()
    want = oracle.scattering1d_backward(x.astype(np.float64), g.astype(np.float64), J, Q,
                                        max_order, oversampling=o)
    worst_max, worst_l2 = 0.0, 0.0
    for p in range(batch):
        d = got[p] - want[p]
        worst_max = max(worst_max, np.abs(d).max() / np.abs(want[p]).max())
        worst_l2 = max(worst_l2, np.linalg.norm(d) / np.linalg.norm(want[p]))
    print("backward 1d", n, J, Q, max_order, o, "max-rel %.2e l2-rel %.2e" % (worst_max, worst_l2),
          flush=True)
    assert worst_max <= TOL_MAX and worst_l2 <= TOL_L2, (worst_max, worst_l2)


@pytest.mark.parametrize("shape,J,LQ,batch", [((64, 64), 3, 4, 7), ((4096,), 5, 4, 5)])
def test_backward_in_chunks_matches_one_pass(shape, J, LQ, batch):
    """A scratch budget that forces one plane per chunk (read once per process, hence the child
    process) gives bit for bit the gradient of the single-chunk pass."""
    import torch
    import subprocess, sys, os, tempfile
    rng = np.random.default_rng(5 + len(shape))
    x = rng.standard_normal((batch,) + shape).astype(np.float32)
    plan = scat.Scattering(shape, J, LQ)
    try:
        g = rng.standard_normal((batch, plan.K) + plan.out_shape).astype(np.float32)
        a = plan.backward(torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda())
        torch.cuda.synchronize()
        a = a.cpu().numpy()
    finally:
        plan.close()
    code = (
        "import sys, numpy as np, torch\n"
        "sys.path.insert(0, %r)\n"
        "import paper_1812_11214_amd as scat\n"
        "d = np.load(sys.argv[1])\n"
        "p = scat.Scattering(%r, %d, %d)\n"
        "y = p.backward(torch.from_numpy(d['x']).cuda(), torch.from_numpy(d['g']).cuda())\n"
        "torch.cuda.synchronize()\n"
        "np.save(sys.argv[2], y.cpu().numpy()); p.close()\n"
    ) % (os.path.dirname(os.path.dirname(os.path.abspath(__file__))), shape, J, LQ)
    with tempfile.TemporaryDirectory() as d:
        inp, out = os.path.join(d, "in.npz"), os.path.join(d, "y.npy")
        np.savez(inp, x=x, g=g)
        env = dict(os.environ, SCAT_SCRATCH_MB="1")
        subprocess.run([sys.executable, "-c", code, inp, out], check=True, env=env, timeout=240)
        b = np.load(out)
    assert np.array_equal(a, b)
