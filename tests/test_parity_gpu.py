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
    ((128, 128), 4, 2, 2), ((32, 32), 2, 5, 2), ((32, 32), 2, 3, 1), ((32, 32), 2, 9, 2),
    ((32, 32), 2, 1, 2),
    # thin images: fewer rows than one wave of the fused row pass transforms at a time
    ((4, 128), 2, 5, 2), ((4, 64), 2, 3, 2), ((8, 64), 3, 2, 2), ((4, 32), 1, 2, 2),
    # coarse octaves whose grids are too small for the fused row pass
    ((32, 128), 4, 2, 2), ((64, 128), 4, 3, 2), ((16, 128), 3, 2, 2), ((16, 256), 4, 2, 2),
    # 64 x 64 leaves with a 32 x 32 output (whole-leaf kernel): first and second order
    ((128, 128), 2, 3, 2), ((64, 64), 1, 4, 2), ((128, 128), 2, 2, 1),
])
def test_2d_shapes(shape, J, L, max_order):
    rng = np.random.default_rng(hash((shape, J, L)) % 2**32)
    x = rng.standard_normal((5,) + shape).astype(np.float32)
    _check_2d(x, J, L, max_order)


@pytest.mark.parametrize("shape,J,L,max_order,batch", [
    ((512, 64), 3, 3, 2, 2), ((64, 512), 2, 5, 2, 2), ((256, 256), 5, 2, 2, 1),
    ((1024, 32), 2, 5, 2, 1), ((512, 512), 2, 6, 1, 1), ((128, 128), 6, 3, 2, 2),
    ((512, 512), 4, 2, 2, 1),  # 64 x 64 leaves of the stored-spectrum schedule
])
def test_2d_stored_spectrum_path(shape, J, L, max_order, batch):
    """Shapes the fused row pass does not take (a side of 512 or more, or more than four
    octaves): full spectra are stored and re-read per level; numbers of angles that are
    not multiples of the filters-per-read of that kernel; rectangular grids."""
    rng = np.random.default_rng(sum(shape) * 13 + J * 5 + L)
    x = rng.standard_normal((batch,) + shape).astype(np.float32)
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
    # rows of 4096 points (n2 = 2^J): the row kernel's largest LDS tile
    (8192, 12, 1, 2), (1 << 18, 3, 2, 2),
    # 256 rows: the column passes of several octaves as segments of one launch, narrow octaves
    # (fewer than 16 columns) beside it; first order only; one octave
    (65536, 4, 1, 2), (1 << 17, 9, 1, 2), (65536, 8, 2, 1), (65536, 1, 3, 2),
    # half spectra between the column and row passes with 128, 64 and 32 rows
    (32768, 4, 2, 2), (8192, 3, 4, 2), (2048, 3, 1, 2),
])
def test_1d_shapes(n, J, Q, max_order):
    rng = np.random.default_rng(n + J + Q)
    x = rng.standard_normal((3, n)).astype(np.float32)
    _check_1d(x, J, Q, max_order)


def test_config4_1d_sample():
    c = workloads.config(4)
    x = workloads.planes(4, 2)
    _check_1d(x, c["J"], c["LQ"])


def test_config2_full_batch_sampled():
    """The benchmark's launch configuration (all 384 planes in one call); planes sampled
    across the batch are compared with the oracle one by one."""
    c = workloads.config(2)
    P = workloads.num_planes(2)
    x = workloads.planes(2)
    plan = scat.Scattering(c["shape"], c["J"], c["LQ"])
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    assert got.shape == (P, 217, 32, 32) and np.isfinite(got).all()
    bank = oracle.bank_2d(256, 256, c["J"], c["LQ"])
    sample = [0, 1, 95, 190, 191, 257, 383]
    want = oracle.scattering2d(x[sample], c["J"], c["LQ"], bank=bank)
    errs = per_order_errors(got[sample], want, order_of_channels(rows), x[sample])
    print("config2 full batch, planes", sample, errs, flush=True)
    assert max(errs.values()) <= TOL, errs
    # every plane's S0 must equal the lowpassed mean structure: cheap whole-batch property
    # (zero-mean input => S0 averages to ~0; S1, S2 non-negative up to rounding)
    order = order_of_channels(rows)
    assert np.abs(got[:, order == 0].mean(axis=(1, 2, 3))).max() < 1e-3
    assert got[:, order > 0].min() > -1e-4


def _full_batch_sampled(wl, sample, dims):
    """Workload `wl` at its full batch in one call (the launch shapes the benchmark times);
    the sampled planes are compared with the oracle one by one, every plane is checked for
    finite values and non-negative S1, S2."""
    c = workloads.config(wl)
    P = workloads.num_planes(wl)
    x = workloads.planes(wl)
    plan = scat.Scattering(c["shape"], c["J"], c["LQ"])
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    assert got.shape[0] == P and np.isfinite(got).all()
    order = order_of_channels(rows)
    assert got[:, order > 0].min() > -1e-4 * np.abs(got).max()
    if dims == 2:
        bank = oracle.bank_2d(c["shape"][0], c["shape"][1], c["J"], c["LQ"])
        want = oracle.scattering2d(x[sample], c["J"], c["LQ"], bank=bank)
    else:
        want = oracle.scattering1d(x[sample], c["J"], c["LQ"])
    errs = per_order_errors(got[sample], want, order, x[sample])
    print("workload", wl, "full batch of", P, "planes sampled", sample, errs, flush=True)
    assert max(errs.values()) <= TOL, errs


def test_config1_full_batch_sampled():
    _full_batch_sampled(1, [0, 1, 2, 1535, 1536, 3070, 3071], 2)


def test_config3_full_batch_sampled():
    _full_batch_sampled(3, [0, 15, 31], 2)


def test_config4_full_batch_sampled():
    _full_batch_sampled(4, [0, 31, 63], 1)


@pytest.mark.parametrize("shape,J,L,batch", [((64, 64), 2, 3, 7), ((64, 128), 3, 5, 3),
                                             ((256, 64), 3, 1, 2), ((32, 32), 1, 8, 5),
                                             ((256, 256), 4, 2, 1), ((128, 64), 4, 3, 2)])
def test_2d_ragged(shape, J, L, batch):
    """Odd numbers of angles and planes (partially filled workgroups and batches), one
    octave only, four octaves on the fast path, rectangular grids."""
    rng = np.random.default_rng(sum(shape) * 31 + J * 7 + L)
    x = rng.standard_normal((batch,) + shape).astype(np.float32)
    _check_2d(x, J, L)


def test_chunked_equals_single_call():
    """A small scratch budget forces the batch to be walked in chunks; results must be
    bit-identical to the single-chunk call."""
    x = workloads.planes(1, 300)
    plan = scat.Scattering((32, 32), 2, 8)
    try:
        a = gpu_forward(plan, x)
    finally:
        plan.close()
    import subprocess, sys, os, tempfile
    code = (
        "import sys, numpy as np, torch\n"
        "sys.path.insert(0, %r)\n"
        "import paper_1812_11214_amd as scat\n"
        "from paper_1812_11214_amd import workloads\n"
        "x = workloads.planes(1, 300)\n"
        "p = scat.Scattering((32, 32), 2, 8)\n"
        "assert p.workspace_bytes(300) <= (1 << 20)\n"
        "y = p.forward(torch.from_numpy(x).cuda()); torch.cuda.synchronize()\n"
        "np.save(sys.argv[1], y.cpu().numpy()); p.close()\n"
    ) % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "y.npy")
        env = dict(os.environ, SCAT_SCRATCH_MB="1")
        subprocess.run([sys.executable, "-c", code, out], check=True, env=env, timeout=240)
        b = np.load(out)
    assert np.array_equal(a, b)


def test_stream_and_plan_independence():
    """Two plans on two streams in flight at once give the same results as alone."""
    import torch
    xa = workloads.planes(0, 4)
    xb = np.random.default_rng(9).standard_normal((6, 64, 64)).astype(np.float32)
    pa, pb = scat.Scattering((32, 32), 2, 8), scat.Scattering((64, 64), 3, 4)
    try:
        ra, rb = gpu_forward(pa, xa), gpu_forward(pb, xb)
        sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
        ta, tb = torch.from_numpy(xa).cuda(), torch.from_numpy(xb).cuda()
        torch.cuda.synchronize()
        for _ in range(3):
            with torch.cuda.stream(sa):
                ya = pa.forward(ta)
            with torch.cuda.stream(sb):
                yb = pb.forward(tb)
        torch.cuda.synchronize()
        assert np.array_equal(ya.cpu().numpy(), ra) and np.array_equal(yb.cpu().numpy(), rb)
    finally:
        pa.close()
        pb.close()


def test_reserve_makes_later_calls_allocation_free():
    """After scat_plan_reserve the forward and backward calls of that size leave the device's
    free memory untouched, and give the results they give without it."""
    import torch
    rng = np.random.default_rng(23)
    x = torch.from_numpy(rng.standard_normal((6, 64, 64)).astype(np.float32)).cuda()
    a, b = scat.Scattering((64, 64), 3, 4), scat.Scattering((64, 64), 3, 4)
    try:
        ref = a.forward(x)
        g = torch.ones_like(ref)
        gref = a.backward(x, g)
        out, gin = torch.empty_like(ref), torch.empty_like(x)
        b.reserve(6, with_backward=True)
        torch.cuda.synchronize()
        free0 = torch.cuda.mem_get_info()[0]
        b.forward(x, out=out)
        b.backward(x, g, grad_in=gin)
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free0
        assert torch.equal(out, ref) and torch.equal(gin, gref)
        free1 = torch.cuda.mem_get_info()[0]   # (torch.equal above may have grown torch's own pool)
        b.reserve(2)   # smaller: a no-op
        assert torch.cuda.mem_get_info()[0] == free1
    finally:
        a.close()
        b.close()


def test_timing_api():
    import torch
    rng = np.random.default_rng(11)
    x = torch.from_numpy(rng.standard_normal((4, 64, 64)).astype(np.float32)).cuda()
    plan = scat.Scattering((64, 64), 3, 4)
    try:
        plan.forward(x)
        plan.timing_begin(None)
        y1 = plan.forward(x)
        table = plan.timing_end()
        assert len(table) >= 3
        for name, row in table.items():
            assert name.startswith("k_") and row["launches"] >= 1 and row["ms"] > 0
            assert row["alg_bytes"] > 0 and row["model_flops"] > 0
        one = max(table, key=lambda k: table[k]["ms"])
        plan.timing_begin(one)
        y2 = plan.forward(x)
        t2 = plan.timing_end()
        assert list(t2) == [one] and t2[one]["launches"] == table[one]["launches"]
        torch.cuda.synchronize()
        assert torch.equal(y1, y2)
    finally:
        plan.close()


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
