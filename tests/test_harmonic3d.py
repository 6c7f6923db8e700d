"""3-D solid harmonic plans of the C-ABI library: host-side checks (no GPU) and parity of
the HIP path with the fp64 oracle, element by element."""
import os
import subprocess
import sys
import tempfile

import numpy as np
import pytest

import paper_1812_11214_amd as scat
from oracle import harmonic3d as o3
from paper_1812_11214_amd import workloads

from parity import TOL, gpu_forward, order_of_channels, per_order_errors


@pytest.mark.parametrize("shape,J,L,mo,status", [
    ((8, 8, 8), 0, 1, 2, 1), ((8, 8, 8), 2, -1, 2, 1), ((8, 8, 8), 2, 9, 2, 1),
    ((8, 8, 8), 2, 1, 3, 1), ((8, 12, 8), 2, 1, 2, 2), ((8, 8, 2), 1, 1, 2, 2),
    ((8, 8, 8), 4, 1, 2, 2), ((512, 8, 8), 2, 1, 2, 2),
])
def test_bad_arguments(shape, J, L, mo, status):
    with pytest.raises(scat.ScatError) as e:
        scat.scat_plan_create_host(shape, J, L, mo)
    assert e.value.status == status


def test_no_padding_oversampling_or_backward():
    for kw in (dict(padded=True), dict(oversampling=1)):
        with pytest.raises(scat.ScatError) as e:
            scat.Scattering((8, 8, 8), 1, 1, host_only=True, **kw)
        assert e.value.status == 1
    p = scat.Scattering((8, 8, 8), 1, 1, host_only=True)
    try:
        assert p.backward_workspace_bytes(4) == 0
        with pytest.raises(scat.ScatError) as e:
            scat.scat_backward(p._plan, 0, 0, 0, 0)
        assert e.value.status == 1
    finally:
        p.close()


@pytest.mark.parametrize("shape,J,L,mo", [((8, 16, 8), 2, 2, 2), ((8, 8, 8), 3, 1, 2),
                                          ((4, 8, 16), 1, 3, 1)])
def test_index_shapes_and_filters_match_oracle(shape, J, L, mo):
    p = scat.Scattering(shape, J, L, mo, host_only=True)
    try:
        rows = [r[:4] for r in p.coeff_index()]
        assert rows == o3.coeff_index_3d(J, L, mo)
        assert p.K == len(rows)
        assert p.out_shape == tuple(s >> J for s in shape)
        assert p.grid_shape == shape
        assert p.workspace_bytes(3) > 0
        bank = o3.bank_3d(shape, J, L)
        phi = p.filter(0, 0)
        assert np.abs(phi - bank['phi_hat'].real).max() <= 1e-12
        for j in range(J):
            for l in range(L + 1):
                t = p.filter(1, j * (L + 1) + l)
                assert t.shape == (2 * l + 1,) + shape
                # the library's tables are real solid harmonics: the modulus non-linearity
                # only sees sum_m |psi^_m|^2 pointwise ...
                mine = (t ** 2).sum(axis=0)
                ref = (np.abs(bank['psi_hat'][j][l]) ** 2).sum(axis=0)
                assert np.abs(mine - ref).max() <= 1e-12 * ref.max()
                # ... and the span of the 2l+1 tables, which must equal the span of the
                # oracle's complex ones (real and imaginary parts up to the factor i^l)
                A = t.reshape(2 * l + 1, -1)
                B = (bank['psi_hat'][j][l] * (1j) ** l).reshape(2 * l + 1, -1)
                Bri = np.concatenate([B.real, B.imag])
                coef, *_ = np.linalg.lstsq(A.T, Bri.T, rcond=None)
                assert np.abs(A.T @ coef - Bri.T).max() <= 1e-10 * np.abs(A).max()
    finally:
        p.close()


def _check(x, J, L, max_order=2):
    shape = x.shape[-3:]
    plan = scat.Scattering(shape, J, L, max_order)
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    want = o3.harmonic_scattering3d(x, J, L, max_order)
    errs = per_order_errors(got, want, order_of_channels(rows), x)
    print("3d", shape, J, L, max_order, errs, flush=True)
    assert max(errs.values()) <= TOL, errs
    return got, want


@pytest.mark.gpu
@pytest.mark.parametrize("shape,J,L,mo", [
    ((16, 16, 16), 2, 2, 2), ((32, 32, 32), 2, 3, 2), ((8, 16, 32), 1, 1, 2),
    ((16, 16, 16), 3, 1, 2), ((32, 16, 8), 2, 2, 1), ((4, 4, 4), 1, 0, 2), ((16, 8, 64), 2, 4, 2),
    # shapes of the fused passes (both fast axes >= 16, slabs of at most 4096 points)
    ((4, 16, 16), 2, 1, 2), ((8, 64, 16), 3, 2, 2), ((16, 16, 256), 2, 1, 2),
    ((8, 256, 16), 1, 1, 2), ((32, 32, 128), 2, 1, 2), ((16, 128, 32), 4, 1, 2),
    ((16, 32, 16), 2, 8, 1), ((128, 16, 64), 2, 0, 2),
    # slabs of 8192 and 16384 points (512 and 1024 threads per slab)
    ((8, 64, 128), 2, 1, 2), ((4, 128, 64), 1, 2, 2), ((4, 32, 256), 2, 1, 2),
    ((8, 256, 32), 3, 1, 2), ((4, 128, 128), 2, 1, 2), ((4, 64, 256), 1, 1, 2),
    # 256 x 64 slabs take the general schedule
    ((4, 256, 64), 2, 1, 2),
    # longest axis 0, deepest supported fold of the fused passes, largest degree
    ((256, 16, 16), 1, 0, 1), ((16, 32, 32), 4, 1, 2), ((8, 16, 16), 1, 8, 2),
])
def test_parity_density_volumes(shape, J, L, mo):
    _check(workloads.volumes(shape, 3), J, L, mo)


@pytest.mark.gpu
def test_parity_white_noise_and_batch_layout():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 3, 16, 16, 16)).astype(np.float32)
    plan = scat.Scattering((16, 16, 16), 2, 2)
    try:
        import torch
        y = plan.forward(torch.from_numpy(x).cuda())
        torch.cuda.synchronize()
        got = y.cpu().numpy()
    finally:
        plan.close()
    assert got.shape == (2, 3, plan.K, 4, 4, 4)
    want = o3.harmonic_scattering3d(x, 2, 2)
    orders = order_of_channels(o3.coeff_index_3d(2, 2))
    errs = per_order_errors(got.reshape((6,) + got.shape[2:]), want.reshape((6,) + want.shape[2:]),
                            orders, x.reshape(6, 16, 16, 16))
    assert max(errs.values()) <= TOL, errs


@pytest.mark.gpu
def test_empty_batch_is_a_no_op():
    import torch
    for shape in ((8, 8, 8), (8, 16, 16)):
        plan = scat.Scattering(shape, 1, 1)
        try:
            x = torch.empty((0,) + shape, dtype=torch.float32, device="cuda")
            y = plan.forward(x)
            torch.cuda.synchronize()
            assert tuple(y.shape) == (0, plan.K) + plan.out_shape
        finally:
            plan.close()


@pytest.mark.gpu
def test_zero_and_constant_volumes():
    x = np.zeros((2, 8, 8, 8), dtype=np.float32)
    x[1] = 2.5
    plan = scat.Scattering((8, 8, 8), 1, 2)
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    assert np.all(got[0] == 0)
    # a constant passes the unit-mass lowpass unchanged; wavelets of degree l >= 1 have zero
    # mean, the degree-0 one has mean 1 (a Gaussian), so those channels equal the constant too
    want = o3.harmonic_scattering3d(x, 1, 2)
    errs = per_order_errors(got, want, order_of_channels(rows), x)
    assert max(errs.values()) <= TOL, errs
    assert np.abs(got[1, 0] - 2.5).max() <= 1e-5


@pytest.mark.gpu
def test_chunked_batches_match_unchunked():
    """The scratch budget is read once per process: the chunked run is a child process."""
    x = workloads.volumes((16, 16, 16), 9)
    plan = scat.Scattering((16, 16, 16), 2, 1)
    try:
        whole = gpu_forward(plan, x)
    finally:
        plan.close()
    code = (
        "import sys, numpy as np, torch\n"
        "sys.path.insert(0, %r)\n"
        "import paper_1812_11214_amd as scat\n"
        "from paper_1812_11214_amd import workloads\n"
        "x = workloads.volumes((16, 16, 16), 9)\n"
        "p = scat.Scattering((16, 16, 16), 2, 1)\n"
        "assert p.workspace_bytes(9) <= (1 << 20) < 9 * p.workspace_bytes(1)\n"
        "y = p.forward(torch.from_numpy(x).cuda()); torch.cuda.synchronize()\n"
        "np.save(sys.argv[1], y.cpu().numpy()); p.close()\n"
    ) % os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "y.npy")
        env = dict(os.environ, SCAT_SCRATCH_MB="1")
        subprocess.run([sys.executable, "-c", code, out], check=True, env=env, timeout=240)
        parts = np.load(out)
    assert np.array_equal(whole, parts)


@pytest.mark.gpu
def test_benchmark_workload_sampled():
    """The 16 x 64^3 batch the benchmark's 3-D mode times, in one call; volumes 0, 7 and 15
    against the oracle."""
    c = workloads.VOLUME_CONFIG
    x = workloads.volumes(c["shape"], c["batch"])
    plan = scat.Scattering(c["shape"], c["J"], c["LQ"])
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    pick = [0, 7, 15]
    want = o3.harmonic_scattering3d(x[pick], c["J"], c["LQ"])
    errs = per_order_errors(got[pick], want, order_of_channels(rows), x[pick])
    print("3d workload", errs, flush=True)
    assert max(errs.values()) <= TOL, errs
