"""scat_forward_static (the entry point for callers that cannot allocate device memory) against
scat_forward, through the C ABI: two calls in a row on one GPU, the second on a smaller input
(the static buffer keeps the first call's contents), plus a plan whose batch runs in several
chunks, the refusal of a plan whose single plane exceeds the buffer, and replays of the call
from a HIP graph."""
import ctypes

import numpy as np
import pytest

import paper_1812_11214_amd as scat
from paper_1812_11214_amd import binding, workloads

pytestmark = pytest.mark.gpu


def _both(plan, x, torch):
    """(scat_forward, scat_forward_static) outputs of the same device input."""
    batch = x.shape[0]
    shp = (batch, plan.K) + plan.out_shape
    ref = torch.full(shp, float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full(shp, float("nan"), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    binding.scat_forward(plan._plan, x.data_ptr(), ref.data_ptr(), batch, stream)
    torch.cuda.synchronize()
    binding.scat_forward_static(plan._plan, x.data_ptr(), got.data_ptr(), batch, stream)
    torch.cuda.synchronize()
    return ref.cpu().numpy(), got.cpu().numpy()


def _check(ref, got):
    assert np.isfinite(ref).all() and np.isfinite(got).all()
    # same kernels, same launch shapes per chunk or not: fp32 results within the parity bar
    err = np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max()
    assert err <= 1e-4, err
    return err


def test_static_two_calls_second_smaller():
    import torch
    torch.cuda.set_device(0)
    plan = scat.Scattering((64, 64), 3, 8)
    try:
        rng = np.random.default_rng(7)
        x_big = torch.from_numpy(rng.standard_normal((24, 64, 64)).astype(np.float32)).cuda()
        x_small = torch.from_numpy(rng.standard_normal((5, 64, 64)).astype(np.float32)).cuda()
        r1, g1 = _both(plan, x_big, torch)
        _check(r1, g1)
        r2, g2 = _both(plan, x_small, torch)
        _check(r2, g2)
    finally:
        plan.close()


def test_static_second_plan_smaller_shape_and_1d():
    import torch
    torch.cuda.set_device(0)
    big = scat.Scattering((512, 512), 4, 8)
    small = scat.Scattering((32, 32), 2, 8)
    one_d = scat.Scattering((4096,), 4, 4)
    try:
        x = torch.from_numpy(workloads.planes(3, 3)).cuda()   # several chunks of the 64 MiB buffer
        assert big.workspace_bytes(1) <= binding.SCAT_STATIC_SCRATCH_MB << 20 < big.workspace_bytes(3)
        r, g = _both(big, x, torch)
        _check(r, g)
        xs = torch.from_numpy(workloads.planes(0)).cuda()
        r, g = _both(small, xs, torch)
        _check(r, g)
        rng = np.random.default_rng(3)
        x1 = torch.from_numpy(rng.standard_normal((3, 4096)).astype(np.float32)).cuda()
        r, g = _both(one_d, x1, torch)
        _check(r, g)
        # the 1-D workload's shape: one signal per pass through the static buffer (merged column
        # passes, half spectra), three signals
        long_1d = scat.Scattering((65536,), 6, 8)
        try:
            assert long_1d.workspace_bytes(1) <= binding.SCAT_STATIC_SCRATCH_MB << 20 < long_1d.workspace_bytes(3)
            x2 = torch.from_numpy(workloads.planes(4, 3)).cuda()
            r, g = _both(long_1d, x2, torch)
            _check(r, g)
        finally:
            long_1d.close()
    finally:
        big.close()
        small.close()
        one_d.close()


def test_static_rejects_oversized_plane_and_bad_arguments():
    import torch
    torch.cuda.set_device(0)
    plan = scat.Scattering((1024, 1024), 3, 8)
    try:
        assert plan.workspace_bytes(1) > binding.SCAT_STATIC_SCRATCH_MB << 20
        x = torch.zeros((1, 1024, 1024), dtype=torch.float32, device="cuda")
        out = torch.zeros((1, plan.K) + plan.out_shape, dtype=torch.float32, device="cuda")
        L = scat.lib()
        st = L.scat_forward_static(plan._plan, ctypes.c_void_p(x.data_ptr()),
                                   ctypes.c_void_p(out.data_ptr()), 1, None)
        assert st == binding.SCAT_ERR_WORKSPACE
        assert "static buffer" in binding.scat_status_string(st)
        assert L.scat_forward_static(plan._plan, None, ctypes.c_void_p(out.data_ptr()), 1, None) == 5
        assert L.scat_forward_static(plan._plan, ctypes.c_void_p(x.data_ptr()),
                                     ctypes.c_void_p(out.data_ptr()), -1, None) == 1
        assert L.scat_forward_static(plan._plan, None, None, 0, None) == 0
        assert L.scat_forward_static(None, None, None, 1, None) == 5
        torch.cuda.synchronize()
    finally:
        plan.close()


# ---- under HIP graph capture: captured once, replayed several times with the program's own
# eager work and synchronisations between the replays, every replay checked against the eager
# result (recording the forward transform into a graph is what this entry point is for)
@pytest.mark.parametrize("shape,J,L,batch", [((256, 256), 3, 4, 3), ((64, 64), 3, 8, 5), ((32, 32), 2, 8, 16)])
def test_static_entry_replays_from_a_graph(shape, J, L, batch):
    import torch
    torch.cuda.set_device(0)
    plan = scat.Scattering(shape, J, L)
    try:
        rng = np.random.default_rng(41)
        x = torch.from_numpy(rng.standard_normal((batch,) + shape).astype(np.float32)).cuda()
        oshape = (batch, plan.K) + plan.out_shape
        ref = torch.empty(oshape, dtype=torch.float32, device="cuda")
        out = torch.full(oshape, float("nan"), dtype=torch.float32, device="cuda")
        # eager: the reference, and the first call's set-up (kernel attributes, scratch address)
        binding.scat_forward_static(plan._plan, x.data_ptr(), ref.data_ptr(), batch,
                                    torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        want = ref.cpu().numpy()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            binding.scat_forward_static(plan._plan, x.data_ptr(), out.data_ptr(), batch,
                                        torch.cuda.current_stream().cuda_stream)
        for rep in range(3):
            out.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            assert np.isfinite(got).all(), rep
            err = np.abs(got.astype(np.float64) - want).max() / np.abs(want).max()
            assert err <= 1e-6, (rep, err)   # the same kernels on the same input
            # eager work of the program's own between the replays
            x2 = (x * 0.5).contiguous()
            binding.scat_forward_static(plan._plan, x2.data_ptr(), ref.data_ptr(), batch,
                                        torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
    finally:
        plan.close()
