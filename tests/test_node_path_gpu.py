"""Parity of the whole-node schedule (one workgroup per node of the tree, first octave of a
256 x 256 image as four polyphase components) against the oracle, through the C ABI: numbers
of angles other than 8, first order only, source counts that do not fill the last group of
eight workgroups, padded plans on a 256 x 256 grid, and the benchmark batch."""
import numpy as np
import pytest

import oracle
import paper_1812_11214_amd as scat
from paper_1812_11214_amd import workloads

from parity import TOL, gpu_forward, order_of_channels, per_order_errors

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,J,L,max_order,batch", [
    (256, 3, 8, 2, 2), (256, 3, 3, 2, 3), (256, 3, 5, 1, 1), (256, 3, 1, 2, 5),
    (256, 3, 2, 2, 9), (256, 3, 6, 2, 1), (256, 3, 7, 2, 2),
    (128, 2, 8, 2, 3), (128, 2, 5, 2, 7), (128, 2, 4, 1, 2), (128, 2, 7, 2, 11),
])
def test_node_schedule_white_noise(n, J, L, max_order, batch):
    rng = np.random.default_rng(1000 * n + 10 * L + batch)
    x = rng.standard_normal((batch, n, n)).astype(np.float32)
    plan = scat.Scattering((n, n), J, L, max_order, node_kernels=True)
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    want = oracle.scattering2d(x, J, L, max_order)
    errs = per_order_errors(got, want, order_of_channels(rows), x)
    print("node", n, J, L, max_order, batch, errs, flush=True)
    assert max(errs.values()) <= TOL, errs


def test_node_schedule_edge_inputs():
    rng = np.random.default_rng(11)
    x = np.zeros((4, 256, 256), dtype=np.float32)
    x[0] = -2.5                      # constant: S1 = S2 = 0
    x[1, 3, 200] = 1.0               # impulse
    x[2] = rng.standard_normal((256, 256)) * 1e4
    x[3] = rng.standard_normal((256, 256)) * 1e-4
    plan = scat.Scattering((256, 256), 3, 4, node_kernels=True)
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    want = oracle.scattering2d(x, 3, 4)
    errs = per_order_errors(got, want, order_of_channels(rows), x)
    print("node edge", errs, flush=True)
    assert max(errs.values()) <= TOL, errs


def test_node_schedule_padded_200x200():
    rng = np.random.default_rng(12)
    x = rng.standard_normal((2, 200, 200)).astype(np.float32)
    plan = scat.Scattering((200, 200), 3, 4, padded=True, node_kernels=True)
    try:
        assert plan.grid_shape == (256, 256)
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    want = oracle.scattering2d_padded(x, 3, 4)
    errs = per_order_errors(got, want, order_of_channels(rows), x)
    print("node padded", errs, flush=True)
    assert max(errs.values()) <= TOL, errs


def test_node_schedule_is_the_one_that_runs():
    """By default the launches are the whole-node kernels; with SCAT_PLAN_PASS_KERNELS the pass
    kernels."""
    import torch
    x = torch.from_numpy(workloads.planes(2, 2)).cuda()
    names = {}
    for flag in (True, False):
        plan = (scat.Scattering((256, 256), 3, 8) if flag
                else scat.Scattering((256, 256), 3, 8, node_kernels=False))
        try:
            plan.timing_begin(None)
            plan.forward(x)
            names[flag] = set(plan.timing_end())
            if flag:
                assert plan.workspace_bytes(1) < 4 << 20   # spectra of x and of one octave only
        finally:
            plan.close()
    assert any(k.startswith("k_node_half<") for k in names[True]), names[True]
    assert not any(k.startswith("k_rows_fused") for k in names[True]), names[True]
    # the pass schedule: row and column passes (and the whole-node kernel only for the
    # 64 x 64 children of the 128 x 128 nodes)
    assert any(k.startswith("k_rows_fused") for k in names[False]), names[False]
    assert not any(k.startswith("k_node_half<") for k in names[False]), names[False]


@pytest.mark.parametrize("n,J,L,batch", [(256, 3, 8, 3), (128, 2, 6, 9)])
def test_pass_schedule_still_matches(n, J, L, batch):
    """The row-and-column-pass schedule of the shapes whose default is the whole-node one."""
    rng = np.random.default_rng(77 * n + L)
    x = rng.standard_normal((batch, n, n)).astype(np.float32)
    plan = scat.Scattering((n, n), J, L, node_kernels=False)
    try:
        got = gpu_forward(plan, x)
        rows = plan.coeff_index()
    finally:
        plan.close()
    want = oracle.scattering2d(x, J, L)
    errs = per_order_errors(got, want, order_of_channels(rows), x)
    print("passes", n, J, L, batch, errs, flush=True)
    assert max(errs.values()) <= TOL, errs


def test_general_schedule_hands_small_children_to_node_kernels():
    """512 x 512 at J = 4 (row and column passes with stored spectra): the second-order nodes
    of 64 and 128 points a side are computed by whole-node kernels that read the parent's whole
    spectrum; parity of the whole transform, and the launches are the ones expected."""
    import torch
    rng = np.random.default_rng(512)
    x = rng.standard_normal((2, 512, 512)).astype(np.float32)
    plan = scat.Scattering((512, 512), 4, 2)
    try:
        xd = torch.from_numpy(x).cuda()
        plan.timing_begin(None)
        got = plan.forward(xd)
        torch.cuda.synchronize()
        names = set(plan.timing_end())
        got = got.cpu().numpy().astype(np.float64)
        rows = plan.coeff_index()
    finally:
        plan.close()
    assert any(k.startswith("k_node_half<4, 1, false, full") for k in names), names
    assert any(k.startswith("k_node<64, 8, 1, false, full") for k in names), names
    want = oracle.scattering2d(x, 4, 2)
    errs = per_order_errors(got, want, order_of_channels(rows), x)
    print("512 general + node children", errs, flush=True)
    assert max(errs.values()) <= TOL, errs
