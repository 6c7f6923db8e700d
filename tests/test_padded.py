"""Signals of any size: symmetric extension to a periodic power-of-two grid.

The paper applies the transform to a 28 x 28 array (section 4, "Interface") without
describing the boundary handling, so the extension rule is this build's reading --
"parity unpinned by the paper".  What is pinned here: the oracle's extension against
numpy's own symmetric padding, the grid and output sizes, exactness for constant signals,
and (GPU) the library against the oracle through the C ABI.
"""
import numpy as np
import pytest

import oracle
import paper_1812_11214_amd as scat
from oracle.scattering import pad_index, padded_size


@pytest.mark.parametrize("n,J", [(28, 2), (5, 3), (100, 4), (32, 2), (1, 2), (3, 1), (1000, 6)])
def test_extension_matches_numpy_symmetric_pad(n, J):
    P = padded_size(n, J)
    assert P & (P - 1) == 0 and P >= n + (1 << J) and P // 2 < n + (1 << J)
    h = (P - n + 1) // 2
    lo = P - n - h
    x = np.arange(n) * 1.5 + 0.25
    want = np.roll(np.pad(x, (lo, h), mode="symmetric"), -lo)
    assert np.array_equal(x[pad_index(n, P)], want)
    # the periodic extension has no jump at either edge of the signal
    xe = x[pad_index(n, P)]
    assert xe[n] == x[n - 1] and xe[P - 1] == x[0]


def test_oracle_padded_shapes_and_constant_signal():
    S = oracle.scattering2d_padded(np.zeros((3, 28, 28)), 2, 8)
    assert S.shape == (3, 81, 7, 7)
    S1 = oracle.scattering1d_padded(np.zeros((2, 1000)), 4, 2)
    assert S1.shape[-1] == 63
    c = oracle.scattering2d_padded(np.full((30, 50), 2.5), 3, 4)
    assert c.shape[-2:] == (4, 7)
    assert np.abs(c[0] - 2.5).max() < 1e-12 and np.abs(c[1:]).max() < 1e-12


def test_oracle_padded_equals_periodic_transform_of_the_extension():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 20, 28))
    J, L = 2, 3
    Pr, Pc = padded_size(20, J), padded_size(28, J)
    xp = x[:, pad_index(20, Pr), :][:, :, pad_index(28, Pc)]
    want = oracle.scattering2d(xp, J, L)[..., :5, :7]
    assert np.array_equal(oracle.scattering2d_padded(x, J, L), want)


def test_host_plan_sizes():
    for shape, J, grid, out in [((28, 28), 2, (32, 32), (7, 7)), ((30, 50), 3, (64, 64), (4, 7)),
                                ((1000,), 4, (1024,), (63,)), ((256, 256), 3, (512, 512), (32, 32)),
                                ((1, 9), 1, (4, 16), (1, 5))]:
        p = scat.Scattering(shape, J, 2, host_only=True, padded=True)
        try:
            assert p.grid_shape == grid and p.out_shape == out
        finally:
            p.close()
    with pytest.raises(scat.ScatError):
        scat.Scattering((5000, 8), 2, 2, host_only=True, padded=True)   # grid 8192 > 4096
    with pytest.raises(scat.ScatError):
        scat.Scattering((0, 8), 2, 2, host_only=True, padded=True)


@pytest.mark.gpu
@pytest.mark.parametrize("shape,J,LQ,batch", [((28, 28), 2, 8, 6), ((30, 50), 3, 4, 3),
                                              ((200, 120), 3, 3, 2), ((5, 7), 2, 2, 4),
                                              ((256, 256), 3, 8, 1), ((1000,), 4, 2, 3),
                                              ((4000,), 6, 8, 2)])
def test_padded_parity_gpu(shape, J, LQ, batch):
    import torch
    rng = np.random.default_rng(sum(shape) + J)
    x = rng.standard_normal((batch,) + shape).astype(np.float32)
    plan = scat.Scattering(shape, J, LQ, padded=True)
    try:
        y = plan.forward(torch.from_numpy(x).cuda())
        torch.cuda.synchronize()
        got = y.cpu().numpy().astype(np.float64)
        assert got.shape[1:] == (plan.K,) + plan.out_shape
        rows = plan.coeff_index()
    finally:
        plan.close()
    if len(shape) == 2:
        want = oracle.scattering2d_padded(x.astype(np.float64), J, LQ)
    else:
        want = oracle.scattering1d_padded(x.astype(np.float64), J, LQ)
    order = np.array([r[0] for r in rows])
    for p in range(batch):
        for o in (0, 1, 2):
            sel = order == o
            err = np.abs(got[p][sel] - want[p][sel]).max() / np.abs(want[p][sel]).max()
            assert err <= 1e-4, (p, o, err)


@pytest.mark.gpu
def test_padded_chunks():
    import torch
    rng = np.random.default_rng(5)
    x = torch.from_numpy(rng.standard_normal((7, 28, 28)).astype(np.float32)).cuda()
    plan = scat.Scattering((28, 28), 2, 8, padded=True)
    try:
        a = plan.forward(x)
        b = torch.cat([plan.forward(x[:3].contiguous()), plan.forward(x[3:].contiguous())])
        torch.cuda.synchronize()
        assert torch.equal(a, b)
    finally:
        plan.close()


def test_oracle_padded_backward_matches_finite_differences():
    rng = np.random.default_rng(1)
    for shape, J, L in [((14, 10), 2, 3), ((5, 7), 1, 2)]:
        x = rng.standard_normal((2,) + shape)
        S = oracle.scattering2d_padded(x, J, L)
        g = rng.standard_normal(S.shape)
        gx = oracle.scattering2d_padded_backward(x, g, J, L)
        d = rng.standard_normal(x.shape)
        eps = 1e-6
        f = lambda z: float(np.sum(g * oracle.scattering2d_padded(z, J, L)))
        fd = (f(x + eps * d) - f(x - eps * d)) / (2 * eps)
        assert abs(fd - np.sum(gx * d)) <= 1e-6 * max(abs(fd), 1e-3)


def test_oracle_padded_backward_1d_and_3d_match_finite_differences():
    from oracle import harmonic3d as o3
    rng = np.random.default_rng(6)
    x = rng.standard_normal((2, 50))
    S = oracle.scattering1d_padded(x, 3, 2)
    g = rng.standard_normal(S.shape)
    gx = oracle.scattering1d_padded_backward(x, g, 3, 2)
    d = rng.standard_normal(x.shape)
    eps = 1e-6
    f = lambda z: float(np.sum(g * oracle.scattering1d_padded(z, 3, 2)))
    fd = (f(x + eps * d) - f(x - eps * d)) / (2 * eps)
    assert abs(fd - np.sum(gx * d)) <= 1e-6 * max(abs(fd), 1e-3)
    x = rng.standard_normal((1, 5, 7, 6)) + 0.3
    S = o3.harmonic_scattering3d_padded(x, 1, 1)
    g = rng.standard_normal(S.shape)
    gx = o3.harmonic_scattering3d_padded_backward(x, g, 1, 1)
    d = rng.standard_normal(x.shape)
    f = lambda z: float(np.sum(g * o3.harmonic_scattering3d_padded(z, 1, 1)))
    fd = (f(x + eps * d) - f(x - eps * d)) / (2 * eps)
    assert abs(fd - np.sum(gx * d)) <= 1e-6 * max(abs(fd), 1e-3)


def test_extension_adjoint_identity():
    """<pad(x), y> = <x, pad^T(y)> with pad^T as used by the oracle's backward pass."""
    rng = np.random.default_rng(2)
    for n, J in [(28, 2), (5, 3), (3, 4)]:
        P = padded_size(n, J)
        idx = pad_index(n, P)
        x, y = rng.standard_normal(n), rng.standard_normal(P)
        yt = np.zeros(n)
        np.add.at(yt, idx, y)
        assert abs(np.dot(x[idx], y) - np.dot(x, yt)) < 1e-12


@pytest.mark.gpu
@pytest.mark.parametrize("shape,J,L,batch", [((28, 28), 2, 8, 4), ((30, 50), 3, 4, 2),
                                             ((5, 7), 2, 2, 3), ((100, 36), 3, 3, 2)])
def test_padded_backward_parity_gpu(shape, J, L, batch):
    import torch
    rng = np.random.default_rng(sum(shape) * 3 + J)
    x = rng.standard_normal((batch,) + shape).astype(np.float32)
    plan = scat.Scattering(shape, J, L, padded=True)
    try:
        g = rng.standard_normal((batch, plan.K) + plan.out_shape).astype(np.float32)
        gi = plan.backward(torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda())
        torch.cuda.synchronize()
        got = gi.cpu().numpy().astype(np.float64)
    finally:
        plan.close()
    want = oracle.scattering2d_padded_backward(x.astype(np.float64), g.astype(np.float64), J, L)
    for p in range(batch):
        err = np.abs(got[p] - want[p]).max() / np.abs(want[p]).max()
        assert err <= 1e-4, (p, err)


@pytest.mark.gpu
@pytest.mark.parametrize("n,J,Q,batch", [(1000, 4, 2, 3), (50, 3, 1, 2), (5000, 5, 4, 2)])
def test_padded_backward_parity_gpu_1d(n, J, Q, batch):
    import torch
    rng = np.random.default_rng(n + J)
    x = rng.standard_normal((batch, n)).astype(np.float32)
    plan = scat.Scattering((n,), J, Q, padded=True)
    try:
        g = rng.standard_normal((batch, plan.K) + plan.out_shape).astype(np.float32)
        gi = plan.backward(torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda())
        torch.cuda.synchronize()
        got = gi.cpu().numpy().astype(np.float64)
    finally:
        plan.close()
    want = oracle.scattering1d_padded_backward(x.astype(np.float64), g.astype(np.float64), J, Q)
    for p in range(batch):
        err = np.abs(got[p] - want[p]).max() / np.abs(want[p]).max()
        assert err <= 1e-4, (p, err)


@pytest.mark.gpu
@pytest.mark.parametrize("shape,J,L,o", [((5, 7, 6), 1, 1, 0), ((20, 24, 28), 2, 2, 0),
                                         ((12, 30, 9), 2, 1, 1)])
def test_padded_backward_parity_gpu_3d(shape, J, L, o):
    import torch
    from oracle import harmonic3d as o3
    rng = np.random.default_rng(sum(shape) + J)
    x = rng.standard_normal((2,) + shape).astype(np.float32)
    plan = scat.Scattering(shape, J, L, padded=True, oversampling=o)
    try:
        g = rng.standard_normal((2, plan.K) + plan.out_shape).astype(np.float32)
        gi = plan.backward(torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda())
        torch.cuda.synchronize()
        got = gi.cpu().numpy().astype(np.float64)
    finally:
        plan.close()
    want = o3.harmonic_scattering3d_padded_backward(x, g, J, L, oversampling=o)
    for p in range(2):
        err = np.abs(got[p] - want[p]).max() / np.abs(want[p]).max()
        assert err <= 1e-4, (p, err)
