"""Oversampling knob: every signal kept 2^o times finer than the default schedule.

The paper only says that intermediate signals are downsampled (section 2,
"Implementation"); with no subsampling at all (o >= J) the cascade IS the section-2
definition evaluated at full resolution, which pins the oracle's handling of the knob
exactly; the library is then checked against the oracle on the GPU.
"""
import numpy as np
import pytest

import oracle
import paper_1812_11214_amd as scat


def test_no_subsampling_equals_the_definition_2d():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 32, 32))
    J, L = 3, 3
    bank = oracle.bank_2d(32, 32, J, L)
    full = oracle.scattering2d(x, J, L, bank=bank, oversampling=J)
    assert full.shape == (2, 1 + J * L + L * L * 3, 32, 32)
    plain = oracle.scattering2d_plain(x, J, L, bank=bank)
    assert np.abs(full[..., ::8, ::8] - plain).max() <= 1e-12 * np.abs(plain).max()
    more = oracle.scattering2d(x, J, L, bank=bank, oversampling=J + 2)
    assert np.array_equal(full, more)


def test_no_subsampling_equals_the_definition_1d():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 256))
    full = oracle.scattering1d(x, 4, 2, oversampling=4)
    plain = oracle.scattering1d_plain(x, 4, 2)
    assert full.shape[-1] == 256
    assert np.abs(full[..., ::16] - plain).max() <= 1e-12 * np.abs(plain).max()


def test_default_is_zero_and_intermediate_values_sit_between():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((32, 32))
    J, L = 3, 2
    bank = oracle.bank_2d(32, 32, J, L)
    s0 = oracle.scattering2d(x, J, L, bank=bank)
    assert np.array_equal(s0, oracle.scattering2d(x, J, L, bank=bank, oversampling=0))
    s1 = oracle.scattering2d(x, J, L, bank=bank, oversampling=1)
    assert s1.shape[-2:] == (8, 8)
    exact = oracle.scattering2d(x, J, L, bank=bank, oversampling=J)[..., ::8, ::8]
    # S0 and the first wavelet layer are exact at any o; with more oversampling the
    # aliasing of the moduli shrinks, so o = 1 is closer to the definition than o = 0
    assert np.allclose(s1[0, ::2, ::2], exact[0], rtol=1e-10, atol=1e-12)
    e0 = np.abs(s0 - exact).max()
    e1 = np.abs(s1[..., ::2, ::2] - exact).max()
    assert e1 < e0


def test_host_plan_output_shapes():
    for shape, J, o, out in [((64, 64), 3, 0, (8, 8)), ((64, 64), 3, 1, (16, 16)),
                             ((64, 64), 3, 5, (64, 64)), ((1024,), 5, 2, (128,))]:
        p = scat.Scattering(shape, J, 2, host_only=True, oversampling=o)
        try:
            assert p.out_shape == out
        finally:
            p.close()
    p = scat.Scattering((28, 28), 2, 2, host_only=True, padded=True, oversampling=1)
    try:
        assert p.grid_shape == (32, 32) and p.out_shape == (14, 14)
    finally:
        p.close()
    with pytest.raises(scat.ScatError):
        scat.Scattering((64, 64), 3, 2, host_only=True, oversampling=-1)


@pytest.mark.gpu
@pytest.mark.parametrize("shape,J,LQ,o,batch,padded", [
    ((64, 64), 3, 4, 1, 3, False), ((64, 64), 3, 4, 3, 2, False), ((32, 32), 2, 8, 1, 4, False),
    ((256, 256), 3, 2, 1, 1, False), ((128, 64), 4, 3, 2, 2, False), ((512, 512), 2, 2, 1, 1, False),
    ((1024,), 5, 2, 2, 3, False), ((4096,), 6, 8, 1, 2, False), ((28, 28), 2, 4, 1, 3, True),
    ((16, 16), 2, 3, 7, 2, False),
    # 1-D rows of 256 and 128 points with nothing / little folded in the row kernel
    ((65536,), 4, 2, 4, 2, False), ((16384,), 5, 1, 3, 2, False),
])
def test_oversampled_parity_gpu(shape, J, LQ, o, batch, padded):
    import torch
    rng = np.random.default_rng(sum(shape) + 7 * J + o)
    x = rng.standard_normal((batch,) + shape).astype(np.float32)
    plan = scat.Scattering(shape, J, LQ, padded=padded, oversampling=o)
    try:
        y = plan.forward(torch.from_numpy(x).cuda())
        torch.cuda.synchronize()
        got = y.cpu().numpy().astype(np.float64)
        rows = plan.coeff_index()
        assert got.shape[1:] == (plan.K,) + plan.out_shape
    finally:
        plan.close()
    xd = x.astype(np.float64)
    if padded:
        from oracle.scattering import pad_index, padded_size
        Pr, Pc = padded_size(shape[0], J), padded_size(shape[1], J)
        xp = xd[:, pad_index(shape[0], Pr), :][:, :, pad_index(shape[1], Pc)]
        want = oracle.scattering2d(xp, J, LQ, oversampling=o)[..., :got.shape[-2], :got.shape[-1]]
    elif len(shape) == 2:
        want = oracle.scattering2d(xd, J, LQ, oversampling=o)
    else:
        want = oracle.scattering1d(xd, J, LQ, oversampling=o)
    order = np.array([r[0] for r in rows])
    for p in range(batch):
        for k in (0, 1, 2):
            sel = order == k
            err = np.abs(got[p][sel] - want[p][sel]).max() / np.abs(want[p][sel]).max()
            assert err <= 1e-4, (p, k, err)


def test_oracle_backward_with_oversampling_matches_finite_differences():
    rng = np.random.default_rng(3)
    shape, J, L = (16, 16), 2, 3
    bank = oracle.bank_2d(16, 16, J, L)
    for o in (1, 2):
        x = rng.standard_normal((2,) + shape)
        S = oracle.scattering2d(x, J, L, bank=bank, oversampling=o)
        g = rng.standard_normal(S.shape)
        gx = oracle.scattering2d_backward(x, g, J, L, bank=bank, oversampling=o)
        d = rng.standard_normal(x.shape)
        eps = 1e-6
        f = lambda z: float(np.sum(g * oracle.scattering2d(z, J, L, bank=bank, oversampling=o)))
        fd = (f(x + eps * d) - f(x - eps * d)) / (2 * eps)
        assert abs(fd - np.sum(gx * d)) <= 1e-6 * max(abs(fd), 1e-3)


@pytest.mark.gpu
@pytest.mark.parametrize("shape,J,L,o,batch", [((32, 32), 2, 3, 1, 3), ((64, 64), 3, 2, 1, 2),
                                               ((32, 32), 3, 4, 3, 2),
                                               # output grids above 1024 points (slab transform
                                               # of the gradient planes): 64 x 64 and 64 x 128
                                               ((128, 128), 2, 2, 1, 2), ((64, 128), 3, 2, 3, 1)])
def test_oversampled_backward_parity_gpu(shape, J, L, o, batch):
    import torch
    rng = np.random.default_rng(sum(shape) + J + o)
    x = rng.standard_normal((batch,) + shape).astype(np.float32)
    plan = scat.Scattering(shape, J, L, oversampling=o)
    try:
        g = rng.standard_normal((batch, plan.K) + plan.out_shape).astype(np.float32)
        gi = plan.backward(torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda())
        torch.cuda.synchronize()
        got = gi.cpu().numpy().astype(np.float64)
    finally:
        plan.close()
    want = oracle.scattering2d_backward(x.astype(np.float64), g.astype(np.float64), J, L,
                                        oversampling=o)
    for p in range(batch):
        err = np.abs(got[p] - want[p]).max() / np.abs(want[p]).max()
        assert err <= 1e-4, (p, err)
