"""CPU-only tests of the C-ABI library: it loads, exports every declared symbol, validates
arguments, and its analytically built filter bank equals the oracle's spatially built one."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from oracle import scattering as oscat
import paper_1812_11214_amd as scat

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "scat.h")).read()
    declared = set(re.findall(r"\b(scat_[a-z_]+)\s*\(", header))
    assert declared == set(scat.EXPORTS)
    L = scat.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings():
    assert scat.scat_status_string(0) == "ok"
    assert len({scat.scat_status_string(s) for s in range(6)}) == 6


@pytest.mark.parametrize("shape,J,LQ,mo,status", [
    ((32, 32), 0, 8, 2, 1), ((32, 32), 2, 0, 2, 1), ((32, 32), 2, 8, 3, 1), ((32, 32), 2, 8, 0, 1),
    ((24, 32), 2, 8, 2, 2), ((32, 2), 2, 8, 2, 2), ((8192, 32), 2, 8, 2, 2), ((100,), 2, 1, 2, 2),
    ((32,), 6, 1, 2, 2), ((8, 8, 8, 8), 2, 1, 2, 1),
])
def test_bad_arguments(shape, J, LQ, mo, status):
    with pytest.raises(scat.ScatError) as e:
        scat.scat_plan_create_host(shape, J, LQ, mo)
    assert e.value.status == status


def test_null_handling():
    L = scat.lib()
    assert L.scat_plan_destroy(None) == 0
    assert L.scat_plan_num_coeffs(None) == -1
    assert L.scat_forward(None, None, None, 1, None) == 5
    shape = (ctypes.c_int * 2)(32, 32)
    assert L.scat_plan_create_host(None, 2, shape, 2, 8, 2) == 5
    h = ctypes.c_void_p()
    assert L.scat_plan_create_host(ctypes.byref(h), 2, None, 2, 8, 2) == 5
    assert h.value is None
    plan = scat.scat_plan_create_host((32, 32), 2, 8)
    try:
        # a host-only plan cannot run; bad batch and null buffers are reported first
        assert L.scat_forward(plan, None, None, -1, None) == 1
        assert L.scat_forward(plan, None, None, 0, None) == 0
        assert L.scat_forward(plan, None, None, 1, None) == 5
        assert L.scat_forward(plan, ctypes.c_void_p(256), ctypes.c_void_p(512), 1, None) == 4
        with pytest.raises(scat.ScatError):
            scat.scat_plan_coeff_index(plan, 81)
        with pytest.raises(scat.ScatError):
            scat.scat_plan_filter(plan, 2, 8, 1, (16, 16))   # j2 = 1 has no table at res 1
    finally:
        scat.scat_plan_destroy(plan)


@pytest.mark.parametrize("shape,J,L,mo", [((32, 32), 2, 8, 2), ((64, 64), 3, 8, 2),
                                          ((16, 64), 3, 4, 1), ((128, 128), 4, 2, 2)])
def test_index_table_and_shapes_2d(shape, J, L, mo):
    p = scat.Scattering(shape, J, L, mo, host_only=True)
    assert p.coeff_index() == oracle.coeff_index_2d(J, L, mo)
    assert p.K == (1 + J * L + (L * L * J * (J - 1) // 2 if mo == 2 else 0))
    assert p.out_shape == (shape[0] >> J, shape[1] >> J)
    assert p.workspace_bytes(3) > 0 and p.workspace_bytes(0) == 0
    p.close()


def test_index_table_1d():
    p = scat.Scattering((4096,), 6, 8, host_only=True)
    assert p.K == 169 and p.out_shape == (64,)
    assert p.coeff_index() == oracle.coeff_index_1d(6, 8)
    p.close()


def test_filter_bank_2d_matches_oracle():
    n_r, n_c, J, L = 64, 32, 3, 4
    p = scat.Scattering((n_r, n_c), J, L, host_only=True)
    bank = oracle.bank_2d(n_r, n_c, J, L)
    for j in range(J):
        for l in range(L):
            ref = bank['psi_hat'][j, l]
            assert np.abs(p.filter(1, j * L + l, 0) - ref.real).max() < 1e-13
            assert p.filter(1, j * L + l, 0)[0, 0] == 0.0
            for r in range(1, j):
                got = p.filter(2, j * L + l, r)
                assert np.abs(got - oscat.fold(ref, r, (-2, -1)).real).max() < 1e-13
    for r in range(J):
        want = oscat.fold(bank['phi_hat'], r, (-2, -1)).real
        assert np.abs(p.filter(0, 0, r) - want).max() < 1e-13
    p.close()


def test_filter_bank_1d_matches_oracle():
    n, J, Q = 2048, 5, 4
    p = scat.Scattering((n,), J, Q, host_only=True)
    bank = oracle.bank_1d(n, J, Q)
    for k in range(J * Q):
        assert np.abs(p.filter(1, k, 0) - bank['psi1_hat'][k].real).max() < 1e-12
    for j2 in range(1, J):
        for r in range(j2):
            want = oscat.fold(bank['psi2_hat'][j2], r, (-1,)).real
            assert np.abs(p.filter(2, j2, r) - want).max() < 1e-12
    for r in range(J):
        assert np.abs(p.filter(0, 0, r) - oscat.fold(bank['phi_hat'], r, (-1,)).real).max() < 1e-13
    p.close()


def test_backward_argument_errors_need_no_gpu():
    """scat_backward rejects unsupported grids and bad arguments before
    it touches the GPU (host-only plans are enough to see it)."""
    import paper_1812_11214_amd as scat
    from paper_1812_11214_amd import binding
    L = binding.lib()
    one_d = scat.scat_plan_create_host((1024,), 4, 2)
    tiny = scat.scat_plan_create_host((4, 4), 2, 2)
    big = scat.scat_plan_create_host((1024, 64), 2, 2)
    ok = scat.scat_plan_create_host((64, 64), 2, 2)
    try:
        assert L.scat_backward(one_d, None, None, None, 1, None) == 5      # supported: NULL args
        pad_1d = scat.scat_plan_create_padded_host((1000,), 4, 2)
        assert L.scat_backward(pad_1d, None, None, None, 1, None) == 5     # supported: NULL args
        assert scat.scat_plan_backward_workspace_bytes(pad_1d, 4) > 0
        scat.scat_plan_destroy(pad_1d)
        long_1d = scat.scat_plan_create_host((1 << 20,), 4, 2)             # 1024 x 1024 matrix
        assert L.scat_backward(long_1d, None, None, None, 1, None) == 2    # SCAT_ERR_SHAPE
        scat.scat_plan_destroy(long_1d)
        assert L.scat_backward(tiny, None, None, None, 1, None) == 2       # SCAT_ERR_SHAPE
        assert L.scat_backward(big, None, None, None, 1, None) == 2
        assert L.scat_backward(ok, None, None, None, -1, None) == 1
        assert L.scat_backward(ok, None, None, None, 0, None) == 0         # no-op
        assert L.scat_backward(ok, None, None, None, 1, None) == 5         # SCAT_ERR_NULL
        assert L.scat_backward(None, None, None, None, 1, None) == 5
        assert scat.scat_plan_backward_workspace_bytes(one_d, 4) > scat.scat_plan_workspace_bytes(one_d, 4)
        assert scat.scat_plan_backward_workspace_bytes(ok, 4) > scat.scat_plan_workspace_bytes(ok, 4)
    finally:
        for p in (one_d, tiny, big, ok):
            scat.scat_plan_destroy(p)


def test_reserve_argument_errors_need_no_gpu():
    """scat_plan_reserve: null plan, bad batch, and a host-only plan (no device to reserve on)."""
    import paper_1812_11214_amd as scat
    from paper_1812_11214_amd import binding
    L = binding.lib()
    ok = scat.scat_plan_create_host((64, 64), 2, 2)
    try:
        assert L.scat_plan_reserve(None, 4, 0) == 5   # SCAT_ERR_NULL
        assert L.scat_plan_reserve(ok, 0, 0) == 1     # SCAT_ERR_ARG
        assert L.scat_plan_reserve(ok, 4, 1) == 4     # SCAT_ERR_DEVICE: host-only plan
    finally:
        scat.scat_plan_destroy(ok)
