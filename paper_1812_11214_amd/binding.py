"""ctypes binding of libscat.so: argument marshalling only.

The functions carry the names of the C entry points declared in include/scat.h.
Every step of the transform runs in the library's HIP kernels; torch is used for
device memory and streams only.  If the shared library has not been built the
binding raises -- there is no CPU fallback.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libscat.so")

SCAT_OK = 0
_lib = None


class ScatError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: %s (status %d)" % (where, scat_status_string(status), status))


def lib():
    """Load (once) and return the ctypes handle of libscat.so."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "%s is missing: build it with `python -m paper_1812_11214_amd.build` "
            "(there is no fallback implementation)" % LIB_PATH)
    L = ctypes.CDLL(LIB_PATH)
    vp, ci, cl = ctypes.c_void_p, ctypes.c_int, ctypes.c_long
    pi = ctypes.POINTER(ctypes.c_int)
    L.scat_plan_create.argtypes = [ctypes.POINTER(vp), ci, pi, ci, ci, ci]
    L.scat_plan_create.restype = ci
    L.scat_plan_create_host.argtypes = [ctypes.POINTER(vp), ci, pi, ci, ci, ci]
    L.scat_plan_create_host.restype = ci
    L.scat_plan_create_padded.argtypes = [ctypes.POINTER(vp), ci, pi, ci, ci, ci]
    L.scat_plan_create_padded.restype = ci
    L.scat_plan_create_padded_host.argtypes = [ctypes.POINTER(vp), ci, pi, ci, ci, ci]
    L.scat_plan_create_padded_host.restype = ci
    L.scat_plan_create_ex.argtypes = [ctypes.POINTER(vp), ci, pi, ci, ci, ci, ci, ci]
    L.scat_plan_create_ex.restype = ci
    L.scat_plan_grid_shape.argtypes = [vp, pi]
    L.scat_plan_grid_shape.restype = ci
    L.scat_forward.argtypes = [vp, vp, vp, cl, vp]
    L.scat_forward.restype = ci
    L.scat_forward_static.argtypes = [vp, vp, vp, cl, vp]
    L.scat_forward_static.restype = ci
    L.scat_plan_reserve.argtypes = [vp, cl, ci]
    L.scat_plan_reserve.restype = ci
    L.scat_backward.argtypes = [vp, vp, vp, vp, cl, vp]
    L.scat_backward.restype = ci
    L.scat_plan_backward_workspace_bytes.argtypes = [vp, cl]
    L.scat_plan_backward_workspace_bytes.restype = ctypes.c_size_t
    L.scat_plan_destroy.argtypes = [vp]
    L.scat_plan_destroy.restype = ci
    L.scat_plan_num_coeffs.argtypes = [vp]
    L.scat_plan_num_coeffs.restype = ci
    L.scat_plan_out_shape.argtypes = [vp, pi]
    L.scat_plan_out_shape.restype = ci
    L.scat_plan_coeff_index.argtypes = [vp, ci, pi]
    L.scat_plan_coeff_index.restype = ci
    L.scat_plan_workspace_bytes.argtypes = [vp, cl]
    L.scat_plan_workspace_bytes.restype = ctypes.c_size_t
    L.scat_plan_filter.argtypes = [vp, ci, ci, ci, ctypes.POINTER(ctypes.c_double)]
    L.scat_plan_filter.restype = ci
    L.scat_plan_timing_begin.argtypes = [vp, ctypes.c_char_p]
    L.scat_plan_timing_begin.restype = ci
    L.scat_plan_timing_end.argtypes = [vp]
    L.scat_plan_timing_end.restype = ci
    L.scat_plan_timing_row.argtypes = [vp, ci, ctypes.c_char_p, ctypes.c_size_t,
                                       ctypes.POINTER(cl), ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(ctypes.c_double)]
    L.scat_plan_timing_row.restype = ci
    L.scat_status_string.argtypes = [ci]
    L.scat_status_string.restype = ctypes.c_char_p
    _lib = L
    return L


EXPORTS = ("scat_plan_create", "scat_plan_create_host", "scat_forward", "scat_plan_destroy",
           "scat_plan_num_coeffs", "scat_plan_out_shape", "scat_plan_coeff_index",
           "scat_plan_workspace_bytes", "scat_plan_filter", "scat_status_string",
           "scat_plan_timing_begin", "scat_plan_timing_end", "scat_plan_timing_row",
           "scat_backward", "scat_plan_backward_workspace_bytes", "scat_plan_create_padded",
           "scat_plan_create_padded_host", "scat_plan_grid_shape", "scat_plan_create_ex",
           "scat_forward_static", "scat_plan_reserve")


def scat_status_string(status):
    return lib().scat_status_string(int(status)).decode()


def _create(fn, shape, J, LQ, max_order):
    shape = tuple(int(s) for s in shape)
    arr = (ctypes.c_int * len(shape))(*shape)
    handle = ctypes.c_void_p()
    st = fn(ctypes.byref(handle), len(shape), arr, int(J), int(LQ), int(max_order))
    if st != SCAT_OK:
        raise ScatError(st, fn.__name__)
    return handle


def scat_plan_create(shape, J, LQ, max_order=2):
    """Plan for signals of `shape` on the current GPU; returns a handle.  1 or 2 sides: the
    Morlet cascade; 3 sides: solid harmonic scattering, LQ = the largest degree L."""
    return _create(lib().scat_plan_create, shape, J, LQ, max_order)


SCAT_PLAN_PADDED = 1
SCAT_PLAN_HOST_ONLY = 2
SCAT_PLAN_NODE_KERNELS = 4
SCAT_PLAN_PASS_KERNELS = 8


def scat_plan_create_ex(shape, J, LQ, max_order=2, oversampling=0, flags=0):
    """General plan creation: oversampling >= 0, flags = SCAT_PLAN_PADDED | SCAT_PLAN_HOST_ONLY |
    SCAT_PLAN_NODE_KERNELS | SCAT_PLAN_PASS_KERNELS."""
    shape = tuple(int(s) for s in shape)
    arr = (ctypes.c_int * len(shape))(*shape)
    handle = ctypes.c_void_p()
    st = lib().scat_plan_create_ex(ctypes.byref(handle), len(shape), arr, int(J), int(LQ),
                                   int(max_order), int(oversampling), int(flags))
    if st != SCAT_OK:
        raise ScatError(st, "scat_plan_create_ex")
    return handle


def scat_plan_create_padded(shape, J, LQ, max_order=2):
    """Plan for signals of any `shape` (symmetric extension to a periodic grid)."""
    return _create(lib().scat_plan_create_padded, shape, J, LQ, max_order)


def scat_plan_create_padded_host(shape, J, LQ, max_order=2):
    return _create(lib().scat_plan_create_padded_host, shape, J, LQ, max_order)


def scat_plan_grid_shape(plan, dims):
    arr = (ctypes.c_int * dims)()
    st = lib().scat_plan_grid_shape(plan, arr)
    if st != SCAT_OK:
        raise ScatError(st, "scat_plan_grid_shape")
    return tuple(arr)


def scat_plan_create_host(shape, J, LQ, max_order=2):
    """Plan with host tables only (no GPU touched)."""
    return _create(lib().scat_plan_create_host, shape, J, LQ, max_order)


def scat_plan_destroy(plan):
    st = lib().scat_plan_destroy(plan)
    if st != SCAT_OK:
        raise ScatError(st, "scat_plan_destroy")


def scat_plan_num_coeffs(plan):
    return lib().scat_plan_num_coeffs(plan)


def scat_plan_out_shape(plan, dims):
    arr = (ctypes.c_int * dims)()
    st = lib().scat_plan_out_shape(plan, arr)
    if st != SCAT_OK:
        raise ScatError(st, "scat_plan_out_shape")
    return tuple(arr)


def scat_plan_coeff_index(plan, c):
    arr = (ctypes.c_int * 5)()
    st = lib().scat_plan_coeff_index(plan, int(c), arr)
    if st != SCAT_OK:
        raise ScatError(st, "scat_plan_coeff_index")
    return tuple(arr)


def scat_plan_workspace_bytes(plan, batch):
    return int(lib().scat_plan_workspace_bytes(plan, int(batch)))


def scat_plan_backward_workspace_bytes(plan, batch):
    return int(lib().scat_plan_backward_workspace_bytes(plan, int(batch)))


def scat_backward(plan, in_ptr, grad_out_ptr, grad_in_ptr, batch, stream_ptr=None):
    """Enqueue the backward pass; the pointers are device addresses (ints)."""
    st = lib().scat_backward(plan, ctypes.c_void_p(in_ptr), ctypes.c_void_p(grad_out_ptr),
                             ctypes.c_void_p(grad_in_ptr), int(batch),
                             ctypes.c_void_p(stream_ptr) if stream_ptr else None)
    if st != SCAT_OK:
        raise ScatError(st, "scat_backward")


def scat_plan_filter(plan, kind, index, res, shape):
    """Unscaled Fourier samples of one filter as a float64 array of `shape`."""
    out = np.empty(shape, dtype=np.float64)
    st = lib().scat_plan_filter(plan, int(kind), int(index), int(res),
                                out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if st != SCAT_OK:
        raise ScatError(st, "scat_plan_filter")
    return out


def scat_plan_timing_begin(plan, kernel_name=None):
    st = lib().scat_plan_timing_begin(plan, kernel_name.encode() if kernel_name else None)
    if st != SCAT_OK:
        raise ScatError(st, "scat_plan_timing_begin")


def scat_plan_timing_end(plan):
    """Stop recording; returns {kernel name: dict(launches, ms, alg_bytes, model_flops)}."""
    n = lib().scat_plan_timing_end(plan)
    if n < 0:
        raise ScatError(4, "scat_plan_timing_end")
    out = {}
    for r in range(n):
        name = ctypes.create_string_buffer(128)
        launches = ctypes.c_long()
        ms, by, fl = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
        st = lib().scat_plan_timing_row(plan, r, name, 128, ctypes.byref(launches),
                                        ctypes.byref(ms), ctypes.byref(by), ctypes.byref(fl))
        if st != SCAT_OK:
            raise ScatError(st, "scat_plan_timing_row")
        out[name.value.decode()] = dict(launches=launches.value, ms=ms.value,
                                        alg_bytes=by.value, model_flops=fl.value)
    return out


def scat_plan_timing_row(plan, row):
    """One row of the last timing table as (name, launches, ms, alg_bytes, model_flops)."""
    name = ctypes.create_string_buffer(128)
    launches = ctypes.c_long()
    ms, by, fl = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    st = lib().scat_plan_timing_row(plan, int(row), name, 128, ctypes.byref(launches),
                                    ctypes.byref(ms), ctypes.byref(by), ctypes.byref(fl))
    if st != SCAT_OK:
        raise ScatError(st, "scat_plan_timing_row")
    return name.value.decode(), launches.value, ms.value, by.value, fl.value


def scat_forward(plan, in_ptr, out_ptr, batch, stream_ptr=None):
    """Raw call: device addresses as integers, stream as a hipStream_t integer or None."""
    st = lib().scat_forward(plan, ctypes.c_void_p(in_ptr), ctypes.c_void_p(out_ptr), int(batch),
                            ctypes.c_void_p(stream_ptr) if stream_ptr else None)
    if st != SCAT_OK:
        raise ScatError(st, "scat_forward")


SCAT_STATIC_SCRATCH_MB = 64
SCAT_ERR_WORKSPACE = 6


def scat_forward_static(plan, in_ptr, out_ptr, batch, stream_ptr=None):
    """scat_forward without any allocation: intermediates in the library's static buffer."""
    st = lib().scat_forward_static(plan, ctypes.c_void_p(in_ptr), ctypes.c_void_p(out_ptr),
                                   int(batch), ctypes.c_void_p(stream_ptr) if stream_ptr else None)
    if st != SCAT_OK:
        raise ScatError(st, "scat_forward_static")


def scat_plan_reserve(plan, batch, with_backward=False):
    """Grow the plan's scratch now so that later calls of up to `batch` planes do not allocate."""
    st = lib().scat_plan_reserve(plan, int(batch), 1 if with_backward else 0)
    if st != SCAT_OK:
        raise ScatError(st, "scat_plan_reserve")


class Scattering:
    """Owner of one plan.  `forward` takes a contiguous float32 CUDA tensor whose trailing
    dims equal `shape`; all leading dims are independent planes.  One or two sides: the Morlet
    cascade (LQ = wavelets per octave Q / number of angles L); three sides: solid harmonic
    scattering (LQ = the largest degree L)."""

    def __init__(self, shape, J, LQ, max_order=2, host_only=False, padded=False, oversampling=0,
                 node_kernels=True):
        """padded=True: signals of any size, extended symmetrically to a periodic grid of
        power-of-two sides (scat_plan_create_padded); else `shape` is that periodic grid.
        oversampling=o: every signal 2^o times finer than the default schedule.
        node_kernels=False: 256x256/J=3 and 128x128/J=2 plans, which by default walk the tree one
        workgroup per node, use the row and column passes instead (SCAT_PLAN_PASS_KERNELS)."""
        self.shape = tuple(int(s) for s in shape)
        self.dims = len(self.shape)
        self.J, self.LQ, self.max_order = int(J), int(LQ), int(max_order)
        self.padded = bool(padded)
        self._plan = None
        self.oversampling = int(oversampling)
        flags = ((SCAT_PLAN_PADDED if padded else 0) | (SCAT_PLAN_HOST_ONLY if host_only else 0)
                 | (0 if node_kernels else SCAT_PLAN_PASS_KERNELS))
        self._plan = scat_plan_create_ex(self.shape, J, LQ, max_order, oversampling, flags)
        self.K = scat_plan_num_coeffs(self._plan)
        self.out_shape = scat_plan_out_shape(self._plan, self.dims)
        self.grid_shape = scat_plan_grid_shape(self._plan, self.dims)

    def coeff_index(self):
        return [scat_plan_coeff_index(self._plan, c) for c in range(self.K)]

    def workspace_bytes(self, batch):
        return scat_plan_workspace_bytes(self._plan, batch)

    def filter(self, kind, index, res=0):
        """Unscaled Fourier samples of one filter.  3-D plans: kind 0 is the lowpass, kind 1
        with index j (L+1) + l the 2l+1 real solid harmonic tables of that scale and degree."""
        shp = tuple(s >> res for s in self.grid_shape)
        if self.dims == 3 and kind == 1:
            shp = (2 * (int(index) % (self.LQ + 1)) + 1,) + shp
        return scat_plan_filter(self._plan, kind, index, res, shp)

    def forward(self, x, out=None):
        import torch
        if not (x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()):
            raise ValueError("input must be a contiguous float32 CUDA tensor")
        if tuple(x.shape[x.dim() - self.dims:]) != self.shape:
            raise ValueError("trailing dims %s do not match the plan's shape %s"
                             % (tuple(x.shape), self.shape))
        lead = tuple(x.shape[:x.dim() - self.dims])
        batch = 1
        for d in lead:
            batch *= d
        oshape = lead + (self.K,) + self.out_shape
        if out is None:
            out = torch.empty(oshape, dtype=torch.float32, device=x.device)
        elif not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous()
                  and tuple(out.shape) == oshape):
            raise ValueError("out must be a contiguous float32 CUDA tensor of shape %s" % (oshape,))
        stream = torch.cuda.current_stream(x.device).cuda_stream
        scat_forward(self._plan, x.data_ptr(), out.data_ptr(), batch, stream)
        return out

    def backward(self, x, grad_out, grad_in=None):
        """Gradient of sum(grad_out * forward(x)) with respect to x."""
        import torch
        for t, nm in ((x, "x"), (grad_out, "grad_out")):
            if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
                raise ValueError("%s must be a contiguous float32 CUDA tensor" % nm)
        if tuple(x.shape[x.dim() - self.dims:]) != self.shape:
            raise ValueError("trailing dims %s do not match the plan's shape %s"
                             % (tuple(x.shape), self.shape))
        lead = tuple(x.shape[:x.dim() - self.dims])
        batch = 1
        for d in lead:
            batch *= d
        if tuple(grad_out.shape) != lead + (self.K,) + self.out_shape:
            raise ValueError("grad_out must have shape %s" % (lead + (self.K,) + self.out_shape,))
        if grad_in is None:
            grad_in = torch.empty_like(x)
        elif not (grad_in.is_cuda and grad_in.dtype == torch.float32 and grad_in.is_contiguous()
                  and grad_in.shape == x.shape):
            raise ValueError("grad_in must be a contiguous float32 CUDA tensor shaped like x")
        stream = torch.cuda.current_stream(x.device).cuda_stream
        scat_backward(self._plan, x.data_ptr(), grad_out.data_ptr(), grad_in.data_ptr(), batch,
                      stream)
        return grad_in

    def backward_workspace_bytes(self, batch):
        return scat_plan_backward_workspace_bytes(self._plan, batch)

    def reserve(self, batch, with_backward=False):
        scat_plan_reserve(self._plan, batch, with_backward)

    def timing_begin(self, kernel_name=None):
        scat_plan_timing_begin(self._plan, kernel_name)

    def timing_end(self):
        return scat_plan_timing_end(self._plan)

    def close(self):
        if self._plan is not None:
            scat_plan_destroy(self._plan)
            self._plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
