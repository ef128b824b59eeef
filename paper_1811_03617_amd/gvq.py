"""Thin ctypes binding of libgvq (see include/gvq.h).  Argument marshalling only: every
step of the codec runs in the HIP kernels of the library.  PyTorch appears here solely as
the owner of device memory and streams.

The functions carry the same names as the C entry points; `Basis` is a small convenience
wrapper that keeps the handle alive and fills in sizes.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

F32, BF16 = 0, 1
OK, EINVAL, EALIGN, ENOTFIT, EHIP, ENOMEM, ENONFINITE, ENOCONV, ETOOBIG = 0, -1, -2, -3, -4, -5, -6, -7, -8
STATIC_MAX_SLICES = 1 << 21
MAX_D = 1024

_lib = None


class GvqError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


def lib():
    """Load libgvq.so (building it with hipcc first if it is not there).  Fails loudly when
    the library cannot be built or loaded: there is no other code path."""
    global _lib
    if _lib is None:
        # PyTorch owns the device memory this library works on, so both must talk to the same
        # HIP runtime: load torch (and with it its libamdhip64) before libgvq resolves its own.
        import torch  # noqa: F401
        if not os.path.exists(_build.LIB):
            _build.build()
        elif _build.needs_build():
            import warnings
            warnings.warn("libgvq.so is older than its sources (csrc/ or include/gvq.h): run "
                          "`python -m paper_1811_03617_amd.build` before trusting tests or timings", RuntimeWarning)
        L = C.CDLL(_build.LIB)
        vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
        L.gvq_basis_create.argtypes = [C.POINTER(vp), i64, i32, i32, i32, C.POINTER(i64), i32]
        L.gvq_basis_destroy.argtypes = [vp]
        L.gvq_num_slices.argtypes = [vp]
        L.gvq_num_slices.restype = i64
        L.gvq_fit_basis.argtypes = [vp, C.POINTER(vp), i32, vp]
        L.gvq_fit_basis_first_slice.argtypes = [vp, C.POINTER(vp), i32, vp]
        L.gvq_fit_status.argtypes = [vp, C.POINTER(i32), vp]
        L.gvq_compress.argtypes = [vp, vp, i32, vp, vp]
        L.gvq_aggregate.argtypes = [vp, C.POINTER(vp), i32, vp, vp]
        L.gvq_decompress.argtypes = [vp, vp, vp, i32, vp]
        L.gvq_basis_export.argtypes = [vp, vp, vp, vp]
        L.gvq_basis_export_cov.argtypes = [vp, vp, vp]
        L.gvq_basis_import.argtypes = [vp, vp, vp]
        L.gvq_compress_segment.argtypes = [vp, vp, i32, i64, i64, vp, vp, vp]
        L.gvq_decompress_segment.argtypes = [vp, vp, i64, i64, vp, i32, vp]
        L.gvq_flatten_conv.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        L.gvq_unflatten_conv.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        L.gvq_local_loss.argtypes = [vp, vp, i32, vp, vp]
        L.gvq_local_loss_static.argtypes = [vp, vp, i32, vp, vp]
        L.gvq_select_k.argtypes = [vp, C.c_double, C.POINTER(i32), vp]
        L.gvq_strerror.argtypes = [i32]
        L.gvq_strerror.restype = C.c_char_p
        L.gvq_set_option.argtypes = [i32, i32]
        for name in ("gvq_basis_create", "gvq_basis_destroy", "gvq_fit_basis", "gvq_fit_status",
                     "gvq_compress", "gvq_aggregate", "gvq_decompress", "gvq_basis_export",
                     "gvq_basis_export_cov", "gvq_basis_import", "gvq_set_option", "gvq_local_loss",
                     "gvq_select_k", "gvq_compress_segment", "gvq_decompress_segment", "gvq_flatten_conv",
                     "gvq_unflatten_conv", "gvq_fit_basis_first_slice", "gvq_local_loss_static"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().gvq_strerror(int(status)).decode()


def _ptr(x):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    raise TypeError(type(x))


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return int(stream)


def _check(status, where):
    if status != OK:
        raise GvqError(status, where)


# ---- the C entry points, same names, raw arguments ---------------------------------------
def gvq_basis_create(n_elems, d, k, block_slice_offsets=None, grad_dtype=F32):
    h = C.c_void_p()
    if block_slice_offsets is None:
        nb, offs = 1, None
    else:
        nb = len(block_slice_offsets) - 1
        offs = (C.c_int64 * (nb + 1))(*[int(o) for o in block_slice_offsets])
    _check(lib().gvq_basis_create(C.byref(h), int(n_elems), int(d), int(k), nb, offs, int(grad_dtype)),
           "gvq_basis_create")
    return h


def gvq_basis_destroy(h):
    _check(lib().gvq_basis_destroy(h), "gvq_basis_destroy")


def gvq_num_slices(h):
    return lib().gvq_num_slices(h)


def gvq_fit_basis(h, grads, stream=None):
    arr = (C.c_void_p * len(grads))(*[_ptr(g) for g in grads])
    _check(lib().gvq_fit_basis(h, arr, len(grads), _stream(stream)), "gvq_fit_basis")


def gvq_fit_basis_first_slice(h, grads, stream=None):
    arr = (C.c_void_p * len(grads))(*[_ptr(g) for g in grads])
    _check(lib().gvq_fit_basis_first_slice(h, arr, len(grads), _stream(stream)), "gvq_fit_basis_first_slice")


def gvq_fit_status(h, stream=None):
    sw = C.c_int(0)
    _check(lib().gvq_fit_status(h, C.byref(sw), _stream(stream)), "gvq_fit_status")
    return sw.value


def gvq_compress(h, grad, n_workers, comp_out, stream=None):
    _check(lib().gvq_compress(h, _ptr(grad), int(n_workers), _ptr(comp_out), _stream(stream)),
           "gvq_compress")


def gvq_aggregate(h, comps, comp_sum, stream=None):
    arr = (C.c_void_p * len(comps))(*[_ptr(c) for c in comps])
    _check(lib().gvq_aggregate(h, arr, len(comps), _ptr(comp_sum), _stream(stream)), "gvq_aggregate")


def gvq_decompress(h, comp_sum, grad_out, out_dtype=F32, stream=None):
    _check(lib().gvq_decompress(h, _ptr(comp_sum), _ptr(grad_out), int(out_dtype), _stream(stream)),
           "gvq_decompress")


def gvq_compress_segment(h, grad, n_workers, first_slice, n_slices, comp_in, comp_out, stream=None):
    _check(lib().gvq_compress_segment(h, _ptr(grad), int(n_workers), int(first_slice), int(n_slices),
                                      _ptr(comp_in), _ptr(comp_out), _stream(stream)), "gvq_compress_segment")


def gvq_decompress_segment(h, comp_sum, first_slice, n_slices, grad_out, out_dtype=F32, stream=None):
    _check(lib().gvq_decompress_segment(h, _ptr(comp_sum), int(first_slice), int(n_slices), _ptr(grad_out),
                                        int(out_dtype), _stream(stream)), "gvq_decompress_segment")


def gvq_flatten_conv(grad, flat, F, D, H, W, dtype=F32, stream=None):
    _check(lib().gvq_flatten_conv(_ptr(grad), _ptr(flat), F, D, H, W, int(dtype), _stream(stream)), "gvq_flatten_conv")


def gvq_unflatten_conv(flat, grad, F, D, H, W, dtype=F32, stream=None):
    _check(lib().gvq_unflatten_conv(_ptr(flat), _ptr(grad), F, D, H, W, int(dtype), _stream(stream)),
           "gvq_unflatten_conv")


def gvq_local_loss(h, grad, n_workers, loss_out, stream=None):
    _check(lib().gvq_local_loss(h, _ptr(grad), int(n_workers), _ptr(loss_out), _stream(stream)), "gvq_local_loss")


def gvq_local_loss_static(h, grad, n_workers, loss_out, stream=None):
    _check(lib().gvq_local_loss_static(h, _ptr(grad), int(n_workers), _ptr(loss_out), _stream(stream)),
           "gvq_local_loss_static")


def gvq_select_k(h, lam, n_bases, stream=None):
    out = (C.c_int * n_bases)()
    _check(lib().gvq_select_k(h, float(lam), out, _stream(stream)), "gvq_select_k")
    return list(out)


def gvq_set_option(option, value):
    _check(lib().gvq_set_option(int(option), int(value)), "gvq_set_option")


class Basis:
    """Owns one gvq_basis_t.  M elements per gradient, slice length d, k kept components."""

    def __init__(self, M, d, k, block_slice_offsets=None, dtype="f32"):
        self.M, self.d, self.k = int(M), int(d), int(k)
        self.dtype = dtype
        self.B = 1 if block_slice_offsets is None else len(block_slice_offsets) - 1
        self._h = gvq_basis_create(M, d, k, block_slice_offsets, BF16 if dtype == "bf16" else F32)
        self.S = gvq_num_slices(self._h)

    def close(self):
        if self._h is not None:
            gvq_basis_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    def fit(self, grads, stream=None, first_slice_only=False):
        if first_slice_only:
            gvq_fit_basis_first_slice(self._h, grads, stream)
        else:
            gvq_fit_basis(self._h, grads, stream)

    def fit_status(self, stream=None):
        return gvq_fit_status(self._h, stream)

    def compress(self, grad, n_workers, comp_out, stream=None):
        gvq_compress(self._h, grad, n_workers, comp_out, stream)

    def aggregate(self, comps, comp_sum, stream=None):
        gvq_aggregate(self._h, comps, comp_sum, stream)

    def decompress(self, comp_sum, grad_out, out_dtype=None, stream=None):
        if out_dtype is None:
            out_dtype = self.dtype
        gvq_decompress(self._h, comp_sum, grad_out, BF16 if out_dtype == "bf16" else F32, stream)

    def compress_segment(self, grad, n_workers, first_slice, n_slices, comp_in, comp_out, stream=None):
        gvq_compress_segment(self._h, grad, n_workers, first_slice, n_slices, comp_in, comp_out, stream)

    def decompress_segment(self, comp_sum, first_slice, n_slices, grad_out, out_dtype=None, stream=None):
        if out_dtype is None:
            out_dtype = self.dtype
        gvq_decompress_segment(self._h, comp_sum, first_slice, n_slices, grad_out,
                               BF16 if out_dtype == "bf16" else F32, stream)

    def local_loss(self, grad, n_workers, loss_out, stream=None):
        gvq_local_loss(self._h, grad, n_workers, loss_out, stream)

    def local_loss_static(self, grad, n_workers, loss_out, stream=None):
        gvq_local_loss_static(self._h, grad, n_workers, loss_out, stream)

    def select_k(self, lam, stream=None):
        return gvq_select_k(self._h, lam, self.B, stream)

    def export(self):
        U = np.empty((self.B, self.d, self.k), dtype=np.float32)
        mu = np.empty((self.B, self.d), dtype=np.float32)
        eig = np.empty((self.B, self.d), dtype=np.float64)
        _check(lib().gvq_basis_export(self._h, U.ctypes.data, mu.ctypes.data, eig.ctypes.data),
               "gvq_basis_export")
        return U, mu, eig

    def export_cov(self):
        cov = np.empty((self.B, self.d, self.d), dtype=np.float64)
        n = np.empty(self.B, dtype=np.int64)
        _check(lib().gvq_basis_export_cov(self._h, cov.ctypes.data, n.ctypes.data), "gvq_basis_export_cov")
        return cov, n

    def import_(self, U, mu):
        U = np.ascontiguousarray(U, dtype=np.float32).reshape(self.B, self.d, self.k)
        mu = np.ascontiguousarray(mu, dtype=np.float32).reshape(self.B, self.d)
        _check(lib().gvq_basis_import(self._h, U.ctypes.data, mu.ctypes.data), "gvq_basis_import")
