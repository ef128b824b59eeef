"""float64 CPU oracle of the GradiVeQ slice-wise PCA codec -- TEST INFRASTRUCTURE ONLY.

Thin ctypes front end over ``gvq_oracle.c`` (plain C, double precision, OpenMP over
slices).  Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s CPU-baseline
leg may import this package; the product package ``paper_1811_03617_amd`` never does
and shares no code with it.

All arrays are numpy.  Gradients are 1-D ``float32`` arrays, or ``uint16`` arrays
holding bf16 bit patterns (``dtype="bf16"``).  U is ``[B, d, k]`` float64, mu ``[B, d]``,
eig ``[B, d]`` (B = number of bases); compressed vectors are ``[slices, k]`` float64.

Section 2 of the paper: Eq. (2) compress, Eq. (3) aggregate, Eq. (4) decompress, and the
PCA paragraph after Eq. (4) for the basis (mean, covariance, eigenvectors of the largest
eigenvalues).
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None
_DT = {"f32": 0, "bf16": 1}
MAX_D = 1024


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        vp, i32, i64, dp = C.c_void_p, C.c_int, C.c_int64, C.POINTER(C.c_double)
        L.gvq_oracle_num_threads.restype = i32
        L.gvq_oracle_set_threads.argtypes = [i32]
        L.gvq_oracle_jacobi_eig.argtypes = [dp, dp, i32, C.c_double, i32]
        L.gvq_oracle_jacobi_eig.restype = i32
        L.gvq_oracle_moments.argtypes = [C.POINTER(vp), i32, i64, i32, i32, i64, i64, dp, dp]
        L.gvq_oracle_moments.restype = i64
        L.gvq_oracle_mean.argtypes = [C.POINTER(vp), i32, i64, i32, i32, i64, i64, dp]
        L.gvq_oracle_mean.restype = i64
        L.gvq_oracle_cov_entry.argtypes = [C.POINTER(vp), i32, i64, i32, i32, i64, i64, i32, i32]
        L.gvq_oracle_cov_entry.restype = C.c_double
        L.gvq_oracle_basis_from_cov.argtypes = [dp, i32, i32, dp, dp]
        L.gvq_oracle_basis_from_cov.restype = i32
        L.gvq_oracle_fit.argtypes = [C.POINTER(vp), i32, i64, i32, i32, i32, i32,
                                     C.POINTER(i64), i32, dp, dp, dp, dp]
        L.gvq_oracle_fit.restype = i32
        L.gvq_oracle_compress.argtypes = [vp, i64, i32, i32, i32, i32, C.POINTER(i64), dp, dp,
                                          i32, i64, i64, dp]
        L.gvq_oracle_compress.restype = None
        L.gvq_oracle_aggregate.argtypes = [C.POINTER(dp), i32, i64, dp]
        L.gvq_oracle_aggregate.restype = None
        L.gvq_oracle_decompress.argtypes = [dp, i32, i32, i32, C.POINTER(i64), dp, dp, i64, i64, dp]
        L.gvq_oracle_decompress.restype = None
        L.gvq_oracle_select_k.argtypes = [dp, i32, C.c_double]
        L.gvq_oracle_select_k.restype = i32
        L.gvq_oracle_local_loss.argtypes = [vp, i64, i32, i32, i32, i32, C.POINTER(i64), dp, dp, i32, dp]
        L.gvq_oracle_local_loss.restype = None
        _lib = L
    return _lib


def num_threads() -> int:
    return lib().gvq_oracle_num_threads()


def set_threads(n: int) -> None:
    lib().gvq_oracle_set_threads(int(n))


def _dptr(a):
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _grad(g, dtype):
    want = np.float32 if dtype == "f32" else np.uint16
    g = np.ascontiguousarray(g)
    if g.dtype != want or g.ndim != 1:
        raise TypeError(f"gradient must be a 1-D {want.__name__} array for dtype {dtype}")
    return g


def _grad_ptrs(grads, dtype):
    keep = [_grad(g, dtype) for g in grads]
    M = keep[0].shape[0]
    for g in keep:
        if g.shape[0] != M:
            raise ValueError("all gradients must have the same length")
    arr = (C.c_void_p * len(keep))(*[g.ctypes.data for g in keep])
    return keep, arr, M


def num_slices(M: int, d: int) -> int:
    return (M + d - 1) // d


def _offsets(offsets, S):
    if offsets is None:
        offsets = [0, S]
    o = np.ascontiguousarray(np.asarray(offsets, dtype=np.int64))
    if o[0] != 0 or o[-1] != S or np.any(np.diff(o) <= 0):
        raise ValueError("block offsets must start at 0, end at the slice count and increase")
    return o


def _optr(o):
    return o.ctypes.data_as(C.POINTER(C.c_int64))


def jacobi_eig(A, tol=1e-15, max_sweeps=100):
    """Eigen-decomposition of a symmetric matrix: returns (eigenvalues unsorted, V, sweeps)."""
    A = np.array(A, dtype=np.float64, order="C")
    n = A.shape[0]
    V = np.empty((n, n), dtype=np.float64)
    sweeps = lib().gvq_oracle_jacobi_eig(_dptr(A), _dptr(V), n, tol, max_sweeps)
    return np.diag(A).copy(), V, sweeps


def moments(grads, d, dtype="f32", s0=0, s1=None):
    """Sample mean and 1/n covariance over the full slices [s0, s1) of every gradient."""
    if d > MAX_D:
        raise ValueError("d too large for the oracle")
    keep, arr, M = _grad_ptrs(grads, dtype)
    if s1 is None:
        s1 = M // d
    mu = np.empty(d, dtype=np.float64)
    Cm = np.empty((d, d), dtype=np.float64)
    n = lib().gvq_oracle_moments(arr, len(keep), M, d, _DT[dtype], s0, s1, _dptr(mu), _dptr(Cm))
    return mu, Cm, n


def mean(grads, d, dtype="f32", s0=0, s1=None):
    """Sample mean over the full slices [s0, s1) of every gradient (the mean of `moments`, on its own)."""
    keep, arr, M = _grad_ptrs(grads, dtype)
    if s1 is None:
        s1 = M // d
    mu = np.empty(d, dtype=np.float64)
    lib().gvq_oracle_mean(arr, len(keep), M, d, _DT[dtype], s0, s1, _dptr(mu))
    return mu


def cov_entry(grads, d, a, b, dtype="f32", s0=0, s1=None):
    keep, arr, M = _grad_ptrs(grads, dtype)
    if s1 is None:
        s1 = M // d
    return lib().gvq_oracle_cov_entry(arr, len(keep), M, d, _DT[dtype], s0, s1, a, b)


def basis_from_cov(Cm, k):
    """(U [d,k], eig [d] descending, sweeps) from a covariance matrix."""
    Cm = np.ascontiguousarray(Cm, dtype=np.float64)
    d = Cm.shape[0]
    U = np.empty((d, k), dtype=np.float64)
    eig = np.empty(d, dtype=np.float64)
    sweeps = lib().gvq_oracle_basis_from_cov(_dptr(Cm), d, k, _dptr(U), _dptr(eig))
    return U, eig, sweeps


def fit(grads, d, k, dtype="f32", offsets=None, return_cov=False, first_slice_only=False):
    """Basis refresh: returns U [B,d,k], mu [B,d], eig [B,d] (and C [B,d,d]).
    first_slice_only: the samples of a basis are the L copies of its first slice only (the
    paper's own sampling, Section 3 "compressor reuse") instead of all its slices."""
    if d > MAX_D:
        raise ValueError("d too large for the oracle")
    keep, arr, M = _grad_ptrs(grads, dtype)
    o = _offsets(offsets, num_slices(M, d))
    B = len(o) - 1
    U = np.empty((B, d, k), dtype=np.float64)
    mu = np.empty((B, d), dtype=np.float64)
    eig = np.empty((B, d), dtype=np.float64)
    Cm = np.empty((B, d, d), dtype=np.float64) if return_cov else None
    rc = lib().gvq_oracle_fit(arr, len(keep), M, d, k, _DT[dtype], B, _optr(o), int(bool(first_slice_only)), _dptr(U),
                              _dptr(mu), _dptr(eig), _dptr(Cm) if return_cov else None)
    if rc != 0:
        raise RuntimeError(f"oracle fit failed (rc={rc})")
    return (U, mu, eig, Cm) if return_cov else (U, mu, eig)


def _basis_args(U, mu, d, k, B):
    U = np.ascontiguousarray(U, dtype=np.float64).reshape(B, d, k)
    mu = np.ascontiguousarray(mu, dtype=np.float64).reshape(B, d)
    return U, mu


def compress(grad, U, mu, n_workers, dtype="f32", offsets=None, j0=0, j1=None):
    """Eq. (2) on slices [j0, j1): returns [j1-j0, k] float64."""
    g = _grad(grad, dtype)
    M = g.shape[0]
    U = np.asarray(U)
    d, k = U.shape[-2], U.shape[-1]
    if d > MAX_D:
        raise ValueError("d too large for the oracle")
    S = num_slices(M, d)
    o = _offsets(offsets, S)
    U, mu = _basis_args(U, mu, d, k, len(o) - 1)
    if j1 is None:
        j1 = S
    out = np.empty((j1 - j0, k), dtype=np.float64)
    lib().gvq_oracle_compress(g.ctypes.data, M, d, k, _DT[dtype], len(o) - 1, _optr(o),
                              _dptr(U), _dptr(mu), int(n_workers), j0, j1, _dptr(out))
    return out


def aggregate(comps):
    """Eq. (3): element-wise sum of the workers' compressed vectors."""
    keep = [np.ascontiguousarray(c, dtype=np.float64) for c in comps]
    out = np.empty_like(keep[0])
    arr = (C.POINTER(C.c_double) * len(keep))(*[_dptr(c) for c in keep])
    lib().gvq_oracle_aggregate(arr, len(keep), keep[0].size, _dptr(out))
    return out


def decompress(Y, U, mu, M, offsets=None, j0=0, j1=None):
    """Eq. (4) on slices [j0, j1): returns the reconstructed elements of those slices that
    lie below M, as a 1-D float64 array."""
    U = np.asarray(U)
    d, k = U.shape[-2], U.shape[-1]
    S = num_slices(M, d)
    o = _offsets(offsets, S)
    U, mu = _basis_args(U, mu, d, k, len(o) - 1)
    if j1 is None:
        j1 = S
    Y = np.ascontiguousarray(Y, dtype=np.float64).reshape(j1 - j0, k)
    out = np.empty(((j1 - j0), d), dtype=np.float64)
    lib().gvq_oracle_decompress(_dptr(Y), d, k, len(o) - 1, _optr(o), _dptr(U), _dptr(mu),
                                j0, j1, _dptr(out))
    out = out.reshape(-1)
    valid = min(M, j1 * d) - j0 * d
    return out[:valid]


def select_k(eig, lam):
    """Eq. (5): smallest k whose leading eigenvalues hold at least 1 - lam of the total.
    eig: [d] or [B, d] (descending); returns an int or a list of ints."""
    e = np.ascontiguousarray(eig, dtype=np.float64)
    if e.ndim == 1:
        return lib().gvq_oracle_select_k(_dptr(e), e.shape[0], float(lam))
    return [lib().gvq_oracle_select_k(_dptr(np.ascontiguousarray(row)), e.shape[1], float(lam)) for row in e]


def local_loss(grad, U, mu, n_workers, dtype="f32", offsets=None):
    """Eq. (6): per-basis || g_n - (U g'_n + mu/N) ||^2 of one worker's gradient, [B] float64."""
    g = _grad(grad, dtype)
    M = g.shape[0]
    U = np.asarray(U)
    d, k = U.shape[-2], U.shape[-1]
    if d > MAX_D:
        raise ValueError("d too large for the oracle")
    o = _offsets(offsets, num_slices(M, d))
    B = len(o) - 1
    U, mu = _basis_args(U, mu, d, k, B)
    out = np.empty(B, dtype=np.float64)
    lib().gvq_oracle_local_loss(g.ctypes.data, M, d, k, _DT[dtype], B, _optr(o), _dptr(U), _dptr(mu),
                                int(n_workers), _dptr(out))
    return out


def flatten_conv(grad):
    """Section 2 / Fig. 2a: gradient of a convolution layer stored [F, D, H, W] -> the flat order
    in which the F collocated gradients of the F filters are adjacent and the groups run along
    depth, then width, then height.  Written as the index formula, one element at a time."""
    g = np.asarray(grad)
    F, D, H, W = g.shape
    flat = np.empty(F * D * H * W, dtype=g.dtype)
    for h in range(H):
        for w in range(W):
            for d in range(D):
                base = ((h * W + w) * D + d) * F
                flat[base:base + F] = g[:, d, h, w]
    return flat


def unflatten_conv(flat, F, D, H, W):
    """Inverse of flatten_conv."""
    flat = np.asarray(flat)
    g = np.empty((F, D, H, W), dtype=flat.dtype)
    for h in range(H):
        for w in range(W):
            for d in range(D):
                base = ((h * W + w) * D + d) * F
                g[:, d, h, w] = flat[base:base + F]
    return g
