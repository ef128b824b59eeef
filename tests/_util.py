"""Helpers shared by the tests: error norms and input plumbing (no codec arithmetic)."""
import numpy as np
import scipy.linalg

REL_TOL = 1e-4      # tolerance on the codec: fp32 kernels vs the float64 oracle, relative
ANGLE_TOL = 1e-3    # radians, largest principal angle between fitted bases


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    nb = np.linalg.norm(b)
    return np.linalg.norm(a - b) / nb if nb > 0 else np.linalg.norm(a - b)


def assert_close(a, b, tol=REL_TOL, what=""):
    """||a-b||_2 <= tol ||b||_2  and  max|a-b| <= tol max|b|."""
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    assert a.shape == b.shape, (what, a.shape, b.shape)
    assert np.all(np.isfinite(a)), f"{what}: non-finite values"
    r = rel_l2(a, b)
    assert r <= tol, f"{what}: relative L2 error {r:.3e} > {tol}"
    if b.size:
        m = np.max(np.abs(a - b))
        assert m <= tol * np.max(np.abs(b)) + 1e-30, f"{what}: max abs error {m:.3e} vs max|ref| {np.max(np.abs(b)):.3e}"


def max_angle(U1, U2):
    return float(scipy.linalg.subspace_angles(np.asarray(U1, np.float64), np.asarray(U2, np.float64)).max())


def bf16_bits_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def f64_to_bf16_bits_rne(x):
    """Round float64 values to bf16 (nearest even), returned as uint16 bit patterns."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)  # double rounding is harmless: 24 >> 8 bits
    u = f.view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)
