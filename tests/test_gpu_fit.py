"""Parity of the HIP basis refresh (gvq_fit_basis) with the float64 oracle."""
import numpy as np
import pytest

import oracle
from paper_1811_03617_amd import Workload, gvq, synth
from _util import ANGLE_TOL, assert_close, max_angle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _wl(M, d, k, N, L, dtype="f32", rank=3, block_elems=0, seed=11, sigma=0.05):
    return Workload("t", M, d, k, N, L, dtype, rank, sigma, block_elems=block_elems, seed=seed)


def _fit_both(w, mean_offset=None):
    fit = synth.fit_gradients(w, "cpu", mean_offset=mean_offset)
    fit_np = [synth.to_numpy(g) for g in fit]
    offs = w.block_offsets()
    Uo, muo, eigo, Co = oracle.fit(fit_np, w.d, w.k, dtype=w.dtype, offsets=offs, return_cov=True)
    b = gvq.Basis(w.M, w.d, w.k, offs, w.dtype)
    dev = [g.to(DEV) for g in fit]
    b.fit(dev)
    sweeps = b.fit_status()
    U, mu, eig = b.export()
    C, n = b.export_cov()
    b.close()
    return (Uo, muo, eigo, Co), (U, mu, eig, C, n, sweeps)


def _check_fit(w, mean_offset=None, angle_rank=None):
    (Uo, muo, eigo, Co), (U, mu, eig, C, n, sweeps) = _fit_both(w, mean_offset)
    assert 0 <= sweeps < 40
    full = w.M // w.d
    offs = w.block_offsets() or [0, w.S]
    for b in range(len(offs) - 1):
        cnt = max(0, min(offs[b + 1], full) - offs[b])
        assert n[b] == cnt * w.L
        lam1 = eigo[b][0]
        scale = max(lam1, np.max(np.abs(muo[b])) ** 2)
        np.testing.assert_allclose(mu[b], muo[b], rtol=2e-7, atol=1e-12 + 1e-7 * np.max(np.abs(muo[b])))
        # covariance: float64 on both sides; one-pass vs two-pass differ by rounding only
        assert np.max(np.abs(C[b] - Co[b])) <= 1e-11 * scale
        assert np.array_equal(C[b], C[b].T)
        np.testing.assert_allclose(eig[b], eigo[b], rtol=0, atol=1e-10 * scale)
        assert np.all(np.diff(eig[b]) <= 0)
        # basis: orthonormal to fp32 rounding, and the same subspace as the oracle's
        Ub = U[b].astype(np.float64)
        assert np.max(np.abs(Ub.T @ Ub - np.eye(w.k))) < 1e-5
        kk = w.k if angle_rank is None else angle_rank
        assert max_angle(Ub[:, :kk], Uo[b][:, :kk]) < ANGLE_TOL
        # sign convention: largest-magnitude entry of every column is positive
        for i in range(w.k):
            assert Ub[np.argmax(np.abs(Ub[:, i])), i] > 0
        # sign-aligned columns agree where the eigenvalue is well separated
        for i in range(w.k):
            gap = min(abs(eigo[b][i] - eigo[b][j]) for j in range(w.d) if j != i)
            if gap > 1e-3 * lam1:
                s = np.sign(np.dot(Ub[:, i], Uo[b][:, i]))
                assert np.max(np.abs(s * Ub[:, i] - Uo[b][:, i])) < 1e-5


@pytest.mark.parametrize("M,d,k,N,L", [
    (16 * 5000, 16, 4, 4, 8),
    (32 * 3000 + 8, 32, 8, 2, 4),
    (64 * 2000 + 40, 64, 16, 2, 3),
    (128 * 1500 + 40, 128, 32, 2, 3),
    (24 * 1000 + 7, 24, 5, 2, 3),       # d not a power of two
    (7 * 999, 7, 7, 2, 2),              # odd d, k = d
    (2 * 500, 2, 1, 1, 1),
    (127 * 300, 127, 9, 2, 2),          # odd d close to the maximum
])
def test_fit_parity(M, d, k, N, L):
    _check_fit(_wl(M, d, k, N, L, rank=min(3, d - 1)))


def test_fit_parity_nonzero_mean():
    w = _wl(32 * 4000 + 5, 32, 8, 4, 4)
    _check_fit(w, mean_offset=np.linspace(-3.0, 4.0, 32))


def test_fit_parity_more_gradients_than_one_launch():
    _check_fit(_wl(16 * 800, 16, 4, 1, 37))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fit_parity_many_bases(dtype):
    _check_fit(_wl(128 * 700 + 40, 128, 16, 2, 3, dtype=dtype, block_elems=128 * 100, rank=5))
    _check_fit(_wl(32 * 900 + 1, 32, 4, 2, 3, dtype=dtype, block_elems=32 * 128, rank=2))


def test_fit_is_bitwise_reproducible():
    w = _wl(64 * 3000 + 40, 64, 16, 2, 3)
    a = _fit_both(w)[1]
    b = _fit_both(w)[1]
    for x, y in zip(a[:4], b[:4]):
        assert np.array_equal(x, y)


def test_block_without_full_slice_gets_the_trivial_basis():
    # last basis covers only the partial tail slice
    M, d, k = 16 * 10 + 3, 16, 4
    offs = [0, 10, 11]
    fit = [torch.randn(M, generator=torch.Generator().manual_seed(3)).to(DEV)]
    b = gvq.Basis(M, d, k, offs)
    b.fit(fit)
    b.fit_status()
    U, mu, eig = b.export()
    _, n = b.export_cov()
    assert n[1] == 0 and np.all(mu[1] == 0) and np.all(eig[1] == 0)
    np.testing.assert_array_equal(U[1], np.eye(d, k, dtype=np.float32))
    b.close()


@pytest.mark.parametrize("d", [16, 192])   # the eigensolver in LDS, and the one out of global memory
def test_fit_reports_non_finite_input(d):
    import ctypes as C
    M, k = d * 200, 4
    g = torch.randn(M, generator=torch.Generator().manual_seed(4))
    g[37] = float("nan")
    b = gvq.Basis(M, d, k)
    b.fit([g.to(DEV)])
    with pytest.raises(gvq.GvqError) as ei:
        b.fit_status()
    assert ei.value.status == gvq.ENONFINITE
    # both routes record "no convergence" for the basis, so no sweep count is reported for it
    sw = C.c_int(-5)
    rc = gvq.lib().gvq_fit_status(b.handle, C.byref(sw), torch.cuda.current_stream().cuda_stream)
    assert rc == gvq.ENONFINITE and sw.value == 0
    b.close()


def test_fit_then_codec_end_to_end_loss_matches_discarded_eigenvalues():
    """Eq. (5) on the device: compressing the fit set with N = 1 loses exactly the mass of
    the discarded eigenvalues (checked against the library's own eig, fp32 codec)."""
    w = _wl(64 * 3000, 64, 8, 1, 2, rank=5, sigma=0.2)
    fit = [g.to(DEV) for g in synth.fit_gradients(w, "cpu")]
    b = gvq.Basis(w.M, w.d, w.k)
    b.fit(fit)
    _, _, eig = b.export()
    err = 0.0
    for g in fit:
        y = torch.empty(b.S * w.k, device=DEV)
        out = torch.empty(w.M, device=DEV)
        b.compress(g, 1, y)
        b.decompress(y, out)
        err += float(((out.double() - g.double()) ** 2).sum().item())
    b.close()
    lost = eig[0][w.k:].sum()
    assert abs(err / (len(fit) * w.S) - lost) < 1e-4 * eig[0].sum()


@pytest.mark.parametrize("M,d,k,L,block_elems,dtype", [
    (64 * 400, 64, 8, 100, 64 * 50, "f32"),      # the paper's L_t = 100 time samples, 8 bases
    (128 * 300 + 40, 128, 16, 40, 128 * 64, "bf16"),   # fewer samples than dimensions
    (16 * 900 + 3, 16, 4, 37, 0, "f32"),
    (24 * 100, 24, 5, 9, 24 * 30, "f32"),
])
def test_fit_first_slice_sampling_mode(M, d, k, L, block_elems, dtype):
    """Section 3 'compressor reuse': L time samples of the first slice of every basis."""
    w = _wl(M, d, k, 2, L, dtype=dtype, block_elems=block_elems, rank=min(6, d // 2), sigma=0.3)
    fit = synth.fit_gradients(w, "cpu")
    offs = w.block_offsets()
    Uo, muo, eigo, Co = oracle.fit([synth.to_numpy(g) for g in fit], d, k, dtype=dtype, offsets=offs,
                                   first_slice_only=True, return_cov=True)
    b = gvq.Basis(M, d, k, offs, dtype)
    b.fit([g.to(DEV) for g in fit], first_slice_only=True)
    assert 0 <= b.fit_status() < 40
    U, mu, eig = b.export()
    C, n = b.export_cov()
    b.close()
    for bb in range(w.n_blocks):
        assert n[bb] == L
        lam1 = eigo[bb][0]
        np.testing.assert_allclose(mu[bb], muo[bb], rtol=2e-7, atol=1e-7 * np.sqrt(lam1))
        assert np.max(np.abs(C[bb] - Co[bb])) <= 1e-12 * lam1
        np.testing.assert_allclose(eig[bb], eigo[bb], rtol=0, atol=1e-11 * lam1)
        kk = min(k, L - 1)                      # what the data determines
        # leave out columns whose eigenvalue is not separated from its neighbours
        while kk > 1 and eigo[bb][kk - 1] - eigo[bb][kk] < 1e-6 * lam1:
            kk -= 1
        assert max_angle(U[bb][:, :kk].astype(np.float64), Uo[bb][:, :kk]) < ANGLE_TOL
        Ub = U[bb].astype(np.float64)
        assert np.max(np.abs(Ub.T @ Ub - np.eye(k))) < 1e-5


def test_fit_degenerate_inputs():
    """Constant gradients (zero covariance) and rank-one data (all but one eigenvalue zero)."""
    M, d, k = 32 * 500, 32, 4
    const = [torch.full((M,), 0.75), torch.full((M,), 0.75)]
    Uo, muo, eigo = oracle.fit([synth.to_numpy(g) for g in const], d, k)
    b = gvq.Basis(M, d, k)
    b.fit([g.to(DEV) for g in const])
    assert b.fit_status() == 0
    U, mu, eig = b.export()
    assert np.all(eig == 0) and np.all(eigo == 0)
    np.testing.assert_array_equal(mu[0], np.full(d, 0.75, np.float32))
    np.testing.assert_array_equal(U[0], np.eye(d, k, dtype=np.float32))
    np.testing.assert_array_equal(Uo[0], np.eye(d, k))
    # rank one: every slice is a multiple of one direction v, with zero mean overall
    gen = torch.Generator().manual_seed(8)
    v = torch.randn(d, generator=gen)
    coef = torch.randn(M // d, generator=gen)
    g1 = (coef[:, None] * v[None, :]).reshape(-1).contiguous()
    Uo, muo, eigo = oracle.fit([synth.to_numpy(g1)], d, k)
    b.fit([g1.to(DEV)])
    b.fit_status()
    U, mu, eig = b.export()
    b.close()
    assert abs(eig[0][0] - eigo[0][0]) < 1e-10 * eigo[0][0]
    assert np.all(np.abs(eig[0][1:]) < 1e-9 * eigo[0][0])
    assert max_angle(U[0][:, :1].astype(np.float64), Uo[0][:, :1]) < ANGLE_TOL
    vn = (v / v.norm()).numpy().astype(np.float64)
    assert abs(abs(np.dot(U[0][:, 0], vn)) - 1) < 1e-6


def test_thousands_of_small_bases():
    """3000 bases of 24 slices each (the basis index is a grid dimension of the fit kernels, and the
    codec's tiles straddle a basis boundary almost every time): fit and codec against the oracle."""
    d, k, per, B = 16, 4, 24, 3000
    M = d * per * B - 5
    w = _wl(M, d, k, 2, 2, block_elems=d * per, rank=2, sigma=0.3)
    assert w.n_blocks == B
    offs = w.block_offsets()
    fit = synth.fit_gradients(w, "cpu")
    Uo, muo, eigo = oracle.fit([synth.to_numpy(g) for g in fit], d, k, offsets=offs)
    b = gvq.Basis(M, d, k, offs)
    b.fit([g.to(DEV) for g in fit])
    assert 0 <= b.fit_status() < 40
    U, mu, eig = b.export()
    np.testing.assert_allclose(eig, eigo, rtol=0, atol=1e-10 * eigo.max())
    np.testing.assert_allclose(mu, muo, rtol=2e-7, atol=1e-7 * np.abs(muo).max())
    worst = max(max_angle(U[i][:, :2].astype(np.float64), Uo[i][:, :2]) for i in range(0, B, 37))
    assert worst < ANGLE_TOL
    # codec with the oracle's basis
    U32, mu32 = Uo.astype(np.float32), muo.astype(np.float32)
    b.import_(U32, mu32)
    g = synth.worker_gradients(w, "cpu")[0]
    comp = torch.empty(b.S * k, device=DEV)
    out = torch.empty(M, device=DEV)
    b.compress(g.to(DEV), 2, comp)
    b.decompress(comp, out)
    torch.cuda.synchronize()
    y = oracle.compress(synth.to_numpy(g), U32.astype(np.float64), mu32.astype(np.float64), 2, offsets=offs)
    assert_close(comp.cpu().numpy().reshape(-1, k), y, 1e-4, "compress")
    xh = oracle.decompress(comp.cpu().numpy().reshape(-1, k).astype(np.float64), U32.astype(np.float64),
                           mu32.astype(np.float64), M, offsets=offs)
    assert_close(out.cpu().numpy(), xh, 1e-4, "decompress")
    b.close()
