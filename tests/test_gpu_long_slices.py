"""Slices longer than 128 elements (Section 3, "slice size": a multiple of filters x depth, 768
in the paper's example): the basis refresh runs its moments in 64 x 64 blocks and a block Jacobi
eigensolver, the codec runs the LDS-tiled long-slice kernels, one pass per 128 comps of a slice.
Same parity bar as the short slices."""
import numpy as np
import pytest

import oracle
from paper_1811_03617_amd import Workload, gvq, synth
from _util import ANGLE_TOL, REL_TOL, assert_close, max_angle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _wl(M, d, k, N, L, dtype="f32", rank=4, block_elems=0, seed=21, sigma=0.05):
    return Workload("t", M, d, k, N, L, dtype, rank, sigma, block_elems=block_elems, seed=seed)


def _check_fit(w, first_slice_only=False, mean_offset=None, angle_rank=None):
    fit = synth.fit_gradients(w, "cpu", mean_offset=mean_offset)
    fit_np = [synth.to_numpy(g) for g in fit]
    offs = w.block_offsets()
    Uo, muo, eigo, Co = oracle.fit(fit_np, w.d, w.k, dtype=w.dtype, offsets=offs, return_cov=True,
                                   first_slice_only=first_slice_only)
    b = gvq.Basis(w.M, w.d, w.k, offs, w.dtype)
    b.fit([g.to(DEV) for g in fit], first_slice_only=first_slice_only)
    sweeps = b.fit_status()
    U, mu, eig = b.export()
    C, n = b.export_cov()
    b.close()
    assert 0 <= sweeps <= 24
    full = w.M // w.d
    offs = offs or [0, w.S]
    for bb in range(len(offs) - 1):
        cnt = max(0, min(offs[bb + 1], full) - offs[bb])
        assert n[bb] == (min(cnt, 1) if first_slice_only else cnt) * w.L
        lam1 = eigo[bb][0]
        scale = max(lam1, np.max(np.abs(muo[bb])) ** 2)
        np.testing.assert_allclose(mu[bb], muo[bb], rtol=2e-7, atol=1e-12 + 1e-7 * np.max(np.abs(muo[bb])))
        assert np.max(np.abs(C[bb] - Co[bb])) <= 1e-11 * scale
        assert np.array_equal(C[bb], C[bb].T)
        np.testing.assert_allclose(eig[bb], eigo[bb], rtol=0, atol=1e-10 * scale)
        assert np.all(np.diff(eig[bb]) <= 0)
        Ub = U[bb].astype(np.float64)
        assert np.max(np.abs(Ub.T @ Ub - np.eye(w.k))) < 1e-5
        kk = w.k if angle_rank is None else angle_rank
        if first_slice_only:
            kk = min(kk, w.L - 1)            # what L samples determine
            while kk > 1 and eigo[bb][kk - 1] - eigo[bb][kk] < 1e-6 * lam1:
                kk -= 1
        assert max_angle(Ub[:, :kk], Uo[bb][:, :kk]) < ANGLE_TOL
        for i in range(w.k):
            assert Ub[np.argmax(np.abs(Ub[:, i])), i] > 0
        for i in range(kk):
            gap = min(abs(eigo[bb][i] - eigo[bb][j]) for j in range(w.d) if j != i)
            if gap > 1e-3 * lam1:
                s = np.sign(np.dot(Ub[:, i], Uo[bb][:, i]))
                assert np.max(np.abs(s * Ub[:, i] - Uo[bb][:, i])) < 1e-5


@pytest.mark.parametrize("M,d,k,L,dtype", [
    (256 * 1500 + 40, 256, 32, 3, "f32"),      # whole 64-element groups
    (320 * 900 + 8, 320, 24, 2, "bf16"),
    (200 * 1000 + 7, 200, 16, 2, "f32"),       # last group partly outside the slice
    (130 * 700 + 3, 130, 8, 2, "f32"),         # d not a multiple of 4: unaligned slices
    (129 * 500, 129, 5, 2, "bf16"),            # odd d: the Jacobi pads to an even size
])
def test_fit_parity_pooled(M, d, k, L, dtype):
    _check_fit(_wl(M, d, k, 2, L, dtype=dtype))


def test_fit_parity_nonzero_mean_and_many_bases():
    w = _wl(192 * 1200 + 50, 192, 12, 2, 2, block_elems=192 * 300)
    _check_fit(w, mean_offset=np.linspace(-2.0, 3.0, 192))


def test_fit_parity_more_gradients_than_one_launch():
    _check_fit(_wl(136 * 150, 136, 6, 1, 35))


def test_fit_parity_first_slice_of_a_768_element_slice():
    """The paper's setting: L time samples of the first slice only, far fewer samples than
    dimensions, so the covariance has rank L - 1 and the kept components span its range."""
    w = _wl(768 * 40 + 100, 768, 16, 2, 24, rank=6, sigma=0.1)
    _check_fit(w, first_slice_only=True)


@pytest.mark.parametrize("M,d,k,L,dtype,block_elems", [
    (256 * 30 + 7, 256, 40, 24, "f32", 0),             # more columns than the samples determine
    (256 * 64, 256, 40, 100, "bf16", 256 * 16),        # a 100 x 100 sample matrix, four bases
    (130 * 9 + 1, 130, 7, 65, "f32", 0),               # as many samples as the small-matrix route takes
    (130 * 9 + 1, 130, 7, 66, "f32", 0),               # one more: the general solver
    (192 * 8, 192, 150, 12, "f32", 0),                 # too many columns for it: the general solver
    (130 * 9 + 1, 130, 96, 65, "f32", 0),              # its scratch just fits the eigenvector work space
    (130 * 9 + 1, 130, 97, 65, "f32", 0),              # ... and just does not: the general solver
    (256 * 140, 256, 16, 128, "f32", 0),               # the largest sample matrix it takes
])
def test_fit_parity_first_slice_few_samples(M, d, k, L, dtype, block_elems):
    _check_fit(_wl(M, d, k, 2, L, dtype=dtype, rank=5, sigma=0.2, block_elems=block_elems), first_slice_only=True)


def test_fit_first_slice_of_identical_samples_gives_unit_vectors():
    M, d, k = 256 * 10, 256, 8
    g = torch.randn(M, generator=torch.Generator().manual_seed(9))
    b = gvq.Basis(M, d, k)
    b.fit([g.to(DEV)] * 6, first_slice_only=True)
    assert b.fit_status() == 0
    U, mu, eig = b.export()
    b.close()
    assert np.all(eig == 0)
    np.testing.assert_array_equal(mu[0], g[:d].numpy())
    np.testing.assert_array_equal(U[0], np.eye(d, k, dtype=np.float32))


def test_fit_is_bitwise_reproducible():
    w = _wl(256 * 2000 + 40, 256, 16, 2, 2)
    fit = [g.to(DEV) for g in synth.fit_gradients(w, "cpu")]
    res = []
    for _ in range(2):
        b = gvq.Basis(w.M, w.d, w.k)
        b.fit(fit)
        b.fit_status()
        res.append(b.export() + b.export_cov())
        b.close()
    for x, y in zip(*res):
        assert np.array_equal(x, y)


def test_fit_at_the_largest_slice_length_by_invariants():
    """d = 1024 is too slow for the oracle's Jacobi in a test; what defines the result is checked
    instead, in float64 on the host: against numpy's symmetric eigensolver for the eigenvalues
    and the kept subspace, and C u = lambda u, U^T U = I, sum(eig) = trace(C) directly."""
    d, k = gvq.MAX_D, 32
    w = _wl(d * 700, d, k, 2, 2, rank=8, sigma=0.2)
    fit = synth.fit_gradients(w, "cpu")
    X = np.concatenate([synth.to_numpy(g).astype(np.float64).reshape(-1, d) for g in fit])
    C_ref = np.cov(X.T, bias=True)
    b = gvq.Basis(w.M, d, k)
    b.fit([g.to(DEV) for g in fit])
    assert 0 <= b.fit_status() <= 24
    U, mu, eig = b.export()
    C, n = b.export_cov()
    b.close()
    assert n[0] == X.shape[0]
    lam1 = eig[0][0]
    np.testing.assert_allclose(mu[0], X.mean(0), rtol=2e-7, atol=1e-7 * np.abs(X.mean(0)).max())
    assert np.max(np.abs(C[0] - C_ref)) <= 1e-11 * lam1
    w_ref, V_ref = np.linalg.eigh(C[0])
    np.testing.assert_allclose(eig[0], w_ref[::-1], rtol=0, atol=1e-10 * lam1)
    assert abs(eig[0].sum() - np.trace(C[0])) <= 1e-10 * lam1
    Ub = U[0].astype(np.float64)
    assert np.max(np.abs(Ub.T @ Ub - np.eye(k))) < 1e-5
    assert np.max(np.abs(C[0] @ Ub - Ub * eig[0][:k])) <= 1e-6 * lam1     # fp32 rounding of U
    assert max_angle(Ub[:, :8], V_ref[:, ::-1][:, :8]) < ANGLE_TOL         # the planted directions


def _check_codec(w, out_dtype=None, fit=True):
    rng = np.random.default_rng(w.seed)
    if fit and w.M // w.d >= 2 * w.d:      # enough samples for a meaningful fit
        fitg = [synth.to_numpy(g) for g in synth.fit_gradients(w, "cpu")]
        U, mu, _ = oracle.fit(fitg, w.d, w.k, dtype=w.dtype, offsets=w.block_offsets())
    else:
        U = np.stack([np.linalg.qr(rng.standard_normal((w.d, w.k)))[0] for _ in range(w.n_blocks)])
        mu = rng.standard_normal((w.n_blocks, w.d))
    U32, mu32 = U.astype(np.float32), mu.astype(np.float32)
    U64, mu64 = U32.astype(np.float64), mu32.astype(np.float64)
    offs = w.block_offsets()
    workers = synth.worker_gradients(w, "cpu")
    workers_np = [synth.to_numpy(g) for g in workers]
    b = gvq.Basis(w.M, w.d, w.k, offs, w.dtype)
    b.import_(U32, mu32)
    comps = [torch.full((b.S * w.k,), float("nan"), device=DEV) for _ in workers]
    for g, c in zip(workers, comps):
        b.compress(g.to(DEV), w.N, c)
    total = torch.full((b.S * w.k,), float("nan"), device=DEV)
    b.aggregate(comps, total)
    out = torch.full((w.M,), float("nan"), device=DEV)
    b.decompress(total, out, "f32")
    loss = torch.empty(w.n_blocks, device=DEV, dtype=torch.float64)
    b.local_loss(workers[0].to(DEV), w.N, loss)
    torch.cuda.synchronize()
    ref = [oracle.compress(g, U64, mu64, w.N, dtype=w.dtype, offsets=offs) for g in workers_np]
    for n, (c, r) in enumerate(zip(comps, ref)):
        assert_close(c.cpu().numpy().reshape(b.S, w.k), r, REL_TOL, f"compress worker {n}")
    ref_total = oracle.aggregate(ref)
    got_total = total.cpu().numpy().reshape(b.S, w.k)
    assert_close(got_total, ref_total, REL_TOL, "aggregate")
    assert_close(out.cpu().numpy(), oracle.decompress(got_total.astype(np.float64), U64, mu64, w.M, offsets=offs),
                 REL_TOL, "decompress")
    assert_close(out.cpu().numpy(), oracle.decompress(ref_total, U64, mu64, w.M, offsets=offs), REL_TOL,
                 "end to end")
    if out_dtype == "bf16":   # the same reconstruction rounded to bf16: half a unit in the last of 8 bits
        out16 = torch.full((w.M,), float("nan"), device=DEV, dtype=torch.bfloat16)
        b.decompress(total, out16, "bf16")
        ref_x = oracle.decompress(got_total.astype(np.float64), U64, mu64, w.M, offsets=offs)
        got16 = out16.float().cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got16 - ref_x) <= 2.0 ** -8 * np.abs(ref_x) + REL_TOL * np.max(np.abs(ref_x)))
    ref_loss = oracle.local_loss(workers_np[0], U64, mu64, w.N, dtype=w.dtype, offsets=offs)
    energy = oracle.local_loss(workers_np[0], np.zeros((w.n_blocks, w.d, 1)), mu64, w.N, dtype=w.dtype, offsets=offs)
    got_loss = loss.cpu().numpy()
    assert np.all(np.abs(got_loss - ref_loss) <= 1e-4 * ref_loss + 1e-9 * energy), (got_loss, ref_loss)
    b.close()


@pytest.mark.parametrize("M,d,k,N,dtype,block_elems", [
    (256 * 700 + 40, 256, 32, 4, "f32", 0),
    (768 * 300 + 500, 768, 96, 3, "f32", 0),         # the paper's example slice, 8x compression
    (768 * 200 + 9, 768, 48, 2, "bf16", 768 * 64),
    (1024 * 100 + 1, 1024, 128, 2, "f32", 0),
    (130 * 900 + 77, 130, 130, 2, "f32", 0),         # k = d: lossless
    (129 * 400 + 128, 129, 3, 2, "bf16", 129 * 100),
    (300, 512, 8, 2, "f32", 0),                      # a single partial slice
    (256 * 10 * 40 + 77, 256, 24, 2, "f32", 256 * 10),   # 41 bases of 10 slices: every tile mostly empty
    (512 * 300 + 100, 512, 256, 3, "f32", 0),        # more than 128 comps: two column passes
    (320 * 500 + 3, 320, 200, 2, "f32", 320 * 150),  # 128 + 72 comps, several bases
    (256 * 260 + 5, 256, 131, 2, "bf16", 0),         # second pass of 3 comps, k not a multiple of 4
    (1024 * 70 + 9, 1024, 520, 2, "f32", 0),         # five passes, the last of 8 comps
])
@pytest.mark.parametrize("pipe", [1, 2, 3], ids=["fp32-products", "bf16-split-products", "bf16-split-lds-tiled-only"])
def test_codec_and_loss_parity(M, d, k, N, dtype, block_elems, pipe):
    assert gvq.lib().gvq_set_option(2, pipe) == gvq.OK
    try:
        _check_codec(_wl(M, d, k, N, 2, dtype=dtype, block_elems=block_elems))
    finally:
        gvq.lib().gvq_set_option(2, 0)


@pytest.mark.parametrize("M,d,k,N", [
    (512 * 200 + 77, 512, 64, 2),
    (1024 * 60 + 5, 1024, 32, 2),
    (768 * 150, 768, 40, 2),        # comps end inside a 32-comp step
    (256 * 500 + 3, 256, 32, 2),    # the smallest slice it takes
    (256 * 300, 256, 128, 2),       # too many column tiles for a wave's strip: the LDS-tiled kernels
    (512 * 100, 512, 52, 3),
    (768 * 20 + 5, 768, 96, 2),     # one whole tile, then 4 slices and one that ends after 5 elements
    (768 * 10, 768, 96, 2),         # no whole tile: the tail tile alone
    (768 * 31 + 767, 768, 96, 2),   # a tail of 16 slices, the last one element short
    (768 * 32, 768, 96, 2),         # whole tiles only
    (1024 * 47 + 2, 1024, 64, 2),   # two buffers in LDS instead of three
    (768 * 4113 + 700, 768, 96, 2), # more tiles than work-groups
])
def test_basis_stationary_kernels(M, d, k, N):
    """fp32 gradients, one basis, d a multiple of 256, the bf16-split pipe: compress, and decompress into fp32, keep U
    in registers while the gradient streams past in 16-slice tiles; compared with the oracle like every other route."""
    # the pipe picked from the shape, exact fp32 products, the bf16 split
    for pipe, out_dtype in ((0, "f32"), (1, "f32"), (2, "bf16"), (2, "f32")):
        assert gvq.lib().gvq_set_option(2, pipe) == gvq.OK
        try:
            _check_codec(_wl(M, d, k, N, 2), out_dtype=out_dtype)
        finally:
            gvq.lib().gvq_set_option(2, 0)


@pytest.mark.parametrize("M,d,k", [
    (768 * (16 * 256 * 6 + 37) + 100, 768, 96),
    (768 * (16 * 256 * 5 + 3), 768, 16),            # exact products by default
    (1024 * (16 * 256 * 5 + 5), 1024, 64),          # two buffers in LDS
    (256 * (16 * 256 * 6 + 9) + 3, 256, 32),
])
def test_basis_stationary_kernels_with_several_tiles_per_work_group(M, d, k):
    """Five or six tiles per work-group on the whole chip: every ring of LDS buffers wraps around, and whole groups of
    16 interleaved tiles, the tiles after the last whole group and the tail tile all occur.  With a random orthonormal
    basis: an oracle fit of this size would take minutes and is not what this test is about."""
    _check_codec(_wl(M, d, k, 1, 2), out_dtype="bf16", fit=False)   # fp32 output, and bf16 output from the same sum


@pytest.mark.parametrize("M,d,k,fit", [
    (768 * 300 + 9, 768, 96, True),
    (256 * 500 + 3, 256, 32, True),
    (1024 * 60 + 5, 1024, 64, True),
    (512 * 100, 512, 52, True),
    (768 * 20 + 5, 768, 96, True),                       # one whole tile and a tail that ends after 5 elements
    (768 * (16 * 256 * 5 + 11) + 100, 768, 96, False),   # five tiles per work-group
])
def test_basis_stationary_kernels_on_bf16_storage(M, d, k, fit):
    """bf16 gradients: the tile sits in LDS as bf16 with swizzled 16-byte chunks and the partial results in a region
    of their own; decompress rounds to bf16 at its row stores.  Same oracle comparison as for fp32 storage."""
    _check_codec(_wl(M, d, k, 2, 2, dtype="bf16"), out_dtype="bf16", fit=fit)


def test_pipe_option_range():
    assert gvq.lib().gvq_set_option(2, 4) == gvq.EINVAL
    assert gvq.lib().gvq_set_option(2, 0) == gvq.OK


def test_select_k_on_a_long_slice():
    w = _wl(256 * 1200, 256, 16, 2, 2, rank=6, sigma=0.3)
    fit = synth.fit_gradients(w, "cpu")
    _, _, eig_o = oracle.fit([synth.to_numpy(g) for g in fit], w.d, w.k)
    b = gvq.Basis(w.M, w.d, w.k)
    b.fit([g.to(DEV) for g in fit])
    for lam in (0.5, 0.1, 0.01, 1e-4):
        got, want = b.select_k(lam), oracle.select_k(eig_o, lam)
        if got[0] != want[0]:      # only when the ratio sits on the threshold
            frac = np.cumsum(eig_o[0]) / eig_o[0].sum()
            assert abs(frac[min(got[0], want[0]) - 1] - (1 - lam)) < 1e-10
    b.close()


@pytest.mark.parametrize("first_slice_only,L", [(False, 2), (True, 6), (True, 200)])
def test_fit_reports_non_finite_input(first_slice_only, L):
    """NaN in a sample reaches the eigenvalues on every route (blocked moments + global-memory Jacobi,
    sample-Gram route, first-slice moments + global-memory Jacobi) and is reported, not hidden."""
    M, d, k = 256 * 40, 256, 8
    gen = torch.Generator().manual_seed(4)
    grads = [torch.randn(M, generator=gen) for _ in range(L)]
    grads[L // 2][37] = float("nan")
    b = gvq.Basis(M, d, k)
    b.fit([g.to(DEV) for g in grads], first_slice_only=first_slice_only)
    with pytest.raises(gvq.GvqError) as ei:
        b.fit_status()
    assert ei.value.status == gvq.ENONFINITE
    b.close()


def test_slice_length_limits():
    import ctypes as C
    L = gvq.lib()
    h = C.c_void_p()
    assert L.gvq_basis_create(C.byref(h), 10000, gvq.MAX_D + 1, 4, 1, None, 0) == gvq.EINVAL
    assert L.gvq_basis_create(C.byref(h), 10000, gvq.MAX_D, gvq.MAX_D, 1, None, 0) == gvq.OK
    assert L.gvq_basis_destroy(h) == gvq.OK
