"""Parity of gvq_local_loss (Eq. 6) and gvq_select_k (Eq. 5) with the float64 oracle."""
import numpy as np
import pytest

import oracle
from paper_1811_03617_amd import Workload, gvq, synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _wl(M, d, k, N, dtype="f32", rank=3, block_elems=0, seed=5, L=2, sigma=0.2):
    return Workload("t", M, d, k, N, L, dtype, rank, sigma, block_elems=block_elems, seed=seed)


def _check_loss(w, mean_offset=None):
    offs = w.block_offsets()
    if w.M < w.d:   # no full slice to fit on: any orthonormal basis serves
        rng = np.random.default_rng(w.seed)
        U = np.linalg.qr(rng.standard_normal((w.d, w.k)))[0][None]
        mu = rng.standard_normal((1, w.d))
    else:
        fit_np = [synth.to_numpy(g) for g in synth.fit_gradients(w, "cpu", mean_offset=mean_offset)]
        U, mu, _ = oracle.fit(fit_np, w.d, w.k, dtype=w.dtype, offsets=offs)
    U32, mu32 = U.astype(np.float32), mu.astype(np.float32)
    U64, mu64 = U32.astype(np.float64), mu32.astype(np.float64)
    workers = synth.worker_gradients(w, "cpu", mean_offset=mean_offset)
    b = gvq.Basis(w.M, w.d, w.k, offs, w.dtype)
    b.import_(U32, mu32)
    out = torch.full((w.n_blocks,), float("nan"), device=DEV, dtype=torch.float64)
    for g in workers[:2]:
        gh = synth.to_numpy(g)
        ref = oracle.local_loss(gh, U64, mu64, w.N, dtype=w.dtype, offsets=offs)
        b.local_loss(g.to(DEV), w.N, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        # energy of the centred gradient per basis: the scale rounding noise is relative to
        Uz = np.zeros((w.n_blocks, w.d, 1))
        energy = oracle.local_loss(gh, Uz, mu64, w.N, dtype=w.dtype, offsets=offs)
        assert np.all(np.isfinite(got))
        assert np.all(np.abs(got - ref) <= 1e-4 * ref + 1e-9 * energy), (got, ref)
        # second call gives the same bits (fixed summation order)
        out2 = torch.empty_like(out)
        b.local_loss(g.to(DEV), w.N, out2)
        torch.cuda.synchronize()
        assert torch.equal(out, out2)
    b.close()


@pytest.mark.parametrize("M,d,k,N", [
    (16 * 1000 + 5, 16, 4, 4), (32 * 2111 + 8, 32, 8, 8), (64 * 1777 + 40, 64, 16, 8),
    (128 * 1531 + 40, 128, 32, 16), (128 * 777 + 127, 128, 16, 3), (128 * 200 + 3, 128, 7, 2),
    (64 * 300 + 1, 64, 32, 2), (32 * 500 + 31, 32, 32, 2), (100, 128, 32, 2),
])
def test_local_loss_mfma_shapes(M, d, k, N):
    _check_loss(_wl(M, d, k, N))


@pytest.mark.parametrize("M,d,k,N", [(24 * 501 + 5, 24, 5, 3), (2 * 1000 + 1, 2, 1, 2),
                                      (100 * 77 + 60, 100, 100, 2), (128 * 65 + 9, 128, 40, 2)])
def test_local_loss_generic_shapes(M, d, k, N):
    _check_loss(_wl(M, d, k, N, rank=1 if d < 4 else 3))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_local_loss_many_bases_and_mean(dtype):
    _check_loss(_wl(128 * 1000 + 40, 128, 16, 4, dtype=dtype, block_elems=128 * 77),
                mean_offset=np.linspace(-3, 5, 128))
    _check_loss(_wl(32 * 4000 + 8, 32, 8, 2, dtype=dtype, block_elems=32 * 1000))
    _check_loss(_wl(24 * 400 + 3, 24, 6, 2, dtype=dtype, block_elems=24 * 50))


def test_local_loss_error_paths():
    L = gvq.lib()
    b = gvq.Basis(16 * 100, 16, 4)
    x = torch.zeros(16 * 100, device=DEV)
    o = torch.zeros(2, device=DEV, dtype=torch.float64)
    st = torch.cuda.current_stream().cuda_stream
    assert L.gvq_local_loss(b.handle, x.data_ptr(), 1, o.data_ptr(), st) == gvq.ENOTFIT
    b.import_(np.zeros((1, 16, 4), np.float32), np.zeros((1, 16), np.float32))
    assert L.gvq_local_loss(b.handle, x.data_ptr(), 0, o.data_ptr(), st) == gvq.EINVAL
    assert L.gvq_local_loss(b.handle, x.data_ptr() + 4, 1, o.data_ptr(), st) == gvq.EALIGN
    assert L.gvq_local_loss(b.handle, x.data_ptr(), 1, o.data_ptr() + 4, st) == gvq.EALIGN
    assert L.gvq_local_loss(b.handle, x.data_ptr(), 1, None, st) == gvq.EINVAL
    b.close()


@pytest.mark.parametrize("M,d,k,block_elems", [(64 * 3000, 64, 16, 0), (16 * 5000, 16, 4, 0),
                                                (128 * 900 + 40, 128, 16, 128 * 100), (24 * 1000, 24, 5, 0)])
def test_select_k_matches_the_oracle(M, d, k, block_elems):
    import ctypes as C
    w = _wl(M, d, k, 2, rank=5 if d > 8 else 2, block_elems=block_elems, L=3)
    offs = w.block_offsets()
    fit = synth.fit_gradients(w, "cpu")
    _, _, eig_o = oracle.fit([synth.to_numpy(g) for g in fit], d, k, offsets=offs)
    b = gvq.Basis(M, d, k, offs)
    st = torch.cuda.current_stream().cuda_stream
    out = (C.c_int * w.n_blocks)()
    assert gvq.lib().gvq_select_k(b.handle, 0.01, out, st) == gvq.ENOTFIT
    b.fit([g.to(DEV) for g in fit])
    _, _, eig = b.export()
    for lam in (0.5, 0.1, 0.01, 1e-3, 1e-5, 0.0):
        got = b.select_k(lam)
        want = oracle.select_k(eig_o, lam)
        for bb in range(w.n_blocks):
            if eig[bb].sum() <= 0:      # a basis without samples: nothing to lose
                assert got[bb] == 1 and want[bb] == 1
                continue
            frac = np.cumsum(eig[bb]) / eig[bb].sum()
            if got[bb] != want[bb]:   # only possible when the ratio sits on the threshold
                assert abs(frac[min(got[bb], want[bb]) - 1] - (1 - lam)) < 1e-10
            assert frac[got[bb] - 1] >= 1 - lam - 1e-12
            assert got[bb] == 1 or frac[got[bb] - 2] < 1 - lam + 1e-12
    assert gvq.lib().gvq_select_k(b.handle, 1.0, out, st) == gvq.EINVAL
    assert gvq.lib().gvq_select_k(b.handle, -0.1, out, st) == gvq.EINVAL
    b.close()
