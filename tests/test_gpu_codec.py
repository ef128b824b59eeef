"""Parity of the HIP codec (compress / aggregate / decompress through the C ABI) with the
float64 oracle, element by element, on seeded synthetic gradients.  The basis is the
oracle's, rounded to fp32 and imported, so both sides use identical parameters."""
import dataclasses

import numpy as np
import pytest

import oracle
from paper_1811_03617_amd import Workload, gvq, synth
from _util import REL_TOL, assert_close, bf16_bits_to_f64, f64_to_bf16_bits_rne

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _wl(M, d, k, N, dtype="f32", rank=None, block_elems=0, seed=7, L=2, sigma=0.05):
    return Workload("t", M, d, k, N, L, dtype, rank or max(1, min(k - 1, d // 4) or 1), sigma,
                    block_elems=block_elems, seed=seed)


def _oracle_basis(w, mean_offset=None):
    if w.M < w.d:  # no full slice to fit on: any orthonormal basis will do for the codec
        rng = np.random.default_rng(w.seed)
        U = np.stack([np.linalg.qr(rng.standard_normal((w.d, w.k)))[0] for _ in range(w.n_blocks)])
        return U.astype(np.float32), rng.standard_normal((w.n_blocks, w.d)).astype(np.float32)
    fitg = [synth.to_numpy(g) for g in synth.fit_gradients(w, "cpu", mean_offset=mean_offset)]
    U, mu, _ = oracle.fit(fitg, w.d, w.k, dtype=w.dtype, offsets=w.block_offsets())
    # what the library will hold: fp32 roundings of the oracle's basis
    U32, mu32 = U.astype(np.float32), mu.astype(np.float32)
    return U32, mu32


def _run_codec(w, U32, mu32, workers_dev, out_dtype=None):
    b = gvq.Basis(w.M, w.d, w.k, w.block_offsets(), w.dtype)
    b.import_(U32, mu32)
    comps = [torch.full((b.S * w.k,), float("nan"), device=DEV) for _ in workers_dev]
    for g, c in zip(workers_dev, comps):
        b.compress(g, len(workers_dev), c)
    total = torch.full((b.S * w.k,), float("nan"), device=DEV)
    b.aggregate(comps, total)
    od = out_dtype or w.dtype
    out = torch.full((w.M,), float("nan"), device=DEV,
                     dtype=torch.bfloat16 if od == "bf16" else torch.float32)
    b.decompress(total, out, od)
    torch.cuda.synchronize()
    res = [c.cpu().numpy().reshape(b.S, w.k) for c in comps], total.cpu().numpy().reshape(b.S, w.k), out
    b.close()
    return res


def _check_codec(w, mean_offset=None, out_dtype=None):
    U32, mu32 = _oracle_basis(w, mean_offset)
    workers = synth.worker_gradients(w, "cpu", mean_offset=mean_offset)
    workers_np = [synth.to_numpy(g) for g in workers]
    workers_dev = [g.to(DEV) for g in workers]
    comps, total, out = _run_codec(w, U32, mu32, workers_dev, out_dtype)

    offs = w.block_offsets()
    U64, mu64 = U32.astype(np.float64), mu32.astype(np.float64)
    ref_comps = [oracle.compress(g, U64, mu64, w.N, dtype=w.dtype, offsets=offs) for g in workers_np]
    for n, (c, r) in enumerate(zip(comps, ref_comps)):
        assert_close(c, r, REL_TOL, f"compress worker {n}")
    ref_total = oracle.aggregate(ref_comps)
    assert_close(total, ref_total, REL_TOL, "aggregate")
    # decompress is checked on the library's own compressed sum widened to float64, and end to end
    ref_out_same_in = oracle.decompress(total.astype(np.float64), U64, mu64, w.M, offsets=offs)
    ref_out = oracle.decompress(ref_total, U64, mu64, w.M, offsets=offs)
    if (out_dtype or w.dtype) == "bf16":
        got_bits = synth.to_numpy(out)
        want_bits = f64_to_bf16_bits_rne(ref_out_same_in)
        exact = np.mean(got_bits == want_bits)
        assert exact >= 0.999, f"bf16 output: only {exact:.5f} of elements equal RNE(oracle)"
        # never more than one bf16 step away (elements near zero: within the fp32 tolerance)
        got, want = bf16_bits_to_f64(got_bits), bf16_bits_to_f64(want_bits)
        assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -7 + REL_TOL * np.max(np.abs(want)))
        assert_close(got, ref_out, 2.0 ** -8, "decompress bf16 end to end")
    else:
        got = out.cpu().numpy()
        assert_close(got, ref_out_same_in, REL_TOL, "decompress")
        assert_close(got, ref_out, REL_TOL, "end to end")


# shapes the MFMA kernels take (d in {16,32,64,128}, k <= 32), several tiles and a ragged tail
MFMA_CASES = [
    # M, d, k, N
    (16 * 1000 + 5, 16, 4, 4),
    (32 * 2111 + 8, 32, 8, 8),
    (64 * 1777 + 40, 64, 16, 8),
    (128 * 1531 + 40, 128, 32, 16),
    (128 * 1024, 128, 32, 2),        # exact multiple of the tile and of d
    (128 * 777 + 127, 128, 16, 3),
    (64 * 300 + 1, 64, 32, 2),
    (32 * 500 + 31, 32, 32, 2),      # k = d on the MFMA path
    (16 * 333 + 3, 16, 16, 2),
    (128 * 200 + 3, 128, 7, 2),      # k not a multiple of 4: scalar stores
    (64 * 200 + 2, 64, 13, 5),
    (16 * 50, 16, 1, 1),             # N = 1, k = 1
    (128 * 3 + 2, 128, 32, 4),       # fewer slices than one tile
    (100, 128, 32, 2),               # M < d: one partial slice
]


@pytest.mark.parametrize("M,d,k,N", MFMA_CASES)
def test_codec_parity_mfma_shapes(M, d, k, N):
    _check_codec(_wl(M, d, k, N))


GENERIC_CASES = [
    (24 * 501 + 5, 24, 5, 3),
    (2 * 1000 + 1, 2, 1, 2),
    (100 * 77 + 60, 100, 100, 2),    # k = d, lossless
    (128 * 65 + 9, 128, 128, 2),
    (128 * 65 + 9, 128, 40, 2),      # d fits the MFMA path but k > 32
    (7 * 300, 7, 3, 4),
]


@pytest.mark.parametrize("M,d,k,N", GENERIC_CASES)
def test_codec_parity_generic_shapes(M, d, k, N):
    _check_codec(_wl(M, d, k, N))


def test_codec_parity_nonzero_mean():
    """The mu/N term of Eq. (2) and the +mu of Eq. (4) only matter with a mean far from 0."""
    w = _wl(64 * 900 + 17, 64, 16, 8)
    _check_codec(w, mean_offset=np.linspace(-30.0, 50.0, 64))


@pytest.mark.parametrize("M,d,k,N,block_elems", [
    (128 * 1000 + 40, 128, 16, 4, 128 * 77),     # basis boundaries inside 16-slice tiles
    (128 * 1000 + 40, 128, 32, 2, 128 * 5),      # several bases inside one tile
    (32 * 4000 + 8, 32, 8, 2, 32 * 1000),        # boundaries on tile boundaries (1000 = 62.5 tiles)
    (64 * 1024, 64, 16, 2, 64 * 256),            # boundaries exactly on tile boundaries
    (24 * 400 + 3, 24, 6, 2, 24 * 50),           # generic kernels with several bases
])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_codec_parity_many_bases(M, d, k, N, block_elems, dtype):
    _check_codec(_wl(M, d, k, N, dtype=dtype, block_elems=block_elems, rank=3), out_dtype="f32")


@pytest.mark.parametrize("M,d,k,N", [(128 * 1500 + 40, 128, 16, 16), (64 * 700 + 6, 64, 16, 2),
                                      (32 * 700 + 30, 32, 8, 2), (16 * 700 + 9, 16, 4, 2),
                                      (24 * 100 + 1, 24, 4, 2)])
def test_codec_parity_bf16_storage(M, d, k, N):
    w = _wl(M, d, k, N, dtype="bf16")
    _check_codec(w, out_dtype="f32")
    _check_codec(w, out_dtype="bf16")


def test_lossless_when_k_equals_d_on_the_gpu():
    """k = d: the reconstructed gradient equals the plain sum of the workers' gradients."""
    w = _wl(32 * 1000 + 12, 32, 32, 4)
    U32, mu32 = _oracle_basis(w)
    workers = synth.worker_gradients(w, "cpu")
    _, _, out = _run_codec(w, U32, mu32, [g.to(DEV) for g in workers])
    total = np.sum([g.numpy().astype(np.float64) for g in workers], axis=0)
    assert_close(out.cpu().numpy(), total, REL_TOL, "k = d round trip")


def test_aggregate_in_place_many_inputs_and_bitwise_determinism():
    w = _wl(16 * 4000 + 3, 16, 4, 40)   # more inputs than fit in one launch
    b = gvq.Basis(w.M, w.d, w.k)
    g = torch.Generator(device="cpu").manual_seed(1)
    comps = [torch.randn(b.S * w.k, generator=g).to(DEV) for _ in range(w.N)]
    ref = oracle.aggregate([c.cpu().numpy() for c in comps])
    out1 = torch.empty_like(comps[0])
    b.aggregate(comps, out1)
    first = comps[0].clone()
    b.aggregate(comps, comps[0])          # output aliases the first input
    torch.cuda.synchronize()
    assert_close(out1.cpu().numpy(), ref, 1e-5, "aggregate N=40")
    assert torch.equal(out1, comps[0])
    comps[0] = first
    out2 = torch.empty_like(out1)
    b.aggregate(comps, out2)
    torch.cuda.synchronize()
    assert torch.equal(out1, out2)
    # fixed summation order: equal to the sequential fp32 sum
    seq = comps[0].clone()
    for c in comps[1:]:
        seq += c
    assert torch.equal(out1, seq)
    b.close()


def test_error_paths_on_the_device():
    import ctypes as C
    L = gvq.lib()
    b = gvq.Basis(16 * 100, 16, 4)
    x = torch.zeros(16 * 100 + 4, device=DEV)
    y = torch.zeros(100 * 4 + 4, device=DEV)
    st = torch.cuda.current_stream().cuda_stream
    assert L.gvq_compress(b.handle, x.data_ptr(), 1, y.data_ptr(), st) == gvq.ENOTFIT
    assert L.gvq_decompress(b.handle, y.data_ptr(), x.data_ptr(), gvq.F32, st) == gvq.ENOTFIT
    assert L.gvq_basis_export(b.handle, None, None, None) == gvq.ENOTFIT
    assert L.gvq_basis_export_cov(b.handle, None, None) == gvq.ENOTFIT
    assert L.gvq_fit_status(b.handle, None, st) == gvq.ENOTFIT
    b.import_(np.zeros((1, 16, 4), np.float32), np.zeros((1, 16), np.float32))
    assert L.gvq_compress(b.handle, x.data_ptr() + 4, 1, y.data_ptr(), st) == gvq.EALIGN
    assert L.gvq_compress(b.handle, x.data_ptr(), 1, y.data_ptr() + 8, st) == gvq.EALIGN
    assert L.gvq_compress(b.handle, x.data_ptr(), 0, y.data_ptr(), st) == gvq.EINVAL
    assert L.gvq_decompress(b.handle, y.data_ptr(), x.data_ptr(), 5, st) == gvq.EINVAL
    arr = (C.c_void_p * 2)(y.data_ptr(), y.data_ptr())
    assert L.gvq_aggregate(b.handle, arr, 2, y.data_ptr(), st) == gvq.EINVAL   # comps[1] aliases out
    assert L.gvq_aggregate(b.handle, arr, 0, y.data_ptr(), st) == gvq.EINVAL
    assert L.gvq_basis_export_cov(b.handle, None, None) == gvq.ENOTFIT          # import is not a fit
    assert L.gvq_compress(b.handle, x.data_ptr(), 1, y.data_ptr(), st) == gvq.OK
    torch.cuda.synchronize()
    b.close()


def _run_ring(w, U32, mu32, workers_dev, first, count, out_dtype):
    """Eq. 3 as a ring of fused compress steps over slices [first, first + count), then Eq. 4 on the same range."""
    b = gvq.Basis(w.M, w.d, w.k, w.block_offsets(), w.dtype)
    b.import_(U32, mu32)
    acc = [torch.full((b.S * w.k,), float("nan"), device=DEV) for _ in range(2)]
    for n, g in enumerate(workers_dev):
        b.compress_segment(g, len(workers_dev), first, count, acc[(n + 1) % 2] if n else None, acc[n % 2])
    total = acc[(len(workers_dev) - 1) % 2]
    out = torch.full((w.M,), float("nan"), device=DEV,
                     dtype=torch.bfloat16 if out_dtype == "bf16" else torch.float32)
    b.decompress_segment(total, first, count, out, out_dtype)
    torch.cuda.synchronize()
    res = total.cpu().numpy(), out
    b.close()
    return res


@pytest.mark.parametrize("M,d,k,N,dtype,out_dtype", [
    (128 * 5000 + 40, 128, 32, 3, "f32", "f32"),
    (128 * 5000 + 40, 128, 16, 2, "f32", "bf16"),
    (128 * 5000 + 40, 128, 32, 2, "bf16", "bf16"),
    (64 * 9000 + 6, 64, 16, 2, "f32", "f32"),
    (32 * 20000 + 8, 32, 8, 2, "f32", "f32"),
    (16 * 30000 + 3, 16, 4, 2, "f32", "bf16"),
])
def test_row_interleave_of_the_register_resident_kernels_changes_no_bit(M, d, k, N, dtype, out_dtype):
    """With one basis, groups of super-tiles exchange their 1 KB rows (option 5: the group size; the groups that do
    not fill up stay as they are).  Which wave computes a slice changes, what it computes does not: every width
    gives the bits of width 1, on the whole gradient and on a ring segment that starts and ends inside a tile."""
    w = _wl(M, d, k, N, dtype=dtype)
    U32, mu32 = _oracle_basis(w)
    dev = [g.to(DEV) for g in synth.worker_gradients(w, "cpu")]
    S = (M + d - 1) // d
    first, count = S // 7 + 3, S // 2 + 5

    def both():
        return _run_codec(w, U32, mu32, dev, out_dtype), _run_ring(w, U32, mu32, dev, first, count, out_dtype)

    assert gvq.lib().gvq_set_option(5, 1) == gvq.OK
    try:
        a, ar = both()
        for width in (0, 2, 3, 7, 16, 64):
            assert gvq.lib().gvq_set_option(5, width) == gvq.OK
            b, br = both()
            for x, y in zip(a[0], b[0]):
                assert np.array_equal(x, y), width
            assert np.array_equal(a[1], b[1]) and torch.equal(a[2], b[2]), width
            lo, hi = first * k, (first + count) * k
            assert np.array_equal(ar[0][lo:hi], br[0][lo:hi]), width
            e0, e1 = first * d, min((first + count) * d, M)
            assert torch.equal(ar[1][e0:e1], br[1][e0:e1]), width
    finally:
        assert gvq.lib().gvq_set_option(5, 0) == gvq.OK


@pytest.mark.parametrize("M,d,k", [
    (128 * 5000 + 40, 128, 32), (128 * 5000 + 40, 128, 16), (64 * 9000 + 6, 64, 16), (32 * 20000 + 8, 32, 8),
    (16 * 30000 + 3, 16, 4),
])
def test_cache_resident_and_streaming_result_stores_give_the_same_bits(M, d, k):
    """When the n_workers results that are summed next fit the last-level cache together, compress writes them with
    ordinary stores, otherwise with non-temporal ones (two kernel variants).  With a zero mean Eq. 2 does not depend
    on n_workers, so a worker count on either side of that limit must give the same bits, and those of the oracle
    to the usual tolerance."""
    w = _wl(M, d, k, 1)
    rng = np.random.default_rng(5)
    U = np.linalg.qr(rng.standard_normal((d, k)))[0][None].astype(np.float32)
    mu = np.zeros((1, d), np.float32)
    g = synth.worker_gradients(w, "cpu")[0]
    b = gvq.Basis(M, d, k, None, "f32")
    b.import_(U, mu)
    many = (224 << 20) // (b.S * k * 4) + 2
    gd = g.to(DEV)
    ys = []
    for n in (1, many):
        c = torch.full((b.S * k,), float("nan"), device=DEV)
        b.compress(gd, n, c)
        torch.cuda.synchronize()
        ys.append(c.cpu().numpy().reshape(b.S, k))
    b.close()
    assert np.array_equal(ys[0], ys[1])
    ref = oracle.compress(synth.to_numpy(g), U.astype(np.float64), mu.astype(np.float64), many)
    assert_close(ys[1], ref, REL_TOL, "compress with streaming stores")


def test_codec_is_bitwise_reproducible():
    w = _wl(128 * 2000 + 40, 128, 32, 3)
    U32, mu32 = _oracle_basis(w)
    dev = [g.to(DEV) for g in synth.worker_gradients(w, "cpu")]
    a = _run_codec(w, U32, mu32, dev)
    b = _run_codec(w, U32, mu32, dev)
    for x, y in zip(a[0], b[0]):
        assert np.array_equal(x, y)
    assert np.array_equal(a[1], b[1]) and torch.equal(a[2], b[2])


@pytest.mark.parametrize("M,d,k,N,dtype,block_elems", [
    (128 * 5000 + 40, 128, 32, 3, "f32", 0),
    (128 * 5000 + 40, 128, 16, 2, "bf16", 128 * 700),    # several bases: super-tiles from the handle's plan
    (64 * 9000 + 6, 64, 16, 2, "bf16", 0),
    (32 * 20000 + 8, 32, 8, 2, "f32", 32 * 3000),
    (16 * 30000 + 3, 16, 4, 2, "f32", 0),
])
def test_both_loops_of_the_register_resident_kernels_agree_bit_for_bit(M, d, k, N, dtype, block_elems):
    """These kernels run whole tiles of one basis through a branch-free loop and the rest through a
    bounds-checked one; option 3 sends everything through the latter.  Same arithmetic in the same order:
    the results must be identical, and the default run is compared with the oracle by the tests above."""
    w = _wl(M, d, k, N, dtype=dtype, block_elems=block_elems)
    U32, mu32 = _oracle_basis(w)
    dev = [g.to(DEV) for g in synth.worker_gradients(w, "cpu")]
    a = _run_codec(w, U32, mu32, dev)
    assert gvq.lib().gvq_set_option(3, 7) == gvq.OK
    try:
        b = _run_codec(w, U32, mu32, dev)
    finally:
        assert gvq.lib().gvq_set_option(3, 0) == gvq.OK
    for x, y in zip(a[0], b[0]):
        assert np.array_equal(x, y)
    assert np.array_equal(a[1], b[1]) and torch.equal(a[2], b[2])
