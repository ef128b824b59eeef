"""Segment-ranged entry points (the building blocks of Algorithm 1) against the oracle, and a
ring all-reduce of Algorithm 1 played out on one GPU with them."""
import numpy as np
import pytest

import oracle
from paper_1811_03617_amd import Workload, gvq, synth
from _util import REL_TOL, assert_close

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _wl(M, d, k, N, dtype="f32", block_elems=0, seed=13):
    return Workload("t", M, d, k, N, 2, dtype, 3, 0.1, block_elems=block_elems, seed=seed)


def _basis(w):
    fit_np = [synth.to_numpy(g) for g in synth.fit_gradients(w, "cpu")]
    U, mu, _ = oracle.fit(fit_np, w.d, w.k, dtype=w.dtype, offsets=w.block_offsets())
    return U.astype(np.float32), mu.astype(np.float32)


CASES = [
    (128 * 1000 + 40, 128, 32, "f32", 0), (128 * 1000 + 40, 128, 16, "bf16", 128 * 77),
    (64 * 700 + 6, 64, 16, "f32", 0), (32 * 900 + 8, 32, 8, "f32", 32 * 100), (16 * 500 + 3, 16, 4, "bf16", 0),
    (24 * 400 + 3, 24, 6, "f32", 24 * 50), (128 * 300 + 5, 128, 7, "f32", 0),
    # long slices: 128-slice work-group tiles that never straddle two bases
    (256 * 700 + 40, 256, 32, "f32", 0), (320 * 500 + 9, 320, 40, "bf16", 320 * 130),
    (192 * 300 + 5, 192, 7, "f32", 192 * 100),
    # more than 128 comps per slice: one pass of the long-slice kernels per 128 columns
    (512 * 200 + 9, 512, 200, "f32", 0), (256 * 300 + 5, 256, 130, "bf16", 256 * 100),
    # the paper's slice length, one basis: whole 16-slice tiles of a segment go to the basis-stationary compress kernel
    (768 * 100 + 9, 768, 96, "f32", 0),
]


@pytest.mark.parametrize("M,d,k,dtype,block_elems", CASES)
def test_segment_calls_match_the_oracle_and_touch_nothing_else(M, d, k, dtype, block_elems):
    if d <= 128:
        _check_segments(M, d, k, dtype, block_elems)
        return
    for pipe in (1, 2, 3):   # long slices: fp32 products, products of bf16 splits, those without the basis-stationary kernel
        assert gvq.lib().gvq_set_option(2, pipe) == gvq.OK
        try:
            _check_segments(M, d, k, dtype, block_elems)
        finally:
            gvq.lib().gvq_set_option(2, 0)


def _check_segments(M, d, k, dtype, block_elems):
    w = _wl(M, d, k, 3, dtype, block_elems)
    offs = w.block_offsets()
    U32, mu32 = _basis(w)
    U64, mu64 = U32.astype(np.float64), mu32.astype(np.float64)
    g = synth.worker_gradients(w, "cpu")[0]
    gh = synth.to_numpy(g)
    b = gvq.Basis(w.M, w.d, w.k, offs, w.dtype)
    b.import_(U32, mu32)
    S = b.S
    ref_y = oracle.compress(gh, U64, mu64, w.N, dtype=dtype, offsets=offs)
    rng = np.random.default_rng(3)
    prev = rng.standard_normal((S, k)).astype(np.float32)
    prev_dev = torch.from_numpy(prev).to(DEV).reshape(-1)
    gd = g.to(DEV)
    segs = [(0, S), (0, 0), (S, 0), (0, 1), (S - 1, 1), (5, 37), (16, 16), (17, S - 30), (S // 3, S // 3 + 1)]
    for (j0, n) in segs:
        j1 = j0 + n
        # plain segment compress: rows outside stay as they were
        out = torch.full((S * k,), 7.5, device=DEV)
        b.compress_segment(gd, w.N, j0, n, None, out)
        got = out.cpu().numpy().reshape(S, k)
        assert np.all(got[:j0] == 7.5) and np.all(got[j1:] == 7.5)
        if n:
            assert_close(got[j0:j1], ref_y[j0:j1], REL_TOL, f"compress_segment [{j0},{j1})")
        # fused ring step, out of place and in place
        out = torch.full((S * k,), 7.5, device=DEV)
        b.compress_segment(gd, w.N, j0, n, prev_dev, out)
        inpl = prev_dev.clone()
        b.compress_segment(gd, w.N, j0, n, inpl, inpl)
        torch.cuda.synchronize()
        got = out.cpu().numpy().reshape(S, k)
        assert np.all(got[:j0] == 7.5) and np.all(got[j1:] == 7.5)
        if n:
            want = ref_y[j0:j1] + prev[j0:j1].astype(np.float64)
            assert_close(got[j0:j1], want, REL_TOL, f"compress+accumulate [{j0},{j1})")
        gi = inpl.cpu().numpy().reshape(S, k)
        assert np.array_equal(gi[j0:j1], got[j0:j1])
        assert np.array_equal(gi[:j0], prev[:j0]) and np.array_equal(gi[j1:], prev[j1:])
        # segment decompress
        Y = torch.from_numpy(ref_y.astype(np.float32)).to(DEV).reshape(-1)
        xo = torch.full((w.M,), 7.5, device=DEV)
        b.decompress_segment(Y, j0, n, xo, "f32")
        torch.cuda.synchronize()
        gx = xo.cpu().numpy()
        lo, hi = j0 * d, min(j1 * d, w.M)
        assert np.all(gx[:lo] == 7.5) and np.all(gx[hi:] == 7.5)
        if n:
            ref_x = oracle.decompress(ref_y.astype(np.float32).astype(np.float64), U64, mu64, w.M, offsets=offs)
            assert_close(gx[lo:hi], ref_x[lo:hi], REL_TOL, f"decompress_segment [{j0},{j1})")
    L = gvq.lib()
    st = torch.cuda.current_stream().cuda_stream
    o = torch.zeros(S * k, device=DEV)
    assert L.gvq_compress_segment(b.handle, gd.data_ptr(), 1, -1, 2, None, o.data_ptr(), st) == gvq.EINVAL
    assert L.gvq_compress_segment(b.handle, gd.data_ptr(), 1, 1, S, None, o.data_ptr(), st) == gvq.EINVAL
    assert L.gvq_decompress_segment(b.handle, o.data_ptr(), S, 1, gd.data_ptr(), gvq.F32, st) == gvq.EINVAL
    b.close()


@pytest.mark.parametrize("M,d,k,N,dtype", [(128 * 1003 + 40, 128, 32, 6, "f32"), (64 * 500 + 1, 64, 16, 4, "bf16")])
def test_algorithm_1_on_one_gpu(M, d, k, N, dtype):
    """Algorithm 1 with the network replaced by pointer hand-over: every 'node' compresses
    segment [n-i] of its own gradient and adds what its predecessor sent; after N-1 steps node n
    holds the fully aggregated segment [n+1], which it decompresses.  The result must equal
    the plain compress / aggregate / decompress of Eqs. 2-4."""
    w = _wl(M, d, k, N, dtype)
    U32, mu32 = _basis(w)
    U64, mu64 = U32.astype(np.float64), mu32.astype(np.float64)
    workers = synth.worker_gradients(w, "cpu")
    dev = [g.to(DEV) for g in workers]
    b = gvq.Basis(w.M, w.d, w.k, None, w.dtype)
    b.import_(U32, mu32)
    S = b.S
    bounds = [S * i // N for i in range(N + 1)]          # N nearly equal segments of whole slices
    seg = lambda s: (bounds[s % N], bounds[s % N + 1] - bounds[s % N])
    # one compressed buffer per node; a "send" hands the segment's rows to the successor's buffer
    bufs = [torch.zeros(S * k, device=DEV) for _ in range(N)]
    for n in range(N):                                    # line 3: compress own segment n
        j0, cnt = seg(n)
        b.compress_segment(dev[n], N, j0, cnt, None, bufs[n])
    for i in range(1, N):                                 # lines 4-8
        for n in range(N):
            j0, cnt = seg(n - i)
            pred = bufs[(n - 1) % N]
            b.compress_segment(dev[n], N, j0, cnt, pred, bufs[n])   # download + compress + add
    out = torch.full((w.M,), float("nan"), device=DEV)
    for n in range(N):                                    # line 9: node n holds segment n+1 complete
        j0, cnt = seg(n + 1)
        b.decompress_segment(bufs[n], j0, cnt, out, "f32")
    torch.cuda.synchronize()
    ys = [oracle.compress(synth.to_numpy(g), U64, mu64, N, dtype=dtype) for g in workers]
    ref = oracle.decompress(oracle.aggregate(ys), U64, mu64, w.M)
    assert_close(out.cpu().numpy(), ref, REL_TOL, "Algorithm 1 result")
