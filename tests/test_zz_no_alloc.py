"""gvq_local_loss_static, the entry point for callers that cannot allocate: same result as gvq_local_loss
(Section 3, Eq. 6), whose scratch lives in the handle, on two calls in a row, the second on a smaller
gradient (the fixed buffer then still holds the first call's numbers beyond what the second one writes)."""
import numpy as np
import pytest

import oracle
from paper_1811_03617_amd import gvq, synth
from _util import REL_TOL

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _case(M, d, k, offs, dtype, N, seed):
    rng = np.random.default_rng(seed)
    B = 1 if offs is None else len(offs) - 1
    U = np.stack([np.linalg.qr(rng.standard_normal((d, k)))[0] for _ in range(B)]).astype(np.float32)
    mu = (0.1 * rng.standard_normal((B, d))).astype(np.float32)
    g = torch.randn(M, generator=torch.Generator().manual_seed(seed)).to(DEV)
    if dtype == "bf16":
        g = g.to(torch.bfloat16)
    b = gvq.Basis(M, d, k, offs, dtype)
    b.import_(U, mu)
    want = torch.full((B,), float("nan"), device=DEV, dtype=torch.float64)
    got = torch.full((B,), float("nan"), device=DEV, dtype=torch.float64)
    b.local_loss(g, N, want)
    b.local_loss_static(g, N, got)
    torch.cuda.synchronize()
    want, got = want.cpu().numpy(), got.cpu().numpy()
    ref = oracle.local_loss(synth.to_numpy(g), U.astype(np.float64), mu.astype(np.float64), N, dtype=dtype, offsets=offs)
    b.close()
    assert np.all(np.isfinite(got))
    # the same kernels in the same order: bit-identical to the handle-scratch entry point ...
    assert np.array_equal(got, want)
    # ... and within the codec tolerance of the oracle
    np.testing.assert_allclose(got, ref, rtol=REL_TOL)


def test_static_scratch_entry_point_matches_on_two_calls_in_a_row():
    # first a larger gradient with several bases (slice lengths of the register-resident kernels) ...
    _case(128 * 40000 + 40, 128, 32, [0, 9000, 9001, 25000, 40001], "f32", 4, 1)
    # ... then a smaller one, which overwrites only the front of the shared buffer
    _case(128 * 3000 + 7, 128, 16, None, "bf16", 2, 2)
    # and the LDS-tiled route (long slices), smaller again
    _case(768 * 500 + 100, 768, 96, [0, 200, 501], "f32", 3, 3)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import ctypes as C
    M, d, k = 2 * (gvq.STATIC_MAX_SLICES + 1), 2, 1
    b = gvq.Basis(M, d, k)
    b.import_(np.ones((1, d, k), np.float32) / np.sqrt(2.0), np.zeros((1, d), np.float32))
    g = torch.zeros(M, device=DEV)
    out = torch.zeros(1, device=DEV, dtype=torch.float64)
    rc = gvq.lib().gvq_local_loss_static(b.handle, g.data_ptr(), 1, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == gvq.ETOOBIG
    assert "static scratch" in gvq.strerror(rc)
    b.close()
