"""A seeded sweep over slice lengths, component counts, gradient lengths, numbers of bases and storage
types: every combination is routed to one of the kernel families (register-resident, LDS-tiled on either
matrix pipe, basis-stationary, column passes, one thread per output), and whatever route it takes, Eq. 2, 3,
4 and 6 must agree with the oracle.  The bases are random orthonormal columns and random means: the codec
does not care where its basis comes from."""
import numpy as np
import pytest

import oracle
from paper_1811_03617_amd import gvq
from _util import REL_TOL, assert_close, bf16_bits_to_f64, f64_to_bf16_bits_rne

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _cases():
    rng = np.random.default_rng(20181103)
    out = []
    pool = [2, 3, 8, 16, 24, 32, 48, 64, 96, 100, 127, 128, 129, 192, 256, 320, 384, 512, 640, 768, 1000, 1024]
    for i in range(56):
        d = int(pool[rng.integers(len(pool))]) if i % 4 else int(rng.integers(2, 1025))
        kmax = d if rng.random() < 0.2 else max(1, d // 4)
        k = int(rng.integers(1, kmax + 1))
        if rng.random() < 0.5 and k >= 4:
            k -= k % 4
        slices = int(rng.integers(1, 420))
        tail = int(rng.integers(0, d)) if rng.random() < 0.6 else 0
        M = max(1, (slices - (1 if tail else 0)) * d + tail)
        S = (M + d - 1) // d
        nb = 1 if rng.random() < 0.55 or S < 4 else int(rng.integers(2, min(6, S) + 1))
        offs = None
        if nb > 1:
            cuts = np.sort(rng.choice(np.arange(1, S), size=nb - 1, replace=False))
            offs = [0] + [int(c) for c in cuts] + [S]
        dtype = "bf16" if rng.random() < 0.35 else "f32"
        N = int(rng.integers(1, 5))
        out.append((i, M, d, k, N, dtype, offs))
    return out


@pytest.mark.parametrize("seed,M,d,k,N,dtype,offs", _cases(), ids=lambda v: str(v) if not isinstance(v, list) else f"B{len(v) - 1}")
def test_whatever_route_a_shape_takes_matches_the_oracle(seed, M, d, k, N, dtype, offs):
    rng = np.random.default_rng(1000 + seed)
    B = 1 if offs is None else len(offs) - 1
    U32 = np.stack([np.linalg.qr(rng.standard_normal((d, k)))[0] for _ in range(B)]).astype(np.float32)
    mu32 = (0.3 * rng.standard_normal((B, d))).astype(np.float32)
    U64, mu64 = U32.astype(np.float64), mu32.astype(np.float64)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    gen = torch.Generator().manual_seed(seed)
    workers = [torch.randn(M, generator=gen).to(tdt) for _ in range(N)]
    workers_np = [(w.view(torch.int16).numpy().view(np.uint16) if dtype == "bf16" else w.numpy()) for w in workers]

    b = gvq.Basis(M, d, k, offs, dtype)
    b.import_(U32, mu32)
    comps = [torch.full((b.S * k,), float("nan"), device=DEV) for _ in workers]
    for g, c in zip(workers, comps):
        b.compress(g.to(DEV), N, c)
    total = torch.full((b.S * k,), float("nan"), device=DEV)
    b.aggregate(comps, total)
    out = torch.full((M,), float("nan"), device=DEV, dtype=tdt)
    b.decompress(total, out, dtype)
    loss = torch.empty(B, device=DEV, dtype=torch.float64)
    b.local_loss(workers[0].to(DEV), N, loss)
    torch.cuda.synchronize()

    ref = [oracle.compress(g, U64, mu64, N, dtype=dtype, offsets=offs) for g in workers_np]
    for n, (c, r) in enumerate(zip(comps, ref)):
        assert_close(c.cpu().numpy().reshape(b.S, k), r, REL_TOL, f"compress worker {n}")
    got_total = total.cpu().numpy().reshape(b.S, k)
    assert_close(got_total, oracle.aggregate(ref), REL_TOL, "aggregate")
    ref_x = oracle.decompress(got_total.astype(np.float64), U64, mu64, M, offsets=offs)
    if dtype == "bf16":
        got = bf16_bits_to_f64(out.view(torch.int16).cpu().numpy().view(np.uint16))
        want = bf16_bits_to_f64(f64_to_bf16_bits_rne(ref_x))
        step = np.maximum(np.abs(want) * 2.0 ** -7, REL_TOL * np.max(np.abs(ref_x)))   # one bf16 step, or the codec tolerance
        assert np.all(np.abs(got - want) <= step)
        assert np.mean(got != want) <= 0.01
    else:
        assert_close(out.cpu().numpy(), ref_x, REL_TOL, "decompress")
    ref_loss = oracle.local_loss(workers_np[0], U64, mu64, N, dtype=dtype, offsets=offs)
    energy = oracle.local_loss(workers_np[0], np.zeros((B, d, 1)), mu64, N, dtype=dtype, offsets=offs)
    got_loss = loss.cpu().numpy()
    assert np.all(np.abs(got_loss - ref_loss) <= 1e-4 * ref_loss + 1e-7 * energy), (got_loss, ref_loss)
    b.close()
