"""The hot path under HIP graph capture: every entry point only enqueues kernels on the caller's
stream, so one aggregation step (N x compress, aggregate, decompress, plus the Eq. 6 monitor) can be
captured once and replayed.  Each replay is checked bit for bit against the same calls made eagerly,
with eager work and synchronisation between the replays."""
import numpy as np
import pytest

from paper_1811_03617_amd import Workload, gvq, synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("M,d,k,N,dtype,block_elems", [
    (128 * 3000 + 40, 128, 32, 4, "f32", 0),            # register-resident kernels
    (128 * 2000 + 40, 128, 16, 3, "bf16", 128 * 300),   # bf16 pipe, several bases
    (768 * 300 + 9, 768, 96, 2, "f32", 0),              # basis-stationary kernels, bf16-split products
    (1024 * 200 + 5, 1024, 16, 2, "f32", 0),            # basis-stationary kernels, exact fp32 products
    (768 * 300 + 9, 768, 96, 2, "bf16", 0),             # LDS-tiled kernels
])
def test_graph_replays_match_eager_calls(M, d, k, N, dtype, block_elems):
    w = Workload("t", M, d, k, N, 2, dtype, 4, 0.1, block_elems=block_elems, seed=31)
    offs = w.block_offsets()
    rng = np.random.default_rng(5)
    U = np.stack([np.linalg.qr(rng.standard_normal((d, k)))[0] for _ in range(w.n_blocks)]).astype(np.float32)
    mu = (0.1 * rng.standard_normal((w.n_blocks, d))).astype(np.float32)
    b = gvq.Basis(M, d, k, offs, dtype)
    b.import_(U, mu)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    S = b.S

    def buffers():
        return ([torch.zeros(M, device=DEV, dtype=tdt) for _ in range(N)],
                [torch.zeros(S * k, device=DEV) for _ in range(N)],
                torch.zeros(S * k, device=DEV), torch.zeros(M, device=DEV, dtype=tdt),
                torch.zeros(w.n_blocks, device=DEV, dtype=torch.float64))

    def step(grads, comps, total, out, loss):
        for g, c in zip(grads, comps):
            b.compress(g, N, c)
        b.aggregate(comps, total)
        b.decompress(total, out)
        b.local_loss(grads[0], N, loss)

    static = buffers()
    eager = buffers()
    step(*static)                       # first launches: one-time runtime queries happen here
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(*static)
    for rep in range(3):
        fresh = synth.worker_gradients(w, DEV, stream=rep + 1)
        for dst_s, dst_e, src in zip(static[0], eager[0], fresh):
            dst_s.copy_(src)
            dst_e.copy_(src)
        graph.replay()
        step(*eager)                    # eager work between the replays
        torch.cuda.synchronize()
        for cs, ce in zip(static[1], eager[1]):
            assert torch.equal(cs, ce), f"replay {rep}: compressed"
        assert torch.equal(static[2], eager[2]), f"replay {rep}: aggregate"
        assert torch.equal(static[3], eager[3]), f"replay {rep}: decompress"
        assert torch.equal(static[4], eager[4]), f"replay {rep}: local loss"
        assert bool(torch.isfinite(static[3].float()).all()) and float(static[2].abs().max()) > 0
    b.close()
