"""gvq_flatten_conv / gvq_unflatten_conv against the oracle's index formula: bit-exact."""
import numpy as np
import pytest

import oracle
from paper_1811_03617_amd import gvq

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
DEV = "cuda:0"

SHAPES = [
    (16, 3, 3, 3),       # the paper's (3,3,16,16)-style first layer, depth 3
    (16, 16, 3, 3),      # the paper's example layer
    (64, 64, 3, 3), (128, 64, 3, 3), (70, 33, 3, 3),   # ragged filter / depth tiles
    (256, 128, 1, 1), (5, 7, 1, 1), (1, 1, 1, 1),
    (96, 3, 11, 11),     # large kernel: few depths per tile
    (32, 20, 5, 5), (64, 3, 7, 7),
    (8, 2, 13, 13),      # H*W too large for a tile: direct kernel
    (512, 512, 3, 3),    # 2.4 M numbers
    # the 128-bit path (F and D*H*W multiples of 4 for fp32, of 8 for bf16): ragged filter tile, ragged depth tile, one depth tile,
    # a fully connected layer (a plain transpose), H*W = 49 with 4 depths per tile, F below one tile
    (68, 36, 3, 3), (64, 28, 5, 5), (128, 4, 3, 3), (1000, 4096, 1, 1), (128, 8, 7, 7), (4, 240, 1, 1), (8, 484, 1, 1),
    (72, 40, 5, 5), (200, 24, 3, 3), (8, 16, 2, 2),   # ... and multiples of 8 for bf16
    (16, 8, 16, 16), (72, 3, 16, 24), (64, 5, 12, 12),   # H*W longer than a tile: one depth per tile, H*W in pieces
]


@pytest.mark.parametrize("F,D,H,W", SHAPES)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_flatten_and_unflatten_are_bit_exact(F, D, H, W, dtype):
    n = F * D * H * W
    rng = np.random.default_rng(F * 1000 + D)
    if dtype == "f32":
        host = rng.standard_normal((F, D, H, W)).astype(np.float32)
        src = torch.from_numpy(host).to(DEV)
        flat = torch.full((n,), float("nan"), device=DEV)
        back = torch.full((n,), float("nan"), device=DEV)
        code = gvq.F32
        bits = lambda t: t.cpu().numpy().view(np.uint32)
        want = oracle.flatten_conv(host).view(np.uint32)
        host_bits = host.view(np.uint32)
    else:
        host = rng.integers(0, 1 << 16, size=(F, D, H, W), dtype=np.uint16)   # arbitrary bf16 bit patterns
        src = torch.from_numpy(host.view(np.int16)).to(DEV)
        flat = torch.zeros(n, device=DEV, dtype=torch.int16)
        back = torch.zeros(n, device=DEV, dtype=torch.int16)
        code = gvq.BF16
        bits = lambda t: t.cpu().numpy().view(np.uint16)
        want = oracle.flatten_conv(host)
        host_bits = host
    gvq.gvq_flatten_conv(src, flat, F, D, H, W, code)
    gvq.gvq_unflatten_conv(flat, back, F, D, H, W, code)
    torch.cuda.synchronize()
    assert np.array_equal(bits(flat), want.ravel())
    assert np.array_equal(bits(back).reshape(F, D, H, W), host_bits)


def test_layout_argument_checks():
    L = gvq.lib()
    x = torch.zeros(64, device=DEV)
    y = torch.zeros(64, device=DEV)
    st = torch.cuda.current_stream().cuda_stream
    assert L.gvq_flatten_conv(x.data_ptr(), y.data_ptr(), 0, 1, 1, 1, gvq.F32, st) == gvq.EINVAL
    assert L.gvq_flatten_conv(x.data_ptr(), x.data_ptr(), 2, 2, 2, 2, gvq.F32, st) == gvq.EINVAL
    assert L.gvq_flatten_conv(None, y.data_ptr(), 2, 2, 2, 2, gvq.F32, st) == gvq.EINVAL
    assert L.gvq_flatten_conv(x.data_ptr() + 2, y.data_ptr(), 2, 2, 2, 2, gvq.F32, st) == gvq.EALIGN
    assert L.gvq_unflatten_conv(x.data_ptr(), y.data_ptr(), 2, 2, 2, 2, 9, st) == gvq.EINVAL
    assert L.gvq_flatten_conv(x.data_ptr() + 2, y.data_ptr(), 2, 2, 2, 2, gvq.BF16, st) == gvq.OK
    torch.cuda.synchronize()
