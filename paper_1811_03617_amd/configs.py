"""The five benchmark workloads and one long-slice workload (shapes only; no arithmetic of
the method here).

Each is a synthetic stand-in for the flattened convolutional gradient of a CNN of that
size: a planted low-rank linear model per slice plus isotropic noise, which gives the
"adjacent gradients are linearly correlated" structure that the paper's Section 2
exploits.
"""
from dataclasses import dataclass
from typing import List, Optional


@dataclass(frozen=True)
class Workload:
    name: str
    M: int                 # elements of one flattened gradient
    d: int                 # slice length (the paper's K)
    k: int                 # kept components (the paper's d)
    N: int                 # simulated workers
    L: int                 # gradients the basis is fitted on (the paper's L_t)
    dtype: str             # "f32" or "bf16": how gradients are stored
    rank: int              # rank of the planted model
    sigma: float           # isotropic noise level
    latent: str = "gauss"  # "gauss" or "laplace" latent coordinates
    layer_scales: int = 0  # >0: that many contiguous segments with log-uniform scales
    block_elems: int = 0   # >0: one basis (and one planted model) per this many elements
    seed: int = 0

    @property
    def S(self) -> int:
        return (self.M + self.d - 1) // self.d

    def block_offsets(self) -> Optional[List[int]]:
        """Slice offsets of the bases, or None for a single basis."""
        if not self.block_elems:
            return None
        per = (self.block_elems + self.d - 1) // self.d
        offs = list(range(0, self.S, per))
        offs.append(self.S)
        return offs

    @property
    def n_blocks(self) -> int:
        o = self.block_offsets()
        return 1 if o is None else len(o) - 1


WORKLOADS = {
    "tiny": Workload("tiny", 460_800, 16, 4, 4, 8, "f32", 3, 0.05, seed=1001),
    "resnet50": Workload("resnet50", 25_557_032, 32, 8, 8, 16, "f32", 6, 0.1,
                         layer_scales=64, seed=1002),
    "alexnet": Workload("alexnet", 61_100_840, 64, 16, 8, 16, "f32", 12, 0.1,
                        latent="laplace", seed=1003),
    "vgg16": Workload("vgg16", 138_357_544, 128, 32, 16, 32, "f32", 24, 0.05, seed=1004),
    "vgg16_bf16": Workload("vgg16_bf16", 138_357_544, 128, 16, 16, 32, "bf16", 24, 0.05,
                           block_elems=1_000_000, seed=1005),
    # the slice size of the paper's own example (Section 3: 768 = 3 x 16 x 16 for a
    # (3,3,16,16) layer) at 8x compression, on a gradient of the vgg16 workload's size
    "conv768": Workload("conv768", 138_357_544, 768, 96, 8, 8, "f32", 24, 0.05, seed=1006),
}
