"""Seeded synthetic gradients for tests and benchmarks.

This module only draws random inputs; it contains none of the codec's arithmetic and is
the one piece of code that both the HIP path's tests and the CPU oracle's tests use.

Recipe (per workload): slice x = scale * (A z + sigma * eps), with A a d x rank matrix
of unit normals fixed by the seed (one per basis block when the workload has blocks),
z the latent coordinates (unit-variance normal or Laplace) and eps unit normal noise.
A "worker gradient" is one such draw over all slices, truncated to M elements; a "fit
gradient" is the sum of N fresh worker draws, because the paper fits its basis on
aggregated gradients.  bf16 workloads are rounded to bf16 once, here.
"""
import math

import numpy as np
import torch

from .configs import Workload

_CHUNK_SLICES = 1 << 18


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def planted_models(w: Workload, device="cpu") -> torch.Tensor:
    """[B, d, rank] float32: the planted mixing matrix of every basis block."""
    g = _gen(w.seed * 7919 + 1, "cpu")
    A = torch.randn(w.n_blocks, w.d, w.rank, generator=g, dtype=torch.float32)
    return A.to(device)


def layer_scale_per_slice(w: Workload, device="cpu") -> torch.Tensor:
    """[S] float32 scale of every slice (all ones unless the workload has layer scales)."""
    if not w.layer_scales:
        return torch.ones(w.S, dtype=torch.float32, device=device)
    g = _gen(w.seed * 7919 + 2, "cpu")
    expo = torch.rand(w.layer_scales, generator=g, dtype=torch.float32) * 3.0 - 4.0
    scales = torch.pow(torch.tensor(10.0), expo)
    per = (w.S + w.layer_scales - 1) // w.layer_scales
    idx = torch.arange(w.S) // per
    return scales[idx].to(device)


def _draw(w: Workload, g: torch.Generator, A: torch.Tensor, scale: torch.Tensor, device,
          mean_offset=None) -> torch.Tensor:
    """One fp32 draw of S*d numbers (before truncation to M)."""
    S, d, r = w.S, w.d, w.rank
    out = torch.empty(S * d, dtype=torch.float32, device=device)
    offs = w.block_offsets() or [0, S]
    per_block = offs[1] - offs[0]
    for s0 in range(0, S, _CHUNK_SLICES):
        s1 = min(S, s0 + _CHUNK_SLICES)
        n = s1 - s0
        z = torch.randn(n, r, generator=g, dtype=torch.float32, device=device)
        if w.latent == "laplace":
            # unit-variance Laplace: sign * Exp(1) / sqrt(2)
            mag = -torch.log1p(-torch.rand(n, r, generator=g, dtype=torch.float32, device=device))
            z = torch.sign(z) * mag / math.sqrt(2.0)
        eps = torch.randn(n, d, generator=g, dtype=torch.float32, device=device)
        if A.shape[0] == 1:
            x = z @ A[0].T
        else:
            blk = torch.arange(s0, s1, device=device) // per_block
            x = torch.einsum("nr,ndr->nd", z, A[blk])
        x = (x + w.sigma * eps) * scale[s0:s1, None]
        if mean_offset is not None:
            x = x + mean_offset[None, :]
        out[s0 * d:s1 * d] = x.reshape(-1)
    return out


def _store(w: Workload, x32: torch.Tensor) -> torch.Tensor:
    x32 = x32[: w.M]
    return x32.to(torch.bfloat16) if w.dtype == "bf16" else x32.contiguous()


def worker_gradients(w: Workload, device="cpu", mean_offset=None, stream=0):
    """List of N worker gradients (1-D tensors of M elements in the storage dtype)."""
    A = planted_models(w, device)
    scale = layer_scale_per_slice(w, device)
    g = _gen(w.seed * 7919 + 100 + stream, device)
    mo = None if mean_offset is None else torch.as_tensor(mean_offset, dtype=torch.float32,
                                                          device=device) / w.N
    return [_store(w, _draw(w, g, A, scale, device, mo)) for _ in range(w.N)]


def fit_gradients(w: Workload, device="cpu", mean_offset=None, L=None):
    """List of L fit gradients, each the sum of N fresh worker draws."""
    A = planted_models(w, device)
    scale = layer_scale_per_slice(w, device)
    g = _gen(w.seed * 7919 + 50, device)
    mo = None if mean_offset is None else torch.as_tensor(mean_offset, dtype=torch.float32,
                                                          device=device) / w.N
    out = []
    for _ in range(w.L if L is None else L):
        acc = _draw(w, g, A, scale, device, mo)
        for _ in range(w.N - 1):
            acc += _draw(w, g, A, scale, device, mo)
        out.append(_store(w, acc))
    return out


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """Host copy for the oracle: float32 array, or uint16 bit patterns for bf16."""
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()
