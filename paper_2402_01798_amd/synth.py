"""Seeded synthetic gradients with the heavy-tailed shape the paper argues for.

The paper measures on gradients of networks trained on an image data set
(Sec. I, Fig. 1; Sec. V); neither is available here, so these generators stand
in for them: symmetric power-law (Pareto) magnitudes, optionally mixed with a
Gaussian bulk or scaled per layer.  "gamma" is the exponent of the density
p(g) ~ |g|^-gamma as in the paper's power-law definition (Sec. IV-A), so the
magnitude is x_min * u^(-1/(gamma-1)) for u uniform in (0, 1].

Nothing here is part of the quantizer: the module only makes inputs, and the
same bytes are handed to the GPU library and to whatever checks it.
"""
from dataclasses import dataclass, field
from typing import Optional, Tuple

import torch

GRID_UNIFORM, GRID_NONUNIFORM = 0, 1


@dataclass(frozen=True)
class Workload:
    name: str
    d: int                       # elements per worker
    workers: int                 # N
    dtype: torch.dtype           # gradient dtype
    bits: Tuple[int, ...]        # b values the configuration names
    grids: Tuple[int, ...]       # grid families the configuration names
    bucket_elems: int            # 0 = one bucket per tensor
    g_min: float                 # 0 = let the library pick the tail edge
    gamma: float
    x_min: float
    gauss_frac: float = 0.0      # share of N(0, gauss_sigma^2) entries
    gauss_sigma: float = 0.0
    layer_scale: Optional[Tuple[float, float]] = None   # log-uniform range


WORKLOADS = {
    "cfg1": Workload("cfg1", 61_706, 4, torch.float32, (3,), (GRID_UNIFORM,), 0,
                     1e-4, 3.0, 1e-4),
    "cfg2": Workload("cfg2", 11_200_000, 8, torch.float32, (2, 4), (GRID_UNIFORM,), 0,
                     0.0, 2.5, 1e-5, gauss_frac=0.1, gauss_sigma=1e-4),
    "cfg3": Workload("cfg3", 25_600_000, 16, torch.float32, (3,), (GRID_NONUNIFORM,),
                     1 << 20, 1e-5, 2.2, 1e-5),
    "cfg4": Workload("cfg4", 124_000_000, 8, torch.float32, (2,),
                     (GRID_UNIFORM, GRID_NONUNIFORM), 1 << 20, 0.0, 3.0, 1.0,
                     layer_scale=(1e-6, 1e-2)),
    "cfg5": Workload("cfg5", 1_000_000_000, 4, torch.bfloat16, (2,), (GRID_NONUNIFORM,),
                     0, 1e-6, 2.1, 1e-6),
}

_CHUNK = 1 << 24


def _seed(wl: Workload, worker: int, salt: int = 0) -> int:
    return (0x7451 << 32) + (sum(map(ord, wl.name)) << 16) + (salt << 8) + worker


def make_gradient(wl: Workload, worker: int, device="cpu", d: Optional[int] = None,
                  dtype: Optional[torch.dtype] = None) -> torch.Tensor:
    """Worker ``worker``'s flat gradient of workload ``wl`` (first ``d`` elements' recipe).

    Deterministic per (workload, worker, device type); generated in chunks so
    the largest workload never needs more than its own size plus 256 MiB.
    """
    d = wl.d if d is None else d
    dtype = wl.dtype if dtype is None else dtype
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(_seed(wl, worker))
    out = torch.empty(d, dtype=dtype, device=dev)
    expo = -1.0 / (wl.gamma - 1.0)
    scale = None
    if wl.layer_scale is not None:
        scale = _layer_scales(wl, worker, d).to(dev)
    for lo in range(0, d, _CHUNK):
        n = min(_CHUNK, d - lo)
        u = 1.0 - torch.rand(n, generator=gen, device=dev, dtype=torch.float32)  # (0, 1]
        mag = wl.x_min * u.double().pow_(expo)
        sign = torch.randint(0, 2, (n,), generator=gen, device=dev, dtype=torch.int8)
        x = torch.where(sign.bool(), mag, -mag)
        if wl.gauss_frac > 0.0:
            pick = torch.rand(n, generator=gen, device=dev, dtype=torch.float32) < wl.gauss_frac
            bulk = torch.randn(n, generator=gen, device=dev, dtype=torch.float64) * wl.gauss_sigma
            x = torch.where(pick, bulk, x)
        if scale is not None:
            x = x * scale[lo:lo + n]
        out[lo:lo + n] = x.to(dtype)
    return out


def _layer_scales(wl: Workload, worker: int, d: int) -> torch.Tensor:
    """Per-element scale: consecutive "layers" of 2^U[10,24] elements, each with one
    scale drawn log-uniformly from ``wl.layer_scale`` (same layers for every worker)."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(_seed(wl, 0, salt=1))
    lo_s, hi_s = wl.layer_scale
    lo_l, hi_l = torch.log10(torch.tensor(lo_s)), torch.log10(torch.tensor(hi_s))
    scales = torch.empty(d, dtype=torch.float64)
    pos = 0
    while pos < d:
        length = int(2.0 ** (10.0 + 14.0 * torch.rand((), generator=gen).item()))
        sc = 10.0 ** (lo_l + (hi_l - lo_l) * torch.rand((), generator=gen)).item()
        scales[pos:pos + length] = sc
        pos += length
    return scales


def layer_segments(wl: Workload, d: Optional[int] = None):
    """Offsets [0, ..., d] of the workload's layers (the same draw as ``_layer_scales``), each interior
    boundary moved down to a multiple of 128: the segment table of a per-layer quantizer."""
    d = wl.d if d is None else d
    gen = torch.Generator(device="cpu")
    gen.manual_seed(_seed(wl, 0, salt=1))
    offs, pos = [0], 0
    while pos < d:
        length = int(2.0 ** (10.0 + 14.0 * torch.rand((), generator=gen).item()))
        torch.rand((), generator=gen)                       # the layer's scale, drawn by _layer_scales
        pos += length
        cut = min(pos, d) // 128 * 128
        if pos < d and cut > offs[-1]:
            offs.append(cut)
    offs.append(d)
    return offs


def as_numpy(t: torch.Tensor):
    """Host numpy view: float32 as is, bfloat16 as its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
