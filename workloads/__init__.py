"""Seeded synthetic inputs for the ISA operator.

This module only draws random tensors with the shapes and the structure of
the benchmark configurations.  It holds none of the operator's arithmetic and
is used by both the CPU oracle's tests and the HIP path's tests / benchmark,
which is what lets the two sides see byte-identical inputs.

Recipe (one per configuration, all seeded):
  * tokens live on a (t, h, w) grid, flattened row-major with w fastest; the
    source segment comes first, then every context reference;
  * K and V: per (batch, head, channel, segment) an independent N(0,1) field
    on the segment's grid, smoothed with a separable Gaussian (sigma = 2
    tokens, radius 6, renormalised at the borders), centred and rescaled to
    unit standard deviation, plus 0.3 * N(0,1) white noise;
  * context keys are multiplied by 0.5 (context is less salient than source);
  * Q: N(0,1) times a per-(batch, head, token) factor drawn log-uniformly
    from [0.5, 4];
  * the result is rounded once to the configuration's storage type (bf16 or
    fp32); every consumer starts from those rounded values.
"""
import math
from dataclasses import dataclass, field
from typing import List, Tuple

import torch

Grid = Tuple[int, int, int]


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    D: int
    dtype: str                      # "bf16" or "f32"
    block: int
    src_grid: Grid
    ctx_grids: Tuple[Tuple[Grid, ...], ...]   # per batch item: one grid per context reference
    keep_ratio: float
    full_frac: float
    seed: int
    exact_frac: float = 0.0
    gamma: float = 0.0              # coarse stacking factor of Alg. 1 Stage 5 (0 in every named configuration)
    centred: bool = True            # subtract each smooth field's mean before rescaling it (every named configuration)
    key_offset: float = 0.0         # a constant added to every channel of every key (0 in every named configuration)

    def seg_len(self, b: int) -> List[int]:
        """Token counts of batch item b: source first, then each context reference."""
        return [math.prod(self.src_grid)] + [math.prod(g) for g in self.ctx_grids[b]]

    def tokens(self, b: int) -> int:
        return sum(self.seg_len(b))

    @property
    def S_max(self) -> int:
        return max(self.tokens(b) for b in range(self.B))

    def with_(self, **kw) -> "Workload":
        d = dict(self.__dict__)
        d.update(kw)
        return Workload(**d)


_G480 = (21, 30, 52)
_G720 = (21, 45, 80)

CONFIGS = {
    "cfg0": Workload("cfg0", 1, 2, 64, "f32", 64, (4, 8, 16), (((4, 8, 16),),), 0.5, 0.25, 20260504),
    "cfg1": Workload("cfg1", 1, 40, 128, "bf16", 128, (5, 30, 52), (((5, 30, 52),),), 0.5, 0.25, 20260505),
    "cfg2": Workload("cfg2", 1, 40, 128, "bf16", 128, _G480, ((_G480,),), 0.5, 0.2, 20260506),
    "cfg3": Workload("cfg3", 2, 40, 128, "bf16", 128, _G480, (((1, 30, 52), _G480), ((11, 30, 52),)), 0.5, 0.2,
                     20260507),
    "cfg4": Workload("cfg4", 1, 40, 128, "bf16", 128, _G720, ((_G720,),), 0.5, 0.2, 20260508),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"bf16": torch.bfloat16, "f32": torch.float32}[name]


def _gauss_weights(sigma: float, radius: int, device) -> torch.Tensor:
    x = torch.arange(-radius, radius + 1, dtype=torch.float32, device=device)
    w = torch.exp(-0.5 * (x / sigma) ** 2)
    return w / w.sum()


def _smooth_axis(x: torch.Tensor, axis: int, w: torch.Tensor) -> torch.Tensor:
    """Filter along one grid axis with zero padding, renormalised at the borders.
    Written as a sum of shifted slices (plain elementwise kernels on any device)."""
    radius = (w.numel() - 1) // 2
    n = x.shape[axis]
    pad = [0, 0] * (x.dim() - 1 - axis) + [radius, radius]
    xp = torch.nn.functional.pad(x, pad)
    ones = torch.nn.functional.pad(torch.ones(n, device=x.device, dtype=x.dtype), [radius, radius])
    y = torch.zeros_like(x)
    norm = torch.zeros(n, device=x.device, dtype=x.dtype)
    for k in range(w.numel()):
        y = y + float(w[k]) * xp.narrow(axis, k, n)
        norm = norm + float(w[k]) * ones[k:k + n]
    shape = [1] * x.dim()
    shape[axis] = n
    return y / norm.view(shape)


def smooth_field(n_fields: int, grid: Grid, gen: torch.Generator, device, sigma=2.0, radius=6, noise=0.3, centred=True):
    """[n_fields, t*h*w] fp32: unit-variance smooth fields plus white noise.  Not `centred`: the filtered field keeps
    whatever mean its few independent samples happen to have (on a grid of a few tokens that mean is as large as the
    field's variation) and is only rescaled."""
    t, h, w_ = grid
    f = torch.randn((n_fields, t, h, w_), generator=gen, device=device, dtype=torch.float32)
    wts = _gauss_weights(sigma, radius, device)
    for axis in (1, 2, 3):
        f = _smooth_axis(f, axis, wts)
    f = f.reshape(n_fields, -1)
    if centred:
        f = f - f.mean(dim=1, keepdim=True)        # small grids: keep the field centred before rescaling
    f = f / f.std(dim=1, unbiased=False, keepdim=True).clamp_min(1e-6)
    f = f + noise * torch.randn(f.shape, generator=gen, device=device, dtype=torch.float32)
    return f


def make_inputs(wl: Workload, device="cpu", heads_per_chunk: int = 8):
    """Q, K, V as [B, H, S_max, D] tensors of the workload's storage type on `device`.

    Rows of a batch item past its own token count are zero and are never read
    by the operator.  Returns (Q, K, V).
    """
    device = torch.device(device)
    dt = torch_dtype(wl.dtype)
    Q = torch.zeros((wl.B, wl.H, wl.S_max, wl.D), dtype=dt, device=device)
    K = torch.zeros_like(Q)
    V = torch.zeros_like(Q)
    gen = torch.Generator(device=device)
    gen.manual_seed(wl.seed)
    for b in range(wl.B):
        segs = [wl.src_grid] + list(wl.ctx_grids[b])
        for h0 in range(0, wl.H, heads_per_chunk):
            nh = min(heads_per_chunk, wl.H - h0)
            off = 0
            for si, grid in enumerate(segs):
                n = math.prod(grid)
                for which, dst in (("k", K), ("v", V)):
                    f = smooth_field(nh * wl.D, grid, gen, device, centred=wl.centred)            # [nh*D, n]
                    if which == "k" and si > 0:
                        f = f * 0.5
                    if which == "k" and wl.key_offset != 0.0:
                        f = f + wl.key_offset
                    dst[b, h0:h0 + nh, off:off + n, :] = f.view(nh, wl.D, n).transpose(1, 2).to(dt)
                qn = torch.randn((nh, n, wl.D), generator=gen, device=device, dtype=torch.float32)
                u = torch.rand((nh, n, 1), generator=gen, device=device, dtype=torch.float32)
                factor = torch.exp(math.log(0.5) + u * (math.log(4.0) - math.log(0.5)))
                Q[b, h0:h0 + nh, off:off + n, :] = (qn * factor).to(dt)
                off += n
    return Q, K, V


def small_variant(base: Workload, name: str, src_grid: Grid, ctx_grids, H: int = None, **kw) -> Workload:
    """A shrunken workload with the same recipe, for element-by-element parity tests."""
    return base.with_(name=name, src_grid=src_grid, ctx_grids=ctx_grids, H=base.H if H is None else H, **kw)
