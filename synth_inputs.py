"""Seeded synthetic inputs and workload descriptions shared by the tests, the
smoke check and the benchmark.

This module holds none of the method's arithmetic: it only draws random
tensors and names shapes.  Both the CPU oracle and the HIP path are fed the
SAME host tensors produced here.

The paper measures on HunyuanVideo activations (latent grid 30x48x80, 24
heads, head dim 128, bf16 -- Sec. 4 and the kernel benchmark table); those
need trained weights, so i.i.d. N(0,1) tensors of the same shapes stand in.
The kernel has no data-dependent control flow, so timing is unaffected.
"""
from dataclasses import dataclass, field
from typing import List, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    H: int
    D: int
    grid: Tuple[int, int, int]
    tile: Tuple[int, int, int]
    window_tiles: Tuple[Tuple[int, int, int], ...]   # one entry per head
    dtype: str                                      # "bf16" or "f32" (dtype of the raster inputs)
    seed: int

    @property
    def N(self) -> int:
        return self.grid[0] * self.grid[1] * self.grid[2]

    @property
    def P(self) -> int:
        return self.tile[0] * self.tile[1] * self.tile[2]

    @property
    def tile_grid(self) -> Tuple[int, int, int]:
        return tuple(g // t for g, t in zip(self.grid, self.tile))

    @property
    def n_tiles(self) -> int:
        a, b, c = self.tile_grid
        return a * b * c


def splitmix64(x: int) -> int:
    """Counter-based 64-bit mixer (public-domain SplitMix64 finaliser)."""
    mask = (1 << 64) - 1
    x = (x + 0x9E3779B97F4A7C15) & mask
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
    return z ^ (z >> 31)


MIXED_WINDOW_CHOICES = ((1, 3, 3), (3, 3, 3), (3, 3, 5), (5, 6, 10))


def mixed_windows(seed: int, H: int):
    """Per-head window drawn from MIXED_WINDOW_CHOICES by a counter-based draw."""
    return tuple(MIXED_WINDOW_CHOICES[splitmix64(seed + h) % len(MIXED_WINDOW_CHOICES)] for h in range(H))


def _uniform(H, w):
    return tuple(tuple(w) for _ in range(H))


def workload(name: str) -> Workload:
    """The five configurations of the benchmark spec, plus the dense variant of C4."""
    if name == "C1":   # tiny 3D, fp32 inputs
        return Workload("C1", 1, 1, 64, (18, 24, 24), (6, 8, 8), _uniform(1, (1, 3, 3)), "f32", 1001)
    if name == "C2":   # 2D, image style
        return Workload("C2", 1, 8, 64, (1, 64, 64), (1, 8, 8), _uniform(8, (1, 3, 3)), "bf16", 1002)
    if name == "C3":   # mid-size 3D
        return Workload("C3", 1, 12, 128, (12, 48, 48), (6, 8, 8), _uniform(12, (1, 3, 3)), "bf16", 1003)
    if name == "C4":   # HunyuanVideo-shaped layer, 3x3x3 tiles
        return Workload("C4", 1, 24, 128, (30, 48, 80), (6, 8, 8), _uniform(24, (3, 3, 3)), "bf16", 1004)
    if name == "C4dense":
        return Workload("C4dense", 1, 24, 128, (30, 48, 80), (6, 8, 8), _uniform(24, (5, 6, 10)), "bf16", 1004)
    if name == "C5":   # per-head windows mixed in one launch
        return Workload("C5", 1, 24, 128, (30, 48, 80), (6, 8, 8), mixed_windows(1005, 24), "bf16", 1005)
    # Not among the task's configurations: head dimension 64 at sizes that fill the chip, for timing and profiling
    if name == "D64-2D":    # 128 heads (batch 16 x 8) of the 2D image shape of C2
        return Workload("D64-2D", 16, 8, 64, (1, 64, 64), (1, 8, 8), _uniform(8, (1, 3, 3)), "bf16", 1006)
    if name == "D64-3D":    # the grid, tile and window of C4 with the head dimension of C1
        return Workload("D64-3D", 1, 24, 64, (30, 48, 80), (6, 8, 8), _uniform(24, (3, 3, 3)), "bf16", 1007)
    raise KeyError(name)


def with_window(w: Workload, window_tiles) -> Workload:
    return Workload(w.name + "_w%dx%dx%d" % tuple(window_tiles), w.B, w.H, w.D, w.grid, w.tile,
                    _uniform(w.H, window_tiles), w.dtype, w.seed)


def custom(name, B, H, D, grid, tile, window_tiles, dtype="bf16", seed=0) -> Workload:
    if len(window_tiles) == 3 and all(isinstance(x, int) for x in window_tiles):
        window_tiles = _uniform(H, window_tiles)
    return Workload(name, B, H, D, tuple(grid), tuple(tile), tuple(tuple(w) for w in window_tiles), dtype, seed)


def make_qkv(w: Workload, device="cpu"):
    """Q, K, V in raster order, [B, H, N, D]; drawn fp32 N(0,1) on the host from
    one generator (Q, then K, then V), then rounded to the workload's dtype."""
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed)
    shape = (w.B, w.H, w.N, w.D)
    out = []
    for _ in range(3):
        x = torch.randn(shape, generator=g, dtype=torch.float32)
        if w.dtype == "bf16":
            x = x.to(torch.bfloat16)
        out.append(x.to(device) if device != "cpu" else x)
    return tuple(out)


def make_dout(w: Workload):
    """Upstream gradient of the attention output for the gradient tests, [B, H, N, D] in raster order: N(0,1)
    drawn on the host from its own generator (seed + 7919), rounded to bf16."""
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed + 7919)
    return torch.randn((w.B, w.H, w.N, w.D), generator=g, dtype=torch.float32).to(torch.bfloat16)


def make_qkv_device(w: Workload, device="cuda:0"):
    """Same distribution drawn directly on the device (benchmark-only inputs
    for sizes where a host draw would dominate the run; not used for parity)."""
    g = torch.Generator(device=device)
    g.manual_seed(w.seed)
    shape = (w.B, w.H, w.N, w.D)
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    return tuple(torch.randn(shape, generator=g, dtype=torch.float32, device=device).to(dt) for _ in range(3))


def strata_tiles(w):
    """Query tiles by stratum of the tile grid: all corners, one tile per edge direction and per face direction
    (where the grid has them), and up to four interior tiles.  Row-major tile ids, no duplicates, corners first."""
    nt, nh, nw = w.tile_grid
    rm = lambda a, b, c: (a * nh + b) * nw + c
    ends = lambda n: sorted({0, n - 1})
    mid = lambda n: n // 2
    picks = [rm(a, b, c) for a in ends(nt) for b in ends(nh) for c in ends(nw)]                      # corners
    picks += [rm(mid(nt), 0, 0), rm(0, mid(nh), nw - 1), rm(nt - 1, nh - 1, mid(nw))]                 # edges
    picks += [rm(0, mid(nh), mid(nw)), rm(mid(nt), nh - 1, mid(nw)), rm(mid(nt), mid(nh), 0)]         # faces
    inner = [(a, b, c) for a in range(1, max(nt - 1, 1)) for b in range(1, max(nh - 1, 1)) for c in range(1, max(nw - 1, 1))]
    step = max(len(inner) // 4, 1)
    picks += [rm(*x) for x in inner[::step][:4]]                                                     # interior
    out = []
    for t in picks:
        if t not in out:
            out.append(t)
    return out
