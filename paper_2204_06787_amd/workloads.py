"""Seeded synthetic inputs shaped like the paper's workloads.

This module is the one thing the HIP path and the CPU oracle share: it only draws random input
tensors.  It holds none of the method's arithmetic (no sign, merge, decode or compensation step)
and imports neither the HIP binding nor the oracle.

The tensors stand in for real training gradients (ImageNet / CIFAR-10 / IMDb runs in Section 5 of
the paper), which need datasets that are not available here.  Only the sizes (Table 2: ResNet-18
about 11 M parameters, ResNet-50 about 25 M) and plausible value distributions are borrowed.
"""

from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    M: int                 # simulated workers
    d: int                 # elements per gradient
    grid_x: int            # 0: ring; X: torus with X columns and M/X rows
    steps: int             # consecutive synchronisations with compensation carried over
    scale: float           # global step size eta_s
    dist: str              # "normal" | "layered" | "heavy_tail"
    std: float = 1.0

    @property
    def n_words(self) -> int:
        return (self.d + 63) // 64

    def algorithmic_bytes(self, with_bitmap: bool = True) -> int:
        """Bytes the fused pass has to move: read g and c, write c' (per worker), write the update
        once and, if asked for, the final packed bitmap."""
        b = 12 * self.M * self.d + 4 * self.d
        if with_bitmap:
            b += 8 * self.n_words
        return b


WORKLOADS = {
    # M=3 ring, d=65,536, N(0,1), c=0, one step: the oracle finishes in well under a second.
    "tiny_ring": Workload("tiny_ring", M=3, d=65_536, grid_x=0, steps=1, scale=1e-3,
                          dist="normal", std=1.0),
    # ResNet-18-sized, N(0, 0.01) (variance 0.01, std 0.1), 10 steps.
    "resnet18": Workload("resnet18", M=8, d=11_200_000, grid_x=0, steps=10, scale=1e-3,
                         dist="normal", std=0.1),
    # ResNet-50-sized, 160 contiguous equal layers, layer std = 10^U, U ~ Unif[-4, -1], 10 steps.
    "resnet50": Workload("resnet50", M=8, d=25_600_000, grid_x=0, steps=10, scale=1e-3,
                         dist="layered"),
    # 4 x 4 torus, N(0, 0.01), 5 steps.
    "torus4x4": Workload("torus4x4", M=16, d=25_600_000, grid_x=4, steps=5, scale=1e-3,
                         dist="normal", std=0.1),
    # 138 M elements, 99 % N(0, 0.01) + 1 % Student-t (nu = 2), 3 steps.
    "large": Workload("large", M=8, d=138_000_000, grid_x=0, steps=3, scale=1e-3,
                      dist="heavy_tail", std=0.1),
}

N_LAYERS = 160
TAIL_FRACTION = 0.01
TAIL_NU = 2.0


def step_seed(seed0: int, t: int) -> int:
    """Seed of the random merge masks of synchronisation ``t``."""
    return (int(seed0) + int(t)) & 0xFFFFFFFFFFFFFFFF


def _generator(seed: int, step: int, device) -> torch.Generator:
    gen = torch.Generator(device=device)
    gen.manual_seed((int(seed) * 1_000_003 + int(step) * 7919 + 12345) & 0x7FFFFFFFFFFFFFFF)
    return gen


def layer_stds(wl: Workload, seed: int) -> torch.Tensor:
    """Per-layer standard deviations of the "layered" distribution (same for all workers/steps)."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed((int(seed) * 2_654_435_761 + 99) & 0x7FFFFFFFFFFFFFFF)
    u = torch.rand(N_LAYERS, generator=gen, dtype=torch.float64) * 3.0 - 4.0
    return torch.pow(torch.tensor(10.0, dtype=torch.float64), u).to(torch.float32)


def make_gradients(wl: Workload, step: int, seed: int, device="cpu", d: int | None = None,
                   ld: int | None = None) -> torch.Tensor:
    """Gradients of all workers for one synchronisation: float32 ``[M, ld]`` (``ld >= d``).

    ``d`` overrides the workload's size (the tests use it for ragged shapes); columns ``>= d`` of a
    padded row are filled with a recognisable constant that no kernel may touch or depend on.
    """
    d = wl.d if d is None else int(d)
    ld = d if ld is None else int(ld)
    assert ld >= d
    dev = torch.device(device)
    gen = _generator(seed, step, dev)
    out = torch.empty((wl.M, ld), dtype=torch.float32, device=dev)
    if ld > d:
        out[:, d:] = 12345.0
    if d == 0:
        return out
    if wl.dist == "layered":
        stds = layer_stds(wl, seed).to(dev)
        layer = max(1, math.ceil(d / N_LAYERS))
        col_std = stds.repeat_interleave(layer)[:d]
    for m in range(wl.M):
        row = out[m, :d]
        row.normal_(mean=0.0, std=1.0, generator=gen)
        if wl.dist == "normal":
            row.mul_(wl.std)
        elif wl.dist == "layered":
            row.mul_(col_std)
        elif wl.dist == "heavy_tail":
            row.mul_(wl.std)
            # Student-t with nu = 2:  Z / sqrt(V / 2), V ~ chi^2(2) = -2 ln U
            pick = torch.rand(d, generator=gen, device=dev) < TAIL_FRACTION
            n_tail = int(pick.sum().item())
            z = torch.randn(n_tail, generator=gen, device=dev)
            u = torch.rand(n_tail, generator=gen, device=dev).clamp_(min=1e-12)
            row[pick] = (wl.std * z / torch.sqrt(-torch.log(u))).to(torch.float32)
        else:
            raise ValueError(f"unknown distribution {wl.dist!r}")
    return out


def zero_compensation(wl: Workload, device="cpu", d: int | None = None,
                      ld: int | None = None) -> torch.Tensor:
    """c_0 = 0 (the initialisation of Algorithm 2)."""
    d = wl.d if d is None else int(d)
    ld = d if ld is None else int(ld)
    return torch.zeros((wl.M, ld), dtype=torch.float32, device=torch.device(device))
