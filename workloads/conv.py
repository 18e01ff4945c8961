"""Synthetic submersive 2-D convolutional networks for Moonwalk (seeded; arrays only, no arithmetic of the method).

Recipe, following the paper's fully parallel 2-D experiment in shape (3x3 kernels, stride 2, padding 1,
a constant number of channels, leaky ReLU, each layer halving the resolution):

* kernel w_i [k][k][C][C] ~ N(0, 1/(k k C)); the tap at (p, p) is made channel-triangular,
  w[p, p, c, c'] = 0 for c < c', with diagonal w[p, p, c, c] ~ U[0.8, 1.2] (conditions (ii), (iii) of the
  lemma on submersive convolutional layers);
* bias ~ N(0, 0.01^2); input x ~ N(0, 1) [B][H][H][C]; target t ~ N(0, 1) of the output shape;
* draw order: per layer w, diagonal, bias; then x; then t; one numpy PCG64 stream; drawn in fp64, rounded to fp32.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np


@dataclass
class ConvWorkload:
    batch: int
    side: int                 # input height = width
    channels: int
    k: int
    s: int
    p: int
    alphas: List[float]
    w: List[np.ndarray]       # fp32 [k][k][C][C]
    b: List[np.ndarray]       # fp32 [C]
    x: np.ndarray             # fp32 [B][H][H][C]
    t: np.ndarray             # fp32 [B][H_L][H_L][C]
    sides: List[int]          # spatial side after each layer, sides[0] = input
    seed: int = 0
    name: str = ""

    @property
    def depth(self) -> int:
        return len(self.w)


def conv_out_side(n: int, k: int, s: int, p: int) -> int:
    return (n + 2 * p - k) // s + 1


def make_convnet(batch: int, side: int, channels, depth: int, k: int = 3, s: int = 2, p: int = 1,
                 alpha: float = 0.1, seed: int = 0, name: str = "") -> ConvWorkload:
    """`channels`: one count for the whole chain (the paper's setting), or depth + 1 counts, the input's
    first, none larger than the one before (C_out <= C_in); `channels` of the result is then the input's."""
    rng = np.random.default_rng(seed)
    cs = [int(channels)] * (depth + 1) if np.isscalar(channels) else [int(c) for c in channels]
    if len(cs) != depth + 1 or any(b > a for a, b in zip(cs, cs[1:])):
        raise ValueError("need depth + 1 channel counts, none larger than the one before")
    sides = [int(side)]
    ws, bs = [], []
    for i in range(depth):
        n = sides[-1]
        no = conv_out_side(n, k, s, p)
        if no < 1 or not (k > p and s > p and n > s * (no - 1)):
            raise ValueError(f"layer with input side {n} violates the spatial bounds of the lemma")
        Ci, Co = cs[i], cs[i + 1]
        w = rng.standard_normal((k, k, Ci, Co)) / np.sqrt(k * k * Ci)
        tap = np.tril(w[p, p])              # rows c, columns c': keep c >= c', zero for c < c'
        d = rng.uniform(0.8, 1.2, size=Co)
        tap[np.arange(Co), np.arange(Co)] = d
        w[p, p] = tap
        bias = 0.01 * rng.standard_normal(Co)
        ws.append(np.ascontiguousarray(w, dtype=np.float32))
        bs.append(np.ascontiguousarray(bias, dtype=np.float32))
        sides.append(no)
    x = rng.standard_normal((batch, side, side, cs[0])).astype(np.float32)
    t = rng.standard_normal((batch, sides[-1], sides[-1], cs[-1])).astype(np.float32)
    return ConvWorkload(batch=int(batch), side=int(side), channels=cs[0], k=k, s=s, p=p, alphas=[float(alpha)] * depth,
                        w=ws, b=bs, x=x, t=t, sides=sides, seed=int(seed), name=name)


def conv_moonwalk_flops(wl: ConvWorkload, h0_full: bool = True) -> int:
    """Algorithmic flops of one Moonwalk step. Per layer, with P = 2 rows' (k k C) C the flops of one
    product with the patch matrix: forward, recomputed forward and weight gradient (3 P), the input
    cotangent (P; not for the first layer unless h_0 is wanted for every input element), and the
    channel solve of the vijp (2 rows' C C), times the (reach + 1)^2 positions that enter an equation when
    the kernel is wider than padding + stride (reach = (k - 1 - p) / s earlier positions per dimension)."""
    total = 0
    reach = (wl.k - 1 - wl.p) // wl.s
    for i in range(wl.depth):
        rows = wl.batch * wl.sides[i + 1] ** 2
        Ci, Co = wl.w[i].shape[2], wl.w[i].shape[3]
        P = 2 * rows * wl.k * wl.k * Ci * Co
        total += 3 * P + (P if (i > 0 or h0_full) else 0) + 2 * rows * Co * Co * (reach + 1) ** 2
    return total


def conv_backprop_flops(wl: ConvWorkload, h0_full: bool = True) -> int:
    """Forward and weight gradient per layer (2 P), the input cotangent (P) for every layer but the first,
    and for the first as well when h_0 is wanted."""
    total = 0
    for i in range(wl.depth):
        rows = wl.batch * wl.sides[i + 1] ** 2
        P = 2 * rows * wl.k * wl.k * wl.w[i].shape[2] * wl.w[i].shape[3]
        total += 2 * P + (P if (i > 0 or h0_full) else 0)
    return total


def make_convnet_on_device(batch: int, side: int, channels: int, depth: int, k: int = 3, s: int = 2, p: int = 1,
                           alpha: float = 0.1, seed: int = 0, name: str = "", device="cuda:0") -> ConvWorkload:
    """The same recipe drawn with torch on `device` (different random stream than make_convnet): for the
    paper-sized configuration, whose input alone is 4 GiB. w, b, x, t are torch tensors on the device."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    C = int(channels)
    sides = [int(side)]
    ws, bs = [], []
    for _ in range(depth):
        n = sides[-1]
        no = conv_out_side(n, k, s, p)
        if no < 1 or not (k > p and s > p and n > s * (no - 1)):
            raise ValueError(f"layer with input side {n} violates the spatial bounds of the lemma")
        w = torch.randn(k, k, C, C, device=device, generator=gen) / float(np.sqrt(k * k * C))
        tap = torch.tril(w[p, p])
        d = 0.8 + 0.4 * torch.rand(C, device=device, generator=gen)
        idx = torch.arange(C, device=device)
        tap[idx, idx] = d
        w[p, p] = tap
        ws.append(w.contiguous())
        bs.append(0.01 * torch.randn(C, device=device, generator=gen))
        sides.append(no)
    x = torch.randn(batch, side, side, C, device=device, generator=gen)
    t = torch.randn(batch, sides[-1], sides[-1], C, device=device, generator=gen)
    return ConvWorkload(batch=int(batch), side=int(side), channels=C, k=k, s=s, p=p, alphas=[float(alpha)] * depth,
                        w=ws, b=bs, x=x, t=t, sides=sides, seed=int(seed), name=name)


# Named configurations. conv2d is the fully parallel 2-D experiment of the paper in shape: 256 x 256 x 128
# input, 3x3x128x128 kernels, stride 2, padding 1, leaky ReLU, batch 128, eight layers (side 256 -> 1).
CONV_CONFIGS = {
    "conv2d_small": dict(batch=8, side=64, channels=32, depth=4, alpha=0.3),
    "conv2d":       dict(batch=128, side=256, channels=128, depth=8, alpha=0.3),
    # a kernel wider than padding + stride: three earlier output positions enter every equation of the vijp
    "conv2d_k5":    dict(batch=32, side=128, channels=128, depth=6, alpha=0.3, k=5, s=2, p=1),
}
