"""Synthetic 1-D convolutional networks for Moonwalk with fragmental checkpointing (seeded; arrays only,
no arithmetic of the method).

Recipe, following the paper's 1-D experiment in shape (kernel size 3, stride 1, padding 1, a constant
number of channels, leaky ReLU, the length kept by every layer):

* kernel w_i [k][C][C]: taps u >= 1 ~ N(0, gain^2 / (k C)); tap 0 lower-triangular over channels,
  w[0, c, c'] = 0 for c < c', strictly lower part ~ N(0, gain^2 / (k C)), diagonal `diag` (1 as the paper
  assumes, or drawn from U[diag]) (the two assumptions of the fragmental update);
* bias ~ N(0, 0.01^2); input x ~ N(0, 1) [S][N][C]; target t ~ N(0, 1) of the same shape;
* draw order: per layer w, diagonal (if drawn), bias; then x; then t; one numpy PCG64 stream; fp64 rounded to fp32.

`gain` scales how fast the block recurrence of the reconstruction amplifies rounding errors: inside a block
each rebuilt position feeds the next, so the error grows like rho^(block - k + 1) with rho the spectral
radius of the recurrence; gain 0.5 keeps rho near 1 (measured in tests/test_frag_oracle_pins.py).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import numpy as np


@dataclass
class FragWorkload:
    batch: int
    length: int
    channels: int
    k: int
    block: int
    alphas: List[float]
    w: List[np.ndarray]       # fp32 [k][C][C]
    b: List[np.ndarray]       # fp32 [C]
    x: np.ndarray             # fp32 [S][N][C]
    t: np.ndarray             # fp32 [S][N][C]
    seed: int = 0
    name: str = ""

    @property
    def depth(self) -> int:
        return len(self.w)


def make_fragnet(batch: int, length: int, channels, depth: int, k: int = 3, block: int = 4, alpha: float = 0.3,
                 gain: float = 0.5, diag=1.0, seed: int = 0, name: str = "") -> FragWorkload:
    """`channels`: one count for the whole chain (the paper's setting), or depth + 1 counts, the input's
    first, none larger than the one before; `channels` of the result is then the input's."""
    if k % 2 != 1 or length % block or block < k - 1:
        raise ValueError("odd kernel size, and a whole number of blocks of at least k - 1 positions")
    rng = np.random.default_rng(seed)
    cs = [int(channels)] * (depth + 1) if np.isscalar(channels) else [int(c) for c in channels]
    if len(cs) != depth + 1 or any(b > a for a, b in zip(cs, cs[1:])):
        raise ValueError("need depth + 1 channel counts, none larger than the one before")
    ws, bs = [], []
    for i in range(depth):
        Ci, Co = cs[i], cs[i + 1]
        w = gain * rng.standard_normal((k, Ci, Co)) / np.sqrt(k * Ci)
        tap = np.tril(w[0])
        if np.isscalar(diag):
            d = np.full(Co, float(diag))
        else:
            d = rng.uniform(diag[0], diag[1], size=Co)
        tap[np.arange(Co), np.arange(Co)] = d
        w[0] = tap
        bias = 0.01 * rng.standard_normal(Co)
        ws.append(np.ascontiguousarray(w, dtype=np.float32))
        bs.append(np.ascontiguousarray(bias, dtype=np.float32))
    x = rng.standard_normal((batch, length, cs[0])).astype(np.float32)
    t = rng.standard_normal((batch, length, cs[-1])).astype(np.float32)
    return FragWorkload(batch=int(batch), length=int(length), channels=cs[0], k=k, block=int(block), alphas=[float(alpha)] * depth,
                        w=ws, b=bs, x=x, t=t, seed=int(seed), name=name)


def frag_moonwalk_flops(wl: FragWorkload) -> int:
    """Algorithmic flops of one step. Per layer, with P = 2 S N (k C) C one product with the patch matrix:
    forward, recomputed forward, input cotangent, weight gradient (4 P), and the block reconstruction:
    k products of 2 S N C C over the (block - k + 1) / block rebuilt positions."""
    total = 0
    for _ in range(wl.depth):
        rows = wl.batch * wl.length
        P = 2 * rows * wl.k * wl.channels * wl.channels
        total += 4 * P + wl.k * 2 * rows * wl.channels * wl.channels * (wl.block - wl.k + 1) // wl.block
    return total


def frag_backprop_flops(wl: FragWorkload, h0: bool = True) -> int:
    total = 0
    for i in range(wl.depth):
        rows = wl.batch * wl.length
        P = 2 * rows * wl.k * wl.channels * wl.channels
        total += 2 * P + (P if (i > 0 or h0) else 0)
    return total


# conv1d is the paper's fragmental-checkpointing experiment in shape: 2048 positions x 256 channels, k = 3,
# stride 1, padding 1, leaky ReLU, batch 128; the depth and block size are the experiment's knobs.
FRAG_CONFIGS = {
    "conv1d_small": dict(batch=4, length=256, channels=32, depth=3, block=4, alpha=0.3),
    "conv1d":       dict(batch=128, length=2048, channels=256, depth=10, block=4, alpha=0.3),
}
