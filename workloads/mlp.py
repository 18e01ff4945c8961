"""Synthetic dense-network workloads for mixed-mode Moonwalk.

Recipe (one generator, seeded, identical arrays go to the CPU oracle and to the GPU):

* layer i has W_i = U_i diag(s_i) V_i^T with U_i Haar-orthogonal (d_out x d_out), V_i a
  d_in x d_out matrix with Haar-distributed orthonormal columns, s_i ~ U[0.8, 1.2] i.i.d.;
  so every W_i has full row rank and the network is submersive (d_out <= d_in).
* b_i ~ N(0, 0.01^2); x, t ~ N(0, 1).
* draw order: per layer U, V, s, b (layers 1..L), then x, then t, all from one
  numpy PCG64 stream seeded with `seed`.
* everything is drawn in fp64 and then rounded to fp32; the fp32 values are what both
  sides consume (the oracle promotes the rounded values back to fp64).

The factors (U, s, V) are returned too: the tests use them for the closed form of the
right inverse.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np


def haar_orthonormal_columns(rng: np.random.Generator, n: int, k: int) -> np.ndarray:
    """n x k matrix (k <= n) with orthonormal columns, Haar-distributed.

    QR of a Gaussian matrix, with the column signs fixed so that diag(R) > 0 (without the
    sign fix the distribution is not Haar).
    """
    if k > n:
        raise ValueError("need k <= n")
    a = rng.standard_normal((n, k))
    q, r = np.linalg.qr(a)
    d = np.sign(np.diagonal(r))
    d[d == 0] = 1.0
    return q * d


@dataclass
class MLPWorkload:
    widths: List[int]                 # d_0 .. d_L
    batch: int
    alphas: List[float]               # per layer; 0 => ReLU
    W: List[np.ndarray]               # fp32, [d_out][d_in]
    b: List[np.ndarray]               # fp32, [d_out]
    x: np.ndarray                     # fp32, [B][d_0]
    t: np.ndarray                     # fp32, [B][d_L]
    reseed_interval: int = 0
    loss_scale: float = 1.0
    seed: int = 0
    name: str = ""
    factors: Optional[List[Dict[str, np.ndarray]]] = field(default=None, repr=False)

    @property
    def depth(self) -> int:
        return len(self.W)


def make_mlp(widths: Sequence[int], batch: int, alpha, seed: int = 0,
             reseed_interval: int = 0, loss_scale: float = 1.0, name: str = "",
             bias_std: float = 0.01, keep_factors: bool = False) -> MLPWorkload:
    widths = [int(w) for w in widths]
    depth = len(widths) - 1
    if depth < 1:
        raise ValueError("need at least one layer")
    alphas = [float(alpha)] * depth if np.isscalar(alpha) else [float(a) for a in alpha]
    if len(alphas) != depth:
        raise ValueError("one alpha per layer")
    rng = np.random.default_rng(seed)
    Ws, bs, factors = [], [], []
    for i in range(depth):
        d_in, d_out = widths[i], widths[i + 1]
        if d_out > d_in:
            raise ValueError(f"layer {i + 1}: d_out={d_out} > d_in={d_in} is not submersive")
        U = haar_orthonormal_columns(rng, d_out, d_out)
        V = haar_orthonormal_columns(rng, d_in, d_out)
        s = rng.uniform(0.8, 1.2, size=d_out)
        bias = bias_std * rng.standard_normal(d_out)
        W = (U * s) @ V.T
        Ws.append(np.ascontiguousarray(W, dtype=np.float32))
        bs.append(np.ascontiguousarray(bias, dtype=np.float32))
        if keep_factors:
            factors.append({"U": U, "s": s, "V": V})
    x = rng.standard_normal((batch, widths[0])).astype(np.float32)
    t = rng.standard_normal((batch, widths[-1])).astype(np.float32)
    return MLPWorkload(widths=widths, batch=int(batch), alphas=alphas, W=Ws, b=bs, x=x, t=t,
                       reseed_interval=int(reseed_interval), loss_scale=float(loss_scale),
                       seed=int(seed), name=name, factors=factors if keep_factors else None)


def make_mlp_on_device(widths: Sequence[int], batch: int, alpha, seed: int = 0, reseed_interval: int = 0,
                       loss_scale: float = 1.0, name: str = "", bias_std: float = 0.01, device="cuda:0"):
    """The same recipe drawn with torch on `device` (fp64 QR on the GPU, then rounded to fp32).

    For the large configurations, whose hundreds of 4096 x 4096 QR factorisations would take the
    host most of an hour. Same distribution, different random stream than make_mlp. W, b, x, t are
    torch tensors on the device; workload_to_host copies them for the CPU oracle, so that both sides
    consume the same fp32 values (the full-depth parity runs of the large configurations do that).
    """
    import torch
    widths = [int(w) for w in widths]
    depth = len(widths) - 1
    alphas = [float(alpha)] * depth if np.isscalar(alpha) else [float(a) for a in alpha]
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))

    def haar(n, k):
        a = torch.randn(n, k, dtype=torch.float64, device=device, generator=gen)
        q, r = torch.linalg.qr(a)
        d = torch.sign(torch.diagonal(r))
        d[d == 0] = 1.0
        return q * d

    Ws, bs = [], []
    for i in range(depth):
        d_in, d_out = widths[i], widths[i + 1]
        if d_out > d_in:
            raise ValueError(f"layer {i + 1}: d_out={d_out} > d_in={d_in} is not submersive")
        U = haar(d_out, d_out)
        V = haar(d_in, d_out)
        s = 0.8 + 0.4 * torch.rand(d_out, dtype=torch.float64, device=device, generator=gen)
        bias = bias_std * torch.randn(d_out, dtype=torch.float64, device=device, generator=gen)
        Ws.append(((U * s) @ V.T).to(torch.float32).contiguous())
        bs.append(bias.to(torch.float32).contiguous())
        del U, V
    x = torch.randn(batch, widths[0], dtype=torch.float64, device=device, generator=gen).to(torch.float32)
    t = torch.randn(batch, widths[-1], dtype=torch.float64, device=device, generator=gen).to(torch.float32)
    return MLPWorkload(widths=widths, batch=int(batch), alphas=alphas, W=Ws, b=bs, x=x, t=t,
                       reseed_interval=int(reseed_interval), loss_scale=float(loss_scale), seed=int(seed),
                       name=name, factors=None)


def workload_to_host(wl: MLPWorkload) -> MLPWorkload:
    """The same workload with every tensor as a numpy array on the host (for the CPU oracle): the values
    a device-drawn workload holds, bit for bit."""
    def host(a):
        return a if isinstance(a, np.ndarray) else a.detach().cpu().numpy()
    return MLPWorkload(widths=list(wl.widths), batch=wl.batch, alphas=list(wl.alphas), W=[host(w) for w in wl.W],
                       b=[host(b) for b in wl.b], x=host(wl.x), t=host(wl.t), reseed_interval=wl.reseed_interval,
                       loss_scale=wl.loss_scale, seed=wl.seed, name=wl.name, factors=None)


def _narrowing_widths() -> List[int]:
    # 32 layers from 4096 down to 512, every width a multiple of 64:
    # the width drops by 64 on every 4th layer and by 128 otherwise.
    w = [4096]
    for i in range(1, 33):
        w.append(w[-1] - (64 if i % 4 == 0 else 128))
    assert w[-1] == 512
    return w


CONFIGS = {
    "tiny":        dict(widths=[64] * 5,            batch=32,   alpha=0.1, reseed_interval=0, loss_scale=1.0),
    "deep_square": dict(widths=[1024] * 65,         batch=256,  alpha=0.1, reseed_interval=4, loss_scale=1.0),
    "narrowing":   dict(widths=_narrowing_widths(), batch=512,  alpha=0.1, reseed_interval=4, loss_scale=1.0),
    "relu_frag":   dict(widths=[2048] * 49,         batch=512,  alpha=0.0, reseed_interval=0, loss_scale=1.0),
    "very_deep":   dict(widths=[4096] * 257,        batch=1024, alpha=0.1, reseed_interval=4, loss_scale=2.0 ** 64),
}


def config_widths(name: str, depth: Optional[int] = None) -> List[int]:
    w = list(CONFIGS[name]["widths"])
    if depth is not None:
        w = w[: depth + 1]
    return w


def make_config(name: str, depth: Optional[int] = None, seed: int = 0,
                keep_factors: bool = False, device=None) -> MLPWorkload:
    """Build one of the named configurations, optionally truncated to its first `depth` layers.
    With `device` the tensors are drawn with torch on that device (see make_mlp_on_device)."""
    c = CONFIGS[name]
    if device is not None:
        return make_mlp_on_device(config_widths(name, depth), c["batch"], c["alpha"], seed=seed,
                                  reseed_interval=c["reseed_interval"], loss_scale=c["loss_scale"],
                                  name=name if depth is None else f"{name}[L={depth}]", device=device)
    return make_mlp(config_widths(name, depth), c["batch"], c["alpha"], seed=seed,
                    reseed_interval=c["reseed_interval"], loss_scale=c["loss_scale"],
                    name=name if depth is None else f"{name}[L={depth}]",
                    keep_factors=keep_factors)


def _sum_din_dout(widths: Sequence[int]) -> int:
    return int(sum(int(a) * int(b) for a, b in zip(widths[:-1], widths[1:])))


def moonwalk_flops(widths: Sequence[int], batch: int) -> int:
    """Algorithmic flops of one Moonwalk gradient step: five B x d_in x d_out GEMMs per layer."""
    return 10 * int(batch) * _sum_din_dout(widths)


def backprop_flops(widths: Sequence[int], batch: int) -> int:
    """Algorithmic flops of one backprop gradient step: three GEMMs per layer."""
    return 6 * int(batch) * _sum_din_dout(widths)
