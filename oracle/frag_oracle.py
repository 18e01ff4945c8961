"""fp64 CPU oracle for Moonwalk with fragmental gradient checkpointing on 1-D convolutional layers.

TEST INFRASTRUCTURE ONLY (see moonwalk_oracle.py): plain numpy, shares no code with the HIP path,
imported only by the tests, the smoke check and the benchmark's CPU-baseline leg.

Layout: activations are [S][N][C] (samples, positions, channels last), kernels are [k][C_in][C_out];
stride 1, padding p with 2 p = k - 1, so the length N is kept (the setting of the section on
fragmental gradient checkpointing: k = 3, p = 1). A layer is

    z[s, i', c'] = sum_{u, c} w[u, c, c'] * x[s, i' + u - p, c] + bias[c']      (zero outside 0 <= . < N)
    x' = leaky_relu(z)

and the loss is J = 0.5 ||x_L - t||^2 / S as for the dense networks. Such a layer is not submersive
(no stride to spare), so its output cotangent cannot be recovered from its input cotangent alone.

What follows which passage of the paper:

* `conv1d`, `conv1d_input_grad`, `conv1d_weight_grad`   the convolution, its vjp (the reverse-pass
        equation of the appendix on fragmental gradient checkpointing) and its parameter vjp, written
        out as their definitions.
* `fragments_of`        what Phase II keeps of a layer's output cotangent: the first k - 1 positions of
        every block of `block` positions (section on fragmental gradient checkpointing).
* `frag_vijp`           the recursive elimination of that section and its appendix: inside a block,
        position t >= k - 1 follows from the input cotangent at t - p and the k - 1 positions before
        t, by forward substitution over channels with the tap u = 0 (lower-triangular over channels,
        non-zero diagonal); blocks are independent of each other.
* `frag_moonwalk`       Phases I-III (Overview section, Algorithm 1) with such layers: Phase I keeps the
        signs, Phase II the input cotangent and the fragments, Phase III rebuilds each layer's output
        cotangent from the two and emits the gradients.
* `conv1d_backprop`     ordinary reverse mode: the plain definition of the result.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np

F64 = np.float64


def _as64(a) -> np.ndarray:
    return np.asarray(a, dtype=F64)


def conv1d(x, w) -> np.ndarray:
    """z[s,i',c'] = sum_{u,c} w[u,c,c'] x[s, i'+u-p, c] with p = (k-1)/2 (zero outside the signal)."""
    x, w = _as64(x), _as64(w)
    S, N, C = x.shape
    k = w.shape[0]
    if k % 2 != 1:
        raise ValueError("the length-preserving convolution needs an odd kernel size")
    p = (k - 1) // 2
    xp = np.zeros((S, N + 2 * p, C))
    xp[:, p:p + N, :] = x
    z = np.zeros((S, N, w.shape[2]))
    for u in range(k):
        z += xp[:, u:u + N, :] @ w[u]
    return z


def conv1d_input_grad(ct, w) -> np.ndarray:
    """vjp w.r.t. the input: h[s,i,c] = sum_{u,c'} w[u,c,c'] ct[s, i+p-u, c'] (zero outside the signal)."""
    ct, w = _as64(ct), _as64(w)
    S, N, Co = ct.shape
    k = w.shape[0]
    p = (k - 1) // 2
    cp = np.zeros((S, N + 2 * p, Co))
    cp[:, p:p + N, :] = ct
    h = np.zeros((S, N, w.shape[1]))
    for u in range(k):
        # position i + p - u of ct sits at index i + 2p - u of the padded array
        h += cp[:, 2 * p - u:2 * p - u + N, :] @ w[u].T
    return h


def conv1d_weight_grad(x, ct, k: int) -> np.ndarray:
    """vjp w.r.t. the kernel: dw[u,c,c'] = sum_{s,i'} x[s, i'+u-p, c] ct[s,i',c']."""
    x, ct = _as64(x), _as64(ct)
    S, N, C = x.shape
    p = (k - 1) // 2
    xp = np.zeros((S, N + 2 * p, C))
    xp[:, p:p + N, :] = x
    dw = np.zeros((k, C, ct.shape[2]))
    for u in range(k):
        dw[u] = np.einsum("snc,snd->cd", xp[:, u:u + N, :], ct)
    return dw


def is_fragmental(w, tol: float = 0.0) -> bool:
    """The assumption of the fragmental update: the tap u = 0 (the one that reaches the newest output
    position) is lower-triangular over channels, w[0, c, c'] = 0 for c < c', with non-zero diagonal;
    C_out <= C_in so that the first C_out input channels carry one equation per unknown."""
    w = _as64(w)
    _, Ci, Co = w.shape
    if Co > Ci:
        return False
    T = w[0, :Co, :Co]
    return bool(np.all(np.abs(np.triu(T, 1)) <= tol) and np.all(np.diag(T) != 0))


def fragments_of(ct, k: int, block: int) -> np.ndarray:
    """[S][N / block][k - 1][C]: the first k - 1 positions of every block."""
    ct = _as64(ct)
    S, N, C = ct.shape
    if N % block or block < k - 1:
        raise ValueError("the signal must be a whole number of blocks of at least k - 1 positions")
    return ct.reshape(S, N // block, block, C)[:, :, :k - 1, :].copy()


def frag_vijp(h, frags, w, block: int) -> np.ndarray:
    """Output cotangent of the convolution from its input cotangent h [S][N][C_in] and the stored
    fragments [S][N / block][k - 1][C_out]. The equation of h[t - p, c] for c < C_out reads

        h[t - p, c] = sum_{c' <= c} w[0, c, c'] ct[t, c'] + sum_{u >= 1} sum_{c'} w[u, c, c'] ct[t - u, c']

    so ct[t, :] follows from positions t - 1 .. t - k + 1 by forward substitution over the channels.
    Positions before the start of the signal do not occur: t >= k - 1 inside every block."""
    h, frags, w = _as64(h), _as64(frags), _as64(w)
    S, N, _ = h.shape
    k, _, Co = w.shape
    p = (k - 1) // 2
    M = N // block
    T = w[0, :Co, :Co]
    ct = np.zeros((S, M, block, Co))
    ct[:, :, :k - 1, :] = frags
    hb = h[:, :, :Co].reshape(S, M, block, Co)
    for j in range(k - 1, block):          # sequential inside a block, all blocks and samples at once
        rhs = hb[:, :, j - p, :].copy()      # j >= k - 1 = 2 p, so the position is inside the block
        for u in range(1, k):
            rhs -= ct[:, :, j - u, :] @ w[u, :Co, :].T
        # T ct = rhs, one channel after the other
        out = np.zeros_like(rhs)
        for c in range(Co):
            out[..., c] = (rhs[..., c] - out[..., :c] @ T[c, :c]) / T[c, c]
        ct[:, :, j, :] = out
    return ct.reshape(S, N, Co)


def sign_mask(z):
    return _as64(z) > 0


def loss_and_cotangent(xL, t, loss_scale: float = 1.0):
    r = _as64(xL) - _as64(t)
    S = r.shape[0]
    return 0.5 * float(np.sum(r * r)) / S, loss_scale * r / S


def conv1d_forward(ws, bs, alphas, x0, forced_masks=None):
    x = _as64(x0)
    xs, zs, masks = [x], [], []
    for i, (w, b, a) in enumerate(zip(ws, bs, alphas)):
        z = conv1d(x, w) + _as64(b)
        m = sign_mask(z) if forced_masks is None else np.asarray(forced_masks[i], dtype=bool)
        x = np.where(m, z, a * z)
        zs.append(z)
        masks.append(m)
        xs.append(x)
    return xs, zs, masks


def conv1d_backprop(ws, bs, alphas, x0, t, forced_masks=None) -> Dict[str, object]:
    """Reverse mode with every activation stored."""
    xs, zs, masks = conv1d_forward(ws, bs, alphas, x0, forced_masks)
    loss, h = loss_and_cotangent(xs[-1], t)
    L = len(ws)
    dW, db, cts = [None] * L, [None] * L, [None] * L
    for i in range(L - 1, -1, -1):
        ct_z = h * np.where(masks[i], 1.0, alphas[i])
        k = np.shape(ws[i])[0]
        dW[i] = conv1d_weight_grad(xs[i], ct_z, k)
        db[i] = ct_z.sum(axis=(0, 1))
        cts[i] = ct_z
        h = conv1d_input_grad(ct_z, ws[i])
    return {"dW": dW, "db": db, "loss": loss, "masks": masks, "h0": h, "ct_z": cts, "xs": xs}


def frag_moonwalk(ws, bs, alphas, x0, t, block: int, forced_masks=None, loss_scale: float = 1.0,
                  dtype=F64) -> Dict[str, object]:
    """Mixed-mode Moonwalk with fragmental checkpointing: Phase I keeps the signs only; Phase II runs
    the reverse pass for the input cotangent h_0 and keeps, per layer, the first k - 1 positions of
    every block of the convolution's output cotangent; Phase III goes forward again, rebuilds each
    layer's output cotangent from the incoming cotangent and the fragments, and emits the gradients.
    `dtype` sets the precision of the stored and propagated values (fp64: the reference itself)."""
    L = len(ws)
    wd = [np.asarray(_as64(w), dtype=dtype) for w in ws]
    bd = [np.asarray(_as64(b), dtype=dtype) for b in bs]
    x = np.asarray(_as64(x0), dtype=dtype)
    # Phase I
    masks = []
    for i in range(L):
        z = (conv1d(x, wd[i]) + bd[i]).astype(dtype)
        m = sign_mask(z) if forced_masks is None else np.asarray(forced_masks[i], dtype=bool)
        masks.append(m)
        x = np.where(m, z, alphas[i] * z).astype(dtype)
    loss, h = loss_and_cotangent(x, t, loss_scale)
    h = h.astype(dtype)
    # Phase II
    frags = [None] * L
    for i in range(L - 1, -1, -1):
        ct_z = (h * np.where(masks[i], 1.0, alphas[i])).astype(dtype)
        frags[i] = fragments_of(ct_z, wd[i].shape[0], block).astype(dtype)
        h = conv1d_input_grad(ct_z, wd[i]).astype(dtype)
    h0 = h
    # Phase III
    x = np.asarray(_as64(x0), dtype=dtype)
    dW, db = [None] * L, [None] * L
    mismatches = 0
    for i in range(L):
        z = (conv1d(x, wd[i]) + bd[i]).astype(dtype)
        mismatches += int(np.count_nonzero(sign_mask(z) != masks[i]))
        ct_z = frag_vijp(h, frags[i], wd[i], block).astype(dtype)
        dW[i] = conv1d_weight_grad(x, ct_z, wd[i].shape[0]) / loss_scale
        db[i] = ct_z.sum(axis=(0, 1)) / loss_scale
        h = (ct_z / np.where(masks[i], 1.0, alphas[i])).astype(dtype)   # vijp of the activation
        x = np.where(masks[i], z, alphas[i] * z).astype(dtype)
    return {"dW": dW, "db": db, "loss": loss, "masks": masks, "h0": h0, "frags": frags,
            "sign_mismatches": mismatches}


def project_constrained(w):
    """The fragmental update constrains the tap u = 0: w[0, c, c'] = 0 for c < c' (within the first C_out
    rows). A training step must leave those entries at zero; this puts them back."""
    w = np.array(_as64(w))
    Co = w.shape[2]
    w[0, :Co, :] = np.tril(w[0, :Co, :])
    return w


def frag_sgd_step(ws, bs, alphas, x0, t, lr: float, block: int, forced_masks=None) -> Dict[str, object]:
    """One training step (Algorithm 1 with "Apply g_i"): theta_i <- theta_i - lr g_i with the gradients of
    frag_moonwalk, the constrained entries of the taps u = 0 kept at zero (a projected step)."""
    g = frag_moonwalk(ws, bs, alphas, x0, t, block, forced_masks=forced_masks)
    new_w = [project_constrained(_as64(w) - lr * dw) for w, dw in zip(ws, g["dW"])]
    new_b = [_as64(b) - lr * db for b, db in zip(bs, g["db"])]
    return {"w": new_w, "b": new_b, "loss": g["loss"], "masks": g["masks"]}

