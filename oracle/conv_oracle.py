"""fp64 CPU oracle for Moonwalk on submersive 2-D convolutional layers.

TEST INFRASTRUCTURE ONLY (see moonwalk_oracle.py): plain numpy, shares no code with the HIP path,
imported only by the tests, the smoke check and the benchmark's CPU-baseline leg.

Layout: activations are [B][H][W][C] (channels last), kernels are [k][k][C_in][C_out]; one stride s
and one padding p for both spatial dimensions. A layer is

    z[b, i', j', c'] = sum_{u, v, c} w[u, v, c, c'] * x[b, s i' + u - p, s j' + v - p, c] + bias[c']
    x' = leaky_relu(z)

(the channel-wise convolution of the lemma on submersive convolutional layers), the loss is
J = 0.5 ||x_L - t||^2 / B as for the dense networks.

What follows which passage of the paper:

* `conv2d`, `conv2d_input_grad`, `conv2d_weight_grad`   the convolution of the lemma, its vjp
        (TransposeConv, Eq. conv-vjp) and its parameter vjp, written out as their definitions.
* `is_submersive`       the three sufficient conditions of the lemma: spatial bounds k > p, s > p,
        n > s (n' - 1); channel-wise triangularity of the tap at (p, p); non-zero diagonal there.
* `conv_vijp`           the constructive proof of the lemma: Gaussian elimination in lexicographic order
        of (i', j', c'), each h'[i', j', c'] recovered from the equation of h[s i', s j', c'].
        For k <= p + s no earlier position enters an equation and the elimination is the paper's
        "fully parallel" algorithm: a triangular solve over channels at every position on its own.
* `conv_moonwalk`       Phases I-III (Overview section, Algorithm 1) with convolutional layers.
* `conv_backprop`       ordinary reverse mode: the plain definition of the result.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F64 = np.float64


def _as64(a) -> np.ndarray:
    return np.asarray(a, dtype=F64)


def out_size(n: int, k: int, s: int, p: int) -> int:
    return (n + 2 * p - k) // s + 1


def conv2d(x, w, s: int, p: int) -> np.ndarray:
    """z[b,i',j',c'] = sum_{u,v,c} w[u,v,c,c'] x[b, s i'+u-p, s j'+v-p, c]  (zero outside the image)."""
    x, w = _as64(x), _as64(w)
    B, H, W, C = x.shape
    k = w.shape[0]
    Ho, Wo = out_size(H, k, s, p), out_size(W, k, s, p)
    xp = np.zeros((B, H + 2 * p + s, W + 2 * p + s, C))
    xp[:, p:p + H, p:p + W, :] = x
    z = np.zeros((B, Ho, Wo, w.shape[3]))
    for u in range(k):
        for v in range(k):
            z += xp[:, u:u + s * Ho:s, v:v + s * Wo:s, :] @ w[u, v]
    return z


def conv2d_input_grad(hp, w, s: int, p: int, in_hw: Tuple[int, int]) -> np.ndarray:
    """h[b,i,j,c] = sum_{u,v,c'} w[u,v,c,c'] h'[b,i',j',c'] over the (i',j') with s i'+u-p = i, s j'+v-p = j
    (TransposeConv of Eq. conv-vjp: the vjp of conv2d with respect to its input)."""
    hp, w = _as64(hp), _as64(w)
    B, Ho, Wo, _ = hp.shape
    H, W = in_hw
    k = w.shape[0]
    acc = np.zeros((B, H + 2 * p + s, W + 2 * p + s, w.shape[2]))
    for u in range(k):
        for v in range(k):
            acc[:, u:u + s * Ho:s, v:v + s * Wo:s, :] += hp @ w[u, v].T
    return acc[:, p:p + H, p:p + W, :].copy()


def conv2d_weight_grad(x, hp, k: int, s: int, p: int) -> np.ndarray:
    """dw[u,v,c,c'] = sum_{b,i',j'} x[b, s i'+u-p, s j'+v-p, c] h'[b,i',j',c']."""
    x, hp = _as64(x), _as64(hp)
    B, H, W, C = x.shape
    _, Ho, Wo, Co = hp.shape
    xp = np.zeros((B, H + 2 * p + s, W + 2 * p + s, C))
    xp[:, p:p + H, p:p + W, :] = x
    dw = np.zeros((k, k, C, Co))
    for u in range(k):
        for v in range(k):
            dw[u, v] = np.einsum("bijc,bijd->cd", xp[:, u:u + s * Ho:s, v:v + s * Wo:s, :], hp)
    return dw


def is_submersive(w, s: int, p: int, n: int) -> bool:
    """The sufficient conditions of the lemma for a square image of side n."""
    w = _as64(w)
    k, _, m, mo = w.shape
    no = out_size(n, k, s, p)
    if not (k > p and s > p and n > s * (no - 1)):
        return False
    if mo > m:
        return False
    tap = w[p, p]                      # [c][c']
    for c in range(m):
        for co in range(mo):
            if c < co and tap[c, co] != 0.0:
                return False
    return all(tap[c, c] != 0.0 for c in range(mo))


def conv_vijp(h, w, s: int, p: int, out_hw: Tuple[int, int]) -> np.ndarray:
    """h' with TransposeConv(h') = h, by elimination in lexicographic order of (i', j', c').

    The equation of h[b, s i', s j', c'] reads (Eq. conv-vjp with i = s i', c = c')
        h[s i', s j', c'] = sum_{u,v,c''} w[u,v,c',c''] hbar'[s i' + p - u, s j' + p - v, c'']
    where hbar' is h' dilated by s. Its terms are h'[i' - a, j' - b, c''] for the taps u = p + a s,
    v = p + b s inside the kernel (a, b >= 0 because s > p), and for a = b = 0 only c'' <= c' by the
    triangularity: everything except h'[i', j', c'] itself comes earlier in the order.
    """
    h, w = _as64(h), _as64(w)
    B = h.shape[0]
    Ho, Wo = out_hw
    k, mo = w.shape[0], w.shape[3]
    reach = (k - 1 - p) // s             # how many earlier positions per dimension an equation touches
    hp = np.zeros((B, Ho, Wo, mo))
    for i in range(Ho):
        for j in range(Wo):
            for c in range(mo):
                v = h[:, s * i, s * j, c].copy()
                for a in range(reach + 1):
                    for b in range(reach + 1):
                        if i - a < 0 or j - b < 0:
                            continue
                        coef = w[p + a * s, p + b * s, c, :]            # over c''
                        if a == 0 and b == 0:
                            v -= hp[:, i, j, :c] @ coef[:c]              # c'' < c'; c'' > c' has coefficient 0
                        else:
                            v -= hp[:, i - a, j - b, :] @ coef
                hp[:, i, j, c] = v / w[p, p, c, c]
    return hp


def conv_vijp_parallel(h, w, s: int, p: int, out_hw: Tuple[int, int]) -> np.ndarray:
    """The "fully parallel" form for k <= p + s: at every output position on its own, a triangular
    solve over channels of  T h'[i', j', :] = h[s i', s j', :m']  with T[c'][c''] = w[p, p, c', c'']."""
    h, w = _as64(h), _as64(w)
    k, mo = w.shape[0], w.shape[3]
    if k > p + s:
        raise ValueError("positions are coupled when k > p + s")
    Ho, Wo = out_hw
    T = w[p, p, :mo, :mo]
    sub = h[:, 0:s * Ho:s, 0:s * Wo:s, :mo]
    hp = np.zeros_like(sub)
    for c in range(mo):                                  # forward substitution over channels
        hp[..., c] = (sub[..., c] - hp[..., :c] @ T[c, :c]) / T[c, c]
    return hp


def sign_mask(z):
    return _as64(z) > 0


def loss_and_cotangent(xL, t, loss_scale: float = 1.0):
    r = _as64(xL) - _as64(t)
    B = r.shape[0]
    return 0.5 * float(np.sum(r * r)) / B, loss_scale * r / B


def conv_forward(ws, bs, alphas, s: int, p: int, x0, forced_masks=None):
    x = _as64(x0)
    xs, zs, masks = [x], [], []
    for i, (w, b, a) in enumerate(zip(ws, bs, alphas)):
        z = conv2d(x, w, s, p) + _as64(b)
        m = sign_mask(z) if forced_masks is None else np.asarray(forced_masks[i], dtype=bool)
        x = np.where(m, z, a * z)
        zs.append(z)
        masks.append(m)
        xs.append(x)
    return xs, zs, masks


def conv_backprop(ws, bs, alphas, s: int, p: int, x0, t, forced_masks=None) -> Dict[str, object]:
    """Reverse mode with every activation stored."""
    xs, zs, masks = conv_forward(ws, bs, alphas, s, p, x0, forced_masks)
    loss, h = loss_and_cotangent(xs[-1], t)
    L = len(ws)
    dW, db, hs = [None] * L, [None] * L, [None] * L
    for i in range(L - 1, -1, -1):
        ct_z = h * np.where(masks[i], 1.0, alphas[i])
        k = np.shape(ws[i])[0]
        dW[i] = conv2d_weight_grad(xs[i], ct_z, k, s, p)
        db[i] = ct_z.sum(axis=(0, 1, 2))
        h = conv2d_input_grad(ct_z, ws[i], s, p, xs[i].shape[1:3])
        hs[i] = h  # the cotangent at the input of layer i (hs[0] is h_0)
    return {"dW": dW, "db": db, "loss": loss, "masks": masks, "h0": h, "hs": hs, "xs": xs}


def conv_moonwalk(ws, bs, alphas, s: int, p: int, x0, t, forced_masks=None, loss_scale: float = 1.0,
                  dtype=F64) -> Dict[str, object]:
    """Mixed-mode Moonwalk with convolutional layers (Overview section, Algorithm 1): Phase I keeps the
    signs only, Phase II gives the input cotangent h_0, Phase III recomputes each layer, maps the
    cotangent forward with the vijp of the convolution and of the activation, and emits the gradients."""
    L = len(ws)
    wd = [np.asarray(_as64(w), dtype=dtype) for w in ws]
    bd = [np.asarray(_as64(b), dtype=dtype) for b in bs]
    x = np.asarray(_as64(x0), dtype=dtype)
    # Phase I
    masks, shapes = [], [x.shape]
    for i in range(L):
        z = (conv2d(x, wd[i], s, p) + bd[i]).astype(dtype)
        m = sign_mask(z) if forced_masks is None else np.asarray(forced_masks[i], dtype=bool)
        masks.append(m)
        x = np.where(m, z, dtype(alphas[i]) * z).astype(dtype)
        shapes.append(x.shape)
    r = x - np.asarray(_as64(t), dtype=dtype)
    B = x.shape[0]
    loss = 0.5 * float(np.sum(_as64(r) ** 2)) / B
    h = (dtype(loss_scale) * r / dtype(B)).astype(dtype)
    # Phase II
    for i in range(L - 1, -1, -1):
        ct_z = (h * np.where(masks[i], dtype(1), dtype(alphas[i]))).astype(dtype)
        h = conv2d_input_grad(ct_z, wd[i], s, p, shapes[i][1:3]).astype(dtype)
    h0 = h
    # Phase III
    x = np.asarray(_as64(x0), dtype=dtype)
    dW, db = [None] * L, [None] * L
    for i in range(L):
        z = (conv2d(x, wd[i], s, p) + bd[i]).astype(dtype)
        ct_z = conv_vijp(h, wd[i], s, p, shapes[i + 1][1:3]).astype(dtype)
        k = wd[i].shape[0]
        dW[i] = conv2d_weight_grad(x, ct_z, k, s, p) / loss_scale
        db[i] = ct_z.sum(axis=(0, 1, 2)) / loss_scale
        slope = np.where(masks[i], dtype(1), dtype(alphas[i]))
        h = (ct_z / slope).astype(dtype)
        x = np.where(masks[i], z, dtype(alphas[i]) * z).astype(dtype)
    return {"dW": dW, "db": db, "loss": loss, "masks": masks, "h0": h0}


def project_constrained(w, p: int):
    """The lemma constrains the tap at (p, p): w[p, p, c, c'] = 0 for c < c' (within the first C_out rows).
    A training step must leave those entries at zero; this puts them back."""
    w = np.array(_as64(w))
    Co = w.shape[3]
    w[p, p, :Co, :] = np.tril(w[p, p, :Co, :])
    return w


def conv_sgd_step(ws, bs, alphas, s: int, p: int, x0, t, lr: float, forced_masks=None) -> Dict[str, object]:
    """One training step (Algorithm 1 with "Apply g_i"): theta_i <- theta_i - lr g_i with the gradients of
    conv_moonwalk, the constrained entries of the (p, p) taps kept at zero (a projected step, so that the
    layers stay submersive). Returns the new kernels and biases and the loss before the update."""
    g = conv_moonwalk(ws, bs, alphas, s, p, x0, t, forced_masks=forced_masks)
    new_w = [project_constrained(_as64(w) - lr * dw, p) for w, dw in zip(ws, g["dW"])]
    new_b = [_as64(b) - lr * db for b, db in zip(bs, g["db"])]
    return {"w": new_w, "b": new_b, "loss": g["loss"], "masks": g["masks"]}

