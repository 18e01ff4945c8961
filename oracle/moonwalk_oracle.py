"""fp64 CPU oracle for mixed-mode Moonwalk on dense (MLP) layers.

TEST INFRASTRUCTURE ONLY. This module is a plain, slow, obviously-correct numpy
implementation of what the GPU library computes. Only the test-suite, the smoke check and
the benchmark's CPU-baseline leg may import it; the product (the HIP library and its Python
binding) never does, and this module shares no code with it.

Network (row-vector convention; X is [B][d], W_i is [d_out][d_in]):

    z_i = x_{i-1} W_i^T + b_i,   m_i = (z_i > 0),   x_i = m_i ? z_i : alpha_i * z_i,   i = 1..L
    J   = 0.5 * ||x_L - t||_F^2 / B

alpha_i in (0, 1] is a leaky ReLU (a submersion when W_i has full row rank); alpha_i == 0 is
a ReLU, whose Jacobian erases cotangent entries and therefore needs the fragment store.

What follows which passage of the Moonwalk paper:

* `backprop`            ordinary reverse mode; it is the plain definition of the result, since
                        the method yields the exact gradient (Moonwalk identity, Eq. ifp-main).
                        `forward_layerwise` / `backprop_layerwise`: the same, one layer in memory at a
                        time (for the 256-layer configuration), pinned to be `backprop` bit for bit.
* `right_inverse`       the (.)^+ of the vijp definition (Notation section) for a dense layer:
                        the Moore-Penrose right inverse of W, kept as P = (W W^T)^{-1} W so that
                        the vijp of the affine map is ct_z = ct_x P^T.  P W^T = I.
* `moonwalk`            Phases I-III of the Overview section and Algorithm 1: a forward pass
                        that keeps only sign bits (Residual Impact section), a reverse pass for
                        the input cotangent h_0 alone, and a forward sweep h_i = vijp(f_i, x_{i-1},
                        h_{i-1}), g_i = vjp(f_i, theta_i, h_i) (Eq. h_i, Eq. g_i).
* fragment store        fragmental cotangent checkpointing (section on Fragmental Gradient
                        Checkpointing) in its elementwise-ReLU form: the minimal subset of the
                        output cotangent that the Jacobian erases is exactly the entries with
                        z <= 0; they are kept in ascending flat order in phase II and put back
                        in phase III.
* re-seeding            plain cotangent checkpointing in phase II (Overview section): every
                        K-th layer-input cotangent is kept and replaces the propagated one in
                        phase III.  K = 0 never re-seeds (the method as printed).

* `sgd_step`            Algorithm 1 with its "Apply g_i" line for plain gradient descent:
                        theta_i <- theta_i - lr g_i with the exact gradient.
* `newton_schulz_refresh`  NOT in the paper, which does not say how the inverse follows the
                        weights: the Schulz iteration for a (pseudo-)inverse, started from the
                        old right inverse carried over to the new weights (see its docstring).

Readings of points the paper leaves open (each is restated in the design notes):
mask bit = (z > 0) strictly, so z = 0, -0.0 and NaN take the slope alpha; every layer is
activated, including the last; packed masks are little-endian in flat row-major order, bit
(e mod 64) of word (e div 64); fragments of a layer are in ascending flat index and layer
bases are an exclusive scan of the per-layer erased counts in reverse-pass order (layer L
first); ReLU layers zero ct_z at erased entries before the parameter vjp; the loss scale
multiplies h_L and is divided out of dW, db.

Pins live in tests/test_oracle_*.py (finite differences, P W^T = I, closed-form P,
Moonwalk == backprop, brute-force packing/compaction, growth law of the rounding error).
No function here is "parity unpinned".
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import scipy.linalg

F64 = np.float64


# --------------------------------------------------------------------------- elementary pieces

def _as64(a) -> np.ndarray:
    return np.asarray(a, dtype=F64)


def sign_mask(z: np.ndarray) -> np.ndarray:
    """m = (z > 0), strictly: 0, -0.0 and NaN give False."""
    return np.greater(z, 0.0)


def activation(z: np.ndarray, m: np.ndarray, alpha: float) -> np.ndarray:
    """x = m ? z : alpha * z."""
    return np.where(m, z, alpha * z)


def activation_slope(m: np.ndarray, alpha: float) -> np.ndarray:
    """f'(z) = m ? 1 : alpha."""
    return np.where(m, 1.0, alpha)


def loss_and_output_cotangent(x_L: np.ndarray, t: np.ndarray, loss_scale: float = 1.0):
    """J = 0.5 ||x_L - t||_F^2 / B and h_L = loss_scale * dJ/dx_L = loss_scale (x_L - t) / B."""
    B = x_L.shape[0]
    r = x_L - t
    return 0.5 * float(np.sum(r * r)) / B, loss_scale * r / B


def forward(Ws, bs, alphas, x0, forced_masks: Optional[Sequence[np.ndarray]] = None):
    """Plain forward pass. Returns (xs = [x_0..x_L], zs = [z_1..z_L], masks = [m_1..m_L]).

    With `forced_masks` the sign decisions are imposed instead of taken from z (the network
    is then the piecewise-linear piece those masks select).
    """
    xs, zs, masks = [_as64(x0)], [], []
    for i, (W, b, a) in enumerate(zip(Ws, bs, alphas)):
        z = xs[-1] @ _as64(W).T + _as64(b)
        m = sign_mask(z) if forced_masks is None else np.asarray(forced_masks[i], dtype=bool)
        xs.append(activation(z, m, a))
        zs.append(z)
        masks.append(m)
    return xs, zs, masks


def loss_value(Ws, bs, alphas, x0, t, forced_masks=None) -> float:
    xs, _, _ = forward(Ws, bs, alphas, x0, forced_masks)
    return loss_and_output_cotangent(xs[-1], _as64(t))[0]


# --------------------------------------------------------------------------- backprop (the definition)

def backprop(Ws, bs, alphas, x0, t, forced_masks=None) -> Dict[str, object]:
    """Reverse-mode gradient of J. Keeps every activation (that is the point of comparison).

    Returns dW[i] ([d_out][d_in]), db[i] ([d_out]), loss, masks (bool, per layer),
    h = [h_0..h_L] with h_i = dJ/dx_i, and zs.
    """
    L = len(Ws)
    xs, zs, masks = forward(Ws, bs, alphas, x0, forced_masks)
    loss, h = loss_and_output_cotangent(xs[-1], _as64(t))
    hs = [None] * (L + 1)
    hs[L] = h
    dW, db = [None] * L, [None] * L
    for i in range(L - 1, -1, -1):                      # layer i+1 in the paper's numbering
        ct_z = hs[i + 1] * activation_slope(masks[i], alphas[i])
        dW[i] = ct_z.T @ xs[i]                          # vjp w.r.t. W
        db[i] = ct_z.sum(axis=0)                        # vjp w.r.t. b
        hs[i] = ct_z @ _as64(Ws[i])                     # vjp w.r.t. the layer input
    return {"dW": dW, "db": db, "loss": loss, "masks": masks, "h": hs, "zs": zs, "xs": xs}


def forward_layerwise(layer, depth: int, alphas, x0, mask_for=None):
    """`forward` for networks whose parameters are fetched one layer at a time: `layer(i)` returns (W_i, b_i)
    (any dtype; used as fp64 and dropped), `mask_for(i, z)` returns the sign decisions to impose on layer i
    given its pre-activation (None, or a None result: the signs of z). Returns (xs = [x_0..x_L], masks)."""
    xs, masks = [_as64(x0)], []
    for i in range(depth):
        W, b = layer(i)
        z = xs[-1] @ _as64(W).T + _as64(b)
        m = mask_for(i, z) if mask_for is not None else None
        m = sign_mask(z) if m is None else np.asarray(m, dtype=bool)
        xs.append(activation(z, m, alphas[i]))
        masks.append(m)
    return xs, masks


def backprop_layerwise(layer, alphas, xs, masks, t):
    """`backprop` for networks whose gradients do not fit in memory at once: a generator over the layers from the
    last to the first, given the activations and masks of `forward_layerwise`. Yields first (L, loss, None, h_L),
    then (i, dW_i, db_i, h_i) for i = L-1 .. 0 with h_i = dJ/dx_i the cotangent at layer i's INPUT (0-based i: the
    paper's layer i+1); xs[i+1] is released once used. Same arithmetic, in the same order, as `backprop`."""
    L = len(masks)
    loss, h = loss_and_output_cotangent(xs[L], _as64(t))
    yield L, loss, None, h
    for i in range(L - 1, -1, -1):
        ct_z = h * activation_slope(masks[i], alphas[i])
        dW = ct_z.T @ xs[i]
        db = ct_z.sum(axis=0)
        W, _ = layer(i)
        h = ct_z @ _as64(W)
        xs[i + 1] = None
        yield i, dW, db, h


# --------------------------------------------------------------------------- right inverse

def right_inverse(W) -> np.ndarray:
    """P = (W W^T)^{-1} W by a Cholesky solve; P W^T = I, W^+ = P^T is the Moore-Penrose right inverse.

    Raises ValueError when d_out > d_in and numpy.linalg.LinAlgError when W W^T is not
    positive definite (W not of full row rank): such a layer is not a submersion.
    """
    W = _as64(W)
    d_out, d_in = W.shape
    if d_out > d_in:
        raise ValueError("not submersive: d_out > d_in")
    G = W @ W.T
    Lc = np.linalg.cholesky(G)                                        # G = Lc Lc^T
    Y = scipy.linalg.solve_triangular(Lc, W, lower=True)              # Lc Y = W
    return scipy.linalg.solve_triangular(Lc.T, Y, lower=False)        # Lc^T P = Y


# --------------------------------------------------------------------------- training step and refresh

def round_to_bf16(a):
    """Every element rounded to the nearest number with an 8-bit significand (bfloat16's: 1 implicit + 7
    stored bits), ties to the even significand. Returned in fp64; bfloat16's exponent range is fp32's, and
    values beyond it (or below its normal range) are not treated specially here."""
    a = _as64(a)
    mant, exp = np.frexp(a)                     # a = mant * 2^exp with 0.5 <= |mant| < 1
    return np.ldexp(np.rint(mant * 256.0) / 256.0, exp)      # rint rounds halves to even


def newton_schulz_refresh(W_new, P_old, iters: int, correction: str = "exact"):
    """Right inverse of W_new from the right inverse P_old = (W_old W_old^T)^{-1} W_old of nearby
    weights, without a factorisation (the library's incremental refresh, written out):

        P_0     = (P_old P_old^T) W_new          since P_old P_old^T = (W_old W_old^T)^{-1}
        P_{k+1} = (2 I - P_k W_new^T) P_k        Schulz iteration, k = 0 .. iters-1

    Every iterate is a left multiple of W_new, so the limit is the minimum-norm right inverse
    (W_new W_new^T)^{-1} W_new, and the residual R_k = I - P_k W_new^T obeys R_{k+1} = R_k^2.
    A square layer has one inverse only and no row space to stay in: there the iteration starts from
    P_0 = P_old itself (residual -P_old dW^T, of the size of the update), which saves the two products
    of the start.
    correction="bf16" is the library's mixed-precision variant: the iteration written as
    P_{k+1} = P_k + R_k P_k, with both operands of the correction product R_k P_k rounded to bfloat16
    and everything else as before. With relative roundings dR, dP of at most 2^-8 per element the
    residual obeys R_{k+1} = R_k^2 - dR (I - R_k) - (R_k + dR) dP W_new^T: it shrinks by a factor of order
    2^-8 per iteration once R_k is below that, to the same limit P W_new^T = I. The rounding of P_k leaves
    the row space of W_new, so for a non-square layer the limit is a right inverse within
    2^-8 ||R_0|| ||P|| of the minimum-norm one rather than that one exactly.
    Returns (P, residuals) with residuals[k] = ||I - P_k W_new^T||_F for k = 0 .. iters.
    """
    if correction not in ("exact", "bf16"):
        raise ValueError(f"unknown correction {correction!r}")
    W = _as64(W_new)
    P_old = _as64(P_old)
    n = W.shape[0]
    eye = np.eye(n)
    P = P_old.copy() if W.shape[0] == W.shape[1] else (P_old @ P_old.T) @ W
    residuals = [float(np.linalg.norm(eye - P @ W.T))]
    for _ in range(int(iters)):
        E = P @ W.T
        if correction == "bf16":
            P = P + round_to_bf16(eye - E) @ round_to_bf16(P)
        else:
            P = (2.0 * eye - E) @ P
        residuals.append(float(np.linalg.norm(eye - P @ W.T)))
    return P, residuals


def sgd_step(Ws, bs, alphas, x0, t, lr: float, forced_masks=None):
    """One step of plain gradient descent on J (Algorithm 1 with "Apply g_i"): the exact gradient
    (backprop) applied to every layer. Returns (new Ws, new bs, loss before the update, masks)."""
    g = backprop(Ws, bs, alphas, x0, t, forced_masks=forced_masks)
    new_W = [_as64(W) - lr * dW for W, dW in zip(Ws, g["dW"])]
    new_b = [_as64(b) - lr * db for b, db in zip(bs, g["db"])]
    return new_W, new_b, g["loss"], g["masks"]


# --------------------------------------------------------------------------- packed masks and fragments

def pack_mask(m: np.ndarray) -> np.ndarray:
    """Pack a bool array (any shape, flattened row-major) into uint64 words, LSB first.

    Element e is bit (e mod 64) of word (e div 64); unused bits of the last word are 0.
    """
    flat = np.asarray(m, dtype=bool).ravel()
    n_words = (flat.size + 63) // 64
    padded = np.zeros(n_words * 64, dtype=np.uint64)
    padded[: flat.size] = flat
    weights = np.uint64(1) << np.arange(64, dtype=np.uint64)          # 2^bit
    return (padded.reshape(n_words, 64) * weights).sum(axis=1, dtype=np.uint64)


def unpack_mask(words: np.ndarray, n: int) -> np.ndarray:
    """Inverse of pack_mask for the first n elements."""
    words = np.asarray(words, dtype=np.uint64)
    bits = (words[:, None] >> np.arange(64, dtype=np.uint64)) & np.uint64(1)
    return bits.ravel()[:n].astype(bool)


def erased_word_offsets(m: np.ndarray) -> np.ndarray:
    """Per 64-element word: number of erased (mask == 0) elements in all earlier words.

    uint32[n_words + 1]; the last entry is the layer's erased count n0. Padding bits of the
    last word are not elements and are not counted.
    """
    flat = np.asarray(m, dtype=bool).ravel()
    n_words = (flat.size + 63) // 64
    erased = np.zeros(n_words * 64, dtype=np.int64)
    erased[: flat.size] = ~flat
    off = np.zeros(n_words + 1, dtype=np.int64)
    off[1:] = np.cumsum(erased.reshape(n_words, 64).sum(axis=1))
    return off.astype(np.uint32)


def compact_fragments(h: np.ndarray, m: np.ndarray) -> np.ndarray:
    """The erased part of a cotangent: h[e] for every flat index e with m[e] == 0, ascending."""
    return np.asarray(h).ravel()[~np.asarray(m, dtype=bool).ravel()].copy()


def erased_rank(m: np.ndarray) -> np.ndarray:
    """rank0(e) = number of erased elements with flat index < e (int64, same shape as m)."""
    z = (~np.asarray(m, dtype=bool)).ravel().astype(np.int64)
    return (np.cumsum(z) - z).reshape(np.shape(m))


def restore_from_fragments(ct_z: np.ndarray, m: np.ndarray, frags: np.ndarray) -> np.ndarray:
    """Output cotangent of a ReLU: kept entries come from ct_z, erased ones from the store."""
    m = np.asarray(m, dtype=bool)
    r = erased_rank(m)
    out = np.array(ct_z, dtype=F64, copy=True)
    out[~m] = np.asarray(frags, dtype=F64)[r[~m]]
    return out


def checkpointed_layers(L: int, K: int) -> List[int]:
    """Indices j in 1..L-1 whose layer-output cotangent h_j is kept for re-seeding (j mod K == 0)."""
    if K <= 0:
        return []
    return [j for j in range(1, L) if j % K == 0]


# --------------------------------------------------------------------------- Moonwalk

def adaptive_reseed_layers(alphas: Sequence[float], budget: float = 700.0, segment: int = 0) -> List[int]:
    """Where the library's reseed_interval = -1 keeps a cotangent (not in the paper: this build's
    answer to the conditioning of the inverse activation slopes, see error_growth_per_layer).

    Walk up the layers with the predicted error growth since the last seed, the product of
    error_growth_per_layer(alpha_j) (1 for a ReLU, whose erased entries come back exactly). Layer
    boundary j (the output of layer j, 1-based, j < L) becomes a seed when taking layer j+1 in as
    well would push the product beyond `budget`. With segment = S > 0 every boundary j = S, 2S, ...
    is an exact seed anyway (Moonwalk with rematerialisation) and is not listed.
    """
    L = len(alphas)
    out: List[int] = []
    growth = 1.0
    g = [error_growth_per_layer(a) if a > 0 else 1.0 for a in alphas]
    for j in range(1, L):
        growth *= g[j - 1]
        if segment > 0 and j % segment == 0:
            growth = 1.0
        elif growth * g[j] > budget:
            out.append(j)
            growth = 1.0
    return out


def moonwalk(Ws, bs, alphas, x0, t, reseed_interval: int = 0, loss_scale: float = 1.0,
             forced_masks=None, Ps: Optional[Sequence[np.ndarray]] = None,
             dtype=F64, reseed_layers: Optional[Sequence[int]] = None) -> Dict[str, object]:
    """Mixed-mode Moonwalk, step by step (Overview section, Algorithm 1).

    `dtype` is the arithmetic type of every step (fp64 for the oracle proper; the tests also
    run it in fp32 to study rounding). `Ps` overrides the right inverses (used by the test
    that any right inverse gives the same result). `reseed_layers` (layer boundaries j, 1 <= j < L)
    overrides the every-K-th rule of `reseed_interval`.

    Returns dW, db (un-scaled), loss, masks (bool), packed (uint64 words per layer),
    fragments (per layer, None for leaky layers), frag_base (per layer start in a store
    filled in reverse-pass order), word_offsets (per ReLU layer), h0, hs (phase-III
    cotangents h_0..h_L, scaled), h_rev (phase-II cotangents), checkpoints.
    """
    L = len(Ws)
    Wd = [np.asarray(_as64(W), dtype=dtype) for W in Ws]
    bd = [np.asarray(_as64(b), dtype=dtype) for b in bs]
    al = [dtype(a) for a in alphas]
    x0 = np.asarray(_as64(x0), dtype=dtype)
    t = np.asarray(_as64(t), dtype=dtype)
    B = x0.shape[0]

    # ---- setup: one right inverse per layer
    if Ps is None:
        Ps = [right_inverse(W) for W in Ws]             # always solved in fp64
    Pd = [np.asarray(P, dtype=dtype) for P in Ps]

    # ---- Phase I: forward, keep sign bits only
    x = x0
    masks = []
    for i in range(L):
        z = x @ Wd[i].T + bd[i]
        m = sign_mask(z) if forced_masks is None else np.asarray(forced_masks[i], dtype=bool)
        masks.append(m)
        x = np.where(m, z, al[i] * z)
    r = x - t
    loss = 0.5 * float(np.sum(_as64(r) ** 2)) / B
    h = (dtype(loss_scale) * r / dtype(B)).astype(dtype)

    # ---- Phase II: reverse, input cotangent only; fragments and checkpoints on the way
    kept = set(checkpointed_layers(L, reseed_interval)) if reseed_layers is None else set(int(j) for j in reseed_layers)
    fragments: List[Optional[np.ndarray]] = [None] * L
    checkpoints: Dict[int, np.ndarray] = {}
    h_rev = [None] * (L + 1)
    h_rev[L] = h
    for i in range(L - 1, -1, -1):
        if al[i] == 0:
            fragments[i] = compact_fragments(h, masks[i])
        ct_z = h * np.where(masks[i], dtype(1), al[i])
        h = ct_z @ Wd[i]
        h_rev[i] = h
        if i in kept:
            checkpoints[i] = h
    h0 = h

    # fragment-store bases: layers are appended in reverse-pass order, layer L first
    frag_base = [None] * L
    running = 0
    for i in range(L - 1, -1, -1):
        if fragments[i] is not None:
            frag_base[i] = running
            running += fragments[i].size
    word_offsets = [erased_word_offsets(masks[i]) if al[i] == 0 else None for i in range(L)]

    # ---- Phase III: forward vijp sweep
    x = x0
    h = h0
    hs = [h0]
    dW, db = [None] * L, [None] * L
    inv_scale = dtype(1.0 / loss_scale)
    for i in range(L):
        if i in checkpoints:                                    # re-seed
            h = checkpoints[i]
            hs[-1] = h
        z = x @ Wd[i].T + bd[i]                                 # recompute the layer
        ct_z = h @ Pd[i].T                                      # vijp of the affine part
        if al[i] == 0:
            m = masks[i]                                        # stored bits: ranks must match phase II
            ct_z = np.where(m, ct_z, dtype(0))
            h_y = restore_from_fragments(ct_z, m, fragments[i]).astype(dtype)
        else:
            m = sign_mask(z) if forced_masks is None else masks[i]
            h_y = ct_z * np.where(m, dtype(1), dtype(1) / al[i])  # vijp of the activation
        dW[i] = (ct_z.T @ x) * inv_scale                        # vjp w.r.t. W
        db[i] = ct_z.sum(axis=0) * inv_scale                    # vjp w.r.t. b
        x = np.where(m, z, al[i] * z)
        h = h_y
        hs.append(h)

    return {"dW": dW, "db": db, "loss": loss, "masks": masks,
            "packed": [pack_mask(m) for m in masks], "fragments": fragments,
            "frag_base": frag_base, "frag_total": running, "word_offsets": word_offsets,
            "h0": h0, "hs": hs, "h_rev": h_rev, "checkpoints": checkpoints, "P": list(Ps)}


# --------------------------------------------------------------------------- error measures and closed forms

def normwise_rel_err(a, ref) -> float:
    """||a - ref||_F / ||ref||_F (0/0 -> 0)."""
    a, ref = _as64(a), _as64(ref)
    den = float(np.linalg.norm(ref))
    num = float(np.linalg.norm(a - ref))
    if den == 0.0:
        return 0.0 if num == 0.0 else np.inf
    return num / den


def max_layer_err(got: Sequence[np.ndarray], ref: Sequence[np.ndarray]) -> float:
    """Largest per-tensor normwise relative error over the layers."""
    return max(normwise_rel_err(g, r) for g, r in zip(got, ref))


def error_growth_per_layer(alpha: float) -> float:
    """Predicted per-layer growth of the relative rounding error in the phase-III cotangent.

    Half of the activation slopes are 1 and half are alpha. Through the inverse Jacobians an
    error component grows like sqrt(E[f'^-2]) per layer, while the true cotangent, which
    undoes the shrinkage of the reverse pass, grows only like 1/sqrt(E[f'^2]). Their ratio is
    sqrt(((1 + alpha^-2)/2) * ((1 + alpha^2)/2)), about 5.05 for alpha = 0.1.
    """
    return float(np.sqrt(((1.0 + alpha ** -2) / 2.0) * ((1.0 + alpha ** 2) / 2.0)))
