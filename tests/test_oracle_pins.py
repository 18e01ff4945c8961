"""Pins for the fp64 oracle: each test ties one of its functions to something other than itself
(finite differences, closed forms, library routines, brute force on tiny inputs, invariants the
paper states), so that a dropped term, wrong sign, wrong index or transposed operand fails here.
"""
import numpy as np
import pytest

from oracle import moonwalk_oracle as O
from workloads import make_mlp, make_config


def tiny(widths, batch, alpha, seed=0, **kw):
    return make_mlp(widths, batch, alpha, seed=seed, keep_factors=True, **kw)


# ---------------------------------------------------------------- backprop vs finite differences

@pytest.mark.parametrize("widths,batch,alpha", [
    ([6, 6, 6], 3, 0.1),
    ([8, 6, 5, 3], 4, 0.3),
    ([7, 7], 2, 0.0),
    ([8, 8, 6], 3, 0.0),
])
def test_backprop_matches_central_differences(widths, batch, alpha):
    wl = tiny(widths, batch, alpha, seed=3)
    Ws = [w.astype(np.float64) for w in wl.W]
    bs = [b.astype(np.float64) for b in wl.b]
    # a bias large enough that some pre-activations are negative, some positive
    rng = np.random.default_rng(5)
    bs = [b + 0.3 * rng.standard_normal(b.shape) for b in bs]
    ref = O.backprop(Ws, bs, wl.alphas, wl.x, wl.t)
    # keep away from the kinks so that central differences see one linear piece
    assert min(np.abs(z).min() for z in ref["zs"]) > 1e-4
    eps = 1e-6

    def J():
        return O.loss_value(Ws, bs, wl.alphas, wl.x, wl.t)

    for i in range(len(Ws)):
        for arr, grad in ((Ws[i], ref["dW"][i]), (bs[i], ref["db"][i])):
            it = np.nditer(arr, flags=["multi_index"])
            for _ in it:
                idx = it.multi_index
                old = arr[idx]
                arr[idx] = old + eps
                jp = J()
                arr[idx] = old - eps
                jm = J()
                arr[idx] = old
                fd = (jp - jm) / (2 * eps)
                assert abs(fd - grad[idx]) <= 1e-7 * max(1.0, abs(grad[idx])), (i, idx, fd, grad[idx])


def test_loss_definition_and_output_cotangent():
    # J = 0.5 * sum over batch and features of (x_L - t)^2, divided by the batch size only
    x = np.array([[1.0, 2.0, 3.0], [0.0, -1.0, 1.0]])
    t = np.array([[0.0, 2.0, 1.0], [1.0, 1.0, 1.0]])
    J, h = O.loss_and_output_cotangent(x, t, loss_scale=4.0)
    assert J == pytest.approx(0.5 * (1 + 0 + 4 + 1 + 4 + 0) / 2)
    np.testing.assert_allclose(h, 4.0 * (x - t) / 2)


# ---------------------------------------------------------------- right inverse

@pytest.mark.parametrize("d_in,d_out", [(8, 8), (12, 5), (64, 64), (96, 32)])
def test_right_inverse_identity_and_closed_form(d_in, d_out):
    wl = tiny([d_in, d_out], 2, 0.1, seed=11)
    W = wl.W[0].astype(np.float64)
    P = O.right_inverse(W)
    assert P.shape == (d_out, d_in)
    np.testing.assert_allclose(P @ W.T, np.eye(d_out), atol=1e-12)
    # Moore-Penrose: numpy's SVD-based pseudo-inverse is an independent library routine
    np.testing.assert_allclose(P, np.linalg.pinv(W).T, atol=1e-12)
    # closed form from the generator's own factors (up to the fp32 rounding of W)
    f = wl.factors[0]
    P_closed = (f["U"] / f["s"]) @ f["V"].T
    assert np.abs(P - P_closed).max() < 5e-6
    if d_in == d_out:
        np.testing.assert_allclose(P, np.linalg.inv(W).T, atol=1e-11)


def test_right_inverse_brute_force_gaussian_elimination():
    rng = np.random.default_rng(0)
    W = rng.standard_normal((4, 6))
    G = W @ W.T
    # solve G P = W by hand-rolled Gauss-Jordan elimination
    aug = np.hstack([G, W]).astype(np.float64)
    n = 4
    for c in range(n):
        aug[c] /= aug[c, c]
        for r in range(n):
            if r != c:
                aug[r] -= aug[r, c] * aug[c]
    np.testing.assert_allclose(O.right_inverse(W), aug[:, n:], atol=1e-12)


def test_right_inverse_rejects_non_submersions():
    with pytest.raises(ValueError):
        O.right_inverse(np.ones((5, 3)))
    W = np.ones((3, 5))                      # rank 1: W W^T is singular
    with pytest.raises(np.linalg.LinAlgError):
        O.right_inverse(W)


def test_vijp_round_trip_and_right_inverse_independence():
    wl = tiny([20, 9], 5, 0.1, seed=2)
    W = wl.W[0].astype(np.float64)
    P = O.right_inverse(W)
    rng = np.random.default_rng(1)
    ct_z = rng.standard_normal((5, 9))
    ct_x = ct_z @ W                                      # vjp
    np.testing.assert_allclose(ct_x @ P.T, ct_z, atol=1e-12)   # vijp undoes it
    # any other right inverse W^+' = W^+ + (I - W^+ W) Y gives the same answer on the row space
    Wp = P.T
    Y = rng.standard_normal((20, 9))
    Wp2 = Wp + (np.eye(20) - Wp @ W) @ Y
    np.testing.assert_allclose(W @ Wp2, np.eye(9), atol=1e-12)
    assert np.abs(Wp2 - Wp).max() > 0.1
    np.testing.assert_allclose(ct_x @ Wp2, ct_z, atol=1e-11)


# ---------------------------------------------------------------- masks and fragments

def test_pack_mask_matches_numpy_packbits_and_brute_force():
    rng = np.random.default_rng(4)
    for shape in [(1, 1), (3, 5), (2, 64), (5, 67), (4, 128), (7, 100)]:
        m = rng.random(shape) < 0.4
        words = O.pack_mask(m)
        n = m.size
        assert words.dtype == np.uint64 and words.size == (n + 63) // 64
        # library routine
        pb = np.packbits(m.ravel(), bitorder="little")
        pb = np.concatenate([pb, np.zeros(words.size * 8 - pb.size, dtype=np.uint8)])
        np.testing.assert_array_equal(words, pb.view("<u8"))
        # brute force, one bit at a time
        for e, bit in enumerate(m.ravel()):
            assert ((int(words[e // 64]) >> (e % 64)) & 1) == int(bit)
        # tail bits are zero
        if n % 64:
            assert int(words[-1]) >> (n % 64) == 0
        np.testing.assert_array_equal(O.unpack_mask(words, n), m.ravel())


def test_sign_mask_special_values():
    z = np.array([1.0, -1.0, 0.0, -0.0, np.nan, np.inf, -np.inf, 5e-324])
    np.testing.assert_array_equal(O.sign_mask(z), [True, False, False, False, False, True, False, True])
    assert O.pack_mask(np.ones((2, 64), bool)).tolist() == [2 ** 64 - 1] * 2
    assert O.pack_mask(np.zeros((2, 64), bool)).tolist() == [0, 0]
    # mask bytes are 32x smaller than fp32 activations when B*d is a multiple of 64
    m = np.zeros((32, 64), bool)
    assert O.pack_mask(m).nbytes * 32 == m.size * 4


def test_fragments_brute_force():
    rng = np.random.default_rng(9)
    for shape in [(3, 5), (4, 64), (5, 70)]:
        m = rng.random(shape) < 0.5
        h = rng.standard_normal(shape)
        F = O.compact_fragments(h, m)
        expect, ranks = [], {}
        for e in range(m.size):
            if not m.ravel()[e]:
                ranks[e] = len(expect)
                expect.append(h.ravel()[e])
        np.testing.assert_array_equal(F, np.array(expect))
        r = O.erased_rank(m).ravel()
        for e, k in ranks.items():
            assert r[e] == k
        off = O.erased_word_offsets(m)
        words = O.pack_mask(m)
        assert off[-1] == len(expect) == m.size - int(m.sum())
        for w in range(words.size):
            lo, hi = 64 * w, min(64 * w + 64, m.size)
            assert off[w + 1] - off[w] == (hi - lo) - bin(int(words[w])).count("1")
        # restoring puts back exactly the erased values and leaves the kept ones
        ct = rng.standard_normal(shape)
        out = O.restore_from_fragments(ct, m, F)
        np.testing.assert_array_equal(out[m], ct[m])
        np.testing.assert_array_equal(out[~m], h[~m])


# ---------------------------------------------------------------- Moonwalk == backprop

@pytest.mark.parametrize("widths,batch,alpha,K", [
    ([64] * 5, 32, 0.1, 0),            # the tiny configuration
    ([48, 40, 32, 32, 16], 8, 0.1, 0),
    ([32] * 9, 8, 0.25, 0),
    ([32] * 9, 8, 0.1, 2),
])
def test_moonwalk_equals_backprop_shallow(widths, batch, alpha, K):
    wl = tiny(widths, batch, alpha, seed=1)
    bp = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    mw = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t, reseed_interval=K)
    assert mw["loss"] == pytest.approx(bp["loss"], rel=1e-14)
    assert O.max_layer_err(mw["dW"], bp["dW"]) < 1e-9
    assert O.max_layer_err(mw["db"], bp["db"]) < 1e-9
    np.testing.assert_allclose(mw["h0"], bp["h"][0], rtol=0, atol=1e-15)
    for i, m in enumerate(bp["masks"]):
        np.testing.assert_array_equal(mw["packed"][i], O.pack_mask(m))


def test_moonwalk_relu_fragments_equals_backprop_at_depth():
    wl = tiny([48] * 41, 16, 0.0, seed=2)
    bp = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    mw = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    assert O.max_layer_err(mw["dW"], bp["dW"]) < 1e-12
    assert O.max_layer_err(mw["db"], bp["db"]) < 1e-12
    # the erased entries of every restored cotangent are bit-identical to phase II's
    for i in range(wl.depth):
        m = bp["masks"][i]
        np.testing.assert_array_equal(mw["hs"][i + 1][~m], mw["h_rev"][i + 1][~m])
        assert mw["fragments"][i].size == m.size - int(m.sum())
    # layer bases: reverse-pass order, layer L first
    assert mw["frag_base"][-1] == 0
    running = 0
    for i in range(wl.depth - 1, -1, -1):
        assert mw["frag_base"][i] == running
        running += mw["fragments"][i].size
    assert mw["frag_total"] == running


def test_moonwalk_mixed_leaky_and_relu_layers():
    alphas = [0.1, 0.0, 0.5, 0.0, 1.0]
    wl = tiny([40, 36, 36, 30, 30, 12], 6, alphas, seed=8)
    bp = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    mw = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    assert O.max_layer_err(mw["dW"], bp["dW"]) < 1e-10
    assert O.max_layer_err(mw["db"], bp["db"]) < 1e-10
    assert [f is not None for f in mw["fragments"]] == [False, True, False, True, False]


def test_forced_masks_select_the_linear_piece():
    wl = tiny([16, 16, 12], 4, 0.1, seed=6)
    free = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    same = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t, forced_masks=free["masks"])
    for a, b in zip(free["dW"], same["dW"]):
        np.testing.assert_array_equal(a, b)
    flipped = [m.copy() for m in free["masks"]]
    flipped[0][0, 0] = ~flipped[0][0, 0]
    other = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t, forced_masks=flipped)
    assert O.normwise_rel_err(other["dW"][0], free["dW"][0]) > 1e-4
    mw = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t, forced_masks=flipped)
    assert O.max_layer_err(mw["dW"], other["dW"]) < 1e-10


# ---------------------------------------------------------------- conditioning, re-seeding, loss scale

def test_error_growth_matches_closed_form():
    alpha = 0.1
    assert O.error_growth_per_layer(alpha) == pytest.approx(5.05, abs=0.01)
    wl = tiny([128] * 17, 32, alpha, seed=0)
    bp = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    mw = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    err = np.array([O.normwise_rel_err(a, b) for a, b in zip(mw["dW"], bp["dW"])])
    assert err[3] < 1e-12 and err[-1] > 1e-7          # grows from rounding level ...
    slope = np.exp(np.polyfit(np.arange(4, 16), np.log(err[4:16]), 1)[0])
    assert slope == pytest.approx(O.error_growth_per_layer(alpha), rel=0.15)   # ... at the predicted rate
    # ReLU + fragments does not grow
    wl0 = tiny([128] * 17, 32, 0.0, seed=0)
    bp0 = O.backprop(wl0.W, wl0.b, wl0.alphas, wl0.x, wl0.t)
    mw0 = O.moonwalk(wl0.W, wl0.b, wl0.alphas, wl0.x, wl0.t)
    assert O.max_layer_err(mw0["dW"], bp0["dW"]) < 1e-13


def test_reseeding_limits_the_growth():
    wl = tiny([64] * 25, 16, 0.1, seed=0)
    bp = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    e = {}
    for K in (0, 1, 4, 24, 100):
        mw = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t, reseed_interval=K)
        e[K] = O.max_layer_err(mw["dW"], bp["dW"])
        assert sorted(mw["checkpoints"]) == O.checkpointed_layers(24, K)
    assert e[0] > 1e-3                      # free-running fp64 has lost the gradient by depth 24
    assert e[1] < 1e-13                     # cotangent kept at every layer: one layer of rounding
    assert e[4] < 1e-10
    assert e[24] == e[0] and e[100] == e[0]   # K >= L never re-seeds
    assert O.checkpointed_layers(8, 4) == [4] and O.checkpointed_layers(9, 4) == [4, 8]


def test_power_of_two_loss_scale_is_exact():
    wl = tiny([32] * 5, 8, 0.1, seed=3)
    a = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t, loss_scale=1.0)
    b = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t, loss_scale=2.0 ** 20)
    for u, v in zip(a["dW"] + a["db"], b["dW"] + b["db"]):
        np.testing.assert_array_equal(u, v)
    np.testing.assert_array_equal(b["h0"], a["h0"] * 2.0 ** 20)


def test_fp32_moonwalk_on_tiny_config_meets_tolerance():
    wl = make_config("tiny")
    bp = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    mw32 = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t, dtype=np.float32, forced_masks=bp["masks"])
    assert O.max_layer_err(mw32["dW"], bp["dW"]) < 1e-3
    assert O.max_layer_err(mw32["db"], bp["db"]) < 1e-3


def test_tiny_golden_fixture_is_reproduced():
    import json
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_oracle.json")
    with open(path) as f:
        g = json.load(f)
    wl = make_config("tiny")
    bp = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    assert bp["loss"] == pytest.approx(g["loss"], rel=1e-12)
    np.testing.assert_allclose([np.linalg.norm(a) for a in bp["dW"]], g["dW_fro"], rtol=1e-11)
    np.testing.assert_allclose([np.linalg.norm(a) for a in bp["db"]], g["db_fro"], rtol=1e-11)
    assert [int(m.sum()) for m in bp["masks"]] == g["mask_popcount"]
    assert [format(int(O.pack_mask(m)[0]), "016x") for m in bp["masks"]] == g["mask_word0_hex"]
    np.testing.assert_array_equal(wl.W[0][0, :4], np.float32(g["W1_first_row_head"]))
    np.testing.assert_array_equal(wl.x[0, :4], np.float32(g["x_head"]))


def test_layerwise_backprop_is_backprop_bit_for_bit():
    """The one-layer-at-a-time form used for the deepest configuration: same loss, gradients, cotangents and masks
    as `backprop`, exactly, with free and with forced masks; activations are released on the way."""
    wl = make_mlp([20, 16, 16, 12, 7], batch=9, alpha=[0.1, 0.0, 0.5, 0.0], seed=13)
    rng = np.random.default_rng(3)
    forced = [rng.random((9, d)) < 0.5 for d in wl.widths[1:]]
    for masks_in in (None, forced):
        ref = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t, forced_masks=masks_in)
        asked = []
        def layer(i):
            asked.append(i)
            return wl.W[i], wl.b[i]
        xs, masks = O.forward_layerwise(layer, wl.depth, wl.alphas, wl.x,
                                        None if masks_in is None else (lambda i, z: masks_in[i]))
        assert asked == list(range(wl.depth))
        for a, b in zip(xs, ref["xs"]):
            np.testing.assert_array_equal(a, b)
        for a, b in zip(masks, ref["masks"]):
            np.testing.assert_array_equal(a, b)
        seen = []
        for i, dW, db, h in O.backprop_layerwise(layer, wl.alphas, xs, masks, wl.t):
            seen.append(i)
            if i == wl.depth:
                assert dW == ref["loss"] and db is None
            else:
                np.testing.assert_array_equal(dW, ref["dW"][i])
                np.testing.assert_array_equal(db, ref["db"][i])
                assert xs[i + 1] is None
            np.testing.assert_array_equal(h, ref["h"][i])
        assert seen == list(range(wl.depth, -1, -1))
    # a mask_for that declines (returns None) leaves the sign of z in charge
    xs2, masks2 = O.forward_layerwise(lambda i: (wl.W[i], wl.b[i]), wl.depth, wl.alphas, wl.x, lambda i, z: None)
    free = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    for a, b in zip(masks2, free["masks"]):
        np.testing.assert_array_equal(a, b)


# ----------------------------------------------------------------------------- training step and refresh
def test_newton_schulz_refresh_squares_the_residual_and_reaches_the_pseudo_inverse():
    """Schulz iteration: R_{k+1} = R_k^2, limit = Moore-Penrose right inverse (library routine pinv)."""
    rng = np.random.default_rng(5)
    wl = make_mlp([24, 16], batch=4, alpha=0.1, seed=11)
    W_old = wl.W[0].astype(np.float64)
    W_new = W_old + 2e-2 * rng.standard_normal(W_old.shape) / np.sqrt(W_old.shape[1])
    P_old = O.right_inverse(W_old)
    P, res = O.newton_schulz_refresh(W_new, P_old, iters=4)
    assert res[0] < 0.2
    for k in range(3):                       # quadratic: ||R^2|| <= ||R||^2 (Frobenius norm is submultiplicative)
        assert res[k + 1] <= res[k] ** 2 * (1 + 1e-9) + 1e-15
    assert res[4] < 1e-13
    assert np.allclose(P, np.linalg.pinv(W_new).T, atol=1e-12, rtol=0)
    # every iterate stays in the row space of W_new: P (I - W^+ W) = 0 already after zero iterations
    P0, _ = O.newton_schulz_refresh(W_new, P_old, iters=0)
    proj_null = np.eye(W_new.shape[1]) - np.linalg.pinv(W_new) @ W_new
    assert np.linalg.norm(P0 @ proj_null) < 1e-12


def test_newton_schulz_refresh_of_a_square_layer_starts_from_the_old_inverse():
    """Square W: P_0 = P_old, residual -P_old dW^T (first order in the update), squared by every iteration,
    limit = the inverse (library routine inv)."""
    rng = np.random.default_rng(8)
    wl = make_mlp([16, 16], batch=4, alpha=0.1, seed=12)
    W_old = wl.W[0].astype(np.float64)
    dW = 1e-2 * rng.standard_normal(W_old.shape) / np.sqrt(W_old.shape[1])
    W_new = W_old + dW
    P_old = O.right_inverse(W_old)
    P0, res0 = O.newton_schulz_refresh(W_new, P_old, iters=0)
    assert np.array_equal(P0, P_old)
    assert res0[0] == pytest.approx(np.linalg.norm(P_old @ dW.T), rel=1e-9)
    P, res = O.newton_schulz_refresh(W_new, P_old, iters=4)
    for k in range(3):
        assert res[k + 1] <= res[k] ** 2 * (1 + 1e-9) + 1e-15
    assert np.allclose(P, np.linalg.inv(W_new).T, atol=1e-12, rtol=0)


def test_round_to_bf16_against_hand_cases_and_the_library_conversion():
    """8-bit significand, ties to even: hand-written cases, then torch's float32 -> bfloat16 conversion
    (a library routine of its own) on random float32 values, which double rounding cannot touch."""
    import torch
    cases = [(1.0, 1.0), (1.0 + 2.0 ** -8, 1.0),                 # tie, even significand below
             (1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -6),             # tie, even significand above
             (1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 2.0 ** -7),    # just above the tie
             (-3.0 - 2.0 ** -7, -3.0), (-3.0 - 3 * 2.0 ** -7, -3.0 - 2.0 ** -5),   # ties in the next binade (spacing 2^-6)
             (-3.0 - 2.0 ** -6, -3.0 - 2.0 ** -6),               # held exactly
             (255.5, 256.0), (0.0, 0.0), (2.0 ** -40 * 1.2345, float(np.ldexp(np.rint(1.2345 * 128) / 128, -40)))]
    for x, want in cases:
        assert float(O.round_to_bf16(np.array([x]))[0]) == want, (x, want)
    rng = np.random.default_rng(17)
    x = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 20, 20000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_to_bf16(x), want)
    # idempotent, odd, and within half a unit in the last place: |r(x) - x| <= 2^-8 |x|
    r = O.round_to_bf16(x)
    np.testing.assert_array_equal(O.round_to_bf16(r), r)
    np.testing.assert_array_equal(O.round_to_bf16(-x.astype(np.float64)), -r)
    assert np.all(np.abs(r - x) <= 2.0 ** -8 * np.abs(x))


@pytest.mark.parametrize("widths", [[24, 16], [16, 16]])
def test_newton_schulz_refresh_with_the_bf16_correction(widths):
    """Operands that bfloat16 holds exactly give the exact iteration bit for bit; otherwise the residual obeys
    R_{k+1} = R_k^2 - dR (I - R_k) - (R_k + dR) dP W^T with |dR| <= 2^-8 |R_k|, |dP| <= 2^-8 |P_k| per element,
    and the limit is still a right inverse, within 2^-8 ||R_0|| ||P|| of the minimum-norm one."""
    rng = np.random.default_rng(23)
    # (a) one iteration on bf16-exact data: P_0 = P_old (square) and R_0 = I - P_old W^T made of small dyadic numbers
    n = 8
    W = np.eye(n) + rng.integers(-2, 3, (n, n)) / 16.0
    P_old = np.eye(n) + rng.integers(-2, 3, (n, n)) / 16.0
    Pe, _ = O.newton_schulz_refresh(W, P_old, 1)
    Pb, _ = O.newton_schulz_refresh(W, P_old, 1, correction="bf16")
    np.testing.assert_array_equal(Pe, Pb)
    # (b) general data
    wl = make_mlp(widths, batch=4, alpha=0.1, seed=11)
    W_old = wl.W[0].astype(np.float64)
    W_new = W_old + 2e-2 * rng.standard_normal(W_old.shape) / np.sqrt(W_old.shape[1])
    P_old = O.right_inverse(W_old)
    iters = 10
    P, res = O.newton_schulz_refresh(W_new, P_old, iters, correction="bf16")
    _, res_exact = O.newton_schulz_refresh(W_new, P_old, 1)
    assert res[0] == res_exact[0]
    assert res[1] != res_exact[1]                                         # the rounding is really there
    Pk = [O.newton_schulz_refresh(W_new, P_old, k, correction="bf16")[0] for k in range(iters)]
    eps = 2.0 ** -8
    w2 = np.linalg.norm(W_new, 2)
    for k in range(iters):
        bound = res[k] ** 2 + eps * res[k] * (1 + res[k]) + (1 + eps) * res[k] * eps * np.linalg.norm(Pk[k]) * w2
        assert res[k + 1] <= bound * (1 + 1e-9) + 1e-15, (k, res[k + 1], bound)
    assert res[iters] < 1e-13                                             # still a right inverse in the limit
    exact = O.right_inverse(W_new)
    assert np.linalg.norm(P - exact) <= eps * res[0] * np.linalg.norm(exact) * 1.5
    if widths[0] == widths[1]:                                            # a square matrix has one inverse only
        assert np.allclose(P, np.linalg.inv(W_new).T, atol=1e-11, rtol=0)
    with pytest.raises(ValueError):
        O.newton_schulz_refresh(W_new, P_old, 1, correction="fp8")


def test_newton_schulz_zero_iterations_is_first_order_accurate():
    """P_0 - P_new = O(||dW||): halving the perturbation halves the error."""
    rng = np.random.default_rng(6)
    wl = make_mlp([20, 12], batch=4, alpha=0.1, seed=3)
    W = wl.W[0].astype(np.float64)
    D = rng.standard_normal(W.shape) / np.sqrt(W.shape[1])
    P = O.right_inverse(W)
    errs = []
    for eps in (1e-3, 5e-4):
        P0, _ = O.newton_schulz_refresh(W + eps * D, P, iters=0)
        errs.append(np.linalg.norm(P0 - O.right_inverse(W + eps * D)))
    assert 1.8 < errs[0] / errs[1] < 2.2


def test_sgd_step_is_a_descent_step_with_the_finite_difference_gradient():
    """J(theta - lr g) = J(theta) - lr ||g||^2 + O(lr^2) with g pinned by finite differences elsewhere."""
    wl = make_mlp([12, 10, 8], batch=6, alpha=0.3, seed=21)
    Ws = [w.astype(np.float64) for w in wl.W]
    bs = [b.astype(np.float64) for b in wl.b]
    g = O.backprop(Ws, bs, wl.alphas, wl.x, wl.t)
    gnorm2 = sum(float(np.sum(d * d)) for d in g["dW"]) + sum(float(np.sum(d * d)) for d in g["db"])
    lr = 1e-4
    W1, b1, loss0, _ = O.sgd_step(Ws, bs, wl.alphas, wl.x, wl.t, lr)
    assert loss0 == g["loss"]
    loss1 = O.loss_value(W1, b1, wl.alphas, wl.x, wl.t)
    assert abs((loss0 - loss1) - lr * gnorm2) < 1e-3 * lr * gnorm2
    for W, Wn, d in zip(Ws, W1, g["dW"]):
        assert np.array_equal(Wn, W - lr * d)


# ----------------------------------------------------------------------------- adaptive re-seeding
def test_adaptive_reseed_rule_on_known_slopes():
    """alpha = 0.1 grows 5.05x per layer: 5.05^4 = 650 <= 700 < 5.05^5, so a seed every 4 layers;
    alpha = 0.5 grows 1.25x: 1.25^29 = 646 <= 700 < 1.25^30; ReLU and alpha = 1 never need one."""
    assert O.adaptive_reseed_layers([0.1] * 20) == [4, 8, 12, 16]
    assert O.adaptive_reseed_layers([0.5] * 64) == [29, 58]
    assert O.adaptive_reseed_layers([0.0] * 30) == []
    assert O.adaptive_reseed_layers([1.0] * 30) == []
    # segment boundaries are seeds by themselves and reset the count
    assert O.adaptive_reseed_layers([0.1] * 20, segment=6) == [4, 10, 16]
    # mixed slopes: the product decides, not the layer count
    got = O.adaptive_reseed_layers([0.1, 0.0, 0.1, 1.0, 0.1, 0.1, 0.1, 0.1])
    assert got == [6]            # growth 5.05 at layers 1,3,5,6 = 650; layer 7 would pass 700


def test_adaptive_reseed_keeps_fp32_moonwalk_accurate_where_none_does_not():
    """The rule is there for a reason: 24 layers of alpha = 0.1 in fp32 arithmetic."""
    wl = make_mlp([48] * 25, batch=16, alpha=0.1, seed=9)
    ref = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    plain = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t, dtype=np.float32, forced_masks=ref["masks"])
    seeds = O.adaptive_reseed_layers(wl.alphas)
    seeded = O.moonwalk(wl.W, wl.b, wl.alphas, wl.x, wl.t, dtype=np.float32, forced_masks=ref["masks"],
                        reseed_layers=seeds)
    assert seeds == [4, 8, 12, 16, 20]
    assert O.max_layer_err(seeded["dW"], ref["dW"]) < 1e-3
    assert O.max_layer_err(plain["dW"], ref["dW"]) > 1e-1


# ----------------------------------------------------------------------------- the error measure
def test_normwise_relative_error_on_hand_computed_vectors():
    """||a - ref|| / ||ref||, worked by hand. a = (3, 4), ref = (0, 5): a - ref = (3, -1), so
    sqrt(10) / 5. Swapping the arguments divides by ||a|| = 5 too, so a second pair with different
    norms tells the two apart: a = (1, 0), ref = (0, 2): sqrt(5) / 2 one way, sqrt(5) / 1 the other.
    Dividing by the squared norm, or taking the max norm instead of the Frobenius norm, fails too."""
    assert O.normwise_rel_err([3.0, 4.0], [0.0, 5.0]) == pytest.approx(np.sqrt(10.0) / 5.0, rel=1e-15)
    assert O.normwise_rel_err([1.0, 0.0], [0.0, 2.0]) == pytest.approx(np.sqrt(5.0) / 2.0, rel=1e-15)
    assert O.normwise_rel_err([0.0, 2.0], [1.0, 0.0]) == pytest.approx(np.sqrt(5.0), rel=1e-15)
    # Frobenius over all entries of a matrix, not per row and not the spectral norm
    a = np.array([[1.0, 2.0], [3.0, 4.0]])
    ref = np.array([[1.0, 0.0], [0.0, 4.0]])
    assert O.normwise_rel_err(a, ref) == pytest.approx(np.sqrt(4.0 + 9.0) / np.sqrt(17.0), rel=1e-15)
    # scale invariance and exactness
    assert O.normwise_rel_err(1e30 * a, 1e30 * ref) == pytest.approx(np.sqrt(13.0 / 17.0), rel=1e-12)
    assert O.normwise_rel_err(ref, ref) == 0.0
    # 0 / 0 is 0 (an all-zero gradient reproduced exactly); x / 0 is infinite
    assert O.normwise_rel_err(np.zeros(3), np.zeros(3)) == 0.0
    assert O.normwise_rel_err([0.0, 1e-3], np.zeros(2)) == np.inf
    # float32 inputs are promoted before the difference is taken: 1 + 2^-24 is not lost
    got = O.normwise_rel_err(np.array([1.0], dtype=np.float32), np.array([1.0 + 2.0 ** -30]))
    assert got == pytest.approx(2.0 ** -30, rel=1e-6)


def test_max_layer_error_picks_the_worst_tensor():
    got = [np.array([1.0, 0.0]), np.array([[3.0, 4.0]]), np.array([2.0])]
    ref = [np.array([1.0, 0.0]), np.array([[0.0, 5.0]]), np.array([1.0])]
    # per layer: 0, sqrt(10)/5 = 0.632.., |2 - 1| / 1 = 1
    assert O.max_layer_err(got, ref) == pytest.approx(1.0, rel=1e-15)
    assert O.max_layer_err(got[:2], ref[:2]) == pytest.approx(np.sqrt(10.0) / 5.0, rel=1e-15)
    # a global norm over all layers would give sqrt(10 + 1) / sqrt(1 + 25 + 1) = 0.638: not this
    assert abs(O.max_layer_err(got, ref) - np.sqrt(11.0 / 27.0)) > 0.3
