"""Pins for the convolutional oracle: everything here is checked against something other than itself
(finite differences, the dense Jacobian and numpy's pseudo-inverse, scipy's correlate, closed forms)."""
import numpy as np
import pytest
from scipy.signal import correlate2d

from oracle import conv_oracle as CO
from workloads import make_convnet


def _jacobian(w, s, p, H, C):
    """Dense Jacobian d vec(z) / d vec(x) of one image, by applying conv2d to basis images."""
    n = H * H * C
    cols = []
    for e in range(n):
        x = np.zeros(n)
        x[e] = 1.0
        cols.append(CO.conv2d(x.reshape(1, H, H, C), w, s, p).ravel())
    return np.stack(cols, axis=1)            # [n_out][n_in]


def test_conv2d_is_scipy_cross_correlation():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, 7, 7, 3))
    w = rng.standard_normal((3, 3, 3, 2))
    for s, p in ((1, 1), (2, 1), (2, 0)):
        z = CO.conv2d(x, w, s, p)
        for b in range(2):
            for co in range(2):
                full = sum(correlate2d(np.pad(x[b, :, :, c], p), w[:, :, c, co], mode="valid") for c in range(3))
                assert np.allclose(z[b, :, :, co], full[::s, ::s][:z.shape[1], :z.shape[2]], atol=1e-12)


def test_input_and_weight_gradients_are_adjoint_to_conv2d():
    """<conv(x, w), g> = <x, input_grad(g)> = <w, weight_grad(x, g)>: the defining property of a vjp."""
    rng = np.random.default_rng(1)
    for (H, k, s, p) in ((8, 3, 2, 1), (9, 3, 2, 1), (7, 5, 2, 1), (6, 3, 1, 1), (8, 2, 2, 0)):
        x = rng.standard_normal((2, H, H, 3))
        w = rng.standard_normal((k, k, 3, 2))
        z = CO.conv2d(x, w, s, p)
        g = rng.standard_normal(z.shape)
        lhs = float(np.sum(z * g))
        assert abs(lhs - float(np.sum(x * CO.conv2d_input_grad(g, w, s, p, (H, H))))) < 1e-10 * max(1, abs(lhs))
        assert abs(lhs - float(np.sum(w * CO.conv2d_weight_grad(x, g, k, s, p)))) < 1e-10 * max(1, abs(lhs))


@pytest.mark.parametrize("H,k,s,p", [(6, 3, 2, 1), (7, 3, 2, 1), (8, 5, 2, 1), (10, 4, 3, 2), (7, 2, 2, 1)])
def test_vijp_is_the_pseudo_inverse_of_the_jacobian(H, k, s, p):
    """h' = h J^+ for the dense Jacobian J of the layer (brute force), including k > p + s where earlier
    positions enter the elimination; and the lemma's conditions hold for the generated kernels."""
    wl = make_convnet(1, H, 4, 1, k=k, s=s, p=p, seed=3)
    w = wl.w[0].astype(np.float64)
    assert CO.is_submersive(w, s, p, H)
    Ho = wl.sides[1]
    J = _jacobian(w, s, p, H, 4)
    assert np.linalg.matrix_rank(J) == J.shape[0]                # right-invertible: a submersion
    rng = np.random.default_rng(4)
    hp = rng.standard_normal((1, Ho, Ho, 4))
    h = CO.conv2d_input_grad(hp, w, s, p, (H, H))
    assert np.allclose(h.ravel(), hp.ravel() @ J, atol=1e-12)    # the vjp is h' J
    got = CO.conv_vijp(h, w, s, p, (Ho, Ho))
    assert np.allclose(got, hp, atol=1e-9)
    assert np.allclose(got.ravel(), h.ravel() @ np.linalg.pinv(J), atol=1e-9)
    if k <= p + s:
        assert np.allclose(CO.conv_vijp_parallel(h, w, s, p, (Ho, Ho)), hp, atol=1e-9)


def test_submersion_conditions_are_checked():
    wl = make_convnet(1, 8, 4, 1, seed=0)
    w = wl.w[0].astype(np.float64)
    assert CO.is_submersive(w, 2, 1, 8)
    bad = w.copy()
    bad[1, 1, 0, 2] = 0.3                       # c < c' at the (p, p) tap
    assert not CO.is_submersive(bad, 2, 1, 8)
    bad = w.copy()
    bad[1, 1, 2, 2] = 0.0                       # zero diagonal
    assert not CO.is_submersive(bad, 2, 1, 8)
    assert not CO.is_submersive(w, 1, 1, 8)     # stride must exceed the padding


def test_conv_backprop_against_finite_differences():
    wl = make_convnet(2, 8, 3, 2, seed=5, alpha=0.3)
    ws = [w.astype(np.float64) for w in wl.w]
    bs = [b.astype(np.float64) for b in wl.b]
    ref = CO.conv_backprop(ws, bs, wl.alphas, 2, 1, wl.x, wl.t)

    def loss(ws_, bs_):
        xs, _, _ = CO.conv_forward(ws_, bs_, wl.alphas, 2, 1, wl.x, forced_masks=ref["masks"])
        return CO.loss_and_cotangent(xs[-1], wl.t)[0]

    rng = np.random.default_rng(6)
    eps = 1e-6
    for layer in range(2):
        for _ in range(6):
            idx = tuple(rng.integers(0, n) for n in ws[layer].shape)
            wp = [w.copy() for w in ws]
            wm = [w.copy() for w in ws]
            wp[layer][idx] += eps
            wm[layer][idx] -= eps
            fd = (loss(wp, bs) - loss(wm, bs)) / (2 * eps)
            assert abs(fd - ref["dW"][layer][idx]) < 1e-6 * max(1.0, abs(fd))
        c = int(rng.integers(0, 3))
        bp = [b.copy() for b in bs]
        bm = [b.copy() for b in bs]
        bp[layer][c] += eps
        bm[layer][c] -= eps
        fd = (loss(ws, bp) - loss(ws, bm)) / (2 * eps)
        assert abs(fd - ref["db"][layer][c]) < 1e-6 * max(1.0, abs(fd))


@pytest.mark.parametrize("k,s,p,H", [(3, 2, 1, 16), (5, 2, 1, 17), (2, 2, 0, 8)])
def test_conv_moonwalk_equals_backprop(k, s, p, H):
    """Moonwalk yields the exact gradient (Moonwalk identity), also with coupled positions (k > p + s)."""
    wl = make_convnet(2, H, 4, 2, k=k, s=s, p=p, seed=7)
    ref = CO.conv_backprop(wl.w, wl.b, wl.alphas, s, p, wl.x, wl.t)
    mw = CO.conv_moonwalk(wl.w, wl.b, wl.alphas, s, p, wl.x, wl.t)
    assert abs(mw["loss"] - ref["loss"]) < 1e-12 * abs(ref["loss"])
    assert np.allclose(mw["h0"], ref["h0"], atol=1e-12)
    for a, b in zip(mw["dW"], ref["dW"]):
        assert np.linalg.norm(a - b) < 1e-9 * np.linalg.norm(b)
    for a, b in zip(mw["db"], ref["db"]):
        assert np.linalg.norm(a - b) < 1e-9 * np.linalg.norm(b)


def test_sgd_step_is_a_projected_descent_step():
    """The training step: stays submersive, leaves the constrained entries at exactly zero, moves every other
    entry by -lr times the gradient backprop gives, and lowers the loss by lr ||projected gradient||^2 to
    first order (pins the sign and the scale of the update)."""
    wl = make_convnet(2, 8, 4, 2, alpha=0.3, seed=5)
    ref = CO.conv_backprop(wl.w, wl.b, wl.alphas, wl.s, wl.p, wl.x, wl.t)
    for lr in (1e-3, 1e-4):
        out = CO.conv_sgd_step(wl.w, wl.b, wl.alphas, wl.s, wl.p, wl.x, wl.t, lr)
        assert abs(out["loss"] - ref["loss"]) < 1e-12
        gnorm2 = 0.0
        for w0, w1, dw in zip(wl.w, out["w"], ref["dW"]):
            free = np.ones(w0.shape, dtype=bool)
            free[wl.p, wl.p] = np.tril(np.ones((4, 4), dtype=bool))
            assert np.all(w1[~free] == 0.0)
            assert np.allclose(w1[free], (w0.astype(np.float64) - lr * dw)[free], rtol=0, atol=1e-15)
            gnorm2 += float(np.sum(dw[free] ** 2))
        for b0, b1, db in zip(wl.b, out["b"], ref["db"]):
            assert np.allclose(b1, b0.astype(np.float64) - lr * db, rtol=0, atol=1e-15)
            gnorm2 += float(np.sum(db ** 2))
        after = CO.conv_backprop(out["w"], out["b"], wl.alphas, wl.s, wl.p, wl.x, wl.t)["loss"]
        drop = ref["loss"] - after
        assert drop > 0
        assert abs(drop - lr * gnorm2) <= 0.05 * lr * gnorm2 + 1e-3 * lr   # first order in lr
        for i, w1 in enumerate(out["w"]):
            assert CO.is_submersive(w1, wl.s, wl.p, wl.sides[i])



def test_loss_and_cotangent_by_hand():
    """J = 0.5 * (sum over every entry of (x_L - t)^2) / batch, h_L = scale (x_L - t) / batch: two 1 x 2 x 1
    images, residuals (1, -2) and (0, 3): J = 0.5 (1 + 4 + 0 + 9) / 2 = 3.5. A mean over all entries, a
    missing half, or a division by the entries per image gives 1.75, 7 or another value."""
    x = np.array([[[[2.0], [0.0]]], [[[1.0], [4.0]]]])          # [2][1][2][1]
    t = np.array([[[[1.0], [2.0]]], [[[1.0], [1.0]]]])
    J, h = CO.loss_and_cotangent(x, t, loss_scale=8.0)
    assert J == 3.5
    np.testing.assert_array_equal(h, 8.0 * np.array([[[[1.0], [-2.0]]], [[[0.0], [3.0]]]]) / 2.0)
    # the cotangent is the gradient of J: central difference on one entry
    eps = 1e-6
    xp, xm = x.copy(), x.copy()
    xp[1, 0, 1, 0] += eps
    xm[1, 0, 1, 0] -= eps
    fd = (CO.loss_and_cotangent(xp, t)[0] - CO.loss_and_cotangent(xm, t)[0]) / (2 * eps)
    assert fd == pytest.approx(CO.loss_and_cotangent(x, t)[1][1, 0, 1, 0], rel=1e-8)
