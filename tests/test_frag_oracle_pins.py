"""Pins for the fragmental 1-D convolutional oracle: everything here is checked against something other
than itself (scipy's correlate, the dense Jacobian and a least-squares solve on it, finite differences,
the sizes the paper prints for its worked example)."""
import os

import numpy as np
import pytest
from scipy.signal import correlate

from oracle import frag_oracle as FO
from workloads.conv1d import make_fragnet


def _rand_kernel(rng, k, Ci, Co, diag=(0.7, 1.3)):
    w = rng.standard_normal((k, Ci, Co)) / np.sqrt(k * Ci)
    tap = np.tril(w[0, :Co, :Co])
    tap[np.arange(Co), np.arange(Co)] = rng.uniform(*diag, size=Co)
    w[0, :Co, :Co] = tap
    return w


def _jacobian(w, N):
    """Dense Jacobian d vec(z) / d vec(x) of one sample, by applying conv1d to basis signals."""
    Ci = w.shape[1]
    cols = []
    for e in range(N * Ci):
        x = np.zeros(N * Ci)
        x[e] = 1.0
        cols.append(FO.conv1d(x.reshape(1, N, Ci), w).ravel())
    return np.stack(cols, axis=1)            # [N Co][N Ci]


@pytest.mark.parametrize("k", [1, 3, 5])
def test_conv1d_is_scipy_correlation_per_channel_pair(k):
    rng = np.random.default_rng(k)
    x = rng.standard_normal((2, 9, 3))
    w = rng.standard_normal((k, 3, 2))
    z = FO.conv1d(x, w)
    for s in range(2):
        for co in range(2):
            want = sum(correlate(x[s, :, ci], w[:, ci, co], mode="same") for ci in range(3))
            assert np.allclose(z[s, :, co], want, atol=1e-12)


def test_vjps_are_the_transposed_jacobian_and_the_weight_derivative():
    rng = np.random.default_rng(0)
    N, Ci, Co, k = 7, 3, 2, 3
    w = rng.standard_normal((k, Ci, Co))
    J = _jacobian(w, N)
    ct = rng.standard_normal((1, N, Co))
    assert np.allclose(FO.conv1d_input_grad(ct, w).ravel(), J.T @ ct.ravel(), atol=1e-12)
    # parameter vjp by central differences of <ct, conv(x, w)> (bilinear in w: exact up to rounding)
    x = rng.standard_normal((1, N, Ci))
    dw = FO.conv1d_weight_grad(x, ct, k)
    for idx in [(0, 0, 0), (1, 2, 1), (2, 1, 0)]:
        e = np.zeros_like(w)
        e[idx] = 1.0
        fd = (np.sum(ct * FO.conv1d(x, w + 0.5 * e)) - np.sum(ct * FO.conv1d(x, w - 0.5 * e)))
        assert abs(dw[idx] - fd) < 1e-10


@pytest.mark.parametrize("k,block,N,Ci,Co", [(3, 4, 12, 3, 3), (3, 6, 12, 4, 2), (5, 6, 12, 3, 3), (3, 2, 8, 2, 2), (1, 3, 6, 3, 3)])
def test_frag_vijp_solves_the_reverse_pass_equations_for_the_unstored_positions(k, block, N, Ci, Co):
    """Brute force on the dense Jacobian: with the fragment entries of ct known, the remaining entries are
    the least-squares (here exact and unique) solution of J^T ct = h."""
    rng = np.random.default_rng(10 * k + block)
    w = _rand_kernel(rng, k, Ci, Co)
    assert FO.is_fragmental(w)
    ct = rng.standard_normal((1, N, Co))
    h = FO.conv1d_input_grad(ct, w)
    frags = FO.fragments_of(ct, k, block)
    got = FO.frag_vijp(h, frags, w, block)
    assert np.allclose(got, ct, atol=1e-10)                       # round trip
    JT = _jacobian(w, N).T                                        # h = JT ct
    known = np.zeros((N, Co), dtype=bool)
    known.reshape(N // block, block, Co)[:, :k - 1, :] = True
    kn = known.ravel()
    rhs = h.ravel() - JT[:, kn] @ ct.ravel()[kn]
    sol, res, rank, _ = np.linalg.lstsq(JT[:, ~kn], rhs, rcond=None)
    assert rank == (~kn).sum()                                    # the stored subset is sufficient
    assert np.allclose(got.ravel()[~kn], sol, atol=1e-9)


def test_fragment_store_sizes_of_the_papers_worked_example():
    path = os.path.join(os.path.dirname(__file__), "golden", "fragment_store_sizes.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 2
    for steps, ch, k, block, stored in (tuple(int(v) for v in r) for r in rows):
        f = FO.fragments_of(np.zeros((1, steps, ch)), k, block)
        assert f.shape[1] * f.shape[2] == stored and f.shape[3] == ch


def test_is_fragmental_checks_triangularity_diagonal_and_channel_counts():
    rng = np.random.default_rng(3)
    w = _rand_kernel(rng, 3, 4, 4)
    assert FO.is_fragmental(w)
    bad = w.copy(); bad[0, 1, 2] = 0.1
    assert not FO.is_fragmental(bad)
    bad = w.copy(); bad[0, 2, 2] = 0.0
    assert not FO.is_fragmental(bad)
    assert not FO.is_fragmental(rng.standard_normal((3, 2, 3)))
    ok = w.copy(); ok[1:] = rng.standard_normal((2, 4, 4))      # the other taps are free
    assert FO.is_fragmental(ok)


@pytest.mark.parametrize("block", [2, 4, 8])
def test_frag_moonwalk_equals_backprop_and_finite_differences(block):
    wl = make_fragnet(2, 16, 4, 3, block=block, gain=1.0, diag=(0.8, 1.2), seed=block)
    ref = FO.conv1d_backprop(wl.w, wl.b, wl.alphas, wl.x, wl.t)
    got = FO.frag_moonwalk(wl.w, wl.b, wl.alphas, wl.x, wl.t, block)
    assert got["sign_mismatches"] == 0
    assert abs(got["loss"] - ref["loss"]) < 1e-12
    for a, b in zip(got["dW"] + got["db"], ref["dW"] + ref["db"]):
        assert np.allclose(a, b, rtol=1e-9, atol=1e-12)
    assert np.allclose(got["h0"], ref["h0"], atol=1e-12)
    # the loss scale cancels
    sc = FO.frag_moonwalk(wl.w, wl.b, wl.alphas, wl.x, wl.t, block, loss_scale=64.0)
    assert np.allclose(sc["dW"][0], ref["dW"][0], rtol=1e-9, atol=1e-12)
    # finite differences of the loss itself (away from kinks: the masks must not change)
    def loss_at(ws):
        xs, _, masks = FO.conv1d_forward(ws, wl.b, wl.alphas, wl.x)
        return FO.loss_and_cotangent(xs[-1], wl.t)[0], masks
    eps = 1e-6
    for (i, idx) in [(0, (0, 1, 0)), (1, (1, 2, 3)), (2, (2, 0, 1))]:
        wp = [np.array(w, dtype=np.float64) for w in wl.w]; wm = [np.array(w, dtype=np.float64) for w in wl.w]
        wp[i][idx] += eps; wm[i][idx] -= eps
        (lp, mp), (lm, mm) = loss_at(wp), loss_at(wm)
        if all(np.array_equal(a, b) for a, b in zip(mp, mm)):
            assert abs((lp - lm) / (2 * eps) - ref["dW"][i][idx]) < 1e-6 * max(1.0, abs(ref["dW"][i][idx]))


def test_fp32_error_of_the_block_recurrence_stays_small_for_the_workload_recipe():
    """The reconstruction feeds each rebuilt position into the next; in fp32 the error against the fp64
    result grows with the block size. For the recipe of workloads/conv1d.py it stays far inside the 1e-3
    parity tolerance even for blocks of 16."""
    for gain, block, bound in [(0.5, 16, 2e-6), (1.0, 4, 2e-6), (1.0, 16, 1e-4)]:
        wl = make_fragnet(2, 64, 32, 4, block=block, gain=gain, seed=1)
        ref = FO.conv1d_backprop(wl.w, wl.b, wl.alphas, wl.x, wl.t)
        m32 = FO.frag_moonwalk(wl.w, wl.b, wl.alphas, wl.x, wl.t, block, forced_masks=ref["masks"], dtype=np.float32)
        err = max(np.linalg.norm(np.asarray(a, dtype=np.float64) - b) / np.linalg.norm(b) for a, b in zip(m32["dW"], ref["dW"]))
        assert err < bound, (gain, block, err)


def test_frag_sgd_step_is_a_projected_descent_step():
    wl = make_fragnet(2, 16, 4, 2, block=4, gain=1.0, diag=(0.8, 1.2), seed=7)
    ref = FO.conv1d_backprop(wl.w, wl.b, wl.alphas, wl.x, wl.t)
    lr = 1e-3
    out = FO.frag_sgd_step(wl.w, wl.b, wl.alphas, wl.x, wl.t, lr, 4)
    gnorm2 = 0.0
    for w0, w1, dw in zip(wl.w, out["w"], ref["dW"]):
        free = np.ones(w0.shape, dtype=bool)
        free[0] = np.tril(np.ones((4, 4), dtype=bool))
        assert np.all(w1[~free] == 0.0) and FO.is_fragmental(w1)
        assert np.allclose(w1[free], (w0.astype(np.float64) - lr * dw)[free], rtol=0, atol=1e-15)
        gnorm2 += float(np.sum(dw[free] ** 2))
    for b0, b1, db in zip(wl.b, out["b"], ref["db"]):
        assert np.allclose(b1, b0.astype(np.float64) - lr * db, rtol=0, atol=1e-15)
        gnorm2 += float(np.sum(db ** 2))
    after = FO.conv1d_backprop(out["w"], out["b"], wl.alphas, wl.x, wl.t)["loss"]
    drop = ref["loss"] - after
    assert drop > 0 and abs(drop - lr * gnorm2) <= 0.05 * lr * gnorm2 + 1e-3 * lr



def test_loss_and_cotangent_by_hand():
    """J = 0.5 * (sum over every entry of (x_L - t)^2) / samples, h_L = scale (x_L - t) / samples: two
    samples of length 2 with one channel, residuals (1, -2) and (0, 3): J = 0.5 * 14 / 2 = 3.5 (a mean over all
    entries would give 1.75, a missing half 7)."""
    x = np.array([[[2.0], [0.0]], [[1.0], [4.0]]])          # [2][2][1]
    t = np.array([[[1.0], [2.0]], [[1.0], [1.0]]])
    J, h = FO.loss_and_cotangent(x, t, loss_scale=0.5)
    assert J == 3.5
    np.testing.assert_array_equal(h, 0.5 * np.array([[[1.0], [-2.0]], [[0.0], [3.0]]]) / 2.0)
    eps = 1e-6
    xp, xm = x.copy(), x.copy()
    xp[0, 1, 0] += eps
    xm[0, 1, 0] -= eps
    fd = (FO.loss_and_cotangent(xp, t)[0] - FO.loss_and_cotangent(xm, t)[0]) / (2 * eps)
    assert fd == pytest.approx(FO.loss_and_cotangent(x, t)[1][0, 1, 0], rel=1e-8)
