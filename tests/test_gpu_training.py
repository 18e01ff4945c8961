"""GPU parity of the in-place training step and the incremental refresh of the right inverses
against the fp64 oracle (Algorithm 1 with "Apply g_i"; Schulz iteration for the refresh)."""
import numpy as np
import pytest
import torch

from oracle import moonwalk_oracle as O
from workloads import make_mlp
from tests.parity import GRAD_TOL, gpu_masks

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mw():
    import paper_2402_14212_amd as m
    m.load_library()
    return m


def _np64(t):
    return t.detach().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("widths", [[64, 64], [200, 136], [96, 40], [640, 512], [1024, 1024]])
@pytest.mark.parametrize("rel", [1e-3, 1e-2])
@pytest.mark.parametrize("correction", ["exact", "bf16"])
def test_refresh_incremental_matches_the_oracle(mw, widths, rel, correction):
    """correction="bf16": the library rounds the operands of the correction product R P to bfloat16; the oracle's
    iteration with the same roundings is the reference, and after one iteration of a 1e-2 update (where the
    two oracles are 2e-5 apart) the library is on the rounded one's side."""
    wl = make_mlp(widths, 4, 0.1, seed=2)
    net = mw.MoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK, refresh_bf16=correction == "bf16")
    P_old = net.fetch_P(0).astype(np.float64)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    W = net.Ws[0]
    D = torch.randn(W.shape, device="cuda", generator=gen)
    W_old = W.clone()
    for iters in (0, 1, 2, 3):
        print("refresh", widths, rel, iters, flush=True)
        W.copy_(W_old + rel * float(W_old.norm() / D.norm()) * D)      # relative change `rel` in Frobenius norm
        W_new = _np64(W)
        res = net.refresh_incremental(iters)
        P = net.fetch_P(0).astype(np.float64)
        P_ref, res_ref = O.newton_schulz_refresh(W_new, P_old, iters, correction=correction)
        err = O.normwise_rel_err(P, P_ref)
        assert err < 1e-5, (iters, err)
        if correction == "bf16" and iters == 1 and rel == 1e-2:
            gap = O.normwise_rel_err(P_ref, O.newton_schulz_refresh(W_new, P_old, iters)[0])
            assert gap > 2e-5 and err < 0.25 * gap, (err, gap)
        if iters >= 1:
            want = res_ref[iters - 1]                                    # measured before the last iteration
            assert abs(float(res.item()) - want) <= 0.02 * want + 2e-5 * np.sqrt(widths[1]), (float(res.item()), want)
        else:
            assert float(res.item()) == -1.0
        if iters >= 2:
            # rounding P leaves the row space of a non-square W: a right inverse still, 2^-8 ||R_0|| off the minimum-norm one
            off_row_space = 2e-5 if correction == "bf16" and widths[0] != widths[1] else 0.0
            assert O.normwise_rel_err(P, O.right_inverse(W_new)) < 2e-5 + off_row_space
            assert np.abs(P @ W_new.T - np.eye(widths[1])).max() < 1e-5
        # put the exact inverse of the OLD weights back for the next round
        W.copy_(W_old)
        net.refresh()
    net.close()


@pytest.mark.parametrize("widths", [[136] * 4, [64] * 12, [96, 96, 96, 40, 40, 40], [70, 50, 50, 50]])
@pytest.mark.parametrize("correction", ["exact", "bf16"])
def test_refresh_incremental_of_layers_of_one_shape_side_by_side(mw, widths, correction):
    """Consecutive layers of one shape are refreshed by grouped products, eight layers at a time: every
    layer's right inverse against the oracle's iteration, for even and odd iteration counts. Layers whose
    widths are not multiples of four are refreshed one at a time, in fp32 whatever was asked for."""
    wl = make_mlp(widths, 4, 0.1, seed=3)
    net = mw.MoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK, refresh_bf16=correction == "bf16")
    plain = lambda i: net.Ws[i].shape[0] % 4 != 0 or net.Ws[i].shape[1] % 4 != 0
    L = len(widths) - 1
    P_old = [net.fetch_P(i).astype(np.float64) for i in range(L)]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(9)
    W_old = [W.clone() for W in net.Ws]
    for iters in (0, 1, 2, 3):
        print("grouped refresh", widths, iters, flush=True)
        for W, W0 in zip(net.Ws, W_old):
            D = torch.randn(W.shape, device="cuda", generator=gen)
            W.copy_(W0 + 3e-3 * float(W0.norm() / D.norm()) * D)
        res = net.refresh_incremental(iters)
        worst = 0.0
        for i in range(L):
            P_ref, res_ref = O.newton_schulz_refresh(_np64(net.Ws[i]), P_old[i], iters,
                                                     correction="exact" if plain(i) else correction)
            assert O.normwise_rel_err(net.fetch_P(i).astype(np.float64), P_ref) < 1e-5, (i, iters)
            if iters >= 1:
                worst = max(worst, res_ref[iters - 1])
        if iters >= 1:   # the reported residual is the largest over the layers, measured before the last iteration
            assert abs(float(res.item()) - worst) <= 0.02 * worst + 2e-5 * np.sqrt(max(widths)), (float(res.item()), worst)
        for W, W0 in zip(net.Ws, W_old):
            W.copy_(W0)
        net.refresh()
    net.close()


TRAIN_CASES = {
    # name: (widths, batch, alpha, K, use_bias)
    "tiny":            ([64] * 5, 32, 0.1, 0, True),
    "ragged_relu":     ([70, 50, 33, 33, 7], 5, 0.0, 0, True),
    "multi_tile_relu": ([200, 168, 136, 136], 77, 0.0, 0, True),
    "mixed":           ([96, 96, 80, 80, 64, 32], 48, [0.1, 0.0, 0.5, 0.0, 1.0], 0, True),
    "reseed4":         ([128] * 13, 64, 0.1, 4, True),
    "no_bias":         ([128, 96, 96, 64], 40, 0.1, 0, False),
    "wide":            ([1024, 1024, 1024], 256, 0.1, 0, True),
}


# (relative size of one update in weight norm, Schulz iterations per refresh): the residual of the
# carried-over inverse is a small multiple of the relative change and is raised to the power 2^iters;
# Phase III then amplifies what is left of it like any other error in P (about 5x per layer for
# alpha = 0.1 between re-seeds), so a 1 % step needs three iterations where a 0.2 % step needs two.
@pytest.mark.parametrize("rel_step,iters", [(2e-3, 2), (1e-2, 3)])
@pytest.mark.parametrize("name", sorted(TRAIN_CASES))
@pytest.mark.parametrize("correction", ["exact", "bf16"])
def test_sgd_steps_match_the_oracle(mw, name, rel_step, iters, correction):
    widths, batch, alpha, K, use_bias = TRAIN_CASES[name]
    bf16 = correction == "bf16"
    wl = make_mlp(widths, batch, alpha, seed=0, reseed_interval=K, name=name)
    if not use_bias:
        wl.b = [np.zeros_like(b) for b in wl.b]
    net = mw.MoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK, refresh_bf16=bf16)
    if not use_bias:
        net.close()
        dev = torch.device("cuda:0")
        Ws = [torch.from_numpy(w).to(dev) for w in wl.W]
        net = mw.MoonwalkNet(Ws, [None] * len(Ws), wl.alphas, wl.batch, reseed_interval=K, plan=mw.PLAN_MOONWALK,
                             refresh_bf16=bf16)
        net.x = torch.from_numpy(wl.x).to(dev)
        net.t = torch.from_numpy(wl.t).to(dev)
    # a step size that changes the weights by about rel_step of their norm
    g0 = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t)
    lr = rel_step * min(np.linalg.norm(w) / np.linalg.norm(d) for w, d in zip(wl.W, g0["dW"]))
    losses = []
    for step in range(3):
        print("sgd", name, rel_step, iters, "step", step, flush=True)
        W_before = [_np64(w) for w in net.Ws]
        b_before = [_np64(b) if b is not None else np.zeros(w.shape[0]) for b, w in zip(net.bs, net.Ws)]
        P_before = [net.fetch_P(i).astype(np.float64) for i in range(len(net.Ws))]
        loss, resid = net.sgd_step(net.x, net.t, lr, refresh_iters=iters)
        torch.cuda.synchronize()
        st = net.memory_stats()
        assert st["sign_mismatches"] == 0
        masks = gpu_masks(net, wl)
        W_ref, b_ref, loss_ref, _ = O.sgd_step(W_before, b_before, wl.alphas, wl.x, wl.t, lr, forced_masks=masks)
        assert abs(float(loss.item()) - loss_ref) <= 1e-5 * abs(loss_ref)
        losses.append(loss_ref)
        worst = 0.0
        for i, w in enumerate(net.Ws):
            got = _np64(w)
            assert O.normwise_rel_err(got - W_before[i], W_ref[i] - W_before[i]) <= GRAD_TOL, (name, step, i)
            assert O.normwise_rel_err(got, W_ref[i]) <= 1e-5
            if use_bias:
                gb = _np64(net.bs[i])
                assert O.normwise_rel_err(gb - b_before[i], b_ref[i] - b_before[i]) <= GRAD_TOL, (name, step, i)
            # the refreshed right inverse: the same two Schulz iterations as the oracle's, and as close to
            # the exact inverse of the NEW weights as the squared residual says (R_{k+1} = R_k^2)
            P = net.fetch_P(i).astype(np.float64)
            # (with the correction product in bfloat16: the oracle's iteration with the same roundings; layers
            # whose widths are not multiples of four stay in fp32; the limit is within 2^-8 ||R_0|| of the
            # minimum-norm inverse, the part of the rounding of P that leaves the row space of W)
            rounded = bf16 and got.shape[0] % 4 == 0 and got.shape[1] % 4 == 0
            P_ref, res_ref = O.newton_schulz_refresh(got, P_before[i], iters, correction="bf16" if rounded else "exact")
            assert O.normwise_rel_err(P, P_ref) < 1e-5, (name, step, i)
            left = 2.0 * res_ref[iters] + 2.0 ** -8 * res_ref[0] if rounded else 2.0 * res_ref[iters - 1] ** 2
            assert O.normwise_rel_err(P, O.right_inverse(got)) < left + 2e-5, (name, step, i)
            worst = max(worst, res_ref[iters - 1])
        r = float(resid.item())
        assert abs(r - worst) <= 0.02 * worst + 1e-4, (r, worst)     # max over layers, before the last iteration
        assert r < 0.2
    assert losses[2] < losses[0]
    net.close()


def test_sgd_step_needs_the_fused_path(mw):
    wl = make_mlp([64, 64, 32], 8, 0.1, seed=0)
    net = mw.MoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK, fuse=False)
    with pytest.raises(mw.MoonwalkError) as e:
        net.sgd_step(net.x, net.t, 0.1)
    assert e.value.code == -7
    net.close()
    net = mw.MoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK)
    with pytest.raises(mw.MoonwalkError) as e:
        net.sgd_step(net.x, net.t, 0.0)
    assert e.value.code == -1
    net.close()


def test_stale_inverse_is_visible_in_the_residual(mw):
    """A large change of the weights must show up in the residual figure so that the caller can fall
    back to the full refresh."""
    wl = make_mlp([256, 256], 4, 0.1, seed=4)
    net = mw.MoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK)
    net.Ws[0].mul_(3.0)                       # P W^T = 3 I now: far outside the iteration's basin
    res = net.refresh_incremental(1)
    torch.cuda.synchronize()
    assert float(res.item()) > 1.0
    net.refresh()
    P = net.fetch_P(0).astype(np.float64)
    assert np.abs(P @ _np64(net.Ws[0]).T - np.eye(256)).max() < 1e-5
    net.close()
