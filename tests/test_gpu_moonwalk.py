"""End-to-end GPU parity of moonwalk_grad / backprop_grad against the fp64 oracle, through the
C ABI, on seeded synthetic networks (recipe in workloads/mlp.py)."""
import numpy as np
import pytest
import torch

from oracle import moonwalk_oracle as O
from workloads import make_mlp, make_config

from parity import check_moonwalk, check_gradients, gpu_masks, grads_to_numpy

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mw():
    import paper_2402_14212_amd as m
    m.load_library()
    return m


CASES = {
    # name: (widths, batch, alpha, K, loss_scale)
    "tiny":            ([64] * 5, 32, 0.1, 0, 1.0),
    "ragged":          ([70, 50, 33, 33, 7], 5, 0.1, 0, 1.0),
    "ragged_relu":     ([70, 50, 33, 33, 7], 5, 0.0, 0, 1.0),
    "multi_tile":      ([200, 168, 136, 136], 77, 0.1, 0, 1.0),
    "multi_tile_relu": ([200, 168, 136, 136], 77, 0.0, 0, 1.0),
    "mixed":           ([96, 96, 80, 80, 64, 32], 48, [0.1, 0.0, 0.5, 0.0, 1.0], 0, 1.0),
    "reseed2":         ([128] * 13, 64, 0.1, 2, 1.0),
    "reseed4_scaled":  ([128] * 13, 64, 0.1, 4, 2.0 ** 20),
    "narrowing_small": ([512, 448, 384, 320, 320, 256, 192, 128], 96, 0.1, 4, 1.0),
    "relu_deep":       ([192] * 25, 64, 0.0, 0, 1.0),
    "one_layer":       ([40, 24], 3, 0.1, 0, 1.0),
    "batch_one":       ([64, 64, 32], 1, 0.1, 0, 1.0),
}


def build(mw, name, **kw):
    widths, batch, alpha, K, scale = CASES[name]
    wl = make_mlp(widths, batch, alpha, seed=0, reseed_interval=K, loss_scale=scale, name=name)
    return wl, mw.MoonwalkNet.from_workload(wl, **kw)


@pytest.mark.parametrize("fuse", [False, True])
@pytest.mark.parametrize("name", list(CASES))
def test_moonwalk_matches_oracle(mw, name, fuse):
    print(f"case {name} fuse={fuse}", flush=True)
    wl, net = build(mw, name, fuse=fuse)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    info = check_moonwalk(net, wl, res)
    print(f"   {info}", flush=True)
    net.close()


def _random_mlp_cases(n_cases, seed):
    """Seeded draws of valid networks: non-increasing widths of any granularity, any batch, leaky and ReLU
    layers mixed, with and without re-seeds (depth kept to what the error growth between re-seeds allows)."""
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n_cases):
        K = int(rng.integers(0, 4))
        depth = int(rng.integers(1, 5 if K == 0 else 9))
        gran = int(rng.choice([1, 4, 32, 64]))
        widths = sorted((gran * int(rng.integers(1, max(2, 260 // gran))) for _ in range(depth + 1)), reverse=True)
        alphas = [float(rng.choice([0.0, 0.1, 0.3, 1.0])) for _ in range(depth)]
        cases.append((widths, int(rng.integers(1, 131)), alphas, K, bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("case", _random_mlp_cases(16, 99), ids=lambda c: "w%s_B%d_K%d_f%d" % ("-".join(map(str, c[0])), c[1], c[3], c[4]))
def test_moonwalk_on_random_valid_networks(mw, case):
    widths, batch, alphas, K, fuse = case
    print("mlp random", case, flush=True)
    wl = make_mlp(widths, batch, alphas, seed=5, reseed_interval=K, name="random")
    net = mw.MoonwalkNet.from_workload(wl, fuse=fuse)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    print(f"   {check_moonwalk(net, wl, res)}", flush=True)
    bp = net.backprop_grad(net.x, net.t)
    torch.cuda.synchronize()
    check_gradients(wl, gpu_masks(net, wl), bp, tol=1e-4)
    net.close()


@pytest.mark.parametrize("name", ["tiny", "ragged", "multi_tile_relu", "mixed", "reseed4_scaled"])
def test_fused_and_unfused_agree_bit_for_bit(mw, name):
    wl, fused = build(mw, name, fuse=True)
    _, plain = build(mw, name, fuse=False)
    a = fused.moonwalk_grad(fused.x, fused.t)
    b = plain.moonwalk_grad(plain.x, plain.t)
    torch.cuda.synchronize()
    for i in range(wl.depth):
        np.testing.assert_array_equal(fused.fetch_mask(i), plain.fetch_mask(i))
        assert torch.equal(a.dW[i], b.dW[i]), f"dW of layer {i}"
        # db: the fused path sums in the weight-gradient kernel's operand order, the plain
        # path in the column-sum kernel's; same value up to fp32 summation order
        assert O.normwise_rel_err(a.db[i].cpu().numpy(), b.db[i].cpu().numpy()) < 1e-5
    np.testing.assert_array_equal(fused.fetch_h0(), plain.fetch_h0())
    assert float(a.loss.item()) == float(b.loss.item())
    fused.close(), plain.close()


@pytest.mark.parametrize("name", ["tiny", "ragged", "multi_tile", "mixed", "relu_deep", "reseed4_scaled"])
def test_backprop_path_matches_oracle(mw, name):
    wl, net = build(mw, name)
    mwres = net.moonwalk_grad(net.x, net.t)
    masks = gpu_masks(net, wl)
    res = net.backprop_grad(net.x, net.t)
    torch.cuda.synchronize()
    _, eW, eb = check_gradients(wl, masks, res, tol=2e-5)      # no inverse sweep: plain fp32 rounding only
    # and the two GPU paths agree with each other within the stated bar
    for a, b in zip(grads_to_numpy(mwres)[0], grads_to_numpy(res)[0]):
        assert O.normwise_rel_err(a, b) < 1e-3
    net.close()


def test_results_are_bit_identical_run_to_run(mw):
    wl, net = build(mw, "mixed")
    a = net.moonwalk_grad(net.x, net.t)
    first = a.flat.clone()
    b = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    assert torch.equal(first, b.flat)
    c = net.backprop_grad(net.x, net.t).flat.clone()
    d = net.backprop_grad(net.x, net.t).flat
    assert torch.equal(c, d)
    net.close()


def test_right_inverse_on_device(mw):
    for widths in ([64, 64], [200, 136], [96, 40], [640, 512], [1024, 1024]):
        wl = make_mlp(widths, 4, 0.1, seed=1, keep_factors=True)
        net = mw.MoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK)
        P = net.fetch_P(0).astype(np.float64)
        W = wl.W[0].astype(np.float64)
        assert np.abs(P @ W.T - np.eye(widths[1])).max() < 1e-5           # P W^T = I
        assert O.normwise_rel_err(P, O.right_inverse(W)) < 1e-5           # the oracle's Cholesky solve
        f = wl.factors[0]
        assert O.normwise_rel_err(P, (f["U"] / f["s"]) @ f["V"].T) < 1e-5  # closed form from the factors
        net.close()


def test_rank_deficient_layer_is_rejected(mw):
    W = torch.ones(8, 16, device="cuda")             # rank 1: W W^T is singular
    with pytest.raises(mw.MoonwalkError) as e:
        mw.MoonwalkNet([W], [None], [0.1], batch=4)
    assert e.value.code == -2


def test_fragment_overflow_is_reported(mw):
    widths, batch, alpha, K, scale = CASES["multi_tile_relu"]
    wl = make_mlp(widths, batch, alpha, seed=0)
    net = mw.MoonwalkNet.from_workload(wl, frag_capacity_factor=0.1)
    net.moonwalk_grad(net.x, net.t)
    st = net.memory_stats(check=False)
    assert st["status"] == -4 and st["frag_overflow"] == 1
    net.close()


def test_nonfinite_loss_is_reported(mw):
    """An input (or target) out of range makes the loss NaN or infinite: both gradient paths raise the flag for that
    step, memory_stats reports it, and the next good step lowers it again."""
    wl = make_mlp([64, 64, 32], 8, 0.1, seed=0)
    net = mw.MoonwalkNet.from_workload(wl)
    for bad in (float("nan"), float("inf"), 3e38):          # 3e38: finite input, squared error beyond fp32
        for step in (net.moonwalk_grad, net.backprop_grad):
            x = net.x.clone()
            t = net.t.clone()
            if bad == 3e38:
                t[3, 5] = bad
            else:
                x[3, 5] = bad
            res = step(x, t)
            st = net.memory_stats(check=False)
            assert st["nonfinite_loss"] == 1 and st["status"] == mw.binding.ERR_NONFINITE, (bad, st["status"])
            assert not np.isfinite(float(res.loss.item())) or bad == 3e38
            with pytest.raises(mw.MoonwalkError):
                net.memory_stats()
            step(net.x, net.t)
            st = net.memory_stats()
            assert st["nonfinite_loss"] == 0 and st["status"] == 0
    net.close()


def test_refresh_after_weight_update(mw):
    wl, net = build(mw, "tiny")
    with torch.no_grad():
        for w in net.Ws:
            w.mul_(1.25)
    net.refresh()
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    wl.W = [w.cpu().numpy() for w in net.Ws]
    check_moonwalk(net, wl, res)
    net.close()


def test_memory_accounting_closed_forms(mw):
    wl, net = build(mw, "reseed4_scaled")
    st = net.memory_stats()
    B, widths, L = wl.batch, wl.widths, wl.depth
    assert st["bytes_P"] == sum(4 * a * b for a, b in zip(widths[:-1], widths[1:]))
    assert st["bytes_masks"] == sum(8 * ((B * d + 63) // 64) for d in widths[1:])
    assert st["bytes_masks"] * 32 == 4 * B * sum(widths[1:])               # sign bits are 32x smaller than fp32
    kept = [j for j in range(1, L) if j % 4 == 0]
    assert st["bytes_checkpoints"] == sum(4 * B * widths[j] for j in kept)
    assert st["bytes_bp_activations"] == 4 * B * sum(widths[1:])
    assert st["bytes_fragments"] == 0
    # phase III keeps a constant number of layer-sized buffers: the scratch does not grow with depth
    wl2 = make_mlp([128] * 25, 64, 0.1, seed=0, reseed_interval=4)
    net2 = mw.MoonwalkNet.from_workload(wl2)
    assert net2.memory_stats()["bytes_mw_scratch"] == st["bytes_mw_scratch"]
    net.close(), net2.close()
