"""The library's own intermediate tensors (cfg.debug_keep), fetched through the C ABI: the integer and
copy steps inside the running network are checked bit for bit against the oracle's definitions applied to
the GPU's OWN pre-activations and cotangents, and the per-layer cotangents against the fp64 oracle."""
import numpy as np
import pytest
import torch

from oracle import moonwalk_oracle as O
from workloads import make_mlp, make_config

from parity import check_moonwalk, check_kept_tensors, gpu_masks

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mw():
    import paper_2402_14212_amd as m
    m.load_library()
    return m


CASES = {
    # name: (widths, batch, alpha, K, loss_scale)
    "multi_tile_relu": ([200, 168, 136, 136], 77, 0.0, 0, 1.0),
    "ragged_relu":     ([70, 50, 33, 33, 7], 5, 0.0, 0, 1.0),
    "mixed":           ([96, 96, 80, 80, 64, 32], 48, [0.1, 0.0, 0.5, 0.0, 1.0], 0, 1.0),
    "reseed4_scaled":  ([128] * 13, 64, 0.1, 4, 2.0 ** 20),
    "relu_deep":       ([192] * 25, 64, 0.0, 0, 1.0),
}


@pytest.mark.parametrize("fuse", [True, False])
@pytest.mark.parametrize("name", list(CASES))
def test_kept_tensors_reproduce_masks_and_fragments_bit_for_bit(mw, name, fuse):
    widths, batch, alpha, K, scale = CASES[name]
    print(f"debug fetch case {name} fuse={fuse}", flush=True)
    wl = make_mlp(widths, batch, alpha, seed=0, reseed_interval=K, loss_scale=scale, name=name)
    net = mw.MoonwalkNet.from_workload(wl, fuse=fuse, debug_keep=True)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    check_moonwalk(net, wl, res)
    masks = gpu_masks(net, wl)
    ref = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t, forced_masks=masks)
    hf_err = check_kept_tensors(net, wl, ref, masks)
    print(f"   Phase-III cotangent errors: first {hf_err[0]:.2e}, worst {max(hf_err):.2e}", flush=True)
    # a kept checkpoint is the Phase-II cotangent itself
    for j in O.checkpointed_layers(wl.depth, K):
        np.testing.assert_array_equal(net.fetch_checkpoint(j - 1), net.fetch_h(j - 1))
    stats = net.memory_stats()
    n_ckpt = len(O.checkpointed_layers(wl.depth, K))
    want = 4 * wl.batch * (3 * sum(wl.widths[1:]) - sum(wl.widths[j] for j in O.checkpointed_layers(wl.depth, K)))
    assert stats["bytes_debug"] == want, (stats["bytes_debug"], want, n_ckpt)
    net.close()


def test_keeping_the_tensors_does_not_change_a_bit_of_the_results(mw):
    wl = make_mlp([200, 168, 136, 136], 77, [0.1, 0.0, 0.1], seed=2, reseed_interval=2, name="keep_vs_plain")
    plain = mw.MoonwalkNet.from_workload(wl)
    kept = mw.MoonwalkNet.from_workload(wl, debug_keep=True)
    a = plain.moonwalk_grad(plain.x, plain.t)
    b = kept.moonwalk_grad(kept.x, kept.t)
    torch.cuda.synchronize()
    assert torch.equal(a.flat, b.flat)
    assert float(a.loss.item()) == float(b.loss.item())
    for i in range(wl.depth):
        np.testing.assert_array_equal(plain.fetch_mask(i), kept.fetch_mask(i))
    np.testing.assert_array_equal(plain.fetch_h0(), kept.fetch_h0())
    assert plain.memory_stats()["bytes_debug"] == 0
    # without the flag the three tensors do not exist
    for fetch in (plain.fetch_z, plain.fetch_h, plain.fetch_h_forward):
        with pytest.raises(mw.MoonwalkError):
            fetch(0)
    plain.close(), kept.close()


def test_forward_sweep_error_grows_between_reseeds_as_predicted(mw):
    """Between two re-seeds the relative error of the Phase-III cotangent grows by about
    error_growth_per_layer(alpha) per layer and falls back at every seed (the reason the seeds exist)."""
    wl = make_mlp([256] * 13, 64, 0.1, seed=4, reseed_interval=4, name="growth")
    net = mw.MoonwalkNet.from_workload(wl, debug_keep=True)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    masks = gpu_masks(net, wl)
    ref = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t, forced_masks=masks)
    err = check_kept_tensors(net, wl, ref, masks)
    print("   per-layer Phase-III cotangent error:", ["%.1e" % e for e in err], flush=True)
    g = O.error_growth_per_layer(0.1)
    for seg in range(3):
        e = err[4 * seg: 4 * seg + 4]
        ratio = (e[3] / e[0]) ** (1.0 / 3.0)
        assert 0.5 * g < ratio < 2.0 * g, (seg, e, ratio, g)
        if seg:
            assert e[0] < 0.1 * err[4 * seg - 1]      # the seed resets the error
    net.close()


def test_full_size_relu_layers_fragments_bit_for_bit(mw):
    """The fragment store of 2048-wide ReLU layers at batch 512 (the relu_frag shape), six layers."""
    wl = make_config("relu_frag", depth=6)
    net = mw.MoonwalkNet.from_workload(wl, debug_keep=True)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    masks = gpu_masks(net, wl)
    ref = O.backprop(wl.W, wl.b, wl.alphas, wl.x, wl.t, forced_masks=masks)
    check_kept_tensors(net, wl, ref, masks)
    net.close()
