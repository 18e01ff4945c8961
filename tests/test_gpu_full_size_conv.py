"""Parity of the convolutional paths at the benchmark's own layer shapes, in the launch configuration
bench.py times (same tiles, same kernels, same slicing)."""
import numpy as np
import pytest
import torch

from oracle import conv_oracle as CO
from oracle import frag_oracle as FO
from oracle import moonwalk_oracle as O
from workloads import CONV_CONFIGS, FRAG_CONFIGS, make_convnet, make_convnet_on_device, make_fragnet
from tests.parity import GRAD_TOL, MASK_GUARD

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mw():
    import paper_2402_14212_amd as m
    m.load_library()
    return m


def _unpack(net, i, shape):
    n = int(np.prod(shape))
    return O.unpack_mask(net.fetch_mask(i), n).reshape(shape)


@pytest.mark.parametrize("block,batch,depth", [(4, 64, 1), (16, 32, 2)])
def test_conv1d_layer_shapes_at_reduced_depth(mw, block, batch, depth):
    """2048 positions, 256 channels: the benchmark's layer at half its batch (131072 patch rows: the same
    128-row tile and the same 85 weight-gradient slices as at 128), one layer deep; and two layers with
    blocks of 16 at a quarter of the batch (same tiles). Sizes the fp64 oracle finishes
    in seconds: every gradient tensor, the loss, h_0 and the fragment store."""
    c = FRAG_CONFIGS["conv1d"]
    wl = make_fragnet(batch, c["length"], c["channels"], depth, block=block, alpha=c["alpha"], seed=0)
    net = mw.ConvMoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    st = net.memory_stats()
    assert st["sign_mismatches"] == 0
    shp = (wl.batch, wl.length, wl.channels)
    masks = [_unpack(net, i, shp) for i in range(depth)]
    _, zs, _ = FO.conv1d_forward(wl.w, wl.b, wl.alphas, wl.x, forced_masks=masks)
    for z, m in zip(zs, masks):
        sure = np.abs(z) > MASK_GUARD * np.sqrt(np.mean(z * z))
        assert not ((m != (z > 0)) & sure).any()
    del zs
    ref = FO.conv1d_backprop(wl.w, wl.b, wl.alphas, wl.x, wl.t, forced_masks=masks)
    assert abs(float(res.loss.item()) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    eW = [O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.dW, ref["dW"])]
    eb = [O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.db, ref["db"])]
    print("conv1d block", block, "dW", eW, "db", eb, flush=True)
    assert max(eW) <= GRAD_TOL and max(eb) <= GRAD_TOL
    assert O.normwise_rel_err(net.fetch_h0().reshape(shp).astype(np.float64), ref["h0"]) <= 1e-4
    for i in range(depth):
        want = FO.fragments_of(ref["ct_z"][i], wl.k, block)
        assert O.normwise_rel_err(net.fetch_fragments(i).reshape(want.shape).astype(np.float64), want) <= 1e-4
    net.close()


def test_conv2d_layer_shapes_at_reduced_batch_and_depth(mw):
    """256 x 256 x 128 input, 3x3x128x128 kernels, stride 2 (the benchmark's first two layers: the 128-row
    tile for the forward, Phase-III, reverse-class and weight-gradient kernels, 113 slices) with 8 images
    instead of 43 per launch and two layers, which the fp64 oracle finishes in seconds: every gradient
    tensor, the loss, h_0."""
    c = CONV_CONFIGS["conv2d"]
    depth, batch = 2, 8
    wl = make_convnet(batch, c["side"], c["channels"], depth, alpha=c["alpha"], seed=0)
    net = mw.ConvMoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK, reseed_interval=1)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    assert net.memory_stats()["sign_mismatches"] == 0
    masks = [_unpack(net, i, (batch, wl.sides[i + 1], wl.sides[i + 1], wl.channels)) for i in range(depth)]
    ref = CO.conv_backprop(wl.w, wl.b, wl.alphas, wl.s, wl.p, wl.x, wl.t, forced_masks=masks)
    assert abs(float(res.loss.item()) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    eW = [O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.dW, ref["dW"])]
    eb = [O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.db, ref["db"])]
    print("conv2d", "dW", eW, "db", eb, flush=True)
    assert max(eW) <= GRAD_TOL and max(eb) <= GRAD_TOL
    assert O.normwise_rel_err(net.fetch_h0().reshape(wl.x.shape).astype(np.float64), ref["h0"]) <= 1e-4
    net.close()


def test_conv2d_full_benchmark_by_sampled_signs_and_properties(mw):
    """The benchmark itself (batch 128, eight layers, three launches of 43/43/42 images per first-layer
    kernel). The oracle cannot run it whole, so: (1) sign bits of the first layer at sampled positions of
    every image chunk against z computed one output at a time from the definition; (2) Phase III's
    recomputed signs equal Phase I's; (3) Moonwalk's gradients equal the library's backprop's (an
    independent route through other kernels: stored activations, no vijp) to 1e-4; (4) the same with the
    input cotangent only as read; (5) bit-identical repeat."""
    c = CONV_CONFIGS["conv2d"]
    wl = make_convnet_on_device(c["batch"], c["side"], c["channels"], c["depth"], alpha=c["alpha"], seed=0)
    net = mw.ConvMoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK, reseed_interval=2)
    grads = net.new_grads()
    net.moonwalk_grad(net.x, net.t, grads)
    torch.cuda.synchronize()
    assert net.memory_stats()["sign_mismatches"] == 0
    # (1) sampled signs of layer 0
    side1 = wl.sides[1]
    n1 = wl.batch * side1 * side1 * wl.channels
    words = net.fetch_mask(0)
    w0 = wl.w[0].double().cpu().numpy()
    b0 = wl.b[0].double().cpu().numpy()
    rng = np.random.default_rng(0)
    picks = [(b, int(rng.integers(side1)), int(rng.integers(side1)), int(rng.integers(wl.channels)))
             for b in (0, 42, 43, 85, 86, 127) for _ in range(40)]
    picks += [(127, side1 - 1, side1 - 1, wl.channels - 1), (0, 0, 0, 0), (43, 0, side1 - 1, 5)]
    zs = []
    for (b, i, j, co) in picks:
        z = b0[co]
        for u in range(wl.k):
            for v in range(wl.k):
                y, x = wl.s * i + u - wl.p, wl.s * j + v - wl.p
                if 0 <= y < wl.side and 0 <= x < wl.side:
                    z += float(wl.x[b, y, x, :].double().cpu().numpy() @ w0[u, v, :, co])
        zs.append(z)
    scale = np.sqrt(np.mean(np.square(zs)))
    for (b, i, j, co), z in zip(picks, zs):
        e = ((b * side1 + i) * side1 + j) * wl.channels + co
        bit = (int(words[e // 64]) >> (e % 64)) & 1
        if abs(z) > MASK_GUARD * scale:
            assert bit == int(z > 0), (b, i, j, co, z)
    assert n1 == words.size * 64
    # (5) repeat
    again = net.new_grads()
    net.moonwalk_grad(net.x, net.t, again)
    torch.cuda.synchronize()
    assert torch.equal(grads, again)
    net.close()
    # (4) as read
    net = mw.ConvMoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK, reseed_interval=2, input_cotangent=mw.CONV_H0_AS_READ)
    net.moonwalk_grad(net.x, net.t, again)
    torch.cuda.synchronize()
    assert net.memory_stats()["sign_mismatches"] == 0
    assert float(((again - grads).double().norm() / grads.double().norm()).item()) <= 1e-5
    net.close()
    # (3) backprop
    net = mw.ConvMoonwalkNet.from_workload(wl, plan=mw.PLAN_BACKPROP)
    net.backprop_grad(net.x, net.t, again)
    torch.cuda.synchronize()
    rel = float(((again - grads).double().norm() / grads.double().norm()).item())
    print("conv2d full: Moonwalk vs backprop", rel, flush=True)
    assert rel <= 1e-4
    net.close()


def test_conv2d_k5_full_benchmark_by_single_images_and_properties(mw):
    """The benchmark with kernels wider than padding + stride (batch 32, six 5 x 5 layers, a sweep over up to
    125 anti-diagonals per layer). Signs and the input cotangent of one image depend on that image alone, so
    the oracle runs on single images: (1) every layer's sign bits of the first and the last image; (2) their
    rows of h_0, which is 1/B of the single-image one; then (3) Phase III's recomputed signs equal Phase I's;
    (4) Moonwalk's gradients equal the library's backprop's (no vijp, no sweep) to 1e-4; (5) bit-identical repeat."""
    c = CONV_CONFIGS["conv2d_k5"]
    wl = make_convnet_on_device(c["batch"], c["side"], c["channels"], c["depth"], k=c["k"], s=c["s"], p=c["p"],
                                alpha=c["alpha"], seed=0)
    net = mw.ConvMoonwalkNet.from_workload(wl, plan=mw.PLAN_MOONWALK, reseed_interval=2)
    grads = net.new_grads()
    net.moonwalk_grad(net.x, net.t, grads)
    torch.cuda.synchronize()
    assert net.memory_stats()["sign_mismatches"] == 0
    B, C = wl.batch, wl.channels
    masks = [_unpack(net, i, (B, wl.sides[i + 1], wl.sides[i + 1], C)) for i in range(wl.depth)]
    h0 = net.fetch_h0().reshape(B, wl.side, wl.side, C)
    ws = [w.cpu().numpy() for w in wl.w]
    bs = [b.cpu().numpy() for b in wl.b]
    for img in (0, B - 1):
        print("conv2d_k5 full: image", img, flush=True)
        x1 = wl.x[img:img + 1].cpu().numpy()
        t1 = wl.t[img:img + 1].cpu().numpy()
        own = [m[img:img + 1] for m in masks]
        _, zs, _ = CO.conv_forward(ws, bs, wl.alphas, wl.s, wl.p, x1, forced_masks=own)
        for z, m in zip(zs, own):
            sure = np.abs(z) > MASK_GUARD * np.sqrt(np.mean(z * z))
            assert not ((m != (z > 0)) & sure).any()
        ref = CO.conv_backprop(ws, bs, wl.alphas, wl.s, wl.p, x1, t1, forced_masks=own)
        assert O.normwise_rel_err(B * h0[img:img + 1].astype(np.float64), ref["h0"]) <= 1e-4
    again = net.new_grads()
    net.moonwalk_grad(net.x, net.t, again)
    torch.cuda.synchronize()
    assert torch.equal(grads, again)
    net.close()
    net = mw.ConvMoonwalkNet.from_workload(wl, plan=mw.PLAN_BACKPROP)
    net.backprop_grad(net.x, net.t, again)
    torch.cuda.synchronize()
    rel = float(((again - grads).double().norm() / grads.double().norm()).item())
    print("conv2d_k5 full: Moonwalk vs backprop", rel, flush=True)
    assert rel <= 1e-4
    net.close()
