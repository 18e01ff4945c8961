"""Parity at the benchmark's own sizes, in the launch configuration bench.py times."""
import numpy as np
import pytest
import torch

from workloads import make_config, workload_to_host

from parity import check_moonwalk, check_moonwalk_layerwise, check_gradients, gpu_masks

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mw():
    import paper_2402_14212_amd as m
    m.load_library()
    return m


def test_deep_square_full_size(mw):
    """Depth 64, width 1024, batch 256, leaky 0.1, re-seed every 4 layers: every gradient tensor, with Phase III
    as bench.py runs it (the library's choice of stretches side by side, on its second stream)."""
    wl = make_config("deep_square")
    net = mw.MoonwalkNet.from_workload(wl, phase3_parallel_segments=0, phase3_overlap=True)
    assert net.memory_stats()["phase3_group_width"] == 4
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    info = check_moonwalk(net, wl, res)
    print("deep_square", info, flush=True)
    bp = net.backprop_grad(net.x, net.t)
    torch.cuda.synchronize()
    check_gradients(wl, gpu_masks(net, wl), bp, tol=5e-5)
    net.close()


@pytest.mark.parametrize("name,depth", [("relu_frag", 6), ("narrowing", 5), ("very_deep", 2)])
def test_large_layer_shapes_at_reduced_depth(mw, name, depth):
    """The layer shapes of the other configurations (2048^2 x 512 ReLU, 4096->3648 x 512,
    4096^2 x 1024) at a depth the fp64 oracle finishes in seconds."""
    wl = make_config(name, depth=depth)
    net = mw.MoonwalkNet.from_workload(wl)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    info = check_moonwalk(net, wl, res)
    print(name, info, flush=True)
    net.close()


@pytest.mark.parametrize("name,depth", [("relu_frag", 48), ("narrowing", 32), ("very_deep", 16)])
def test_large_configurations_at_the_stated_depth(mw, name, depth):
    """relu_frag (48 ReLU layers of 2048, batch 512: a fragment store with 48 layer bases) and narrowing
    (32 layers, 4096 -> 512, batch 512, every tile choice of the taper) whole; very_deep's layers (4096 x 4096,
    batch 1024, loss scale 2^64, a re-seed every 4 layers) at depth 16, three re-seeds taken. The weights are
    drawn on the device (the host QR of these sizes takes minutes) and the same fp32 arrays go to the oracle.
    Everything check_moonwalk checks: masks, every dW and db, h_0, fragment index, bases and values."""
    print(f"full depth: {name} L={depth}", flush=True)
    dev = make_config(name, depth=depth, device="cuda:0")
    net = mw.MoonwalkNet.from_workload(dev, plan=1)
    wl = workload_to_host(dev)
    del dev
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    info = check_moonwalk(net, wl, res)
    print(name, depth, info, flush=True)
    stats = net.memory_stats()
    kept = [j for j in range(1, depth) if wl.reseed_interval and j % wl.reseed_interval == 0]
    assert stats["bytes_checkpoints"] == 4 * wl.batch * sum(wl.widths[j] for j in kept)
    if name == "very_deep":
        assert len(kept) == 3
        # the scaled cotangent really is far outside what fp32 would hold unscaled at full depth
        assert float(np.abs(net.fetch_h0()).max()) > 2.0 ** 40
    net.close()


def test_very_deep_whole(mw, capsys):
    """very_deep at its stated depth: 256 layers of 4096 x 4096, batch 1024, loss scale 2^64, a re-seed every 4
    layers. Every dW and db, the loss and h_0 against the fp64 oracle with the GPU's masks forced, one layer in host
    memory at a time (about 26 TFLOP of fp64 on the host: a minute or two, with progress lines)."""
    def say(msg):
        with capsys.disabled():
            print(msg, flush=True)

    say("very_deep L=256: drawing the weights on the device")
    dev = make_config("very_deep", device="cuda:0")
    net = mw.MoonwalkNet.from_workload(dev, plan=1)
    say("very_deep L=256: gradient step")
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    info = check_moonwalk_layerwise(net, dev, res, say)
    say(f"very_deep L=256: {info}")
    stats = net.memory_stats()
    assert stats["bytes_checkpoints"] == 4 * dev.batch * 4096 * 63
    # what the scale is for: at this depth the unscaled input cotangent lies below fp32's normal range
    top = float(np.abs(net.fetch_h0()).max())
    assert 0.0 < top / dev.loss_scale < 2.0 ** -126 < top
    net.close()
