"""Parity at the benchmark's own sizes, in the launch configuration bench.py times."""
import numpy as np
import pytest
import torch

from workloads import make_config

from parity import check_moonwalk, check_gradients, gpu_masks

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mw():
    import paper_2402_14212_amd as m
    m.load_library()
    return m


def test_deep_square_full_size(mw):
    """Depth 64, width 1024, batch 256, leaky 0.1, re-seed every 4 layers: every gradient tensor."""
    wl = make_config("deep_square")
    net = mw.MoonwalkNet.from_workload(wl)
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
