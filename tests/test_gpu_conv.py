"""GPU parity of Moonwalk on submersive 2-D convolutional layers against the fp64 convolutional oracle."""
import numpy as np
import pytest
import torch

from oracle import conv_oracle as CO
from oracle import moonwalk_oracle as O
from workloads import make_convnet
from tests.parity import GRAD_TOL, MASK_GUARD

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mw():
    import paper_2402_14212_amd as m
    m.load_library()
    return m


def _patches_by_definition(x, k, s, p):
    """[B Ho Wo][k k C] patch matrix written out from its definition (test-side, numpy)."""
    B, H, W, C = x.shape
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    xp = np.zeros((B, H + 2 * p, W + 2 * p, C), dtype=x.dtype)
    xp[:, p:p + H, p:p + W] = x
    out = np.zeros((B, Ho, Wo, k, k, C), dtype=x.dtype)
    for u in range(k):
        for v in range(k):
            out[:, :, :, u, v, :] = xp[:, u:u + s * (Ho - 1) + 1:s, v:v + s * (Wo - 1) + 1:s, :]
    return out.reshape(B * Ho * Wo, k * k * C)


@pytest.mark.parametrize("shape,k,s,p", [((2, 9, 11, 8), 3, 2, 1), ((3, 8, 8, 6), 3, 2, 1), ((2, 7, 7, 5), 2, 2, 0),
                                         ((1, 12, 10, 4), 3, 1, 1), ((2, 10, 10, 12), 5, 2, 1)])
def test_im2col_and_col2im(mw, shape, k, s, p):
    rng = np.random.default_rng(0)
    x = rng.standard_normal(shape).astype(np.float32)
    want = _patches_by_definition(x, k, s, p)
    got = mw.conv_im2col(torch.from_numpy(x).cuda(), k, s, p).cpu().numpy()
    assert np.array_equal(got, want)                                         # pure data movement: bit-exact
    part = mw.conv_im2col(torch.from_numpy(x).cuda(), k, s, p, row0=3, n_rows=7).cpu().numpy()
    assert np.array_equal(part, want[3:10])
    # col2im is the transpose of im2col: <im2col(x), d> = <x, col2im(d)>; against the oracle's scatter too
    d = rng.standard_normal(want.shape).astype(np.float32)
    back = mw.conv_col2im(torch.from_numpy(d).cuda(), shape, k, s, p).cpu().numpy().astype(np.float64)
    B, H, W, C = shape
    Ho, Wo = (H + 2 * p - k) // s + 1, (W + 2 * p - k) // s + 1
    ref = np.zeros((B, H + 2 * p + s, W + 2 * p + s, C))
    d6 = d.astype(np.float64).reshape(B, Ho, Wo, k, k, C)
    for u in range(k):
        for v in range(k):
            ref[:, u:u + s * Ho:s, v:v + s * Wo:s, :] += d6[:, :, :, u, v, :]
    ref = ref[:, p:p + H, p:p + W, :]
    assert np.abs(back - ref).max() <= 1e-6 * max(1.0, np.abs(ref).max())


def _masks(net, wl):
    out = []
    for i in range(wl.depth):
        shp = (wl.batch, wl.sides[i + 1], wl.sides[i + 1], wl.channels)
        n = int(np.prod(shp))
        words = net.fetch_mask(i)
        assert words.size == (n + 63) // 64
        if n % 64:
            assert int(words[-1]) >> (n % 64) == 0
        out.append(O.unpack_mask(words, n).reshape(shp))
    return out


CONV_CASES = {
    # name: (batch, side, channels, depth, k, s, p, alpha, K, patch_bytes, kernels)
    "small":        (2, 16, 8, 2, 3, 2, 1, 0.3, 0, 0, 0),
    "odd_side":     (3, 21, 16, 2, 3, 2, 1, 0.3, 0, 0, 0),
    "chunks":       (5, 16, 8, 3, 3, 2, 1, 0.3, 0, 40000, 0),   # patch buffer of about one image: several fills
    "not_vec":      (2, 12, 6, 2, 3, 2, 1, 0.3, 0, 0, 0),        # channels not a multiple of 4
    "k2":           (2, 16, 8, 3, 2, 2, 0, 0.3, 0, 0, 0),
    "deep_reseed":  (2, 64, 16, 5, 3, 2, 1, 0.1, 2, 0, 0),
    # channel counts that take the kernels gathering the patch matrix inside the product
    "wide":         (2, 32, 64, 3, 3, 2, 1, 0.2, 0, 0, 0),
    "wide_patches": (2, 32, 64, 3, 3, 2, 1, 0.2, 0, 0, 1),       # the same network through the patch buffer
    "gather_odd":   (3, 21, 32, 3, 3, 2, 1, 0.3, 0, 0, 0),       # sides 21 -> 11 -> 6 -> 3: ragged tiles, padding on all edges
    "gather_k2":    (2, 16, 32, 2, 2, 2, 0, 0.3, 0, 0, 0),
    "gather_deep":  (2, 64, 32, 5, 3, 2, 1, 0.1, 2, 40000, 0),   # re-seeds; Phase II still in several patch fills
    "gather_128":   (2, 128, 128, 2, 3, 2, 1, 0.3, 0, 0, 0),     # 8192 and 2048 rows, K = 1152: the split-K tiles
    "gather_tall":  (1, 512, 32, 2, 3, 2, 1, 0.3, 0, 0, 0),      # 65536 rows: the 128-row tile, then 16384 rows
    "gather_mid":   (2, 256, 32, 1, 3, 2, 1, 0.3, 0, 0, 0),      # 32768 rows: the 64 x 128 tile
    # kernels wider than padding + stride: earlier positions enter the vijp, swept diagonal by diagonal
    "general_k5":   (2, 32, 32, 2, 5, 2, 1, 0.3, 0, 0, 0),       # reach 1: sides 32 -> 15 -> 7
    "general_k4":   (3, 29, 32, 3, 4, 2, 1, 0.3, 2, 0, 0),       # reach 1, even kernel, a re-seed kept whole
    "general_s1":   (2, 12, 32, 2, 3, 1, 0, 0.3, 0, 0, 0),       # stride 1 without padding: reach 2, eight earlier positions
    "general_wide": (2, 40, 64, 1, 5, 2, 1, 0.3, 0, 0, 0),       # non-square diagonals' worth of rows over several tiles
}


@pytest.mark.parametrize("name", sorted(CONV_CASES))
def test_conv_moonwalk_matches_the_oracle(mw, name):
    _parity_of_case(mw, name)


def test_conv_nonfinite_loss_is_reported(mw):
    """A NaN in the input: the step's loss is not finite, memory_stats says so; the next good step lowers the flag."""
    B, side, C, depth, k, s, p, alpha, K, patch_bytes, kernels = CONV_CASES[sorted(CONV_CASES)[0]]
    wl = make_convnet(B, side, C, depth, k=k, s=s, p=p, alpha=alpha, seed=1)
    net = mw.ConvMoonwalkNet.from_workload(wl, reseed_interval=K, patch_bytes=patch_bytes, kernels=kernels)
    for step in (net.moonwalk_grad, net.backprop_grad):
        x = net.x.clone()
        x.view(-1)[7] = float("nan")
        step(x, net.t)
        st = net.memory_stats(check=False)
        assert st["nonfinite_loss"] == 1 and st["status"] == mw.binding.ERR_NONFINITE
        step(net.x, net.t)
        st = net.memory_stats()
        assert st["nonfinite_loss"] == 0 and st["status"] == 0
    net.close()


def _parity_of_case(mw, name, **net_kw):
    B, side, C, depth, k, s, p, alpha, K, patch_bytes, kernels = CONV_CASES[name]
    wl = make_convnet(B, side, C, depth, k=k, s=s, p=p, alpha=alpha, seed=1, name=name)
    print("conv", name, net_kw, flush=True)
    net = mw.ConvMoonwalkNet.from_workload(wl, reseed_interval=K, patch_bytes=patch_bytes, kernels=kernels, **net_kw)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    st = net.memory_stats()
    assert st["sign_mismatches"] == 0
    masks = _masks(net, wl)
    # masks: equal to the oracle's signs outside a guard band around zero
    _, zs, _ = CO.conv_forward(wl.w, wl.b, wl.alphas, s, p, wl.x, forced_masks=masks)
    for z, m in zip(zs, masks):
        sure = np.abs(z) > MASK_GUARD * np.sqrt(np.mean(z * z))
        assert not ((m != (z > 0)) & sure).any()
    ref = CO.conv_backprop(wl.w, wl.b, wl.alphas, s, p, wl.x, wl.t, forced_masks=masks)
    assert abs(float(res.loss.item()) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    eW = [O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.dW, ref["dW"])]
    eb = [O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.db, ref["db"])]
    assert max(eW) <= GRAD_TOL, eW
    assert max(eb) <= GRAD_TOL, eb
    h0 = net.fetch_h0().reshape(wl.x.shape).astype(np.float64)
    assert O.normwise_rel_err(h0, ref["h0"]) <= 1e-4
    # the re-seed cotangents: kept as the next layer's vijp reads them (strided positions, its C_out channels)
    if K > 0:
        for j in range(K, depth, K):
            side = wl.sides[j + 1]
            want = ref["hs"][j] if k > p + s else ref["hs"][j][:, ::s, ::s, :C][:, :side, :side]
            got = net.fetch_checkpoint(j - 1).reshape(want.shape).astype(np.float64)
            assert O.normwise_rel_err(got, want) <= 1e-4, j
    # the tap inverses
    for i in range(depth):
        T = wl.w[i][p, p].astype(np.float64)
        assert O.normwise_rel_err(net.fetch_tap_inverse(i), np.linalg.inv(T)) < 1e-5
    # the library's own backprop, same oracle
    bp = net.backprop_grad(net.x, net.t)
    torch.cuda.synchronize()
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(bp.dW, ref["dW"])) <= 1e-4
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(bp.db, ref["db"])) <= 1e-4
    assert O.normwise_rel_err(net.fetch_h0().reshape(wl.x.shape).astype(np.float64), ref["h0"]) <= 1e-5   # backprop's h_0
    # determinism
    res2 = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    assert torch.equal(res.flat, res2.flat)
    # memory: one bit per output element against backprop's 32
    n_out = [B * wl.sides[i + 1] ** 2 * C for i in range(depth)]
    assert st["bytes_masks"] == 8 * sum((n + 63) // 64 for n in n_out)
    assert st["bytes_bp_activations"] == 4 * sum(n_out)
    assert st["bytes_input_cotangent"] == 4 * wl.x.size
    net.close()


NARROWING_CASES = {
    # name: (batch, side, channel counts input first, k, s, p, K, h_0 mode)
    "patch":        (2, 16, [12, 8, 6], 3, 2, 1, 0, 0),          # through the patch buffer
    "gather":       (3, 21, [96, 64, 32, 32], 3, 2, 1, 2, 0),    # gathered kernels; the re-seed keeps 32 of 64 channels
    "gather_read":  (2, 32, [64, 32, 32], 3, 2, 1, 0, 1),        # h_0 as the first vijp reads it: 32 of 64 channels
    "general":      (2, 29, [64, 32, 32], 5, 2, 1, 2, 0),        # coupled positions, re-seed kept whole
}


@pytest.mark.parametrize("name", sorted(NARROWING_CASES))
def test_conv_moonwalk_with_fewer_output_than_input_channels(mw, name):
    """C_out < C_in: the vijp's equations are those of the first C_out input channels at the strided positions."""
    B, side, cs, k, s, p, K, h0_mode = NARROWING_CASES[name]
    depth = len(cs) - 1
    wl = make_convnet(B, side, cs, depth, k=k, s=s, p=p, alpha=0.3, seed=5, name=name)
    print("conv narrowing", name, flush=True)
    net = mw.ConvMoonwalkNet.from_workload(wl, reseed_interval=K, input_cotangent=h0_mode)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    assert net.memory_stats()["sign_mismatches"] == 0
    shapes = [(B, wl.sides[i + 1], wl.sides[i + 1], cs[i + 1]) for i in range(depth)]
    masks = [O.unpack_mask(net.fetch_mask(i), int(np.prod(sh))).reshape(sh) for i, sh in enumerate(shapes)]
    _, zs, _ = CO.conv_forward(wl.w, wl.b, wl.alphas, s, p, wl.x, forced_masks=masks)
    for z, m in zip(zs, masks):
        sure = np.abs(z) > MASK_GUARD * np.sqrt(np.mean(z * z))
        assert not ((m != (z > 0)) & sure).any()
    ref = CO.conv_backprop(wl.w, wl.b, wl.alphas, s, p, wl.x, wl.t, forced_masks=masks)
    assert abs(float(res.loss.item()) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.dW, ref["dW"])) <= GRAD_TOL
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.db, ref["db"])) <= GRAD_TOL
    whole = k > p + s
    if h0_mode == 0:
        assert O.normwise_rel_err(net.fetch_h0().reshape(wl.x.shape).astype(np.float64), ref["h0"]) <= 1e-4
    else:
        want = ref["h0"][:, ::s, ::s, :cs[1]][:, :wl.sides[1], :wl.sides[1]]
        assert O.normwise_rel_err(net.fetch_h0().reshape(want.shape).astype(np.float64), want) <= 1e-4
    for j in range(K, depth, K) if K > 0 else ():
        n = wl.sides[j + 1]
        want = ref["hs"][j] if whole else ref["hs"][j][:, ::s, ::s, :cs[j + 1]][:, :n, :n]
        assert O.normwise_rel_err(net.fetch_checkpoint(j - 1).reshape(want.shape).astype(np.float64), want) <= 1e-4, j
    for i in range(depth):
        T = wl.w[i][p, p, :cs[i + 1], :].astype(np.float64)
        assert O.normwise_rel_err(net.fetch_tap_inverse(i), np.linalg.inv(T)) < 1e-5
    if h0_mode == 0:
        bp = net.backprop_grad(net.x, net.t)
        torch.cuda.synchronize()
        assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(bp.dW, ref["dW"])) <= 1e-4
    net.close()


@pytest.mark.parametrize("H,W,C,depth,k,s,p,K", [
    (20, 13, 8, 2, 3, 2, 1, 0),       # patch buffer
    (13, 37, 32, 2, 3, 2, 1, 0),      # gathered kernels, wide images
    (29, 19, 32, 2, 5, 2, 1, 0),      # coupled positions: diagonals of a 14 x 9, then a 6 x 4 grid
    (9, 14, 32, 2, 3, 1, 0, 1),       # reach 2, grids 7 x 12 and 5 x 10, every cotangent re-seeded
    (17, 3, 32, 1, 5, 2, 1, 0),       # an 8 x 1 grid: every diagonal is one position
])
def test_conv_moonwalk_on_images_that_are_not_square(mw, H, W, C, depth, k, s, p, K):
    B = 3
    kernels = make_convnet(1, 64, C, depth, k=k, s=s, p=p, alpha=0.3, seed=11)   # the recipe's kernels and biases
    rng = np.random.default_rng(12)
    x = rng.standard_normal((B, H, W, C)).astype(np.float32)
    hs, ws_ = [H], [W]
    for _ in range(depth):
        hs.append((hs[-1] + 2 * p - k) // s + 1)
        ws_.append((ws_[-1] + 2 * p - k) // s + 1)
        assert hs[-2] > s * (hs[-1] - 1) and ws_[-2] > s * (ws_[-1] - 1) and hs[-1] >= 1 and ws_[-1] >= 1
    t = rng.standard_normal((B, hs[-1], ws_[-1], C)).astype(np.float32)
    print("conv not square", H, W, k, s, p, flush=True)
    dev = torch.device("cuda:0")
    net = mw.ConvMoonwalkNet([torch.from_numpy(w).to(dev) for w in kernels.w], [torch.from_numpy(b).to(dev) for b in kernels.b],
                             kernels.alphas, B, H, W, s, p, reseed_interval=K)
    dx, dt = torch.from_numpy(x).to(dev), torch.from_numpy(t).to(dev)
    res = net.moonwalk_grad(dx, dt)
    torch.cuda.synchronize()
    assert net.memory_stats()["sign_mismatches"] == 0
    shapes = [(B, hs[i + 1], ws_[i + 1], C) for i in range(depth)]
    masks = [O.unpack_mask(net.fetch_mask(i), int(np.prod(sh))).reshape(sh) for i, sh in enumerate(shapes)]
    ref = CO.conv_backprop(kernels.w, kernels.b, kernels.alphas, s, p, x, t, forced_masks=masks)
    assert abs(float(res.loss.item()) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.dW, ref["dW"])) <= GRAD_TOL
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.db, ref["db"])) <= GRAD_TOL
    assert O.normwise_rel_err(net.fetch_h0().reshape(x.shape).astype(np.float64), ref["h0"]) <= 1e-4
    bp = net.backprop_grad(dx, dt)
    torch.cuda.synchronize()
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(bp.dW, ref["dW"])) <= 1e-4
    net.close()


@pytest.mark.parametrize("name,per_launch", [("gather_odd", 2), ("gather_deep", 1), ("general_k4", 2), ("general_s1", 1)])
def test_conv_moonwalk_in_several_launches_per_layer(mw, name, per_launch):
    """The batch taken in image chunks, as the 2 GiB operand limit forces at the benchmark's size: the same
    parity with the oracle (chunks of two and one image, or one launch per image)."""
    _parity_of_case(mw, name, max_images_per_launch=per_launch)
    wl = make_convnet(2, 16, 32, 1, seed=0)
    with pytest.raises(mw.MoonwalkError) as e:
        mw.ConvMoonwalkNet.from_workload(wl, max_images_per_launch=-1)
    assert e.value.code == -1


def _random_conv_cases(n_cases, seed):
    """Seeded draws of valid chains: channel counts, kernel, stride, padding, image sides that meet the
    lemma's spatial bounds, one or two layers, any re-seed interval."""
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n_cases:
        k, s = int(rng.integers(1, 6)), int(rng.integers(1, 4))
        p = int(rng.integers(0, min(s, k)))
        depth = int(rng.integers(1, 3))
        wide = k > p + s
        pool = [32, 64] if wide else [4, 6, 8, 12, 32, 64]
        cs = sorted((int(rng.choice(pool)) for _ in range(depth + 1)), reverse=True)
        H, W = int(rng.integers(k, 27)), int(rng.integers(k, 27))
        hs, ws_, ok = [H], [W], True
        for _ in range(depth):
            ho, wo = (hs[-1] + 2 * p - k) // s + 1, (ws_[-1] + 2 * p - k) // s + 1
            ok = ok and hs[-1] + 2 * p >= k and ws_[-1] + 2 * p >= k and ho >= 1 and wo >= 1
            ok = ok and hs[-1] > s * (ho - 1) and ws_[-1] > s * (wo - 1)
            hs.append(ho)
            ws_.append(wo)
        if ok:
            cases.append((int(rng.integers(1, 4)), H, W, cs, k, s, p, int(rng.integers(0, 2)), hs, ws_))
    return cases


@pytest.mark.parametrize("case", _random_conv_cases(24, 2024), ids=lambda c: "B%d_%dx%d_c%s_k%d_s%d_p%d_K%d" % (
    c[0], c[1], c[2], "-".join(map(str, c[3])), c[4], c[5], c[6], c[7]))
def test_conv_moonwalk_on_random_valid_chains(mw, case):
    B, H, W, cs, k, s, p, K, hs, ws_ = case
    depth = len(cs) - 1
    kernels = make_convnet(1, 64, cs, depth, k=k, s=max(s, p + 1), p=p, alpha=0.3, seed=31)   # kernels and biases only
    rng = np.random.default_rng(32)
    x = rng.standard_normal((B, H, W, cs[0])).astype(np.float32)
    t = rng.standard_normal((B, hs[-1], ws_[-1], cs[-1])).astype(np.float32)
    print("conv random", case[:8], flush=True)
    dev = torch.device("cuda:0")
    net = mw.ConvMoonwalkNet([torch.from_numpy(w).to(dev) for w in kernels.w], [torch.from_numpy(b).to(dev) for b in kernels.b],
                             kernels.alphas, B, H, W, s, p, reseed_interval=K)
    dx, dt = torch.from_numpy(x).to(dev), torch.from_numpy(t).to(dev)
    res = net.moonwalk_grad(dx, dt)
    torch.cuda.synchronize()
    assert net.memory_stats()["sign_mismatches"] == 0
    shapes = [(B, hs[i + 1], ws_[i + 1], cs[i + 1]) for i in range(depth)]
    masks = [O.unpack_mask(net.fetch_mask(i), int(np.prod(sh))).reshape(sh) for i, sh in enumerate(shapes)]
    ref = CO.conv_backprop(kernels.w, kernels.b, kernels.alphas, s, p, x, t, forced_masks=masks)
    assert abs(float(res.loss.item()) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.dW, ref["dW"])) <= GRAD_TOL
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.db, ref["db"])) <= GRAD_TOL
    assert O.normwise_rel_err(net.fetch_h0().reshape(x.shape).astype(np.float64), ref["h0"]) <= 1e-4
    bp = net.backprop_grad(dx, dt)
    torch.cuda.synchronize()
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(bp.dW, ref["dW"])) <= 1e-4
    net.close()


def test_conv_setup_rejects_what_is_not_submersive_or_not_built(mw):
    wl = make_convnet(2, 16, 8, 1, seed=0)
    dev = torch.device("cuda:0")
    w = torch.from_numpy(wl.w[0]).to(dev)
    with pytest.raises(mw.MoonwalkError) as e:            # a non-zero entry above the diagonal of the (p, p) tap
        bad = w.clone()
        bad[1, 1, 0, 3] = 0.5
        mw.ConvMoonwalkNet([bad], [None], [0.3], 2, 16, 16, 2, 1)
    assert e.value.code == -2
    with pytest.raises(mw.MoonwalkError) as e:            # zero diagonal
        bad = w.clone()
        bad[1, 1, 2, 2] = 0.0
        mw.ConvMoonwalkNet([bad], [None], [0.3], 2, 16, 16, 2, 1)
    assert e.value.code == -2
    with pytest.raises(mw.MoonwalkError) as e:            # stride must exceed the padding
        mw.ConvMoonwalkNet([w], [None], [0.3], 2, 16, 16, 1, 1)
    assert e.value.code == -2
    with pytest.raises(mw.MoonwalkError) as e:            # k > p + s: coupled positions need channels in 32s ...
        w5 = torch.zeros(5, 5, 8, 8, device=dev)
        w5[1, 1] = torch.eye(8, device=dev)
        mw.ConvMoonwalkNet([w5], [None], [0.3], 2, 17, 17, 2, 1)
    assert e.value.code == -1
    with pytest.raises(mw.MoonwalkError) as e:            # ... and the whole input cotangent
        w5 = torch.zeros(5, 5, 32, 32, device=dev)
        w5[1, 1] = torch.eye(32, device=dev)
        mw.ConvMoonwalkNet([w5], [None], [0.3], 2, 17, 17, 2, 1, input_cotangent=mw.CONV_H0_AS_READ)
    assert e.value.code == -1
    with pytest.raises(mw.MoonwalkError) as e:            # ReLU is not supported on this path
        mw.ConvMoonwalkNet([w], [None], [0.0], 2, 16, 16, 2, 1)
    assert e.value.code == -1
    for shape in ((0, 16, 16), (2, 0, 16), (2, 16, 0)):  # an empty batch or image
        with pytest.raises(mw.MoonwalkError) as e:
            mw.ConvMoonwalkNet([w], [None], [0.3], *shape, 2, 1)
        assert e.value.code == -1
    with pytest.raises(mw.MoonwalkError) as e:            # an image too small for the kernel: no output position
        mw.ConvMoonwalkNet([torch.zeros(5, 5, 8, 8, device=dev)], [None], [0.3], 2, 2, 2, 2, 1)
    assert e.value.code in (-1, -2)


def test_conv_refresh_follows_the_kernel(mw):
    wl = make_convnet(2, 16, 8, 2, seed=2)
    net = mw.ConvMoonwalkNet.from_workload(wl)
    net.ws[0][1, 1].mul_(1.5)
    net.refresh()
    T = net.ws[0][1, 1].cpu().numpy().astype(np.float64)
    assert O.normwise_rel_err(net.fetch_tap_inverse(0), np.linalg.inv(T)) < 1e-5
    net.close()


def test_conv_refresh_rebuilds_what_both_paths_derive_from_the_weights(mw):
    """After a weight change and refresh(), Moonwalk and the library's backprop follow the new weights
    (tap inverses and the regrouped taps of the input-cotangent kernel)."""
    wl = make_convnet(2, 16, 32, 2, seed=3)
    net = mw.ConvMoonwalkNet.from_workload(wl)
    net.moonwalk_grad(net.x, net.t)
    for w in net.ws:
        w.mul_(torch.tril(torch.full((32, 32), 1.25, device=w.device)) + torch.triu(torch.full((32, 32), 0.8, device=w.device), 1))
    net.refresh()
    w_new = [w.cpu().numpy() for w in net.ws]
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    assert net.memory_stats()["sign_mismatches"] == 0
    masks = _masks(net, wl)
    ref = CO.conv_backprop(w_new, wl.b, wl.alphas, wl.s, wl.p, wl.x, wl.t, forced_masks=masks)
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.dW, ref["dW"])) <= GRAD_TOL
    assert O.normwise_rel_err(net.fetch_h0().reshape(wl.x.shape).astype(np.float64), ref["h0"]) <= 1e-4
    bp = net.backprop_grad(net.x, net.t)
    torch.cuda.synchronize()
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(bp.dW, ref["dW"])) <= 1e-4
    net.close()


@pytest.mark.parametrize("name", ["small", "gather_odd", "gather_deep", "wide_patches"])
def test_conv_moonwalk_with_the_input_cotangent_as_read(mw, name):
    """CONV_H0_AS_READ: Phase II stops at what the first layer's vijp reads; the gradients are the same
    (to rounding: the first layer's right-hand sides are the same numbers) and h_0 shrinks to
    [B][H'][W'][C_out]."""
    B, side, C, depth, k, s, p, alpha, K, patch_bytes, kernels = CONV_CASES[name]
    wl = make_convnet(B, side, C, depth, k=k, s=s, p=p, alpha=alpha, seed=1, name=name)
    net = mw.ConvMoonwalkNet.from_workload(wl, reseed_interval=K, patch_bytes=patch_bytes, kernels=kernels,
                                           plan=mw.PLAN_MOONWALK, input_cotangent=mw.CONV_H0_AS_READ)
    res = net.moonwalk_grad(net.x, net.t)
    torch.cuda.synchronize()
    st = net.memory_stats()
    assert st["sign_mismatches"] == 0
    masks = _masks(net, wl)
    ref = CO.conv_backprop(wl.w, wl.b, wl.alphas, s, p, wl.x, wl.t, forced_masks=masks)
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.dW, ref["dW"])) <= GRAD_TOL
    assert max(O.normwise_rel_err(g.cpu().numpy(), r) for g, r in zip(res.db, ref["db"])) <= GRAD_TOL
    s1 = wl.sides[1]
    want = ref["h0"][:, ::s, ::s, :C][:, :s1, :s1]
    got = net.fetch_h0().reshape(want.shape).astype(np.float64)
    assert O.normwise_rel_err(got, want) <= 1e-4
    assert st["bytes_input_cotangent"] == 4 * want.size
    full = mw.ConvMoonwalkNet.from_workload(wl, reseed_interval=K, patch_bytes=patch_bytes, kernels=kernels,
                                            plan=mw.PLAN_MOONWALK)
    res_full = full.moonwalk_grad(full.x, full.t)
    torch.cuda.synchronize()
    assert O.normwise_rel_err(res.flat.cpu().numpy(), res_full.flat.cpu().numpy().astype(np.float64)) <= 1e-5
    full.close()
    net.close()
