"""Element-by-element parity of the three products that gather the patch matrix inside the MFMA main loop
(forward, input cotangent, weight gradient), through their C-ABI entry points, against the fp64 oracle's
definitions of the convolution and its two vjps; shapes outside what Moonwalk's layers need included
(stride 1 and 3, more output than input channels, wide kernels, one-row images)."""
import numpy as np
import pytest
import torch

from oracle import conv_oracle as CO
from oracle import frag_oracle as FO
from oracle import moonwalk_oracle as O
from tests.parity import MASK_GUARD

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mw():
    import paper_2402_14212_amd as m
    m.load_library()
    return m


SHAPES = [
    # B, H, W, C_in, C_out, k, s, p
    (2, 9, 11, 32, 32, 3, 2, 1),
    (1, 16, 16, 64, 32, 3, 1, 1),      # stride 1: one class with all nine taps
    (3, 7, 7, 32, 64, 2, 2, 0),        # more output than input channels
    (2, 13, 10, 32, 32, 5, 3, 2),      # stride 3: nine classes, some with a single tap
    (2, 12, 12, 32, 32, 1, 1, 0),      # pointwise
    (1, 33, 35, 96, 64, 3, 2, 1),      # odd sizes, ragged tiles in every dimension
    (4, 64, 64, 32, 32, 3, 2, 1),      # 4096 patch rows
    (2, 64, 64, 128, 128, 3, 2, 1),    # the experiment's channel count: K = 1152
]


def _draw(shape, seed):
    B, H, W, Ci, Co, k, s, p = shape
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, H, W, Ci)).astype(np.float32)
    w = (rng.standard_normal((k, k, Ci, Co)) / np.sqrt(k * k * Ci)).astype(np.float32)
    b = (0.1 * rng.standard_normal(Co)).astype(np.float32)
    Ho, Wo = CO.out_size(H, k, s, p), CO.out_size(W, k, s, p)
    ct = rng.standard_normal((B, Ho, Wo, Co)).astype(np.float32)
    return x, w, b, ct


def _close(got, want, tol):
    err = np.abs(got.astype(np.float64) - want).max()
    scale = np.sqrt(np.mean(want * want)) + 1e-30
    assert err <= tol * scale, (err, scale)


@pytest.mark.parametrize("shape", SHAPES)
def test_forward_product_is_the_convolution(mw, shape):
    B, H, W, Ci, Co, k, s, p = shape
    x, w, b, _ = _draw(shape, 1)
    z = CO.conv2d(x, w, s, p) + b.astype(np.float64)
    dx, dw, db = (torch.from_numpy(a).cuda() for a in (x, w, b))
    out, mask = mw.conv_forward(dx, dw, db, s, p, p, alpha=0.25, want_mask=True)
    _close(out.cpu().numpy(), np.where(z > 0, z, 0.25 * z), 2e-5)
    bits = O.unpack_mask(mask.cpu().numpy().view(np.uint64), z.size).reshape(z.shape)
    sure = np.abs(z) > MASK_GUARD * np.sqrt(np.mean(z * z))
    assert not ((bits != (z > 0)) & sure).any()
    plain = mw.conv_forward(dx, dw, None, s, p, p)                      # no bias, no activation
    _close(plain.cpu().numpy(), CO.conv2d(x, w, s, p), 2e-5)


@pytest.mark.parametrize("shape", SHAPES)
def test_input_cotangent_product_is_the_transposed_convolution(mw, shape):
    B, H, W, Ci, Co, k, s, p = shape
    _, w, _, ct = _draw(shape, 2)
    want = CO.conv2d_input_grad(ct, w, s, p, (H, W))
    got = mw.conv_input_cotangent(torch.from_numpy(ct).cuda(), torch.from_numpy(w).cuda(), (H, W), s, p, p)
    _close(got.cpu().numpy(), want, 2e-5)


@pytest.mark.parametrize("shape", SHAPES)
def test_weight_gradient_product(mw, shape):
    B, H, W, Ci, Co, k, s, p = shape
    x, _, _, ct = _draw(shape, 3)
    want = CO.conv2d_weight_grad(x, ct, k, s, p)
    dw, db = mw.conv_weight_grad(torch.from_numpy(x).cuda(), torch.from_numpy(ct).cuda(), k, k, s, p, p, scale=0.5)
    assert O.normwise_rel_err(dw.cpu().numpy(), 0.5 * want) <= 2e-6
    _close(dw.cpu().numpy(), 0.5 * want, 2e-5 * np.sqrt(B * ct.shape[1] * ct.shape[2]) / 8 + 2e-5)
    assert O.normwise_rel_err(db.cpu().numpy(), 0.5 * ct.astype(np.float64).sum(axis=(0, 1, 2))) <= 2e-6
    again, _ = mw.conv_weight_grad(torch.from_numpy(x).cuda(), torch.from_numpy(ct).cuda(), k, k, s, p, p, scale=0.5)
    assert torch.equal(dw, again)                                       # slices are added in a fixed order


@pytest.mark.parametrize("S,N,Ci,Co,k", [(2, 50, 32, 32, 3), (3, 64, 64, 32, 5), (1, 2048, 32, 32, 3)])
def test_one_row_images_with_1_x_k_kernels(mw, S, N, Ci, Co, k):
    """The 1-D layers: a one-row image and a 1 x k kernel, against the 1-D definitions."""
    rng = np.random.default_rng(k)
    x = rng.standard_normal((S, N, Ci)).astype(np.float32)
    w = (rng.standard_normal((k, Ci, Co)) / np.sqrt(k * Ci)).astype(np.float32)
    ct = rng.standard_normal((S, N, Co)).astype(np.float32)
    p = (k - 1) // 2
    dx, dw4, dct = torch.from_numpy(x[:, None]).cuda(), torch.from_numpy(w[None]).cuda(), torch.from_numpy(ct[:, None]).cuda()
    out = mw.conv_forward(dx, dw4, None, 1, 0, p)
    _close(out.cpu().numpy()[:, 0], FO.conv1d(x, w), 2e-5)
    h = mw.conv_input_cotangent(dct, dw4, (1, N), 1, 0, p)
    _close(h.cpu().numpy()[:, 0], FO.conv1d_input_grad(ct, w), 2e-5)
    g, _ = mw.conv_weight_grad(dx, dct, 1, k, 1, 0, p)
    assert O.normwise_rel_err(g.cpu().numpy()[0], FO.conv1d_weight_grad(x, ct, k)) <= 2e-6


def test_kernel_level_entries_reject_what_they_cannot_take(mw):
    x = torch.zeros(1, 8, 8, 24, device="cuda")
    w = torch.zeros(3, 3, 24, 32, device="cuda")
    with pytest.raises(mw.MoonwalkError):                               # channels not a multiple of 32
        mw.conv_forward(x, w, None, 2, 1, 1)
    x = torch.zeros(1, 2, 2, 32, device="cuda")
    w = torch.zeros(5, 5, 32, 32, device="cuda")
    with pytest.raises(mw.MoonwalkError):                               # kernel larger than the padded image
        mw.conv_forward(x, w, None, 1, 1, 1)
    ct = torch.zeros(1, 2, 2, 32, device="cuda")
    w = torch.zeros(3, 3, 32, 32, device="cuda")
    with pytest.raises(mw.MoonwalkError):                               # stride 4: more classes than the kernel holds
        mw.conv_input_cotangent(ct, w, (8, 8), 4, 1, 1)
