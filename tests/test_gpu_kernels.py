"""GPU parity of the individual device steps against the oracle's definitions.

Integer work (packed masks, erased offsets, compaction order, restored values) must match bit
for bit; the GEMMs are compared with an fp64 numpy product at a tolerance derived from fp32
accumulation: K products with unit roundoff 2^-24 give a normwise error of about
sqrt(K) * 6e-8, far below the 2e-6 bound used here for K <= 4096.
"""
import numpy as np
import pytest
import torch

from oracle import moonwalk_oracle as O

pytestmark = pytest.mark.gpu

GEMM_TOL = 2e-6


@pytest.fixture(scope="module")
def mw():
    import paper_2402_14212_amd as m
    m.load_library()
    return m


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def as_u64(t):
    return t.cpu().numpy().view(np.uint64)


GEMM_SHAPES = [
    # (M, N, K): tile multiples, ragged tails, tiny, K not a multiple of 4, several tiles
    (128, 128, 64), (256, 192, 160), (64, 64, 32), (32, 32, 128), (1, 1, 1), (5, 7, 3),
    (77, 130, 45), (130, 77, 257), (200, 96, 1000), (33, 260, 129), (300, 300, 36),
]


@pytest.mark.parametrize("op", [0, 1, 2])
@pytest.mark.parametrize("tile", [1, 2, 3, 4, 5, 6, 7])
def test_gemm_matches_fp64_product(mw, op, tile):
    rng = np.random.default_rng(100 * op + tile)
    for (M, N, K) in GEMM_SHAPES:
        print(f"gemm op={op} tile={tile} M={M} N={N} K={K}", flush=True)
        A = rng.standard_normal((M, K)).astype(np.float32)
        B = rng.standard_normal((N, K)).astype(np.float32)
        ref = A.astype(np.float64) @ B.astype(np.float64).T
        if op == mw.GEMM_NT:
            got = mw.gemm_f32(op, dev(A), dev(B), tile=tile)
        elif op == mw.GEMM_NN:
            got = mw.gemm_f32(op, dev(A), dev(B.T.copy()), tile=tile)
        else:
            got = mw.gemm_f32(op, dev(A.T.copy()), dev(B.T.copy()), tile=tile)
        torch.cuda.synchronize()
        assert O.normwise_rel_err(got.cpu().numpy(), ref) < GEMM_TOL, (op, tile, M, N, K)


def test_gemm_alpha_beta_and_auto_tile(mw):
    rng = np.random.default_rng(7)
    for (M, N, K) in [(256, 1024, 1024), (512, 2048, 256), (1024, 1024, 256), (96, 40, 72)]:
        A = rng.standard_normal((M, K)).astype(np.float32)
        B = rng.standard_normal((N, K)).astype(np.float32)
        C0 = rng.standard_normal((M, N)).astype(np.float32)
        ref = -0.5 * (A.astype(np.float64) @ B.astype(np.float64).T) + 2.0 * C0
        c = dev(C0)
        mw.gemm_f32(mw.GEMM_NT, dev(A), dev(B), C_out=c, alpha=-0.5, beta=2.0)
        assert O.normwise_rel_err(c.cpu().numpy(), ref) < GEMM_TOL


def test_gemm_is_deterministic(mw):
    rng = np.random.default_rng(1)
    A, B = dev(rng.standard_normal((256, 1024)).astype(np.float32)), dev(rng.standard_normal((1024, 1024)).astype(np.float32))
    for tile in (1, 2, 3, 4, 5, 6, 7):
        a = mw.gemm_f32(mw.GEMM_NT, A, B, tile=tile).clone()
        b = mw.gemm_f32(mw.GEMM_NT, A, B, tile=tile)
        assert torch.equal(a, b)


SHAPES_EW = [(1, 1), (3, 5), (4, 64), (5, 67), (32, 64), (77, 130), (256, 1024), (33, 2048)]


@pytest.mark.parametrize("alpha", [0.1, 0.0])
def test_bias_act_mask_bit_exact(mw, alpha):
    rng = np.random.default_rng(2)
    for rows, d in SHAPES_EW:
        z = rng.standard_normal((rows, d)).astype(np.float32)
        z.ravel()[:: 7] = 0.0
        if z.size > 3:
            z.ravel()[1], z.ravel()[2], z.ravel()[3] = -0.0, np.nan, np.inf
        b = rng.standard_normal(d).astype(np.float32)
        for bias in (None, b):
            x, mask = mw.bias_act_mask(dev(z), None if bias is None else dev(bias), alpha)
            zz = z if bias is None else z + bias            # fp32 add, as on the device
            m = O.sign_mask(zz)
            np.testing.assert_array_equal(as_u64(mask)[: (z.size + 63) // 64], O.pack_mask(m))
            with np.errstate(invalid="ignore"):                 # alpha = 0 times the planted infinity
                want = np.where(m, zz, np.float32(alpha) * zz)
            np.testing.assert_array_equal(x.cpu().numpy(), want.astype(np.float32))


def test_mask_special_cases(mw):
    ones = np.ones((4, 64), np.float32)
    _, mask = mw.bias_act_mask(dev(ones), None, 0.1)
    assert as_u64(mask).tolist() == [2 ** 64 - 1] * 4
    _, mask = mw.bias_act_mask(dev(-ones), None, 0.1)
    assert as_u64(mask).tolist() == [0] * 4
    z = np.array([[0.0, -0.0, np.nan, 1e-45, -1e-45, 1.0]], np.float32)
    _, mask = mw.bias_act_mask(dev(z), None, 0.1)
    assert int(as_u64(mask)[0]) == int(O.pack_mask(O.sign_mask(z))[0])


@pytest.mark.parametrize("alpha", [0.1, 0.0])
def test_rev_scale_and_fragments_bit_exact(mw, alpha):
    rng = np.random.default_rng(3)
    for rows, d in SHAPES_EW:
        n = rows * d
        m = rng.random((rows, d)) < 0.5
        h = rng.standard_normal((rows, d)).astype(np.float32)
        words = O.pack_mask(m)
        mask = dev(words.view(np.int64))
        ct = mw.rev_scale(dev(h), mask, alpha)
        np.testing.assert_array_equal(ct.cpu().numpy(), h * np.where(m, np.float32(1), np.float32(alpha)))
        off = mw.frag_offsets(mask, n)
        np.testing.assert_array_equal(off.cpu().numpy().view(np.uint32), O.erased_word_offsets(m))
        frag, flag = mw.frag_compact(dev(h), mask, off)
        want = O.compact_fragments(h, m)
        assert int(flag.item()) == 0
        np.testing.assert_array_equal(frag.cpu().numpy()[: want.size], want)
        # overflow: nothing past the capacity is written and the flag is raised
        if want.size > 1:
            cap = want.size // 2
            frag2, flag2 = mw.frag_compact(dev(h), mask, off, capacity=cap)
            assert int(flag2.item()) == 1
            np.testing.assert_array_equal(frag2.cpu().numpy()[:cap], want[:cap])


def test_fragment_edge_masks(mw):
    for m in (np.ones((2, 64), bool), np.zeros((2, 64), bool), np.zeros((1, 3), bool)):
        h = np.arange(m.size, dtype=np.float32).reshape(m.shape) + 1
        mask = dev(O.pack_mask(m).view(np.int64))
        off = mw.frag_offsets(mask, m.size)
        np.testing.assert_array_equal(off.cpu().numpy().view(np.uint32), O.erased_word_offsets(m))
        frag, _ = mw.frag_compact(dev(h), mask, off)
        want = O.compact_fragments(h, m)
        np.testing.assert_array_equal(frag.cpu().numpy()[: want.size], want)


def test_vijp_epilogue_leaky_and_relu(mw):
    rng = np.random.default_rng(4)
    for rows, d in SHAPES_EW:
        z = rng.standard_normal((rows, d)).astype(np.float32)
        c = rng.standard_normal((rows, d)).astype(np.float32)
        # leaky
        a = np.float32(0.1)
        x, hy = mw.vijp_epilogue(dev(z), dev(c), float(a))
        m = z > 0
        np.testing.assert_array_equal(x.cpu().numpy(), np.where(m, z, a * z))
        np.testing.assert_array_equal(hy.cpu().numpy(), np.where(m, c, c * (np.float32(1) / a)))
        # ReLU with stored mask and fragments
        h_prev = rng.standard_normal((rows, d)).astype(np.float32)
        F = O.compact_fragments(h_prev, m)
        mask = dev(O.pack_mask(m).view(np.int64))
        off = mw.frag_offsets(mask, z.size)
        ct = dev(c)
        x, hy = mw.vijp_epilogue(dev(z), ct, 0.0, mask=mask, offsets=off, frag=dev(F if F.size else np.zeros(1, np.float32)))
        np.testing.assert_array_equal(ct.cpu().numpy(), np.where(m, c, np.float32(0)))
        np.testing.assert_array_equal(hy.cpu().numpy(), O.restore_from_fragments(c, m, F).astype(np.float32))
        assert np.array_equal(hy.cpu().numpy()[~m], h_prev[~m])      # erased entries come back bit-identical
        np.testing.assert_array_equal(x.cpu().numpy(), np.where(m, z, np.float32(0) * z))


def test_colsum_and_loss(mw):
    rng = np.random.default_rng(5)
    for rows, d in SHAPES_EW:
        a = rng.standard_normal((rows, d)).astype(np.float32)
        got = mw.colsum(dev(a), 0.5).cpu().numpy()
        ref = 0.5 * a.astype(np.float64).sum(axis=0)
        assert np.abs(got - ref).max() <= 1e-5 * max(1.0, np.abs(ref).max())
        t = rng.standard_normal((rows, d)).astype(np.float32)
        hL, loss = mw.loss_grad(dev(a), dev(t), scale=4.0)
        J, h = O.loss_and_output_cotangent(a.astype(np.float64), t.astype(np.float64), 4.0)
        assert abs(float(loss.item()) - J) <= 1e-6 * J
        assert O.normwise_rel_err(hL.cpu().numpy(), h) < 1e-6


@pytest.mark.parametrize("rows,d", [(1, 4), (7, 12), (300, 128), (5000, 32), (70001, 256), (2048, 1000), (1025, 130), (999, 7)])
def test_colsum_of_tall_matrices(mw, rows, d):
    """Row ranges summed side by side, then added in range order: the 128-bit kernel (d a multiple of 4) and
    the scalar one, ragged row ranges, more than 128 columns; bit-identical on repetition."""
    rng = np.random.default_rng(6)
    a = rng.standard_normal((rows, d)).astype(np.float32)
    got = mw.colsum_wide(dev(a), 0.25)
    ref = 0.25 * a.astype(np.float64).sum(axis=0)
    assert np.abs(got.cpu().numpy() - ref).max() <= 2e-6 * np.sqrt(rows) * max(1.0, np.abs(a).max())
    assert torch.equal(got, mw.colsum_wide(dev(a), 0.25))
    view = dev(np.concatenate([np.zeros(1, np.float32), a.ravel()]))[1:].view(rows, d)   # not 16-byte aligned
    assert np.abs(mw.colsum_wide(view, 0.25).cpu().numpy() - ref).max() <= 2e-6 * np.sqrt(rows) * max(1.0, np.abs(a).max())


def test_copy(mw):
    for n in (1, 5, 1024, 1_000_003):
        src = torch.arange(n, dtype=torch.float32, device="cuda")
        dst = torch.zeros_like(src)
        mw.copy_f32(src, dst)
        assert torch.equal(src, dst)


def test_operand_stream_probe(mw):
    """The load-only probe reads every operand element exactly once per tile: with one tile per
    dimension pair its checksums add up to sum(A) * tiles_n + sum(B) * tiles_m."""
    M, N, K = 64, 128, 512
    A = torch.randint(-3, 4, (M, K), device="cuda").float()
    B = torch.randint(-3, 4, (N, K), device="cuda").float()
    for tile in (16, 32, 64):
        sink = mw.probe_operand_stream(A, B, tile)
        want = float(A.double().sum()) * (N // tile) + float(B.double().sum()) * (M // tile)
        assert float(sink.double().sum()) == want
    with pytest.raises(mw.MoonwalkError):
        mw.probe_operand_stream(A, B, 48)
    with pytest.raises(mw.MoonwalkError):
        mw.probe_operand_stream(A[:, :384].contiguous(), B[:, :384].contiguous(), 32)
