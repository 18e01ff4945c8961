"""mw_colsum_wide_noalloc (the entry point for callers that cannot allocate) against mw_colsum_wide, through
the C ABI: the same bits, on calls in a row that share the library's fixed array, the later ones with
smaller inputs; and against the fp64 column sums. Sizes beyond the array are refused."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mw():
    import paper_2402_14212_amd as m
    m.load_library()
    return m


def _case(mw, rows, d, seed, scale):
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((rows, d)).astype(np.float32)
    dev = torch.from_numpy(a).cuda()
    out = torch.full((d,), float("nan"), dtype=torch.float32, device="cuda")
    got = mw.colsum_wide_noalloc(dev, out, scale)
    want = mw.colsum_wide(dev, scale)
    torch.cuda.synchronize()
    assert got.data_ptr() == out.data_ptr()
    assert torch.equal(got, want), f"rows={rows} d={d}: differs from mw_colsum_wide"
    ref = scale * a.astype(np.float64).sum(axis=0)
    tol = 2e-6 * np.sqrt(rows) * max(1.0, float(np.abs(a).max())) * abs(scale)
    assert np.abs(got.cpu().numpy() - ref).max() <= tol


def test_two_calls_in_a_row_the_second_smaller(mw):
    print("no-alloc colsum: 200000 x 256, then 3000 x 96", flush=True)
    _case(mw, 200000, 256, seed=1, scale=0.25)      # many row ranges: most of the partial-sum slots in use
    _case(mw, 3000, 96, seed=2, scale=-2.0)         # fewer ranges, fewer columns: stale slots must not be read
    _case(mw, 77, 4, seed=3, scale=1.0)             # one range
    _case(mw, 5000, 33, seed=4, scale=1.0)          # the kernel for widths that are not a multiple of 4
    _case(mw, 200000, 256, seed=1, scale=0.25)      # and the first one again


def test_the_library_allocates_nothing(mw):
    rng = np.random.default_rng(5)
    dev = torch.from_numpy(rng.standard_normal((4096, 512)).astype(np.float32)).cuda()
    out = torch.empty(512, dtype=torch.float32, device="cuda")
    mw.colsum_wide_noalloc(dev, out)                 # first call on the device done
    torch.cuda.synchronize()
    free_before, _ = torch.cuda.mem_get_info()
    reserved_before = torch.cuda.memory_reserved()
    for _ in range(3):
        mw.colsum_wide_noalloc(dev, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_reserved() == reserved_before
    assert torch.cuda.mem_get_info()[0] == free_before


def test_sizes_beyond_the_array_are_refused(mw):
    lib = mw.load_library()
    cap = int(lib.mw_colsum_noalloc_max_floats())
    assert cap == 1 << 20
    d = cap + 4                                       # one row range already needs more than the array
    a = torch.zeros((2, d), dtype=torch.float32, device="cuda")
    out = torch.full((d,), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(mw.MoonwalkError) as err:
        mw.colsum_wide_noalloc(a, out)
    assert err.value.code == mw.binding.ERR_TOO_LARGE
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                  # nothing was launched
    # the largest width that fits with one range is accepted
    a = torch.ones((3, cap), dtype=torch.float32, device="cuda")
    out = torch.empty(cap, dtype=torch.float32, device="cuda")
    mw.colsum_wide_noalloc(a, out)
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())
