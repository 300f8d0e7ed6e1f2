"""dat_conv_backward_weight_static (the entry point that allocates nothing: its split partial sums live in a
buffer of the library's device image) against dat_conv_backward_weight, through the C ABI: two calls in a row,
the second with a smaller input, then a shape beyond the limit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dat():
    import paper_2206_06257_amd as dat
    return dat


def _case(dat, B, H, Cin, Cout, k, stride, pad, seed):
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    x = torch.randn(B, H, H, Cin, device="cuda", generator=g).to(torch.bfloat16)
    Ho = (H + 2 * pad - k) // stride + 1
    dy = torch.randn(B, Ho, Ho, Cout, device="cuda", generator=g).to(torch.bfloat16)
    want = dat.conv_backward_weight(x, dy, k, stride, pad)
    dw = torch.full((Cout, k, k, Cin), float("nan"), dtype=torch.float32, device="cuda")   # allocated by the caller
    got = dat.conv_backward_weight(x, dy, k, stride, pad, dw=dw, static=True)
    torch.cuda.synchronize()
    return want.cpu().numpy(), got.cpu().numpy()


def test_static_scratch_entry_point_matches_the_allocating_one(dat):
    # first call: 25 splits of a 128 x 1152 tile set (14.7 MB of partial sums)
    want, got = _case(dat, 8, 28, 128, 128, 3, 1, 1, seed=1)
    assert np.isfinite(got).all() and np.abs(want).max() > 0
    assert np.array_equal(got, want)
    # second call, smaller input: fewer splits, fewer columns -- the first call's partial sums are still in the buffer
    want2, got2 = _case(dat, 3, 14, 64, 72, 3, 2, 1, seed=2)
    assert np.isfinite(got2).all() and np.abs(want2).max() > 0
    assert np.array_equal(got2, want2)
    # and the first shape again
    want3, got3 = _case(dat, 8, 28, 128, 128, 3, 1, 1, seed=1)
    assert np.array_equal(got3, want) and np.array_equal(want3, want)


def test_static_scratch_entry_point_rejects_shapes_beyond_its_limit(dat):
    assert dat.conv_backward_weight_static_limit() == 32 << 20
    x = torch.zeros(64, 14, 14, 512, dtype=torch.bfloat16, device="cuda")
    dy = torch.zeros(64, 14, 14, 512, dtype=torch.bfloat16, device="cuda")
    dw = torch.full((512, 3, 3, 512), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(dat.DatError) as e:
        dat.conv_backward_weight(x, dy, 3, 1, 1, dw=dw, static=True)
    assert e.value.status == 6
    torch.cuda.synchronize()
    assert float(dw.min()) == 7.0 and float(dw.max()) == 7.0      # nothing was launched
