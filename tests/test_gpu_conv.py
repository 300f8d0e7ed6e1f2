"""GPU parity of the three MFMA convolution kernels against the CPU reference's direct
convolution, per layer shape (bf16 operands, fp32 accumulate): the inputs are bf16 values, so
the exact result is the fp64 sum; the kernel may differ from it by fp32 accumulation error
before its single rounding to bf16."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

# (B, H, W, Cin, Cout, k, stride, pad): the distinct kinds of layers in the four networks at
# reduced spatial size, with ragged tiles (pixel counts and channel counts off the tile sizes)
SHAPES = [
    (2, 9, 7, 16, 24, 3, 1, 1),        # everything ragged
    (3, 8, 8, 64, 64, 3, 1, 1),        # ResNet 3x3
    (2, 8, 8, 64, 128, 3, 2, 1),       # strided 3x3
    (2, 7, 7, 64, 256, 1, 1, 0),       # bottleneck expand
    (2, 8, 8, 256, 64, 1, 1, 0),       # bottleneck reduce
    (2, 8, 8, 128, 256, 1, 2, 0),      # projection shortcut
    (2, 18, 14, 8, 64, 7, 2, 3),       # ImageNet stem (3 channels padded to 8)
    (2, 8, 8, 8, 16, 3, 1, 1),         # CIFAR stem
    (1, 6, 6, 160, 320, 3, 2, 1),      # wide-ResNet widths
    (5, 12, 12, 32, 40, 3, 1, 1),      # several pixel tiles + ragged channel tile
    (2, 9, 7, 16, 32, 3, 2, 1),        # stride 2 on odd sizes (parity classes of unequal size)
    (2, 15, 13, 8, 64, 7, 2, 3),       # stem on odd sizes
    (2, 7, 9, 64, 128, 1, 2, 0),       # 1x1 stride 2: three parity classes receive zeros
    (3, 16, 16, 128, 128, 3, 1, 1),    # full 128x128 tiles
    (130, 2, 2, 64, 64, 1, 2, 0),      # 1x1 output maps: every pixel of a 64-pixel tile is another image
    (70, 3, 3, 16, 40, 3, 1, 1),       # output rows shorter than a tile: several row and image wraps per tile step
    (32, 64, 64, 8, 128, 1, 1, 0),     # enough pixel tiles for the 128x256 configuration
    (32, 64, 64, 8, 64, 3, 1, 1),      # ... and the 64x256 one
    (33, 63, 65, 16, 136, 3, 1, 1),    # wide tiles with ragged pixel and channel tails
    (5, 7, 7, 128, 128, 3, 1, 1),      # 3x3 on 7x7 images: a pixel tile spans several images, ragged tail
    (3, 14, 14, 256, 72, 3, 1, 1),     # 3x3, four channel chunks, ragged channel tile
    (2, 28, 28, 64, 64, 3, 1, 1),      # 3x3 into 64 channels (narrow tile), several tiles per image
    (1, 56, 56, 64, 128, 3, 1, 1),     # widest image the LDS-resident patch supports at this size
    (3, 10, 10, 160, 160, 3, 1, 1),    # wide-ResNet stage 1: a contraction of 160 channels (register-staged 32-wide k-tiles)
    (2, 12, 12, 64, 160, 3, 1, 1),     # ... and one the direct-to-LDS kernel takes
    (3, 8, 8, 320, 320, 3, 1, 1),      # stage 2 width
    (2, 16, 16, 128, 320, 1, 1, 0),    # ... 1x1
    (2, 16, 16, 160, 320, 1, 2, 0),    # ... strided projection of the wide nets
    (5, 9, 11, 160, 160, 3, 1, 1),     # 160-channel tiles with a ragged pixel tail
    (2, 8, 8, 96, 160, 3, 1, 1),       # k-tiles of 64 over 96-channel taps: a tile ends two thirds into a tap
    (2, 9, 9, 32, 160, 5, 1, 2),       # ... and two taps per k-tile (5x5 window)
    (8, 4, 4, 512, 512, 3, 1, 1),      # last stage of the CIFAR ResNets: few tiles, long contraction
    (2, 8, 8, 1024, 256, 1, 1, 0),     # reducing 1x1 layer with a long contraction
]
WIDE_NET_SHAPES = [s for s in SHAPES if s[4] in (160, 320) or s[3] in (160, 320)]


@pytest.fixture(scope="module")
def dat():
    import paper_2206_06257_amd as dat
    return dat


def _bf16_values(rng, shape, scale=1.0):
    t = torch.tensor(rng.standard_normal(shape) * scale, dtype=torch.float32).to(torch.bfloat16)
    return t


def _check(got_bf16, exact64, what):
    got = got_bf16.float().cpu().numpy().astype(np.float64)
    # one rounding to bf16 (2^-9 relative) plus fp32 accumulation noise on the largest terms
    tol = 2.0 ** -8 * np.abs(exact64) + 1e-5 * np.abs(exact64).max()
    bad = np.abs(got - exact64) > tol
    assert not bad.any(), (what, int(bad.sum()), float(np.abs(got - exact64).max()))


@pytest.mark.parametrize("shape", SHAPES)
def test_conv_forward_backward_parity(dat, shape):
    B, H, W, Ci, Co, k, st, pad = shape
    rng = np.random.default_rng(hash(shape) % (2 ** 31))
    x = _bf16_values(rng, (B, H, W, Ci))
    w = _bf16_values(rng, (Co, k, k, Ci), 1.0 / np.sqrt(Ci * k * k))
    x64, w64 = x.double().numpy(), w.double().numpy()
    y64 = oracle.conv_forward(x64, w64, st, pad)
    y = dat.conv_forward(x.cuda(), w.cuda(), st, pad)
    torch.cuda.synchronize()
    assert tuple(y.shape) == y64.shape
    _check(y, y64, "forward")
    dy = _bf16_values(rng, y64.shape)
    dx64, dw64 = oracle.conv_backward(x64, w64, dy.double().numpy(), st, pad)
    dx = dat.conv_backward_data(dy.cuda(), w.cuda(), (H, W), st, pad)
    _check(dx, dx64, "backward_data")
    dw = dat.conv_backward_weight(x.cuda(), dy.cuda(), k, st, pad).cpu().numpy().astype(np.float64)
    err = np.abs(dw - dw64).max() / np.abs(dw64).max()
    assert err < 2e-5, ("backward_weight", err)



# long contractions into more than 64 channels: at these sizes they have few tiles and run in 32-channel tiles
FEW_TILE_SHAPES = [s for s in SHAPES if s[3] % 64 == 0 and s[4] > 64 and s[5] * s[5] * s[3] >= 1024]


def _ab(dat, shape, option, what):
    B, H, W, Ci, Co, k, st, pad = shape
    rng = np.random.default_rng(hash(shape) % (2 ** 31) + 1)
    x = _bf16_values(rng, (B, H, W, Ci)).cuda()
    w = _bf16_values(rng, (Co, k, k, Ci), 1.0 / np.sqrt(Ci * k * k)).cuda()
    Ho, Wo = (H + 2 * pad - k) // st + 1, (W + 2 * pad - k) // st + 1
    dy = _bf16_values(rng, (B, Ho, Wo, Co)).cuda()
    res = []
    try:
        for on in (1, 0):
            dat.set_kernel_option(option, on)
            y = dat.conv_forward(x, w, st, pad)
            dx = dat.conv_backward_data(dy, w, (H, W), st, pad)
            torch.cuda.synchronize()
            res.append((y.view(torch.int16).cpu().numpy(), dx.view(torch.int16).cpu().numpy()))
    finally:
        dat.set_kernel_option(option, 1)
    _check(y, oracle.conv_forward(x.double().cpu().numpy(), w.double().cpu().numpy(), st, pad), "forward, " + what)
    _check(dx, oracle.conv_backward(x.double().cpu().numpy(), w.double().cpu().numpy(), dy.double().cpu().numpy(), st, pad)[0],
           "backward_data, " + what)
    assert np.array_equal(res[0][0], res[1][0]) and np.array_equal(res[0][1], res[1][1])


@pytest.mark.parametrize("shape", WIDE_NET_SHAPES)
def test_160_channel_tiles_give_the_bits_of_128_channel_tiles(dat, shape):
    """Layers 160 or 320 channels wide run in 160-channel tiles (no partly empty last tile).  Every output element is
    the same chain of MFMA accumulations over the same k order under either tiling, so forward and backward-data
    results must not differ by a bit; the 128-channel launches stay covered by this test."""
    _ab(dat, shape, dat.KOPT_TILE_160, "128-channel tiles")


@pytest.mark.parametrize("shape", FEW_TILE_SHAPES)
def test_32_channel_tiles_of_underfilled_layers_give_the_bits_of_128_channel_tiles(dat, shape):
    """A long contraction with too few 128x128 tiles to keep the compute units busy runs in 32-channel tiles.  Same k order
    per accumulator, so the same bits; with the switch off these shapes go through the 128-channel kernels, which this
    test thereby keeps covered at small sizes."""
    assert len(FEW_TILE_SHAPES) >= 6
    _ab(dat, shape, dat.KOPT_NARROW_UNDERFILLED, "128-channel tiles")
