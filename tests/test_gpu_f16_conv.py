"""GPU parity on 16-bit float storage: conv2d, depthwiseConv2d and the MobileNet forward against the CPU oracle."""
import numpy as np
import pytest

import oracle
from oracle import ACT_NONE, ACT_RELU, ACT_RELU6, PAD_SAME, PAD_VALID
from paper_1901_05350_amd import inputs
from util import assert_close_f16, dev16, host

pytestmark = pytest.mark.gpu


def h(a):
    return np.ascontiguousarray(a).astype(np.float16)


def conv_case(seed, n, hh, ww, cin, cout, fh, fw):
    d = inputs.conv_general(seed, n, hh, ww, cin, cout, fh, fw)
    return h(d["x"]), h(d["filter"]), h(d["bias"] * 30)     # a bias large enough to matter in binary16


@pytest.mark.parametrize("shape,stride,pad,act", [
    ((2, 56, 56, 128, 128, 1, 1), 1, PAD_SAME, ACT_RELU6),      # pointwise: matMul path, B stored [K,N]
    ((8, 56, 56, 128, 128, 1, 1), 1, PAD_SAME, ACT_RELU6),      # M >= 16384 with a thin filter: filter-stationary kernel
    ((2, 112, 112, 32, 64, 1, 1), 1, PAD_SAME, ACT_RELU6),
    ((7, 57, 53, 64, 128, 1, 1), 1, PAD_SAME, ACT_RELU),        # M = 21147: ragged last unit
    ((6, 56, 56, 128, 256, 1, 1), 1, PAD_SAME, ACT_NONE),
    ((1, 14, 14, 512, 512, 1, 1), 1, PAD_SAME, ACT_RELU6),
    ((3, 9, 7, 24, 40, 1, 1), 1, PAD_VALID, ACT_NONE),
    ((2, 10, 10, 6, 10, 1, 1), 1, PAD_SAME, ACT_RELU),          # channel counts that are not multiples of 8
    ((2, 224, 224, 3, 32, 3, 3), 2, PAD_SAME, ACT_RELU6),       # the stem
    ((1, 97, 101, 3, 8, 3, 3), 2, PAD_SAME, ACT_RELU6),
    ((1, 40, 75, 3, 32, 3, 3), 2, PAD_SAME, ACT_RELU6),         # matrix-core stem: ragged last slab of a row, borders
    ((2, 21, 53, 3, 32, 3, 3), 1, PAD_VALID, ACT_NONE),         # all slabs interior
    ((3, 18, 34, 3, 32, 3, 3), 1, PAD_SAME, ACT_RELU),
    ((1, 2, 2, 3, 32, 3, 3), 2, PAD_SAME, ACT_RELU6),
    ((1, 33, 35, 3, 24, 3, 3), 1, PAD_VALID, ACT_NONE),
    ((2, 17, 19, 5, 7, 3, 3), 2, PAD_SAME, ACT_RELU6),          # general direct kernel
    ((1, 12, 12, 16, 8, 5, 2), 3, PAD_VALID, ACT_RELU),
    ((2, 8, 8, 32, 16, 1, 1), 2, PAD_SAME, ACT_NONE),           # 1x1 with stride 2 is not a plain matMul
])
def test_conv2d_f16(shape, stride, pad, act):
    import paper_1901_05350_amd as tfx
    n, hh, ww, cin, cout, fh, fw = shape
    x, f, b = conv_case(100 + cin + cout, n, hh, ww, cin, cout, fh, fw)
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), dev16(b), stride, pad, act))
    assert_close_f16(got, oracle.conv2d_f16(x, f, b, stride, pad, act), "conv2d_f16 %r s%d" % (shape, stride))
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), None, stride, pad, ACT_NONE))
    assert_close_f16(got, oracle.conv2d_f16(x, f, None, stride, pad, ACT_NONE), "conv2d_f16 no bias %r" % (shape,))


@pytest.mark.parametrize("shape,stride,pad,act", [
    ((2, 56, 56, 64, 64, 3, 3), 1, PAD_SAME, ACT_RELU6),        # several row tiles, every tap inside one 64-half slice
    ((2, 56, 56, 64, 64, 3, 3), 2, PAD_SAME, ACT_RELU6),
    ((1, 30, 29, 72, 136, 3, 3), 1, PAD_VALID, ACT_NONE),       # Ci not a divisor of 64, ragged column tile (136 = 128 + 8)
    ((3, 19, 23, 24, 40, 3, 3), (2, 1), PAD_SAME, ACT_RELU),    # three tap carries per slice, ragged last slice (K = 216)
    ((2, 21, 17, 8, 24, 5, 5), 1, PAD_SAME, ACT_RELU6),         # 8 channels: a slice spans 8 taps; 25 taps
    ((1, 40, 33, 16, 8, 2, 7), (3, 2), PAD_SAME, ACT_NONE),
    ((1, 9, 9, 128, 256, 4, 4), 1, PAD_VALID, ACT_RELU6),       # K = 2048: 32 slices, 36 rows (one ragged tile)
    ((1, 1, 1, 64, 64, 3, 3), 1, PAD_SAME, ACT_NONE),           # a single pixel: 8 of 9 taps outside
])
def test_conv2d_f16_implicit_gemm(shape, stride, pad, act):
    """Channel counts that are multiples of 8 take the matrix-core implicit GEMM."""
    import paper_1901_05350_amd as tfx
    n, hh, ww, cin, cout, fh, fw = shape
    x, f, b = conv_case(400 + cin + cout + fh, n, hh, ww, cin, cout, fh, fw)
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), dev16(b), stride, pad, act))
    assert_close_f16(got, oracle.conv2d_f16(x, f, b, stride, pad, act), "conv2d_f16 gemm %r" % (shape,))
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), None, stride, pad, ACT_NONE))
    assert_close_f16(got, oracle.conv2d_f16(x, f, None, stride, pad, ACT_NONE), "conv2d_f16 gemm no bias %r" % (shape,))


def test_conv2d_f16_implicit_gemm_one_hot_and_unaligned_output():
    import torch
    import paper_1901_05350_amd as tfx
    # one-hot filters: output channel o copies input channel (o * 5) % 16 under tap (o % 3, (o // 3) % 3): every
    # (tap, channel) position of the window is located exactly, borders included
    rng = np.random.default_rng(11)
    x = h(rng.uniform(-1, 1, (1, 7, 9, 16)))
    f = np.zeros((3, 3, 16, 24), np.float16)
    for o in range(24):
        f[o % 3, (o // 3) % 3, (o * 5) % 16, o] = 1
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), None, 1, PAD_SAME, ACT_NONE))
    assert np.array_equal(got, oracle.conv2d_f16(x, f, None, 1, PAD_SAME, ACT_NONE))
    # an output buffer 2 bytes off a 16-byte boundary: element stores, nothing written outside
    x, f, b = conv_case(412, 1, 10, 11, 16, 24, 3, 3)
    out = torch.zeros(10 * 11 * 24 + 2, dtype=torch.float16, device="cuda:0")
    tfx.tfx_conv2d_f16(dev16(x), dev16(f), dev16(b), 1, PAD_SAME, ACT_RELU6, out=out[1:-1].view(1, 10, 11, 24))
    o = host(out)
    assert o[0] == 0 and o[-1] == 0
    assert_close_f16(o[1:-1].reshape(1, 10, 11, 24), oracle.conv2d_f16(x, f, b, 1, PAD_SAME, ACT_RELU6), "unaligned y")


def test_conv2d_f16_3x3_benchmark_size_every_image():
    import paper_1901_05350_amd as tfx
    n = 64
    x, f, b = conv_case(420, n, 56, 56, 64, 64, 3, 3)
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), dev16(b), 1, PAD_SAME, ACT_RELU6))
    assert_close_f16(got, oracle.conv2d_f16(x, f, b, 1, PAD_SAME, ACT_RELU6), "conv 3x3 f16 batch 64")


@pytest.mark.parametrize("shape,stride,pad,act", [
    ((6, 56, 56, 64, 64, 3, 3), 1, PAD_SAME, ACT_RELU6),        # M = 18816, whole 4 x 8 patches
    ((6, 57, 53, 32, 64, 3, 3), 1, PAD_SAME, ACT_RELU),         # ragged last patch row (1 of 4) and column (5 of 8)
    ((9, 47, 45, 32, 128, 3, 3), 1, PAD_VALID, ACT_NONE),       # no tap outside the image; 45 x 43 outputs
    ((10, 44, 41, 64, 32, 3, 3), 1, PAD_SAME, ACT_RELU6),
    ((17, 33, 31, 32, 32, 3, 3), 1, PAD_SAME, ACT_NONE),
    ((4, 150, 38, 64, 64, 3, 3), 1, PAD_VALID, ACT_RELU6),      # tall images: a workgroup's units cross image boundaries
    ((1100, 3, 5, 32, 32, 3, 3), 1, PAD_SAME, ACT_RELU6),       # images smaller than a 4 x 8 patch: every window is mostly padding
    ((50, 21, 20, 64, 64, 3, 3), 1, PAD_VALID, ACT_RELU),       # 19 x 18 outputs: 3 of 4 rows and 2 of 8 columns in the last patches
    ((9, 45, 47, 128, 32, 3, 3), 1, PAD_SAME, ACT_RELU6),       # 128 channels in: the tiled implicit GEMM
    ((23, 57, 53, 32, 64, 3, 3), 2, PAD_SAME, ACT_RELU),        # stride 2: the tiled implicit GEMM
])
def test_conv2d_f16_filter_stationary(shape, stride, pad, act):
    """Few channels, stride 1 and at least 16384 output pixels: the kernel that keeps the whole 3 x 3 filter in LDS."""
    import paper_1901_05350_amd as tfx
    n, hh, ww, cin, cout, fh, fw = shape
    x, f, b = conv_case(500 + cin + cout, n, hh, ww, cin, cout, fh, fw)
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), dev16(b), stride, pad, act))
    assert_close_f16(got, oracle.conv2d_f16(x, f, b, stride, pad, act), "conv2d_f16 stationary %r" % (shape,))
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), None, stride, pad, ACT_NONE))
    assert_close_f16(got, oracle.conv2d_f16(x, f, None, stride, pad, ACT_NONE), "conv2d_f16 stationary no bias %r" % (shape,))


def test_conv2d_f16_filter_stationary_one_hot():
    """One-hot filters: output channel o copies input channel (o * 5) % 32 under tap (o % 3, (o // 3) % 3), so every
    (tap, channel) position of the window is located exactly, image borders and image-to-image boundaries included."""
    import paper_1901_05350_amd as tfx
    rng = np.random.default_rng(12)
    x = h(rng.uniform(-1, 1, (5, 60, 58, 32)))
    f = np.zeros((3, 3, 32, 64), np.float16)
    for o in range(64):
        f[o % 3, (o // 3) % 3, (o * 5) % 32, o] = 1
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), None, 1, PAD_SAME, ACT_NONE))
    assert got.shape[0] * got.shape[1] * got.shape[2] >= 16384
    assert np.array_equal(got, oracle.conv2d_f16(x, f, None, 1, PAD_SAME, ACT_NONE))


@pytest.mark.parametrize("shape,act", [
    ((8, 14, 14, 512, 512), ACT_RELU6),      # M = 1568: 49 units of 32 rows against 4 column slabs
    ((2, 29, 29, 256, 256), ACT_RELU),       # M = 1682: ragged last unit, 2 slabs
    ((3, 28, 28, 256, 512), ACT_RELU6),      # some wavefronts take two units
    ((16, 7, 7, 512, 1024), ACT_NONE),       # M = 784 < 1536: the tiled kernel (same shapes, other path)
    ((33, 7, 7, 512, 1024), ACT_RELU6),      # M = 1617, 8 slabs
    ((2, 28, 28, 256, 2048), ACT_RELU6),     # 16 slabs: one part of the rows per XCD pair
    ((40, 14, 14, 512, 512), ACT_RELU6),     # M = 7840: several units per wavefront
    ((1, 56, 56, 64, 128), ACT_RELU6),       # K = 64 (two k-steps), one slab
    ((2, 28, 29, 128, 256), ACT_RELU),       # K = 128, M = 1624
    ((1, 56, 56, 128, 128), ACT_NONE),
])
def test_conv2d_f16_pointwise_column_slabs(shape, act):
    """Pointwise layers with K = 64 ... 512 and N a multiple of 128, from 1536 output pixels on (below 16384 for the
    filters that fit in LDS whole): a workgroup keeps a 128-column slab of the filter in LDS and streams rows against
    it."""
    import paper_1901_05350_amd as tfx
    n, hh, ww, cin, cout = shape
    x, f, b = conv_case(700 + cin + cout + n, n, hh, ww, cin, cout, 1, 1)
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), dev16(b), 1, PAD_SAME, act))
    assert_close_f16(got, oracle.conv2d_f16(x, f, b, 1, PAD_SAME, act), "conv2d_f16 slabs %r" % (shape,))
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), None, 1, PAD_SAME, ACT_NONE))
    assert_close_f16(got, oracle.conv2d_f16(x, f, None, 1, PAD_SAME, ACT_NONE), "conv2d_f16 slabs no bias %r" % (shape,))


def test_conv2d_f16_pointwise_column_slabs_one_hot():
    """A one-hot filter: output channel o copies input channel (o * 37) % 512, so every (row, k, column) position of
    the slab layout is located exactly; bit-exact."""
    import paper_1901_05350_amd as tfx
    rng = np.random.default_rng(13)
    x = h(rng.uniform(-1, 1, (9, 14, 14, 512)))
    f = np.zeros((1, 1, 512, 1024), np.float16)
    for o in range(1024):
        f[0, 0, (o * 37) % 512, o] = 1
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), None, 1, PAD_SAME, ACT_NONE))
    assert np.array_equal(got, x[..., (np.arange(1024) * 37) % 512])
    assert np.array_equal(got, oracle.conv2d_f16(x, f, None, 1, PAD_SAME, ACT_NONE))


def test_stem_f16_matrix_core_form_walks_over_several_slabs():
    """Batch 20 at 224 x 224 is 15680 slabs for at most 8192 wavefronts: wavefronts move on across row and image
    boundaries.  Every image is compared."""
    import paper_1901_05350_amd as tfx
    x, f, b = conv_case(77, 20, 224, 224, 3, 32, 3, 3)
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), dev16(b), 2, PAD_SAME, ACT_RELU6))
    assert got.shape == (20, 112, 112, 32)
    assert_close_f16(got, oracle.conv2d_f16(x, f, b, 2, PAD_SAME, ACT_RELU6), "stem f16 batch 20")


@pytest.mark.parametrize("shape,stride,pad,mult", [
    ((2, 112, 112, 64), 1, PAD_SAME, 1), ((2, 112, 112, 64), 2, PAD_SAME, 1), ((64, 56, 56, 128), 1, PAD_SAME, 1),
    ((1, 14, 14, 512), 1, PAD_SAME, 1), ((3, 7, 7, 1024), 1, PAD_SAME, 1), ((1, 14, 14, 512), 2, PAD_SAME, 1),
    ((2, 13, 17, 16), 1, PAD_VALID, 1), ((2, 31, 29, 8), 2, PAD_SAME, 1), ((16, 28, 28, 256), 2, PAD_SAME, 1),
    ((2, 9, 11, 12), 1, PAD_SAME, 1),          # C % 8 != 0: general kernel
    ((1, 10, 10, 8), 1, PAD_SAME, 2), ((1, 12, 9, 5), 2, PAD_VALID, 3),
])
def test_depthwise_f16(shape, stride, pad, mult):
    import paper_1901_05350_amd as tfx
    n, hh, ww, c = shape
    rng = np.random.default_rng(200 + c + stride)
    x = h(rng.uniform(-1, 1, shape))
    f = h(rng.standard_normal((3, 3, c, mult)) * (2.0 / 9) ** 0.5)
    b = h(rng.standard_normal(c * mult) * 0.3)
    got = host(tfx.tfx_depthwise_conv2d_f16(dev16(x), dev16(f), dev16(b), stride, pad, ACT_RELU6))
    assert_close_f16(got, oracle.depthwise_conv2d_f16(x, f, b, stride, pad, ACT_RELU6), "depthwise_f16 %r s%d" % (shape, stride))


def test_f16_benchmark_sizes_every_image():
    """The sizes the benchmark times (batch 64); every image is compared."""
    import paper_1901_05350_amd as tfx
    n = 64
    x, f, b = conv_case(300, n, 56, 56, 128, 128, 1, 1)
    got = host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), dev16(b), 1, PAD_SAME, ACT_RELU6))
    assert_close_f16(got, oracle.conv2d_f16(x, f, b, 1, PAD_SAME, ACT_RELU6), "pointwise f16 batch 64")
    rng = np.random.default_rng(301)
    x = h(rng.uniform(-1, 1, (n, 112, 112, 64)))
    f = h(rng.standard_normal((3, 3, 64, 1)) * (2.0 / 9) ** 0.5)
    b = h(rng.standard_normal(64) * 0.3)
    for stride in (1, 2):
        got = host(tfx.tfx_depthwise_conv2d_f16(dev16(x), dev16(f), dev16(b), stride, PAD_SAME, ACT_RELU6))
        assert_close_f16(got, oracle.depthwise_conv2d_f16(x, f, b, stride, PAD_SAME, ACT_RELU6),
                         "depthwise f16 batch 64 s%d" % stride)


@pytest.mark.parametrize("batch", [8, 64])
def test_mobilenet_f16_benchmark_batches_every_image(batch):
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1_f16(seed=9, batch=batch)
    model = tfx.MobileNetV1F16(data["weights"], batch=batch)
    p, l = model.forward(dev16(data["image"]))
    p, l = host(p).copy(), host(l).copy()
    probs, logits = oracle.mobilenet_v1_forward_f16(data["image"], data["weights"])
    end_to_end_bar(l, logits, "f16 logits batch %d" % batch, 8)
    end_to_end_bar(p, probs, "f16 probs batch %d" % batch, 16)
    assert np.array_equal(p.argmax(axis=1), probs.argmax(axis=1))


def test_f16_nan_and_inf_through_the_fused_activations():
    """As on fp32 storage: a NaN passes through relu and relu6, -inf becomes 0, +inf the upper bound (or stays +inf
    under relu), and a NaN in the input reaches exactly the outputs whose window holds it.  Covers the tiled,
    small-tile, filter-stationary and column-slab pointwise kernels, the implicit GEMM, the filter-stationary 3 x 3 kernel, both stems, the direct kernel, both
    depthwise kernels and the matMul epilogue."""
    import paper_1901_05350_amd as tfx
    rng = np.random.default_rng(46)

    def same(got, ref, what):
        assert np.isnan(ref).any() and not np.isnan(ref).all(), what
        assert_close_f16(got, ref, what)      # requires NaNs and infinities to coincide

    for (n, hh, ww, ci, co, fh, fw, s) in [(1, 14, 14, 64, 96, 1, 1, 1), (2, 56, 56, 128, 128, 1, 1, 1),
                                           (8, 56, 56, 128, 128, 1, 1, 1), (2, 20, 20, 32, 40, 3, 3, 1),
                                           (6, 56, 56, 64, 64, 3, 3, 1), (6, 57, 53, 32, 64, 3, 3, 1), (9, 14, 14, 512, 512, 1, 1, 1), (2, 28, 28, 256, 256, 1, 1, 1),
                                           (1, 30, 30, 3, 32, 3, 3, 2), (1, 30, 30, 3, 16, 3, 3, 2), (1, 9, 9, 5, 4, 3, 3, 1)]:
        x, f, b = conv_case(500 + ci, n, hh, ww, ci, co, fh, fw)
        x[n - 1, hh // 2, ww // 3, ci - 1] = np.nan
        x[0, 1, 2, 0] = np.inf
        x[0, hh - 2, ww - 1, ci // 2] = -np.inf
        f[..., 0] = np.abs(f[..., 0])
        for act in (ACT_RELU6, ACT_RELU, ACT_NONE):
            same(host(tfx.tfx_conv2d_f16(dev16(x), dev16(f), dev16(b), s, PAD_SAME, act)),
                 oracle.conv2d_f16(x, f, b, s, PAD_SAME, act), "conv f16 NaN/Inf %r act %d" % ((n, hh, ww, ci, co, fh, fw, s), act))
    for (n, hh, ww, c, mult, s) in [(1, 28, 28, 32, 1, 1), (16, 28, 28, 64, 1, 2), (2, 9, 11, 5, 2, 1)]:
        x = h(rng.uniform(-1, 1, (n, hh, ww, c)))
        f = h(rng.standard_normal((3, 3, c, mult)) * (2.0 / 9) ** 0.5)
        b = h(rng.standard_normal(c * mult) * 0.3)
        x[n - 1, hh // 2, ww // 3, c - 1] = np.nan
        x[0, 1, 2, 0] = np.inf
        x[0, hh - 2, ww - 1, c // 2] = -np.inf
        for act in (ACT_RELU6, ACT_RELU, ACT_NONE):
            same(host(tfx.tfx_depthwise_conv2d_f16(dev16(x), dev16(f), dev16(b), s, PAD_SAME, act)),
                 oracle.depthwise_conv2d_f16(x, f, b, s, PAD_SAME, act), "depthwise f16 NaN/Inf %r act %d" % ((n, hh, ww, c, mult, s), act))
    a = h(rng.uniform(-1, 1, (2, 300, 136)))
    bm = h(rng.uniform(-1, 1, (2, 200, 136)))
    bias = h(rng.standard_normal(200))
    a[1, 7, 3], a[0, 9, 5], a[0, 11, 2] = np.nan, np.inf, -np.inf
    bm[..., 0:8] = np.abs(bm[..., 0:8])
    for act in (ACT_RELU6, ACT_RELU):
        same(host(tfx.tfx_batch_matmul_f16(dev16(a), dev16(bm), False, True, dev16(bias), act)),
             oracle.batch_matmul_f16(a, bm, False, True, bias, act), "matMul f16 NaN/Inf act %d" % act)


def test_f16_conv_rounds_once_and_handles_unaligned_buffers():
    import torch
    import paper_1901_05350_amd as tfx
    # 2048 + 1 + 1 across three taps must give 2050 (a binary16 running sum would stay at 2048)
    xs = np.array([2048, 1, 1], np.float16).reshape(1, 1, 3, 1)
    ws = np.ones((1, 3, 1, 1), np.float16)
    assert host(tfx.tfx_conv2d_f16(dev16(xs), dev16(ws), None, 1, PAD_VALID))[0, 0, 0, 0] == np.float16(2050)
    assert host(tfx.tfx_depthwise_conv2d_f16(dev16(xs), dev16(ws), None, 1, PAD_VALID))[0, 0, 0, 0] == np.float16(2050)
    # operands that start 2 bytes off a 16-byte boundary take the general paths
    rng = np.random.default_rng(7)
    x = h(rng.uniform(-1, 1, (1, 12, 12, 16)))
    f = h(rng.standard_normal((3, 3, 16, 1)) * 0.4)
    b = h(rng.standard_normal(16) * 0.1)
    off = lambda a: dev16(np.concatenate([np.zeros(1, np.float16), a.ravel()]))[1:].view(a.shape)
    got = host(tfx.tfx_depthwise_conv2d_f16(off(x), off(f), off(b), 1, PAD_SAME, ACT_RELU6))
    assert_close_f16(got, oracle.depthwise_conv2d_f16(x, f, b, 1, PAD_SAME, ACT_RELU6), "unaligned depthwise_f16")
    fp = h(rng.standard_normal((1, 1, 16, 24)) * 0.3)
    bp = h(rng.standard_normal(24) * 0.1)
    out = torch.zeros(12 * 12 * 24 + 2, dtype=torch.float16, device="cuda:0")
    tfx.tfx_conv2d_f16(off(x), off(fp), off(bp), 1, PAD_SAME, ACT_RELU6, out=out[1:-1].view(1, 12, 12, 24))
    o = host(out)
    assert o[0] == 0 and o[-1] == 0
    assert_close_f16(o[1:-1].reshape(1, 12, 12, 24), oracle.conv2d_f16(x, fp, bp, 1, PAD_SAME, ACT_RELU6), "unaligned pointwise f16")
    with pytest.raises(TypeError):
        tfx.tfx_conv2d_f16(dev16(x), dev16(fp).float(), None)


@pytest.fixture(scope="module")
def net16():
    data = inputs.mobilenet_v1_f16(seed=4, batch=1)
    probs, logits, acts = oracle.mobilenet_v1_forward_f16(data["image"], data["weights"], return_activations=True)
    return data, probs, logits, acts


def test_mobilenet_f16_layer_by_layer_each_fed_the_oracle_input(net16):
    import paper_1901_05350_amd as tfx
    data, probs, logits, acts = net16
    w = data["weights"]
    got = host(tfx.tfx_conv2d_f16(dev16(data["image"]), dev16(w["conv0_w"]), dev16(w["conv0_b"]), 2, PAD_SAME, ACT_RELU6))
    assert_close_f16(got, acts[0], "f16 conv0")
    for i in range(13):
        s = oracle.MOBILENET_V1_STRIDES[i]
        got = host(tfx.tfx_depthwise_conv2d_f16(dev16(acts[2 * i]), dev16(w["dw_w"][i]), dev16(w["dw_b"][i]), s, PAD_SAME, ACT_RELU6))
        assert_close_f16(got, acts[2 * i + 1], "f16 dw%d" % (i + 1))
        got = host(tfx.tfx_conv2d_f16(dev16(acts[2 * i + 1]), dev16(w["pw_w"][i]), dev16(w["pw_b"][i]), 1, PAD_SAME, ACT_RELU6))
        assert_close_f16(got, acts[2 * i + 2], "f16 pw%d" % (i + 1))


def end_to_end_bar(got, ref, what, steps):
    """End to end, a one-step rounding difference in one layer's output moves the next layers' sums by a few
    hundredths of a step each, so outputs may differ by a few binary16 steps; the exact bar applies layer by
    layer (above).  Here: at most `steps` binary16 steps at the magnitude of the row's largest entry (a logit
    near zero is a sum of terms of that magnitude)."""
    g, r = got.astype(np.float64), ref.astype(np.float64)
    bound = steps * np.spacing(np.abs(ref).max(axis=-1, keepdims=True)).astype(np.float64)
    assert np.isfinite(g).all() and (np.abs(g - r) <= bound).all(), (what, float(np.abs(g - r).max()), float(bound.min()))


@pytest.mark.parametrize("size,q,classes,batch", [(224, 4, 1000, 1), (224, 4, 1000, 3), (128, 1, 10, 2), (160, 2, 100, 1),
                                                  (192, 3, 1000, 1), (100, 2, 5, 2)])
def test_mobilenet_f16_end_to_end(size, q, classes, batch):
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1_f16(seed=30 + q, batch=batch, image_size=size, width_quarters=q, classes=classes)
    probs, logits = oracle.mobilenet_v1_forward_f16(data["image"], data["weights"])
    model = tfx.MobileNetV1F16(data["weights"], batch=batch, image_size=size, width_quarters=q)
    p, l = model.forward(dev16(data["image"]))
    p, l = host(p).copy(), host(l).copy()
    assert p.dtype == np.float16 and p.shape == (batch, classes)
    end_to_end_bar(l, logits, "f16 logits", 8)
    end_to_end_bar(p, probs, "f16 probs", 16)
    assert np.array_equal(p.argmax(axis=1), probs.argmax(axis=1))
    assert np.abs(p.astype(np.float64).sum(axis=1) - 1).max() < 2e-3
    p2, l2 = model.forward(dev16(data["image"]))
    assert np.array_equal(host(p2), p) and np.array_equal(host(l2), l)


@pytest.mark.parametrize("size,batch,blocks", [(224, 8, (1, 2, 3, 4)), (200, 12, (1, 2, 3)), (224, 3, (1, 2, 3, 5, 13)),
                                               (224, 22, (4, 5)), (200, 27, (3, 4))])
def test_mobilenet_f16_internal_activations(size, batch, blocks):
    """tfx_mobilenet_v1_features_f16 against the oracle's own feature maps.  From 16384 output pixels on, blocks 1, 2,
    3 and 4 of the full-width network run as one filter-stationary launch each (blocks 1 - 3 at batch 8 and 12, block
    4 -- from 6272 pixels on; one slab per unit, 256 output channels in two passes -- at batch 8, 22 and 27; 200 x 200 images give 100 x 100,
    50 x 50 and 25 x 25 maps: ragged last patches, an odd padding under stride 2); batch 3 takes the single-op kernels
    throughout.  The maps are the end of a chain of layers that each round once, so the end-to-end bar
    applies (4 steps at the pixel's largest channel up to block 5, 8 -- the bar of the logits -- beyond), and in the
    first four blocks all but a small share of the
    values -- growing with the depth -- must be the oracle's bit for bit."""
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1_f16(seed=52, batch=batch, image_size=size, width_quarters=4, classes=10)
    probs, logits, acts = oracle.mobilenet_v1_forward_f16(data["image"], data["weights"], return_activations=True)
    model = tfx.MobileNetV1F16(data["weights"], batch=batch, image_size=size, width_quarters=4)
    img = dev16(data["image"])
    for k in blocks:
        got, ref = host(model.features(img, k)), acts[2 * k]
        assert got.dtype == np.float16 and got.shape == ref.shape
        end_to_end_bar(got, ref, "f16 features batch %d size %d block %d" % (batch, size, k), 4 if k <= 5 else 8)
        differ = float((got.view(np.uint16) != ref.view(np.uint16)).mean())
        assert k > 4 or differ <= 0.005 * 4.0 ** (k - 1), (k, differ)
    p, l = model.forward(img)
    end_to_end_bar(host(l), logits, "f16 logits batch %d size %d" % (batch, size), 8)


@pytest.mark.parametrize("batch,blocks", [(8, (1, 2, 3)), (21, (4,))])
def test_mobilenet_f16_nan_and_inf_through_the_fused_blocks_at_large_batch(batch, blocks):
    """A NaN in one image reaches exactly the outputs whose windows hold it, block after block, and no other image;
    +inf and -inf clamp as the oracle's relu6 does (the fused kernel clamps both layers with a median of three and
    must notice the NaN on the side)."""
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1_f16(seed=53, batch=batch, image_size=224, width_quarters=4, classes=10)
    img = data["image"].copy()
    img[3, 100, 37, 1] = np.nan
    img[1, 5, 7, 0] = np.inf
    img[6, 200, 220, 2] = -np.inf
    probs, logits, acts = oracle.mobilenet_v1_forward_f16(img, data["weights"], return_activations=True)
    model = tfx.MobileNetV1F16(data["weights"], batch=batch, image_size=224, width_quarters=4)
    for k in blocks:
        got, ref = host(model.features(dev16(img), k)), acts[2 * k]
        assert np.isnan(ref).any() and not np.isnan(ref[3]).all() and not np.isnan(np.delete(ref, 3, axis=0)).any()
        assert np.array_equal(np.isnan(got), np.isnan(ref)), "NaN positions after block %d" % k
        keep = ~np.isnan(ref).any(axis=-1)
        end_to_end_bar(got[keep], ref[keep], "finite pixels after block %d" % k, 4)


@pytest.mark.parametrize("size,q,classes,batch", [(64, 1, 40, 16), (96, 2, 1000, 17), (64, 4, 8, 40), (64, 1, 37, 16),
                                                  (64, 2, 24, 1), (128, 1, 16, 3), (64, 1, 1001, 5)])
def test_mobilenet_f16_tail_at_large_batch(size, q, classes, batch):
    """With a class count that is a multiple of 8 the tail is pool, GEMM, softmax as three launches, with the pooled
    vectors -- and the logits, if the caller passes no buffer for them -- in the workspace; 37 and 1001 classes take
    the two-launch tail.  With and without a logits buffer the probabilities have the same bits."""
    import ctypes
    import torch
    import paper_1901_05350_amd as tfx
    data = inputs.mobilenet_v1_f16(seed=60 + classes, batch=batch, image_size=size, width_quarters=q, classes=classes)
    probs, logits = oracle.mobilenet_v1_forward_f16(data["image"], data["weights"])
    model = tfx.MobileNetV1F16(data["weights"], batch=batch, image_size=size, width_quarters=q)
    img = dev16(data["image"])
    p, l = model.forward(img)
    p, l = host(p).copy(), host(l).copy()
    end_to_end_bar(l, logits, "f16 logits", 8)
    end_to_end_bar(p, probs, "f16 probs", 16)
    assert np.array_equal(p.argmax(axis=1), probs.argmax(axis=1))
    p2 = torch.zeros_like(model.probs)
    rc = tfx.lib().tfx_mobilenet_v1_forward_f16(ctypes.byref(model.variant), img.data_ptr(), batch, ctypes.byref(model.struct),
                                                model.workspace.data_ptr(), model.workspace.numel(), p2.data_ptr(), None, None)
    assert rc == 0
    assert np.array_equal(host(p2), p)


def test_mobilenet_f16_argument_checks():
    import ctypes
    import paper_1901_05350_amd as tfx
    from paper_1901_05350_amd import binding
    L = tfx.lib()
    V = binding.TfxVariant
    n32 = tfx.tfx_mobilenet_v1_variant_workspace_bytes(V(224, 4, 1000), 1)
    n16 = int(L.tfx_mobilenet_v1_workspace_bytes_f16(ctypes.byref(V(224, 4, 1000)), 1))
    assert 0 < n16 < n32 and n16 % 256 == 0
    assert int(L.tfx_mobilenet_v1_workspace_bytes_f16(ctypes.byref(V(224, 9, 1000)), 1)) == 0
    data = inputs.mobilenet_v1_f16(seed=4, batch=1, image_size=64, width_quarters=1, classes=10)
    model = tfx.MobileNetV1F16(data["weights"], batch=1, image_size=64, width_quarters=1)
    img = dev16(data["image"])
    rc = L.tfx_mobilenet_v1_forward_f16(ctypes.byref(model.variant), img.data_ptr(), 1, ctypes.byref(model.struct),
                                        model.workspace.data_ptr(), 16, model.probs.data_ptr(), None, None)
    assert rc == -5
    rc = L.tfx_mobilenet_v1_forward_f16(ctypes.byref(V(64, 0, 10)), img.data_ptr(), 1, ctypes.byref(model.struct),
                                        model.workspace.data_ptr(), model.workspace.numel(), model.probs.data_ptr(), None, None)
    assert rc == -3
