"""GPU parity: tfx_conv2d / tfx_depthwise_conv2d against the CPU oracle, through the C ABI."""
import itertools

import numpy as np
import pytest

import oracle
from oracle import ACT_NONE, ACT_RELU, ACT_RELU6, PAD_SAME, PAD_VALID
from paper_1901_05350_amd import inputs
from util import assert_close, dev, host

pytestmark = pytest.mark.gpu


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def gpu_conv(x, f, b, stride, pad, act):
    import paper_1901_05350_amd as tfx
    return host(tfx.tfx_conv2d(dev(x), dev(f), None if b is None else dev(b), stride, pad, act))


def gpu_dw(x, f, b, stride, pad, act):
    import paper_1901_05350_amd as tfx
    return host(tfx.tfx_depthwise_conv2d(dev(x), dev(f), None if b is None else dev(b), stride, pad, act))


def test_config_pointwise_conv():
    d = inputs.pointwise_conv(seed=1)
    got = gpu_conv(d["x"], d["filter"], d["bias"], 1, PAD_SAME, ACT_RELU6)
    ref = oracle.conv2d(d["x"], d["filter"], d["bias"], 1, PAD_SAME, ACT_RELU6)
    assert got.shape == (1, 56, 56, 128)
    assert_close(got, ref, "pointwise 56x56x128->128")
    assert got.min() == 0.0 and (ref > 0).mean() > 0.2


@pytest.mark.parametrize("stride", [1, 2])
def test_config_depthwise_conv(stride):
    d = inputs.depthwise_conv(seed=2)
    got = gpu_dw(d["x"], d["filter"], d["bias"], stride, PAD_SAME, ACT_RELU6)
    ref = oracle.depthwise_conv2d(d["x"], d["filter"], d["bias"], stride, PAD_SAME, ACT_RELU6)
    assert got.shape == ((1, 112, 112, 64) if stride == 1 else (1, 56, 56, 64))
    assert_close(got, ref, "depthwise 112x112x64 s%d" % stride)


def test_pointwise_shape_sweep():
    # every MobileNet pointwise GEMM shape plus ragged channel counts and batch > 1
    cases = [(1, 112, 112, 32, 64), (1, 56, 56, 64, 128), (1, 28, 28, 128, 256), (1, 28, 28, 256, 256),
             (1, 14, 14, 256, 512), (1, 14, 14, 512, 512), (1, 7, 7, 512, 1024), (1, 7, 7, 1024, 1024),
             (2, 9, 7, 5, 3), (3, 1, 1, 1, 1), (1, 15, 15, 33, 65), (2, 14, 14, 130, 36), (1, 1, 3, 4, 130)]
    r = rng(21)
    for i, (n, h, w, ci, co) in enumerate(cases):
        x = r.uniform(-1, 1, (n, h, w, ci)).astype(np.float32)
        f = (r.standard_normal((1, 1, ci, co)) * np.sqrt(2.0 / ci)).astype(np.float32)
        b = (r.standard_normal((co,)) * 0.5).astype(np.float32)
        act = [ACT_RELU6, ACT_NONE, ACT_RELU][i % 3]
        bias = None if i % 4 == 3 else b
        for pad in (PAD_SAME, PAD_VALID):
            got = gpu_conv(x, f, bias, 1, pad, act)
            assert_close(got, oracle.conv2d(x, f, bias, 1, pad, act), "pointwise %r" % ((n, h, w, ci, co),))


def test_pointwise_large_m_thin_filters():
    # large N*H*W with the four thin MobileNet filter shapes (filter-stationary kernel), M ragged
    cases = [(6, 112, 112, 32, 64), (2, 181, 183, 64, 128), (2, 181, 183, 128, 128), (4, 129, 130, 128, 256),
             (8, 56, 56, 128, 128), (64, 56, 56, 128, 128)]
    r = rng(22)
    for i, (n, h, w, ci, co) in enumerate(cases):
        x = r.uniform(-1, 1, (n, h, w, ci)).astype(np.float32)
        f = (r.standard_normal((1, 1, ci, co)) * np.sqrt(2.0 / ci)).astype(np.float32)
        b = (r.standard_normal((co,)) * 0.5).astype(np.float32)
        act = [ACT_RELU6, ACT_NONE, ACT_RELU][i % 3]
        got = gpu_conv(x, f, b if i != 1 else None, 1, PAD_SAME, act)
        # every image of the batch, the benchmark's batch 8 and 64 included
        assert_close(got, oracle.conv2d(x, f, b if i != 1 else None, 1, PAD_SAME, act),
                     "pointwise large M %r" % ((n, h, w, ci, co),))


def test_stem_conv_config_shape():
    d = inputs.conv_general(31, 1, 224, 224, 3, 32, 3, 3)
    got = gpu_conv(d["x"], d["filter"], d["bias"], 2, PAD_SAME, ACT_RELU6)
    assert got.shape == (1, 112, 112, 32)
    assert_close(got, oracle.conv2d(d["x"], d["filter"], d["bias"], 2, PAD_SAME, ACT_RELU6), "stem 224x224x3->32")


def test_stem_conv_small_and_ragged():
    r = rng(32)
    for (n, h, w, s, pad) in [(2, 9, 11, 2, PAD_SAME), (1, 8, 8, 2, PAD_SAME), (1, 7, 5, 1, PAD_SAME),
                              (1, 10, 9, 2, PAD_VALID), (1, 3, 3, 3, PAD_VALID), (1, 1, 1, 2, PAD_SAME)]:
        x = r.uniform(-1, 1, (n, h, w, 3)).astype(np.float32)
        f = r.standard_normal((3, 3, 3, 32)).astype(np.float32)
        b = r.standard_normal((32,)).astype(np.float32)
        got = gpu_conv(x, f, b, s, pad, ACT_RELU6)
        assert_close(got, oracle.conv2d(x, f, b, s, pad, ACT_RELU6), "stem %r" % ((n, h, w, s, pad),))


def test_stem_conv_matrix_core_form_slab_walk_and_borders():
    """32 filters take the matrix-core stem kernel: 16-pixel slabs of an output row, interior slabs with
    unconditional loads, border slabs with per-tap checks, a ragged last slab per row, and (batch 20 at 224 x 224:
    15680 slabs for at most 8192 wavefronts) wavefronts that walk over several slabs, across row and image
    boundaries; every image of the large batch is compared."""
    r = rng(36)
    f = r.standard_normal((3, 3, 3, 32)).astype(np.float32)
    b = r.standard_normal((32,)).astype(np.float32)
    for (n, h, w, s, pad, act, bias) in [(1, 40, 75, 2, PAD_SAME, ACT_RELU6, True), (2, 21, 53, 1, PAD_VALID, 0, False),
                                         (1, 35, 130, (2, 1), PAD_SAME, ACT_RELU6, True), (3, 18, 34, 1, PAD_SAME, 0, True),
                                         (1, 50, 64, (1, 2), PAD_VALID, ACT_RELU6, True)]:
        x = r.uniform(-1, 1, (n, h, w, 3)).astype(np.float32)
        got = gpu_conv(x, f, b if bias else None, s, pad, act)
        assert_close(got, oracle.conv2d(x, f, b if bias else None, s, pad, act), "stem %r" % ((n, h, w, s, pad),))
    x = r.uniform(-1, 1, (20, 224, 224, 3)).astype(np.float32)
    got = gpu_conv(x, f, b, 2, PAD_SAME, ACT_RELU6)
    assert got.shape == (20, 112, 112, 32)
    assert_close(got, oracle.conv2d(x, f, b, 2, PAD_SAME, ACT_RELU6), "stem batch 20")


def test_general_conv_sweep():
    r = rng(33)
    hw = [(1, 1), (2, 3), (7, 7), (14, 15)]
    for (h, w), (fh, fw), s, pad, (ci, co) in itertools.product(
            hw, [(3, 3), (2, 5), (1, 1)], [1, 2, 3], [PAD_SAME, PAD_VALID], [(1, 1), (3, 4), (5, 32), (4, 5)]):
        if pad == PAD_VALID and (h < fh or w < fw):
            continue
        if fh == 1 and s == 1:
            continue
        x = r.uniform(-1, 1, (2, h, w, ci)).astype(np.float32)
        f = r.standard_normal((fh, fw, ci, co)).astype(np.float32)
        b = r.standard_normal((co,)).astype(np.float32)
        got = gpu_conv(x, f, b, (s, 1 + (s % 2)), pad, ACT_RELU6)
        ref = oracle.conv2d(x, f, b, (s, 1 + (s % 2)), pad, ACT_RELU6)
        assert_close(got, ref, "conv %r" % ((h, w, fh, fw, s, pad, ci, co),))


def test_conv_implicit_gemm_sweep():
    # enough channels for the matrix-core path: filters 3x3 / 5x2 / 1x1-strided, strides 1-3, both paddings,
    # channel counts that are and are not multiples of 4 (vector and scalar loaders), ragged M and N
    r = rng(35)
    for (n, h, w), (fh, fw), s, pad, (ci, co) in itertools.product(
            [(1, 14, 15), (2, 9, 7), (1, 33, 31)], [(3, 3), (5, 2), (1, 1)], [1, 2, 3], [PAD_SAME, PAD_VALID],
            [(8, 8), (16, 40), (9, 10), (64, 72), (12, 130)]):
        if fh == 1 and s == 1:
            continue
        x = r.uniform(-1, 1, (n, h, w, ci)).astype(np.float32)
        f = (r.standard_normal((fh, fw, ci, co)) * np.sqrt(2.0 / (fh * fw * ci))).astype(np.float32)
        b = (r.standard_normal((co,)) * 0.5).astype(np.float32)
        st = (s, 1 + (s % 2))
        got = gpu_conv(x, f, b, st, pad, ACT_RELU6)
        assert_close(got, oracle.conv2d(x, f, b, st, pad, ACT_RELU6), "implicit gemm %r" % ((n, h, w, fh, fw, s, pad, ci, co),))


def test_conv_3x3_small_maps_tap_per_wavefront():
    """3x3 convolutions of small feature maps with 16 / 32 / 64 / 128 input channels (the kernel that gives every
    filter tap a wavefront and loads the matrix-core operands straight from memory): both paddings, strides 1 and
    2, borders everywhere (maps down to 1 x 1 ... 3 x 3), filter counts that are not multiples of the 32-column tile,
    a one-hot filter that must copy a shifted input channel exactly, and the benchmark's 56 x 56 x 64 -> 64 layer."""
    r = rng(61)
    for ci, (n, h, w), co, s, pad in itertools.product(
            [16, 32, 64, 128], [(1, 1, 1), (1, 3, 3), (2, 7, 5), (1, 14, 14), (3, 8, 9)], [4, 36, 64], [1, 2], [PAD_SAME, PAD_VALID]):
        if pad == PAD_VALID and (h < 3 or w < 3):
            continue
        x = r.uniform(-1, 1, (n, h, w, ci)).astype(np.float32)
        f = (r.standard_normal((3, 3, ci, co)) * np.sqrt(2.0 / (9 * ci))).astype(np.float32)
        b = (r.standard_normal((co,)) * 0.5).astype(np.float32)
        got = gpu_conv(x, f, b, s, pad, ACT_RELU6)
        assert_close(got, oracle.conv2d(x, f, b, s, pad, ACT_RELU6), "conv3x3 small %r" % ((n, h, w, ci, co, s, pad),))
        # one-hot filter: output channel j = input channel c under tap (kh, kw), shifted copy, bit-exact
        kh, kw, c, j = int(r.integers(3)), int(r.integers(3)), int(r.integers(ci)), int(r.integers(co))
        f1 = np.zeros((3, 3, ci, co), np.float32)
        f1[kh, kw, c, j] = 1
        got = gpu_conv(x, f1, None, s, pad, ACT_NONE)
        assert np.array_equal(got, oracle.conv2d(x, f1, None, s, pad, ACT_NONE).astype(np.float32)), (n, h, w, ci, co, s, pad, kh, kw, c, j)
    d = inputs.conv_general(36, 1, 56, 56, 64, 64, 3, 3)
    got = gpu_conv(d["x"], d["filter"], d["bias"], 1, PAD_SAME, ACT_RELU6)
    assert_close(got, oracle.conv2d(d["x"], d["filter"], d["bias"], 1, PAD_SAME, ACT_RELU6), "conv3x3 56x56x64->64")


def test_conv_3x3_large_batches_every_image():
    # 3x3 convolutions at the sizes the benchmark times (batch 8 and 64 of 56 x 56 x 64 -> 64; 128 x 128 and
    # 64 x 64 tiles, XCD-remapped tile order); every output of every image is compared
    for (n, hw, ci, co, s) in [(8, 56, 64, 64, 1), (64, 56, 64, 64, 1), (8, 56, 64, 128, 2), (4, 28, 128, 256, 1),
                               (16, 28, 128, 256, 1)]:
        d = inputs.conv_general(36, n, hw, hw, ci, co, 3, 3)
        got = gpu_conv(d["x"], d["filter"], d["bias"], s, PAD_SAME, ACT_RELU6)
        ref = oracle.conv2d(d["x"], d["filter"], d["bias"], s, PAD_SAME, ACT_RELU6)
        assert_close(got, ref, "conv3x3 %r" % ((n, hw, ci, co, s),))


def test_general_conv_3x3_many_channels():
    d = inputs.conv_general(34, 1, 14, 14, 64, 48, 3, 3)
    got = gpu_conv(d["x"], d["filter"], d["bias"], 1, PAD_SAME, ACT_RELU)
    assert_close(got, oracle.conv2d(d["x"], d["filter"], d["bias"], 1, PAD_SAME, ACT_RELU), "conv 3x3 64->48")


def test_depthwise_fast_path_sweep():
    # 3x3, multiplier 1, channels a multiple of 4: every MobileNet depthwise shape, odd / even
    # extents, tiny images, both strides and both paddings
    r = rng(41)
    shapes = [(1, 112, 112, 32), (1, 56, 56, 128), (1, 28, 28, 256), (1, 14, 14, 512), (1, 7, 7, 1024),
              (2, 15, 14, 8), (3, 1, 1, 4), (1, 2, 3, 12), (1, 3, 3, 4), (2, 33, 9, 64), (1, 5, 70, 20)]
    for (n, h, w, c), s, pad in itertools.product(shapes, [1, 2], [PAD_SAME, PAD_VALID]):
        if pad == PAD_VALID and (h < 3 or w < 3):
            continue
        x = r.uniform(-1, 1, (n, h, w, c)).astype(np.float32)
        f = (r.standard_normal((3, 3, c, 1)) * np.sqrt(2.0 / 9)).astype(np.float32)
        b = (r.standard_normal((c,)) * 0.5).astype(np.float32)
        got = gpu_dw(x, f, b, s, pad, ACT_RELU6)
        assert_close(got, oracle.depthwise_conv2d(x, f, b, s, pad, ACT_RELU6), "dw %r s%d pad%d" % ((n, h, w, c), s, pad))
    x = r.uniform(-1, 1, (1, 9, 9, 8)).astype(np.float32)
    f = r.standard_normal((3, 3, 8, 1)).astype(np.float32)
    assert_close(gpu_dw(x, f, None, 1, PAD_SAME, ACT_NONE), oracle.depthwise_conv2d(x, f, None, 1, PAD_SAME, ACT_NONE),
                 "dw no bias")


@pytest.mark.parametrize("n", [8, 64])
@pytest.mark.parametrize("stride", [1, 2])
def test_depthwise_benchmark_batches_every_image(n, stride):
    # the batch sizes the benchmark times (they select the kernel variants with several rows per
    # thread and the XCD-remapped strip order); every image is compared
    d = inputs.depthwise_conv(seed=2, n=n)
    got = gpu_dw(d["x"], d["filter"], d["bias"], stride, PAD_SAME, ACT_RELU6)
    ref = oracle.depthwise_conv2d(d["x"], d["filter"], d["bias"], stride, PAD_SAME, ACT_RELU6)
    assert_close(got, ref, "depthwise batch %d s%d" % (n, stride))


def test_depthwise_rows_per_thread_variants_ragged_heights():
    # output heights that are not multiples of the 2 / 4 / 6 rows a thread covers, at sizes that
    # select each variant; heights that are multiples of 7 at sizes that select 7 rows per thread
    # (several strips, and a 7-row map as a single strip)
    r = rng(44)
    for (n, h, w, c) in [(16, 37, 45, 64), (44, 53, 61, 32), (200, 31, 33, 32), (4, 9, 200, 128), (36, 28, 45, 128),
                         (48, 7, 9, 1024)]:
        x = r.uniform(-1, 1, (n, h, w, c)).astype(np.float32)
        f = (r.standard_normal((3, 3, c, 1)) * np.sqrt(2.0 / 9)).astype(np.float32)
        b = (r.standard_normal((c,)) * 0.5).astype(np.float32)
        for s in (1, 2):
            got = gpu_dw(x, f, b, s, PAD_SAME, ACT_RELU6)
            assert_close(got, oracle.depthwise_conv2d(x, f, b, s, PAD_SAME, ACT_RELU6), "dw variants %r s%d" % ((n, h, w, c), s))


def test_depthwise_generic_sweep():
    r = rng(42)
    for (h, w), (fh, fw), s, pad, (c, mult) in itertools.product(
            [(1, 1), (3, 2), (7, 7), (14, 15)], [(3, 3), (5, 2), (1, 1)], [1, 2, 3], [PAD_SAME, PAD_VALID],
            [(1, 1), (3, 1), (5, 2), (4, 3), (64, 1)]):
        if pad == PAD_VALID and (h < fh or w < fw):
            continue
        x = r.uniform(-1, 1, (2, h, w, c)).astype(np.float32)
        f = r.standard_normal((fh, fw, c, mult)).astype(np.float32)
        b = r.standard_normal((c * mult,)).astype(np.float32)
        got = gpu_dw(x, f, b, (s, 1 + (s % 2)), pad, ACT_RELU)
        ref = oracle.depthwise_conv2d(x, f, b, (s, 1 + (s % 2)), pad, ACT_RELU)
        assert_close(got, ref, "dw generic %r" % ((h, w, fh, fw, s, pad, c, mult),))


def test_one_hot_tap_is_a_shifted_copy_bit_exact():
    # which side the odd padding unit goes to (stride 2, even input) shows up as a shift
    r = rng(43)
    x = r.standard_normal((1, 8, 8, 4)).astype(np.float32)
    for kh, kw in [(0, 0), (2, 2), (0, 2), (1, 1)]:
        f = np.zeros((3, 3, 4, 1), np.float32)
        f[kh, kw, :, 0] = 1
        for s in (1, 2):
            got = gpu_dw(x, f, None, s, PAD_SAME, ACT_NONE)
            assert np.array_equal(got, oracle.depthwise_conv2d(x, f, None, s, PAD_SAME, ACT_NONE))


def test_epilogue_activation_table_and_tiny_bias():
    vals = np.array([-1, 0, 3, 6, 7, 1e-8, -1e-8, 5.9999995], np.float32)
    x = np.ones((1, 2, 2, 4), np.float32)
    zf = np.zeros((1, 1, 4, 8), np.float32)
    for act in (ACT_NONE, ACT_RELU, ACT_RELU6):
        assert np.array_equal(gpu_conv(x, zf, vals, 1, PAD_SAME, act), oracle.conv2d(x, zf, vals, 1, PAD_SAME, act))
    xd = np.ones((1, 2, 2, 8), np.float32)
    zd = np.zeros((3, 3, 8, 1), np.float32)
    for act in (ACT_NONE, ACT_RELU, ACT_RELU6):
        assert np.array_equal(gpu_dw(xd, zd, vals, 1, PAD_SAME, act), oracle.depthwise_conv2d(xd, zd, vals, 1, PAD_SAME, act))


def test_nan_and_inf_through_the_fused_activations():
    """A NaN passes through relu and relu6 (a clamp must not erase it), -inf becomes 0, +inf the upper bound; a NaN
    in the input reaches exactly the outputs whose window holds it.  Every conv2d / depthwise kernel family: pointwise
    (16-row, tiled and filter-stationary kernels), implicit GEMM 3x3, tap-per-wavefront 3x3, the stems, the direct
    kernel, depthwise fast path and generic."""
    r = rng(46)

    def same(got, ref, what):
        assert np.array_equal(np.isnan(got), np.isnan(ref)), what
        assert np.isnan(ref).any() and not np.isnan(ref).all(), what
        ok = ~np.isnan(ref)
        assert np.array_equal(np.isinf(got[ok]), np.isinf(ref[ok])), what
        fin = ok & ~np.isinf(ref)
        assert_close(got[fin], ref[fin], what)

    conv_cases = [(1, 14, 14, 64, 96, 1, 1, 1), (2, 56, 56, 128, 128, 1, 1, 1), (6, 112, 112, 32, 64, 1, 1, 1),
                  (8, 56, 56, 128, 128, 1, 1, 1), (2, 20, 20, 32, 40, 3, 3, 1), (1, 14, 14, 64, 36, 3, 3, 2),
                  (8, 56, 56, 64, 64, 3, 3, 1), (1, 30, 30, 3, 32, 3, 3, 2), (1, 30, 30, 3, 16, 3, 3, 2),
                  (1, 9, 9, 5, 4, 3, 3, 1)]
    for (n, h, w, ci, co, fh, fw, s) in conv_cases:
        x = r.uniform(-1, 1, (n, h, w, ci)).astype(np.float32)
        f = (r.standard_normal((fh, fw, ci, co)) * np.sqrt(2.0 / (fh * fw * ci))).astype(np.float32)
        b = (r.standard_normal((co,)) * 0.5).astype(np.float32)
        x[n - 1, h // 2, w // 3, ci - 1] = np.nan
        x[0, 1, 2, 0] = np.inf
        x[0, h - 2, w - 1, ci // 2] = -np.inf
        f[..., 0] = np.abs(f[..., 0])          # output channel 0 sees +inf / -inf with a known sign
        for act in (ACT_RELU6, ACT_RELU, ACT_NONE):
            same(gpu_conv(x, f, b, s, PAD_SAME, act), oracle.conv2d(x, f, b, s, PAD_SAME, act),
                 "conv NaN/Inf %r act %d" % ((n, h, w, ci, co, fh, fw, s), act))
    for (n, h, w, c, mult, s) in [(1, 28, 28, 32, 1, 1), (64, 28, 28, 64, 1, 1), (8, 56, 56, 64, 1, 2), (1, 7, 7, 1024, 1, 1),
                                  (2, 9, 11, 5, 2, 1)]:
        x = r.uniform(-1, 1, (n, h, w, c)).astype(np.float32)
        f = (r.standard_normal((3, 3, c, mult)) * np.sqrt(2.0 / 9)).astype(np.float32)
        b = (r.standard_normal((c * mult,)) * 0.5).astype(np.float32)
        x[n - 1, h // 2, w // 3, c - 1] = np.nan
        x[0, 1, 2, 0] = np.inf
        x[0, h - 2, w - 1, c // 2] = -np.inf
        for act in (ACT_RELU6, ACT_RELU, ACT_NONE):
            same(gpu_dw(x, f, b, s, PAD_SAME, act), oracle.depthwise_conv2d(x, f, b, s, PAD_SAME, act),
                 "depthwise NaN/Inf %r act %d" % ((n, h, w, c, mult, s), act))
    # bias-only table: NaN, +inf, -inf straight into each activation, bit for bit
    vals = np.array([np.nan, np.inf, -np.inf, 2.0, np.nan, -1, 7, 0], np.float32)
    x1 = np.ones((1, 2, 2, 4), np.float32)
    for act in (ACT_NONE, ACT_RELU, ACT_RELU6):
        got, ref = gpu_conv(x1, np.zeros((1, 1, 4, 8), np.float32), vals, 1, PAD_SAME, act), oracle.conv2d(x1, np.zeros((1, 1, 4, 8), np.float32), vals, 1, PAD_SAME, act)
        assert np.array_equal(got, ref, equal_nan=True)
        xd = np.ones((1, 2, 2, 8), np.float32)
        got, ref = gpu_dw(xd, np.zeros((3, 3, 8, 1), np.float32), vals, 1, PAD_SAME, act), oracle.depthwise_conv2d(xd, np.zeros((3, 3, 8, 1), np.float32), vals, 1, PAD_SAME, act)
        assert np.array_equal(got, ref, equal_nan=True)


def test_unaligned_buffers_take_the_scalar_paths():
    # tensors that start 4 bytes past a 16-byte boundary: the 128-bit-load kernels must not be chosen
    import torch
    import paper_1901_05350_amd as tfx

    def shifted(a):
        buf = torch.empty(a.size + 1, dtype=torch.float32, device="cuda:0")
        v = buf[1:].view(*a.shape)
        v.copy_(torch.from_numpy(a))
        assert v.data_ptr() % 16 != 0
        return v

    r = rng(45)
    x = r.uniform(-1, 1, (1, 12, 12, 32)).astype(np.float32)
    f = r.standard_normal((1, 1, 32, 64)).astype(np.float32)
    fd = r.standard_normal((3, 3, 32, 1)).astype(np.float32)
    f3 = r.standard_normal((3, 3, 32, 16)).astype(np.float32)
    b = r.standard_normal((64,)).astype(np.float32)
    bd = r.standard_normal((32,)).astype(np.float32)
    b3 = r.standard_normal((16,)).astype(np.float32)
    got = host(tfx.tfx_conv2d(shifted(x), shifted(f), shifted(b), 1, PAD_SAME, ACT_RELU6))
    assert_close(got, oracle.conv2d(x, f, b, 1, PAD_SAME, ACT_RELU6), "pointwise, unaligned operands")
    got = host(tfx.tfx_depthwise_conv2d(shifted(x), shifted(fd), shifted(bd), 2, PAD_SAME, ACT_RELU6))
    assert_close(got, oracle.depthwise_conv2d(x, fd, bd, 2, PAD_SAME, ACT_RELU6), "depthwise, unaligned operands")
    got = host(tfx.tfx_conv2d(shifted(x), shifted(f3), shifted(b3), 1, PAD_SAME, ACT_RELU))
    assert_close(got, oracle.conv2d(x, f3, b3, 1, PAD_SAME, ACT_RELU), "conv 3x3, unaligned operands")
    out = torch.empty(12 * 12 * 64 + 1, dtype=torch.float32, device="cuda:0")[1:].view(1, 12, 12, 64)
    tfx.tfx_conv2d(dev(x), dev(f), dev(b), 1, PAD_SAME, ACT_RELU6, out=out)
    assert_close(host(out), oracle.conv2d(x, f, b, 1, PAD_SAME, ACT_RELU6), "pointwise, unaligned output")
    # large M with the thin filter but a bias that is not 16-byte aligned: not the filter-stationary kernel
    xl = r.uniform(-1, 1, (2, 100, 100, 32)).astype(np.float32)
    got = host(tfx.tfx_conv2d(dev(xl), dev(f), shifted(b), 1, PAD_SAME, ACT_RELU6))
    assert_close(got, oracle.conv2d(xl, f, b, 1, PAD_SAME, ACT_RELU6), "pointwise large M, unaligned bias")
