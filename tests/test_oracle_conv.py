"""Pins for the oracle's conv2d / depthwiseConv2d / epilogue (CPU only).

The paper gives the index order of the conv2d input (batch, row, column, depth: Section 4.1)
and nothing else, so the ops are pinned by what the mathematics fixes: 1x1 convolution is a
matrix product, one-hot filters are shifted copies, all-ones inputs count in-bounds taps, tiny
integer cases are brute-forced with independent pure-Python loops, and torch's float64
convolution (explicitly padded) is a library special case.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from oracle import ACT_NONE, ACT_RELU, ACT_RELU6, PAD_SAME, PAD_VALID


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def ints(r, shape, lo=-3, hi=4):
    return r.integers(lo, hi, shape).astype(np.float32)


# ---------- independent brute force: pure Python, integers, explicit zero-padded copy ----------
def brute_conv(x, w, bias, sh, sw, pads, act, depthwise=False):
    n_, h_, w_, c_ = x.shape
    fh, fw = w.shape[:2]
    pt, pb, pl, pr = pads
    xp = np.zeros((n_, h_ + pt + pb, w_ + pl + pr, c_), dtype=np.float64)
    xp[:, pt:pt + h_, pl:pl + w_, :] = x
    oh = (xp.shape[1] - fh) // sh + 1
    ow = (xp.shape[2] - fw) // sw + 1
    oc = c_ * w.shape[3] if depthwise else w.shape[3]
    y = np.zeros((n_, oh, ow, oc), dtype=np.float64)
    for n, i, j, o in itertools.product(range(n_), range(oh), range(ow), range(oc)):
        s = 0.0
        for a, b in itertools.product(range(fh), range(fw)):
            if depthwise:
                c, q = divmod(o, w.shape[3])
                s += xp[n, i * sh + a, j * sw + b, c] * float(w[a, b, c, q])
            else:
                for c in range(c_):
                    s += xp[n, i * sh + a, j * sw + b, c] * float(w[a, b, c, o])
        if bias is not None:
            s += float(bias[o])
        if act == ACT_RELU:
            s = max(s, 0.0)
        elif act == ACT_RELU6:
            s = min(max(s, 0.0), 6.0)
        y[n, i, j, o] = s
    return y


CASES = [
    # n, h, w, ci, co/mult, fh, fw, sh, sw, pad
    (1, 5, 5, 3, 2, 3, 3, 1, 1, PAD_SAME),
    (1, 5, 5, 3, 2, 3, 3, 2, 2, PAD_SAME),
    (2, 4, 6, 2, 3, 3, 3, 2, 2, PAD_SAME),   # even extents: the single pad unit goes after
    (1, 5, 4, 2, 2, 2, 3, 1, 2, PAD_SAME),
    (1, 5, 5, 1, 1, 3, 3, 1, 1, PAD_VALID),
    (1, 6, 5, 2, 2, 3, 2, 2, 1, PAD_VALID),
    (1, 3, 3, 2, 2, 5, 5, 1, 1, PAD_SAME),   # filter larger than the image
    (1, 1, 1, 3, 2, 3, 3, 1, 1, PAD_SAME),
    (1, 7, 5, 2, 2, 1, 1, 3, 2, PAD_SAME),   # 1x1 filter with stride: no padding, subsampling
]


@pytest.mark.parametrize("case", CASES, ids=str)
@pytest.mark.parametrize("act", [ACT_NONE, ACT_RELU6])
def test_conv2d_brute_force_exact(case, act):
    n, h, w, ci, co, fh, fw, sh, sw, pad = case
    r = rng(10)
    x, f, b = ints(r, (n, h, w, ci)), ints(r, (fh, fw, ci, co)), ints(r, (co,))
    oshape, pads = oracle.conv2d_out_shape(x.shape, f.shape, (sh, sw), pad)
    want = brute_conv(x, f, b, sh, sw, pads, act)
    got = oracle.conv2d(x, f, b, (sh, sw), pad, act)
    assert got.shape == oshape == want.shape
    assert np.array_equal(got, want.astype(np.float32))


@pytest.mark.parametrize("case", CASES, ids=str)
@pytest.mark.parametrize("act", [ACT_NONE, ACT_RELU])
def test_depthwise_brute_force_exact(case, act):
    n, h, w, c, mult, fh, fw, sh, sw, pad = case
    r = rng(11)
    x, f, b = ints(r, (n, h, w, c)), ints(r, (fh, fw, c, mult)), ints(r, (c * mult,))
    oshape, pads = oracle.depthwise_conv2d_out_shape(x.shape, f.shape, (sh, sw), pad)
    want = brute_conv(x, f, b, sh, sw, pads, act, depthwise=True)
    got = oracle.depthwise_conv2d(x, f, b, (sh, sw), pad, act)
    assert got.shape == oshape == want.shape
    assert np.array_equal(got, want.astype(np.float32))


# ---------- 1x1 convolution is a matrix product (bit-exact inside the oracle) ----------
def test_pointwise_conv_equals_matmul():
    r = rng(12)
    x = r.uniform(-1, 1, (2, 5, 7, 19)).astype(np.float32)
    f = r.standard_normal((1, 1, 19, 23)).astype(np.float32)
    y = oracle.conv2d(x, f, None, 1, PAD_SAME, ACT_NONE)
    assert np.array_equal(y.reshape(-1, 23), oracle.matmul(x.reshape(-1, 19), f.reshape(19, 23)))
    # and against numpy float64
    want = x.reshape(-1, 19).astype(np.float64) @ f.reshape(19, 23).astype(np.float64)
    assert np.allclose(y.reshape(-1, 23), want, rtol=1e-6, atol=1e-7)


# ---------- one-hot filter = shifted, strided copy with zeros where padded ----------
@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("hw", [(6, 6), (7, 5)])
def test_conv2d_one_hot_filter_is_shifted_copy(stride, hw):
    h, w = hw
    r = rng(13)
    x = r.standard_normal((1, h, w, 3)).astype(np.float32)
    (_, oh, ow, _), (pt, _, pl, _) = oracle.conv2d_out_shape(x.shape, (3, 3, 3, 2), stride, PAD_SAME)
    for kh, kw, c0, o0 in [(0, 0, 0, 0), (2, 2, 1, 1), (1, 0, 2, 0), (0, 2, 1, 1)]:
        f = np.zeros((3, 3, 3, 2), np.float32)
        f[kh, kw, c0, o0] = 1
        y = oracle.conv2d(x, f, None, stride, PAD_SAME, ACT_NONE)
        assert not y[..., 1 - o0].any()
        for i in range(oh):
            for j in range(ow):
                ih, iw = i * stride - pt + kh, j * stride - pl + kw
                want = x[0, ih, iw, c0] if (0 <= ih < h and 0 <= iw < w) else 0.0
                assert y[0, i, j, o0] == want


def test_depthwise_one_hot_tap_shifts_one_channel():
    r = rng(14)
    x = r.standard_normal((1, 6, 6, 4)).astype(np.float32)
    f = np.zeros((3, 3, 4, 2), np.float32)
    f[0, 2, 3, 1] = 1        # top-right tap of channel 3, multiplier slot 1 -> output channel 7
    y = oracle.depthwise_conv2d(x, f, None, 2, PAD_SAME, ACT_NONE)   # even input, stride 2: pad (0,1)
    assert y.shape == (1, 3, 3, 8)
    assert not y[..., :7].any()
    for i in range(3):
        for j in range(3):
            ih, iw = 2 * i + 0, 2 * j + 2
            want = x[0, ih, iw, 3] if iw < 6 else 0.0
            assert y[0, i, j, 7] == want


# ---------- all-ones input and filter count the in-bounds taps ----------
def test_all_ones_tap_counts_stride1():
    ci = 5
    y = oracle.conv2d(np.ones((1, 6, 7, ci), np.float32), np.ones((3, 3, ci, 2), np.float32), None, 1, PAD_SAME)
    assert y[0, 2, 3, 0] == 9 * ci and y[0, 0, 3, 1] == 6 * ci and y[0, 3, 0, 0] == 6 * ci
    for (i, j) in [(0, 0), (0, 6), (5, 0), (5, 6)]:
        assert y[0, i, j, 0] == 4 * ci
    d = oracle.depthwise_conv2d(np.ones((1, 6, 7, ci), np.float32), np.ones((3, 3, ci, 1), np.float32), None, 1, PAD_SAME)
    assert d[0, 2, 3, 0] == 9 and d[0, 0, 3, 1] == 6 and d[0, 5, 6, 4] == 4


def test_all_ones_tap_counts_stride2_even_input_pads_after():
    # 8x8 input, 3x3, stride 2, SAME: pad (0,1).  The top-left output sees all 9 taps,
    # the last row/column lose one tap row/column, the bottom-right corner keeps 4.
    ci = 3
    y = oracle.conv2d(np.ones((1, 8, 8, ci), np.float32), np.ones((3, 3, ci, 1), np.float32), None, 2, PAD_SAME)
    assert y.shape == (1, 4, 4, 1)
    assert y[0, 0, 0, 0] == 9 * ci
    assert y[0, 3, 1, 0] == 6 * ci and y[0, 1, 3, 0] == 6 * ci
    assert y[0, 3, 3, 0] == 4 * ci
    d = oracle.depthwise_conv2d(np.ones((1, 8, 8, ci), np.float32), np.ones((3, 3, ci, 1), np.float32), None, 2, PAD_SAME)
    assert d[0, 0, 0, 0] == 9 and d[0, 3, 0, 1] == 6 and d[0, 3, 3, 2] == 4
    # odd input 7x7, stride 2: pad (1,1), corners see 4 taps on all four sides
    y7 = oracle.depthwise_conv2d(np.ones((1, 7, 7, 1), np.float32), np.ones((3, 3, 1, 1), np.float32), None, 2, PAD_SAME)
    assert y7.shape == (1, 4, 4, 1)
    assert y7[0, 0, 0, 0] == 4 and y7[0, 3, 3, 0] == 4 and y7[0, 1, 1, 0] == 9 and y7[0, 0, 2, 0] == 6


# ---------- linearity ----------
def test_conv2d_is_linear_in_input_and_filter():
    r = rng(15)
    x1, x2 = ints(r, (1, 6, 5, 3)), ints(r, (1, 6, 5, 3))
    f1, f2 = ints(r, (3, 3, 3, 4)), ints(r, (3, 3, 3, 4))
    c = lambda x, f: oracle.conv2d(x, f, None, 2, PAD_SAME, ACT_NONE)
    assert np.array_equal(c(x1 + 2 * x2, f1), c(x1, f1) + 2 * c(x2, f1))
    assert np.array_equal(c(x1, f1 - 3 * f2), c(x1, f1) - 3 * c(x1, f2))


# ---------- depthwise = conv2d with a block-diagonal filter; channels are independent ----------
@pytest.mark.parametrize("mult", [1, 2, 3])
@pytest.mark.parametrize("stride", [1, 2])
def test_depthwise_equals_block_diagonal_conv2d(mult, stride):
    r = rng(16)
    c = 4
    x = r.standard_normal((2, 6, 5, c)).astype(np.float32)
    f = r.standard_normal((3, 3, c, mult)).astype(np.float32)
    b = r.standard_normal((c * mult,)).astype(np.float32)
    full = np.zeros((3, 3, c, c * mult), np.float32)
    for ch in range(c):
        for q in range(mult):
            full[:, :, ch, ch * mult + q] = f[:, :, ch, q]
    got = oracle.depthwise_conv2d(x, f, b, stride, PAD_SAME, ACT_RELU6)
    want = oracle.conv2d(x, full, b, stride, PAD_SAME, ACT_RELU6)
    assert np.array_equal(got, want)   # the zero products add exactly nothing


def test_depthwise_channel_independence():
    r = rng(17)
    x = r.standard_normal((1, 5, 5, 3)).astype(np.float32)
    f = r.standard_normal((3, 3, 3, 2)).astype(np.float32)
    y0 = oracle.depthwise_conv2d(x, f)
    x2 = x.copy()
    x2[..., 1] += 1.0
    y1 = oracle.depthwise_conv2d(x2, f)
    changed = np.any(y0 != y1, axis=(0, 1, 2))
    assert changed.tolist() == [False, False, True, True, False, False]


# ---------- library special case: torch float64 convolution with explicit padding ----------
def torch_conv(x, f, b, stride, pads, groups=1):
    pt, pb, pl, pr = pads
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    xt = F.pad(xt, (pl, pr, pt, pb))
    wt = torch.from_numpy(f.astype(np.float64)).permute(3, 2, 0, 1)   # HWIO -> OIHW
    bt = None if b is None else torch.from_numpy(b.astype(np.float64))
    return F.conv2d(xt, wt, bt, stride=stride, groups=groups).permute(0, 2, 3, 1).numpy()


@pytest.mark.parametrize("shape", [(2, 9, 8, 5, 7, 3, 3, 1), (1, 14, 14, 6, 4, 3, 3, 2), (1, 10, 7, 3, 8, 5, 2, 3),
                                   (1, 12, 12, 16, 16, 1, 1, 1)])
@pytest.mark.parametrize("pad", [PAD_SAME, PAD_VALID])
def test_conv2d_against_torch_float64(shape, pad):
    n, h, w, ci, co, fh, fw, s = shape
    r = rng(18)
    x = r.uniform(-1, 1, (n, h, w, ci)).astype(np.float32)
    f = r.standard_normal((fh, fw, ci, co)).astype(np.float32)
    b = r.standard_normal((co,)).astype(np.float32)
    _, pads = oracle.conv2d_out_shape(x.shape, f.shape, s, pad)
    want = torch_conv(x, f, b, s, pads)
    got = oracle.conv2d(x, f, b, s, pad, ACT_NONE)
    assert got.shape == want.shape
    assert np.allclose(got, want, rtol=2e-7, atol=1e-6)
    got6 = oracle.conv2d(x, f, b, s, pad, ACT_RELU6)
    assert np.allclose(got6, np.clip(want, 0, 6), rtol=2e-7, atol=1e-6)


@pytest.mark.parametrize("shape", [(2, 9, 8, 5, 1, 3, 3, 1), (1, 14, 14, 6, 1, 3, 3, 2), (1, 10, 7, 3, 2, 5, 2, 3)])
@pytest.mark.parametrize("pad", [PAD_SAME, PAD_VALID])
def test_depthwise_against_torch_float64(shape, pad):
    n, h, w, c, mult, fh, fw, s = shape
    r = rng(19)
    x = r.uniform(-1, 1, (n, h, w, c)).astype(np.float32)
    f = r.standard_normal((fh, fw, c, mult)).astype(np.float32)
    b = r.standard_normal((c * mult,)).astype(np.float32)
    _, pads = oracle.depthwise_conv2d_out_shape(x.shape, f.shape, s, pad)
    # torch grouped conv: weight [C*mult, 1, fh, fw], output channel c*mult+q uses input channel c
    wt = f.transpose(2, 3, 0, 1).reshape(c * mult, 1, fh, fw)         # [(c,q),1,fh,fw]
    pt, pb, pl, pr = pads
    xt = F.pad(torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2), (pl, pr, pt, pb))
    want = F.conv2d(xt, torch.from_numpy(wt.astype(np.float64)), torch.from_numpy(b.astype(np.float64)),
                    stride=s, groups=c).permute(0, 2, 3, 1).numpy()
    got = oracle.depthwise_conv2d(x, f, b, s, pad, ACT_NONE)
    assert got.shape == want.shape
    assert np.allclose(got, want, rtol=2e-7, atol=1e-6)


# ---------- epilogue: bias first, then activation ----------
def test_bias_only_and_activation_table():
    vals = np.array([-1, 0, 3, 6, 7], np.float32)
    x = np.ones((1, 2, 2, 1), np.float32)
    zero_f = np.zeros((1, 1, 1, 5), np.float32)
    assert oracle.conv2d(x, zero_f, vals, 1, PAD_SAME, ACT_RELU6)[0, 0, 0].tolist() == [0, 0, 3, 6, 6]
    assert oracle.conv2d(x, zero_f, vals, 1, PAD_SAME, ACT_RELU)[0, 1, 1].tolist() == [0, 0, 3, 6, 7]
    assert oracle.conv2d(x, zero_f, vals, 1, PAD_SAME, ACT_NONE)[0, 1, 0].tolist() == [-1, 0, 3, 6, 7]
    zero_d = np.zeros((3, 3, 5, 1), np.float32)
    xd = np.ones((1, 2, 2, 5), np.float32)
    assert oracle.depthwise_conv2d(xd, zero_d, vals, 1, PAD_SAME, ACT_RELU6)[0, 1, 1].tolist() == [0, 0, 3, 6, 6]
    # activation is applied after the bias: conv = -2, bias = +5 -> relu6(3) = 3, not relu6(-2)+5 = 5
    f = np.full((1, 1, 1, 1), -2, np.float32)
    assert oracle.conv2d(np.ones((1, 1, 1, 1), np.float32), f, np.array([5], np.float32), 1, PAD_SAME, ACT_RELU6).item() == 3
    # a tiny bias is not flushed in fp32 (the fp16 epsilon pitfall of Section 4.1, device support)
    tiny = oracle.conv2d(np.ones((1, 1, 1, 1), np.float32), np.zeros((1, 1, 1, 1), np.float32),
                         np.array([1e-8], np.float32), 1, PAD_SAME, ACT_RELU6).item()
    assert tiny == np.float32(1e-8)


def test_nan_and_inf_through_the_activations():
    # a NaN survives relu and relu6 (it must not be erased by a clamp); -inf -> 0; +inf -> inf under relu, 6 under relu6
    vals = np.array([np.nan, np.inf, -np.inf, 2.0], np.float32)
    x = np.ones((1, 1, 1, 1), np.float32)
    zero_f = np.zeros((1, 1, 1, 4), np.float32)
    for fn, xx, ff in ((oracle.conv2d, x, zero_f), (oracle.depthwise_conv2d, np.ones((1, 1, 1, 4), np.float32), np.zeros((1, 1, 4, 1), np.float32))):
        y = fn(xx, ff, vals, 1, PAD_SAME, ACT_NONE)[0, 0, 0]
        assert np.isnan(y[0]) and y[1] == np.inf and y[2] == -np.inf and y[3] == 2
        y = fn(xx, ff, vals, 1, PAD_SAME, ACT_RELU)[0, 0, 0]
        assert np.isnan(y[0]) and y[1] == np.inf and y[2] == 0 and y[3] == 2
        y = fn(xx, ff, vals, 1, PAD_SAME, ACT_RELU6)[0, 0, 0]
        assert np.isnan(y[0]) and y[1] == 6 and y[2] == 0 and y[3] == 2
    # a NaN in the input reaches exactly the outputs whose window holds it (3x3, SAME): a 3x3 patch of one channel
    xi = np.zeros((1, 5, 5, 2), np.float32)
    xi[0, 2, 2, 1] = np.nan
    y = oracle.depthwise_conv2d(xi, np.ones((3, 3, 2, 1), np.float32), None, 1, PAD_SAME, ACT_RELU6)
    want = np.zeros((5, 5), bool)
    want[1:4, 1:4] = True
    assert np.array_equal(np.isnan(y[0, :, :, 1]), want) and not np.isnan(y[0, :, :, 0]).any()
    # in a conv2d the NaN of one input channel reaches every output channel of those pixels, under relu too
    y = oracle.conv2d(xi, np.ones((3, 3, 2, 3), np.float32), None, 1, PAD_SAME, ACT_RELU)
    assert np.array_equal(np.isnan(y[0]), np.repeat(want[:, :, None], 3, axis=2))


def test_relu6_range_on_random_input():
    r = rng(20)
    x = r.uniform(-1, 1, (1, 9, 9, 8)).astype(np.float32)
    f = (r.standard_normal((3, 3, 8, 8)) * 2).astype(np.float32)
    y = oracle.conv2d(x, f, None, 1, PAD_SAME, ACT_RELU6)
    assert y.min() == 0.0 and y.max() == 6.0 and np.isfinite(y).all()


def test_rejects_bad_arguments():
    x = np.ones((1, 4, 4, 2), np.float32)
    with pytest.raises(oracle.OracleError):
        oracle.conv2d(x, np.ones((3, 3, 3, 2), np.float32))           # channel mismatch
    with pytest.raises(oracle.OracleError):
        oracle.conv2d(x, np.ones((5, 5, 2, 2), np.float32), pad=PAD_VALID)   # filter > image
    with pytest.raises(oracle.OracleError):
        oracle.conv2d(x, np.ones((3, 3, 2, 2), np.float32), stride=0)
    with pytest.raises(oracle.OracleError):
        oracle.conv2d(x, np.ones((3, 3, 2, 2), np.float32), act=9)
