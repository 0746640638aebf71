"""Pins for the oracle's 16-bit float storage ops and element-wise addition (CPU only).

Section 4.1: one matMul implementation renders to a 32-bit or a 16-bit float texture; Fig. 3: the
element-wise addition program.  The oracle's own binary16 encode / decode is checked against numpy's
float16 casts (an independent implementation) over every bit pattern, every rounding tie and random
values, and against hand-worked encodings; the ops against float64 numpy, exact integer cases and
exact rational arithmetic.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def all_halfs():
    return np.arange(65536, dtype=np.uint32).astype(np.uint16)


def test_decode_every_bit_pattern():
    h = all_halfs()
    got = oracle.half_to_double(h)
    want = h.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))   # -0.0 keeps its sign


@pytest.mark.parametrize("bits,value", [
    (0x3c00, 1.0), (0xc000, -2.0), (0x7bff, 65504.0), (0x0001, 2.0 ** -24), (0x0400, 2.0 ** -14),
    (0x03ff, 1023 * 2.0 ** -24), (0x3555, 0.333251953125), (0x2e66, 0.0999755859375), (0x7c00, np.inf),
    (0xfc00, -np.inf), (0x0000, 0.0), (0x4248, 3.140625)])
def test_hand_worked_encodings(bits, value):
    assert oracle.half_to_double(np.array([bits], dtype=np.uint16))[0] == value
    assert oracle.double_to_half(np.array([value])).view(np.uint16)[0] == bits


def test_encode_round_trip_of_every_finite_half():
    h = all_halfs()
    v = h.view(np.float16).astype(np.float64)
    finite = np.isfinite(v)
    back = oracle.double_to_half(v[finite]).view(np.uint16)
    assert np.array_equal(back, h[finite])


def test_encode_ties_and_their_neighbours():
    """Midpoints between consecutive halfs go to the even neighbour; one double-ulp to either side
    goes to the nearer one.  Includes the subnormal range and the overflow threshold 65520."""
    pos = np.arange(0, 0x7c00, dtype=np.uint32).astype(np.uint16)           # +0 ... largest finite
    lo = pos.view(np.float16).astype(np.float64)
    hi = np.append(lo[1:], 65536.0)                                         # the value after 65504 on the grid
    mid = (lo + hi) / 2
    cases = np.concatenate([mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf)])
    cases = np.concatenate([cases, -cases])
    with np.errstate(over="ignore"):
        want = cases.astype(np.float16).view(np.uint16)
    got = oracle.double_to_half(cases).view(np.uint16)
    assert np.array_equal(got, want)
    # explicit: ties to even, overflow from 65520 up, largest value that still rounds to 65504
    enc = lambda x: int(oracle.double_to_half(np.array([x])).view(np.uint16)[0])
    assert enc(1.0 + 2.0 ** -11) == 0x3c00 and enc(1.0 + 3 * 2.0 ** -11) == 0x3c02
    assert enc(65520.0) == 0x7c00 and enc(np.nextafter(65520.0, 0)) == 0x7bff and enc(-65520.0) == 0xfc00
    assert enc(2.0 ** -25) == 0x0000 and enc(np.nextafter(2.0 ** -25, 1)) == 0x0001 and enc(3 * 2.0 ** -25) == 0x0002
    assert enc(-0.0) == 0x8000 and enc(1e-30) == 0 and enc(-1e-30) == 0x8000 and enc(1e30) == 0x7c00
    assert enc(float("nan")) & 0x7c00 == 0x7c00 and enc(float("nan")) & 0x3ff != 0


def test_encode_random_values_match_numpy():
    rng = np.random.default_rng(5)
    v = np.concatenate([rng.standard_normal(200000), rng.standard_normal(100000) * 1e-6,
                        np.exp2(rng.uniform(-30, 17, 200000)) * rng.choice([-1.0, 1.0], 200000)])
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    assert np.array_equal(oracle.double_to_half(v).view(np.uint16), want)


def test_add_f32_is_the_correctly_rounded_sum():
    rng = np.random.default_rng(6)
    a = (rng.standard_normal(100001) * np.exp2(rng.integers(-20, 20, 100001))).astype(np.float32)
    b = (rng.standard_normal(100001) * np.exp2(rng.integers(-20, 20, 100001))).astype(np.float32)
    got = oracle.add(a, b)
    assert np.array_equal(got.view(np.uint32), (a + b).view(np.uint32))           # IEEE float add
    assert np.array_equal(got, (a.astype(np.float64) + b.astype(np.float64)).astype(np.float32))
    x = np.array([1.0, -1.0, 0.5, 16777216.0, np.inf, 3e38], dtype=np.float32)
    y = np.array([2.0, 1.0, 0.25, 1.0, 1.0, 3e38], dtype=np.float32)
    with np.errstate(over="ignore"):
        assert np.array_equal(oracle.add(x, y), np.array([3.0, 0.0, 0.75, 16777216.0, np.inf, np.inf], dtype=np.float32))
    assert np.isnan(oracle.add(np.array([np.inf], np.float32), np.array([-np.inf], np.float32))[0])
    assert oracle.add(np.zeros(0, np.float32), np.zeros(0, np.float32)).shape == (0,)
    m = rng.standard_normal((3, 5, 7)).astype(np.float32)
    assert oracle.add(m, m).shape == (3, 5, 7) and np.array_equal(oracle.add(m, m), 2 * m)


def test_add_f16_exact_rational_and_numpy():
    # every pair from a spread of patterns, against exact rational arithmetic rounded by numpy
    pats = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x03ff, 0x0400, 0x0401, 0x3bff, 0x3c00, 0x3c01, 0xbc00, 0x4000,
                     0x4001, 0x6800, 0x6801, 0x6bff, 0x7bff, 0xfbff, 0x7800, 0x1400, 0x1401, 0x2e66, 0x3555, 0xb555],
                    dtype=np.uint16)
    a, b = np.meshgrid(pats, pats, indexing="ij")
    got = oracle.add_f16(a.ravel(), b.ravel()).view(np.uint16)
    vals = pats.view(np.float16).astype(np.float64)
    for i, (x, y) in enumerate(zip(a.ravel(), b.ravel())):
        fx = Fraction(float(np.array([x], np.uint16).view(np.float16)[0]))
        fy = Fraction(float(np.array([y], np.uint16).view(np.float16)[0]))
        s = fx + fy                      # exact; any such sum is representable in double
        assert Fraction(float(s)) == s
        with np.errstate(over="ignore"):
            want = np.array([float(s)]).astype(np.float16).view(np.uint16)[0]
        if s == 0:                       # x + (-x) = +0, (-0) + (-0) = -0
            want = 0x8000 if (x & 0x8000 and y & 0x8000) else 0
        assert got[i] == want, (hex(x), hex(y), hex(got[i]), hex(want))
    # random, against numpy's float16 addition (fp32 add then one more rounding: harmless for 11-bit operands)
    rng = np.random.default_rng(7)
    p = rng.integers(0, 0x7c00, 200000).astype(np.uint16) | (rng.integers(0, 2, 200000).astype(np.uint16) << 15)
    q = rng.integers(0, 0x7c00, 200000).astype(np.uint16) | (rng.integers(0, 2, 200000).astype(np.uint16) << 15)
    with np.errstate(over="ignore"):
        want = (p.view(np.float16) + q.view(np.float16)).view(np.uint16)
    assert np.array_equal(oracle.add_f16(p, q).view(np.uint16), want)


def test_matmul_f16_exact_small_integer_case():
    # integers small enough that every product, sum and result is exact in binary16
    a = np.array([[[1, 2, 3], [4, 5, 6]]], dtype=np.float16)                   # [1,2,3]
    b = np.array([[[1, 0], [0, 1], [2, -1]]], dtype=np.float16)                # [1,3,2]
    want = np.array([[[7, -1], [16, -1]]], dtype=np.float16)
    assert np.array_equal(oracle.batch_matmul_f16(a, b), want)
    # the same product through every transpose combination
    at, bt = np.ascontiguousarray(a.transpose(0, 2, 1)), np.ascontiguousarray(b.transpose(0, 2, 1))
    assert np.array_equal(oracle.batch_matmul_f16(at, b, transpose_a=True), want)
    assert np.array_equal(oracle.batch_matmul_f16(a, bt, transpose_b=True), want)
    assert np.array_equal(oracle.batch_matmul_f16(at, bt, transpose_a=True, transpose_b=True), want)
    # bias then activation: relu6 clamps 7+1 and 16+1 to 6, -1-2 to 0
    bias = np.array([1, -2], dtype=np.float16)
    assert np.array_equal(oracle.batch_matmul_f16(a, b, bias=bias, act=oracle.ACT_RELU6),
                          np.array([[[6, 0], [6, 0]]], dtype=np.float16))
    assert np.array_equal(oracle.batch_matmul_f16(a, b, bias=bias, act=oracle.ACT_RELU),
                          np.array([[[8, 0], [17, 0]]], dtype=np.float16))
    assert np.array_equal(oracle.batch_matmul_f16(a, b, bias=bias), np.array([[[8, -3], [17, -3]]], dtype=np.float16))


def test_matmul_f16_rounds_once_from_the_exact_sum():
    # 2048 + 1 + 1: summing in binary16 would stay at 2048 (spacing 2); the exact sum 2050 is representable
    a = np.array([[[2048, 1, 1]]], dtype=np.float16)
    b = np.ones((1, 3, 1), dtype=np.float16)
    assert oracle.batch_matmul_f16(a, b)[0, 0, 0] == np.float16(2050)
    # 1 + 2^-11 + 2^-11 = 1 + 2^-10 exactly: rounding after each addition would give 1
    a = np.array([[[1, 2.0 ** -11, 2.0 ** -11]]], dtype=np.float16)
    assert oracle.batch_matmul_f16(a, b)[0, 0, 0].view(np.uint16) == 0x3c01
    # overflow of the result saturates to infinity, not to 65504
    a = np.full((1, 1, 4), 200, dtype=np.float16)
    b = np.full((1, 4, 1), 200, dtype=np.float16)
    assert np.isposinf(oracle.batch_matmul_f16(a, b)[0, 0, 0])
    # identity
    rng = np.random.default_rng(8)
    m = rng.standard_normal((2, 9, 9)).astype(np.float16)
    eye = np.broadcast_to(np.eye(9, dtype=np.float16), (2, 9, 9)).copy()
    assert np.array_equal(oracle.batch_matmul_f16(m, eye), m) and np.array_equal(oracle.batch_matmul_f16(eye, m), m)


@pytest.mark.parametrize("ta,tb", [(False, False), (True, False), (False, True), (True, True)])
def test_matmul_f16_against_float64_numpy(ta, tb):
    rng = np.random.default_rng(9 + 2 * ta + tb)
    B, M, N, K = 3, 37, 29, 53
    a = rng.standard_normal((B, K, M) if ta else (B, M, K)).astype(np.float16)
    b = rng.standard_normal((B, N, K) if tb else (B, K, N)).astype(np.float16)
    bias = rng.standard_normal(N).astype(np.float16)
    a64 = a.astype(np.float64).transpose(0, 2, 1) if ta else a.astype(np.float64)
    b64 = b.astype(np.float64).transpose(0, 2, 1) if tb else b.astype(np.float64)
    exact = np.einsum("bmk,bkn->bmn", a64, b64) + bias.astype(np.float64)
    got = oracle.batch_matmul_f16(a, b, ta, tb, bias=bias, act=oracle.ACT_RELU6)
    want = np.clip(exact, 0.0, 6.0).astype(np.float16)
    # float64 summation order differs between the two (1e-16 relative): allow the one-in-a-million
    # element whose exact sum sits on a rounding boundary to differ by one binary16 step
    diff = np.abs(got.view(np.uint16).astype(np.int32) - want.view(np.uint16).astype(np.int32))
    assert diff.max() <= 1 and (diff != 0).sum() <= 1


def test_matmul_f16_brute_force_rationals():
    rng = np.random.default_rng(10)
    a = rng.standard_normal((1, 4, 6)).astype(np.float16)
    b = (rng.standard_normal((1, 6, 5)) * 8).astype(np.float16)
    got = oracle.batch_matmul_f16(a, b)
    for i in range(4):
        for j in range(5):
            s = sum(Fraction(float(a[0, i, k])) * Fraction(float(b[0, k, j])) for k in range(6))
            want = oracle.double_to_half(np.array([float(s)]))[0]      # float(Fraction) is correctly rounded
            lo, hi = sorted((float(np.nextafter(want, np.float16(-np.inf))), float(np.nextafter(want, np.float16(np.inf)))))
            assert abs(Fraction(float(got[0, i, j])) - s) <= min(abs(Fraction(lo) - s), abs(Fraction(hi) - s))
            assert got[0, i, j] == want


def test_f16_argument_checks():
    a = np.zeros((2, 3, 4), np.float16)
    with pytest.raises(oracle.OracleError):
        oracle.batch_matmul_f16(a, np.zeros((2, 5, 6), np.float16))          # K mismatch
    with pytest.raises(oracle.OracleError):
        oracle.batch_matmul_f16(a, np.zeros((3, 4, 6), np.float16))          # batch mismatch
    with pytest.raises(oracle.OracleError):
        oracle.batch_matmul_f16(a, np.zeros((2, 4, 6), np.float16), act=7)
    with pytest.raises(TypeError):
        oracle.batch_matmul_f16(np.zeros((2, 3, 4), np.float32), np.zeros((2, 4, 6), np.float16))


# ---------------------------------------------------------------------------------------------
# conv2d / depthwiseConv2d / MobileNet tail on 16-bit float storage
# ---------------------------------------------------------------------------------------------
def conv_f64(x, w, bias, stride, pad, depthwise=False):
    """Independent float64 reference: explicit zero padding (shape rule pinned elsewhere) + window sums in numpy."""
    x, w = x.astype(np.float64), w.astype(np.float64)
    shape_fn = oracle.depthwise_conv2d_out_shape if depthwise else oracle.conv2d_out_shape
    (n, oh, ow, oc), (pt, pb, pl, pr) = shape_fn(x.shape, w.shape, stride, pad)
    xp = np.pad(x, ((0, 0), (pt, pb), (pl, pr), (0, 0)))
    out = np.zeros((n, oh, ow, oc))
    fh, fw = w.shape[:2]
    for kh in range(fh):
        for kw in range(fw):
            win = xp[:, kh:kh + (oh - 1) * stride + 1:stride, kw:kw + (ow - 1) * stride + 1:stride, :]
            if depthwise:
                out += (win[..., :, None] * w[kh, kw][None, None, None]).reshape(n, oh, ow, oc)
            else:
                out += win @ w[kh, kw]
    return out if bias is None else out + bias.astype(np.float64)


def steps_apart(a, b):
    """Distance in binary16 steps between finite arrays of equal sign pattern (or across zero)."""
    ka = a.view(np.uint16).astype(np.int32)
    kb = b.view(np.uint16).astype(np.int32)
    ka = np.where(ka & 0x8000, -(ka & 0x7fff), ka)
    kb = np.where(kb & 0x8000, -(kb & 0x7fff), kb)
    return np.abs(ka - kb)


@pytest.mark.parametrize("stride,pad,fh,fw", [(1, oracle.PAD_SAME, 3, 3), (2, oracle.PAD_SAME, 3, 3), (1, oracle.PAD_VALID, 2, 3),
                                              (2, oracle.PAD_VALID, 1, 1), (3, oracle.PAD_SAME, 5, 2)])
def test_conv2d_f16_against_float64_numpy(stride, pad, fh, fw):
    rng = np.random.default_rng(50 + stride + fh)
    x = rng.standard_normal((2, 9, 11, 5)).astype(np.float16)
    w = (rng.standard_normal((fh, fw, 5, 7)) / 3).astype(np.float16)
    b = rng.standard_normal(7).astype(np.float16)
    got = oracle.conv2d_f16(x, w, b, stride, pad, oracle.ACT_RELU6)
    want = np.clip(conv_f64(x, w, b, stride, pad), 0, 6).astype(np.float16)
    d = steps_apart(got, want)
    assert got.shape == want.shape and d.max() <= 1 and (d != 0).sum() <= 1      # float64 summation order only


@pytest.mark.parametrize("stride,pad,mult", [(1, oracle.PAD_SAME, 1), (2, oracle.PAD_SAME, 1), (1, oracle.PAD_VALID, 2), (2, oracle.PAD_SAME, 3)])
def test_depthwise_f16_against_float64_numpy(stride, pad, mult):
    rng = np.random.default_rng(60 + stride + mult)
    x = rng.standard_normal((2, 10, 9, 6)).astype(np.float16)
    w = (rng.standard_normal((3, 3, 6, mult)) / 2).astype(np.float16)
    b = rng.standard_normal(6 * mult).astype(np.float16)
    got = oracle.depthwise_conv2d_f16(x, w, b, stride, pad, oracle.ACT_RELU)
    want = np.maximum(conv_f64(x, w, b, stride, pad, depthwise=True), 0).astype(np.float16)
    d = steps_apart(got, want)
    assert got.shape == want.shape and d.max() <= 1 and (d != 0).sum() <= 1


def test_conv_f16_exact_cases():
    rng = np.random.default_rng(70)
    # small integers: every product and sum is exact in binary16, so the fp32 oracle gives the same numbers
    x = rng.integers(-4, 5, (2, 7, 8, 4)).astype(np.float16)
    w = rng.integers(-3, 4, (3, 3, 4, 5)).astype(np.float16)
    b = rng.integers(-5, 6, 5).astype(np.float16)
    for stride in (1, 2):
        got = oracle.conv2d_f16(x, w, b, stride, oracle.PAD_SAME, oracle.ACT_NONE)
        ref32 = oracle.conv2d(x.astype(np.float32), w.astype(np.float32), b.astype(np.float32), stride, oracle.PAD_SAME, oracle.ACT_NONE)
        assert np.array_equal(got.astype(np.float32), ref32)
    wd = rng.integers(-3, 4, (3, 3, 4, 2)).astype(np.float16)
    bd = rng.integers(-5, 6, 8).astype(np.float16)
    got = oracle.depthwise_conv2d_f16(x, wd, bd, 2, oracle.PAD_SAME, oracle.ACT_RELU6)
    ref32 = oracle.depthwise_conv2d(x.astype(np.float32), wd.astype(np.float32), bd.astype(np.float32), 2, oracle.PAD_SAME, oracle.ACT_RELU6)
    assert np.array_equal(got.astype(np.float32), ref32)
    # one-hot depthwise tap (kh, kw) = (0, 2) with SAME padding: y[h, w] = x[h - 1, w + 1], zero outside
    xr = rng.standard_normal((1, 5, 6, 3)).astype(np.float16)
    tap = np.zeros((3, 3, 3, 1), np.float16)
    tap[0, 2, :, 0] = 1
    y = oracle.depthwise_conv2d_f16(xr, tap, None, 1, oracle.PAD_SAME, oracle.ACT_NONE)
    want = np.zeros_like(xr)
    want[:, 1:, :-1, :] = xr[:, :-1, 1:, :]
    assert np.array_equal(y.view(np.uint16), want.view(np.uint16))
    # a 1x1 convolution is the matMul of the pixel rows with the filter (same sums, same order: same bits)
    xc = rng.standard_normal((2, 6, 5, 16)).astype(np.float16)
    wc = rng.standard_normal((1, 1, 16, 24)).astype(np.float16)
    bc = rng.standard_normal(24).astype(np.float16)
    yc = oracle.conv2d_f16(xc, wc, bc, 1, oracle.PAD_SAME, oracle.ACT_RELU6)
    ym = oracle.batch_matmul_f16(xc.reshape(1, 60, 16), wc.reshape(1, 16, 24), bias=bc, act=oracle.ACT_RELU6)
    assert np.array_equal(yc.reshape(1, 60, 24).view(np.uint16), ym.view(np.uint16))
    # one rounding: 2048 + 1 + 1 over three taps is 2050, not 2048
    xs = np.array([2048, 1, 1], np.float16).reshape(1, 1, 3, 1)
    ws = np.ones((1, 3, 1, 1), np.float16)
    assert oracle.conv2d_f16(xs, ws, None, 1, oracle.PAD_VALID)[0, 0, 0, 0] == np.float16(2050)
    assert oracle.depthwise_conv2d_f16(xs, ws, None, 1, oracle.PAD_VALID)[0, 0, 0, 0] == np.float16(2050)


def test_pool_and_softmax_f16():
    x = np.array([1, 2, 3, 4], np.float16).reshape(1, 2, 2, 1)
    assert oracle.global_avg_pool_f16(x)[0, 0] == np.float16(2.5)
    rng = np.random.default_rng(71)
    x = rng.standard_normal((3, 7, 7, 10)).astype(np.float16)
    got = oracle.global_avg_pool_f16(x)
    for n in range(3):
        for c in range(10):
            s = sum(Fraction(float(v)) for v in x[n, :, :, c].ravel()) / 49
            lo, hi = float(s) - abs(float(s)) * 1e-15, float(s) + abs(float(s)) * 1e-15    # float(Fraction) is correctly rounded
            assert got[n, c] in (oracle.double_to_half(np.array([lo]))[0], oracle.double_to_half(np.array([hi]))[0])
    # softmax: three equal logits give 1/3 -> 0x3555; shift invariance; agreement with float64 numpy
    assert np.array_equal(oracle.softmax_f16(np.full((1, 3), 5, np.float16)).view(np.uint16), np.full((1, 3), 0x3555, np.uint16))
    l = (rng.standard_normal((4, 1000)) * 3).astype(np.float16)
    p = oracle.softmax_f16(l)
    z = l.astype(np.float64)
    e = np.exp(z - z.max(axis=1, keepdims=True))
    want = (e / e.sum(axis=1, keepdims=True)).astype(np.float16)
    d = steps_apart(p, want)
    assert d.max() <= 1 and (d != 0).sum() <= 4
    assert np.abs(p.astype(np.float64).sum(axis=1) - 1).max() < 2e-3          # each of 1000 terms rounded to 11 bits
    assert np.array_equal(p.argmax(axis=1), z.argmax(axis=1))
    big = np.array([[60000, 60000, -60000]], np.float16)
    assert np.array_equal(oracle.softmax_f16(big).view(np.uint16), np.array([[0x3800, 0x3800, 0]], np.uint16))


def test_mobilenet_forward_f16_chain():
    from paper_1901_05350_amd import inputs
    d = inputs.mobilenet_v1_f16(seed=13, batch=1, image_size=96, width_quarters=1, classes=10)
    probs, logits, acts = oracle.mobilenet_v1_forward_f16(d["image"], d["weights"], return_activations=True)
    assert probs.dtype == np.float16 and probs.shape == (1, 10) and len(acts) == 28
    assert acts[0].shape == (1, 48, 48, 8) and acts[-2].shape == (1, 3, 3, 256) and acts[-1].shape == (1, 256)
    # each stage is the single op applied to the previous stage
    w = d["weights"]
    a1 = oracle.depthwise_conv2d_f16(acts[0], w["dw_w"][0], w["dw_b"][0], 1, oracle.PAD_SAME, oracle.ACT_RELU6)
    assert np.array_equal(a1.view(np.uint16), acts[1].view(np.uint16))
    assert np.array_equal(oracle.global_avg_pool_f16(acts[-2]).view(np.uint16), acts[-1].view(np.uint16))
    assert np.array_equal(oracle.softmax_f16(logits).view(np.uint16), probs.view(np.uint16))
    # 16-bit storage stays close to the fp32 chain on the same (binary16-representable) inputs
    w32 = {k: ([t.astype(np.float32) for t in v] if isinstance(v, list) else v.astype(np.float32)) for k, v in w.items()}
    p32, l32 = oracle.mobilenet_v1_forward(d["image"].astype(np.float32), w32)
    assert np.abs(logits.astype(np.float64) - l32).max() < 5e-3 and int(probs.argmax()) == int(p32.argmax())
