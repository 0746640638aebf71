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
