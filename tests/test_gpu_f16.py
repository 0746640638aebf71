"""GPU parity: element-wise addition and batchMatMul on 16-bit float storage against the CPU oracle."""
import numpy as np
import pytest

import oracle
from paper_1901_05350_amd import inputs
from util import assert_close_f16, dev, dev16, host

pytestmark = pytest.mark.gpu


def bits(a):
    return np.asarray(a).view(np.uint32 if a.dtype == np.float32 else np.uint16)


def same_bits(got, ref):
    nan = np.isnan(ref)
    return np.array_equal(np.isnan(got), nan) and np.array_equal(bits(got)[~nan], bits(ref)[~nan])


@pytest.mark.parametrize("n", [1, 5, 4095, 4096, 4097, 8192, (1 << 20) + 3])
def test_add_f32_bit_exact(n):
    import paper_1901_05350_amd as tfx
    d = inputs.add_operands(seed=8, n=n, dtype=np.float32)
    got = host(tfx.tfx_add(dev(d["a"]), dev(d["b"])))
    assert same_bits(got, oracle.add(d["a"], d["b"]))


@pytest.mark.parametrize("n", [1, 7, 8191, 8192, 8193, 16384, (1 << 20) + 5])
def test_add_f16_bit_exact(n):
    import paper_1901_05350_amd as tfx
    d = inputs.add_operands(seed=9, n=n, dtype=np.float16)
    got = host(tfx.tfx_add_f16(dev16(d["a"]), dev16(d["b"])))
    assert same_bits(got, oracle.add_f16(d["a"], d["b"]))


def test_add_special_values_empty_unaligned_and_in_place():
    import torch
    import paper_1901_05350_amd as tfx
    # every pair from a set of special binary16 patterns (ties, subnormals, signed zeros, overflow, inf, nan)
    pats = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x03ff, 0x0400, 0x3c00, 0x3c01, 0xbc00, 0x6800, 0x6801, 0x7bff,
                     0xfbff, 0x7c00, 0xfc00, 0x7e00, 0x1400, 0x1401], dtype=np.uint16)
    a, b = [m.ravel().view(np.float16) for m in np.meshgrid(pats, pats, indexing="ij")]
    assert same_bits(host(tfx.tfx_add_f16(dev16(a), dev16(b))), oracle.add_f16(a, b))
    f = np.array([0.0, -0.0, 1.0, 16777216.0, 3e38, np.inf, -np.inf, np.nan, 1e-45, -1e-45], dtype=np.float32)
    x, y = [m.ravel() for m in np.meshgrid(f, f, indexing="ij")]
    with np.errstate(all="ignore"):
        assert same_bits(host(tfx.tfx_add(dev(x), dev(y))), oracle.add(x, y))
    # empty
    e = torch.empty(0, dtype=torch.float32, device="cuda:0")
    assert tfx.tfx_add(e, e).numel() == 0
    # operands that are not 16-byte aligned take the scalar path
    d = inputs.add_operands(seed=10, n=10001, dtype=np.float32)
    A, B = dev(np.concatenate([[0], d["a"]])), dev(np.concatenate([[0, 0, 0], d["b"]]))
    out = torch.zeros(10003, dtype=torch.float32, device="cuda:0")
    tfx.tfx_add(A[1:], B[3:], out=out[1:10002])
    o = host(out)
    assert same_bits(o[1:10002], oracle.add(d["a"], d["b"])) and o[0] == 0 and o[10002] == 0
    h = inputs.add_operands(seed=11, n=9001, dtype=np.float16)
    A16 = dev16(np.concatenate([np.zeros(1, np.float16), h["a"]]))
    assert same_bits(host(tfx.tfx_add_f16(A16[1:], dev16(h["b"]))), oracle.add_f16(h["a"], h["b"]))
    # in place: out is one of the operands
    p, q = dev(d["a"]), dev(d["b"])
    tfx.tfx_add(p, q, out=p)
    assert same_bits(host(p), oracle.add(d["a"], d["b"]))
    big = inputs.add_operands(seed=12, n=40000, dtype=np.float16)
    p, q = dev16(big["a"]), dev16(big["b"])
    tfx.tfx_add_f16(p, q, out=q)
    assert same_bits(host(q), oracle.add_f16(big["a"], big["b"]))
    with pytest.raises(TypeError):
        tfx.tfx_add(dev(d["a"]), dev16(h["a"]))


def run_mm(d, act=oracle.ACT_NONE):
    import paper_1901_05350_amd as tfx
    got = host(tfx.tfx_batch_matmul_f16(dev16(d["a"]), dev16(d["b"]), d["transpose_a"], d["transpose_b"],
                                        None if d["bias"] is None else dev16(d["bias"]), act))
    ref = oracle.batch_matmul_f16(d["a"], d["b"], d["transpose_a"], d["transpose_b"], d["bias"], act)
    return got, ref


@pytest.mark.parametrize("ta,tb", [(False, False), (True, False), (False, True), (True, True)])
@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (3, 37, 29, 53), (2, 130, 70, 64), (1, 64, 64, 200), (2, 300, 200, 136)])
def test_matmul_f16_layouts_and_ragged_shapes(ta, tb, shape):
    b, m, n, k = shape
    d = inputs.batch_matmul_f16(seed=30 + m, batch=b, m=m, n=n, k=k, transpose_a=ta, transpose_b=tb, bias=True)
    got, ref = run_mm(d, oracle.ACT_RELU6 if m % 2 else oracle.ACT_NONE)
    assert_close_f16(got, ref, "f16 matmul %r ta=%d tb=%d" % (shape, ta, tb))


@pytest.mark.parametrize("shape,ta,tb", [((1, 256, 256, 64), False, True), ((4, 512, 1024, 128), False, True),
                                         ((2, 4096, 2048, 64), False, True), ((1, 200, 1000, 1024), False, True),
                                         ((1, 3136, 128, 128), False, True), ((1, 2048, 2100, 72), False, True),
                                         ((1, 2048, 2048, 24), True, False), ((1, 2050, 2047, 33), False, False),
                                         ((1, 100, 72, 8), False, True), ((3, 257, 129, 200), False, True),
                                         ((1, 4100, 4090, 136), False, True), ((2, 1, 1, 16), False, True),
                                         ((1, 2048, 2048, 72), False, False), ((2, 4096, 2048, 64), False, False),
                                         ((1, 3136, 128, 128), False, False), ((3, 100, 8, 8), False, False),
                                         ((1, 4100, 4088, 136), False, False),
                                         ((1, 196, 512, 512), False, False), ((1, 49, 1024, 1024), False, False),
                                         ((1, 3136, 128, 64), False, False), ((2, 50, 40, 72), False, False),
                                         ((1, 12544, 64, 32), False, False), ((1, 700, 520, 1032), False, False)])
def test_matmul_f16_tile_configurations(shape, ta, tb):
    """Each tile size of the 16-byte-load kernel (A [M,K], B stored [N,K]) and of the element-wise
    loader (other layouts); every output is compared."""
    import paper_1901_05350_amd as tfx
    b, m, n, k = shape
    d = inputs.batch_matmul_f16(seed=40 + n, batch=b, m=m, n=n, k=k, transpose_a=ta, transpose_b=tb, bias=True)
    got = host(tfx.tfx_batch_matmul_f16(dev16(d["a"]), dev16(d["b"]), ta, tb, dev16(d["bias"]), oracle.ACT_RELU))
    ref = oracle.batch_matmul_f16(d["a"], d["b"], ta, tb, d["bias"], oracle.ACT_RELU)
    assert_close_f16(got, ref, "f16 matmul %r" % (shape,))


def test_matmul_f16_rounding_overflow_subnormals_and_nan():
    import paper_1901_05350_amd as tfx
    mm = lambda a, b, **kw: host(tfx.tfx_batch_matmul_f16(dev16(a), dev16(b), **kw))
    # the sum is taken wider than binary16 and rounded once
    a = np.array([[[2048, 1, 1, 0, 0, 0, 0, 0]]], dtype=np.float16)
    b = np.ones((1, 8, 1), dtype=np.float16)
    assert mm(a, b)[0, 0, 0] == np.float16(2050)
    a = np.array([[[1, 2.0 ** -11, 2.0 ** -11, 0, 0, 0, 0, 0]]], dtype=np.float16)
    assert mm(a, b)[0, 0, 0].view(np.uint16) == 0x3c01
    # overflow saturates to infinity
    a = np.full((1, 1, 8), 200, dtype=np.float16)
    b = np.full((1, 8, 1), 200, dtype=np.float16)
    assert np.isposinf(mm(a, b)[0, 0, 0]) and np.isneginf(mm(-a, b)[0, 0, 0])
    # subnormal operands and subnormal results are kept: 2^-24 * 2^10 = 2^-14, 2^-24 * 1 = 2^-24
    a = np.zeros((1, 2, 8), dtype=np.float16)
    a[0, 0, 0] = a[0, 1, 0] = np.float16(2.0 ** -24)
    b = np.zeros((1, 8, 2), dtype=np.float16)
    b[0, 0, 0], b[0, 0, 1] = 1024, 1
    got = mm(a, b)
    assert np.array_equal(got.view(np.uint16), oracle.batch_matmul_f16(a, b).view(np.uint16))
    assert got[0, 0, 0] == np.float16(2.0 ** -14) and got[0, 0, 1] == np.float16(2.0 ** -24)
    # NaN and Inf propagate when there is no activation
    a = np.ones((1, 4, 8), dtype=np.float16)
    b = np.ones((1, 8, 4), dtype=np.float16)
    a[0, 1, 3], a[0, 2, 5] = np.nan, np.inf
    got, ref = mm(a, b), oracle.batch_matmul_f16(a, b)
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(np.isinf(got), np.isinf(ref))
    assert np.isnan(got[0, 1]).all() and np.isposinf(got[0, 2]).all() and (got[0, 0] == 8).all()


def test_matmul_f16_unaligned_and_output_buffer():
    import torch
    import paper_1901_05350_amd as tfx
    d = inputs.batch_matmul_f16(seed=50, batch=1, m=96, n=72, k=64, bias=True)
    ref = oracle.batch_matmul_f16(d["a"], d["b"], False, True, d["bias"])
    # operands and result offset by one element: neither 16-byte loads nor 8-byte stores apply
    A = dev16(np.concatenate([np.zeros(1, np.float16), d["a"].ravel()]))[1:].view(1, 96, 64)
    B = dev16(np.concatenate([np.zeros(1, np.float16), d["b"].ravel()]))[1:].view(1, 72, 64)
    out = torch.zeros(96 * 72 + 2, dtype=torch.float16, device="cuda:0")
    tfx.tfx_batch_matmul_f16(A, B, False, True, dev16(d["bias"]), out=out[1:-1].view(1, 96, 72))
    o = host(out)
    assert o[0] == 0 and o[-1] == 0
    assert_close_f16(o[1:-1].reshape(1, 96, 72), ref, "unaligned f16 matmul")
    with pytest.raises(tfx.TfxError) as e:
        tfx.tfx_batch_matmul_f16(dev16(d["a"]), dev16(d["b"]))          # K mismatch without transposeB
    assert e.value.status == -2


def test_matmul_f16_full_size():
    """8 x 1024^3 with transposeB, the configuration the benchmark times; every output is compared."""
    import paper_1901_05350_amd as tfx
    d = inputs.batch_matmul_f16(seed=6)
    got = host(tfx.tfx_batch_matmul_f16(dev16(d["a"]), dev16(d["b"]), False, True))
    ref = oracle.batch_matmul_f16(d["a"], d["b"], False, True)
    frac = assert_close_f16(got, ref, "8x1024^3 f16")
    assert frac < 0.05   # only sums near a rounding boundary may land on the neighbouring binary16 value
