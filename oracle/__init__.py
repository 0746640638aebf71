"""CPU oracle for the dense ops of the TensorFlow.js paper (arxiv 1901.05350).

TEST INFRASTRUCTURE ONLY.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the product path never does.  The
arithmetic lives in ``tfx_ref.c`` (plain C loops, fp32 in/out, one double
accumulator per output element); this module compiles that file with gcc,
loads it with ctypes and marshals numpy arrays.  Nothing here touches the GPU
library, and nothing in the GPU library touches this.

The MobileNet-v1 forward pass below is a chain of the single-op oracle
functions, in the layer order the MobileNet-v1 1.0/224 benchmark of Section
3.9 / Table 1 runs: conv 3x3 s2 -> 13 x (depthwise 3x3 -> pointwise 1x1), bias
and ReLU6 after each of the 27 convolutions, global average pool, fully
connected layer, softmax.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tfx_ref.c")
_LIB = os.path.join(_HERE, "libtfx_ref.so")

PAD_VALID, PAD_SAME = 0, 1
ACT_NONE, ACT_RELU, ACT_RELU6 = 0, 1, 2

# MobileNet-v1 1.0: output channels and strides of the 13 depthwise-separable blocks.
MOBILENET_V1_CHANNELS = (64, 128, 128, 256, 256, 512, 512, 512, 512, 512, 512, 1024, 1024)
MOBILENET_V1_STRIDES = (1, 2, 1, 2, 1, 2, 1, 1, 1, 1, 1, 2, 1)


def build(force=False):
    """Compile tfx_ref.c into libtfx_ref.so (gcc -O2, OpenMP, no intrinsics, no BLAS)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-fPIC", "-shared",
           "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__("oracle status %d" % code)
        self.code = code


def _check(rc):
    if rc != 0:
        raise OracleError(rc)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _fp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _shape(dims):
    return (ctypes.c_int64 * len(dims))(*[int(d) for d in dims])


def set_threads(n):
    """Set the OpenMP thread count used by the oracle loops (via libgomp)."""
    gomp = ctypes.CDLL("libgomp.so.1")
    gomp.omp_set_num_threads(int(n))


def get_max_threads():
    gomp = ctypes.CDLL("libgomp.so.1")
    return int(gomp.omp_get_max_threads())


def out_extent(in_size, k, s, pad):
    """(out, pad_before, pad_after) of one spatial dimension."""
    o, pb, pa = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    _check(_load().tfx_ref_out_extent(ctypes.c_int64(in_size), ctypes.c_int64(k), ctypes.c_int64(s),
                                      int(pad), ctypes.byref(o), ctypes.byref(pb), ctypes.byref(pa)))
    return o.value, pb.value, pa.value


def matmul_out_shape(a_shape, b_shape, transpose_a=False, transpose_b=False):
    o = _shape((0, 0))
    _check(_load().tfx_ref_matmul_out_shape(_shape(a_shape), _shape(b_shape), int(transpose_a),
                                            int(transpose_b), o))
    return tuple(o)


def conv2d_out_shape(x_shape, f_shape, stride, pad):
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    o, p = _shape((0,) * 4), _shape((0,) * 4)
    _check(_load().tfx_ref_conv2d_out_shape(_shape(x_shape), _shape(f_shape), int(sh), int(sw), int(pad), o, p))
    return tuple(o), tuple(p)


def depthwise_conv2d_out_shape(x_shape, f_shape, stride, pad):
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    o, p = _shape((0,) * 4), _shape((0,) * 4)
    _check(_load().tfx_ref_depthwise_conv2d_out_shape(_shape(x_shape), _shape(f_shape), int(sh), int(sw),
                                                      int(pad), o, p))
    return tuple(o), tuple(p)


def matmul(a, b, transpose_a=False, transpose_b=False):
    a, b = _f32(a), _f32(b)
    assert a.ndim == 2 and b.ndim == 2
    m, n = matmul_out_shape(a.shape, b.shape, transpose_a, transpose_b)
    c = np.empty((m, n), dtype=np.float32)
    _check(_load().tfx_ref_matmul(_fp(a), _shape(a.shape), _fp(b), _shape(b.shape),
                                  int(transpose_a), int(transpose_b), _fp(c)))
    return c


def batch_matmul(a, b, transpose_a=False, transpose_b=False):
    a, b = _f32(a), _f32(b)
    assert a.ndim == 3 and b.ndim == 3
    if a.shape[0] != b.shape[0]:
        raise OracleError(-2)
    m, n = matmul_out_shape(a.shape[1:], b.shape[1:], transpose_a, transpose_b)
    c = np.empty((a.shape[0], m, n), dtype=np.float32)
    _check(_load().tfx_ref_batch_matmul(_fp(a), _shape(a.shape), _fp(b), _shape(b.shape),
                                        int(transpose_a), int(transpose_b), _fp(c)))
    return c


def conv2d(x, w, bias=None, stride=1, pad=PAD_SAME, act=ACT_NONE):
    x, w = _f32(x), _f32(w)
    assert x.ndim == 4 and w.ndim == 4
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    oshape, _ = conv2d_out_shape(x.shape, w.shape, (sh, sw), pad)
    y = np.empty(oshape, dtype=np.float32)
    bp = None
    if bias is not None:
        bias = _f32(bias)
        assert bias.shape == (w.shape[3],)
        bp = _fp(bias)
    _check(_load().tfx_ref_conv2d(_fp(x), _shape(x.shape), _fp(w), _shape(w.shape), bp,
                                  int(sh), int(sw), int(pad), int(act), _fp(y)))
    return y


def depthwise_conv2d(x, w, bias=None, stride=1, pad=PAD_SAME, act=ACT_NONE):
    x, w = _f32(x), _f32(w)
    assert x.ndim == 4 and w.ndim == 4
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    oshape, _ = depthwise_conv2d_out_shape(x.shape, w.shape, (sh, sw), pad)
    y = np.empty(oshape, dtype=np.float32)
    bp = None
    if bias is not None:
        bias = _f32(bias)
        assert bias.shape == (w.shape[2] * w.shape[3],)
        bp = _fp(bias)
    _check(_load().tfx_ref_depthwise_conv2d(_fp(x), _shape(x.shape), _fp(w), _shape(w.shape), bp,
                                            int(sh), int(sw), int(pad), int(act), _fp(y)))
    return y


def global_avg_pool(a):
    a = _f32(a)
    assert a.ndim == 4
    p = np.empty((a.shape[0], a.shape[3]), dtype=np.float32)
    _check(_load().tfx_ref_global_avg_pool(_fp(a), _shape(a.shape), _fp(p)))
    return p


def softmax(logits):
    logits = _f32(logits)
    assert logits.ndim == 2
    probs = np.empty_like(logits)
    _check(_load().tfx_ref_softmax(_fp(logits), ctypes.c_int64(logits.shape[0]),
                                   ctypes.c_int64(logits.shape[1]), _fp(probs)))
    return probs


def _u16(a):
    """Contiguous uint16 bit patterns of a float16 (or uint16) array."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("16-bit float storage is passed as float16 or uint16 bit patterns")
    return a


def _hp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def half_to_double(h):
    """binary16 bit patterns -> float64 values (the oracle's own decoding)."""
    h = _u16(h)
    out = np.empty(h.shape, dtype=np.float64)
    _check(_load().tfx_ref_half_to_double(_hp(h), ctypes.c_int64(h.size),
                                          out.ctypes.data_as(ctypes.POINTER(ctypes.c_double))))
    return out


def double_to_half(v):
    """float64 values -> binary16 (returned as a float16 array), round to nearest even."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    _check(_load().tfx_ref_double_to_half(v.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                          ctypes.c_int64(v.size), _hp(out)))
    return out.view(np.float16)


def add(a, b):
    a, b = _f32(a), _f32(b)
    assert a.shape == b.shape
    c = np.empty_like(a)
    _check(_load().tfx_ref_add(_fp(a), _fp(b), ctypes.c_int64(a.size), _fp(c)))
    return c


def add_f16(a, b):
    a, b = _u16(a), _u16(b)
    assert a.shape == b.shape
    c = np.empty(a.shape, dtype=np.uint16)
    _check(_load().tfx_ref_add_f16(_hp(a), _hp(b), ctypes.c_int64(a.size), _hp(c)))
    return c.view(np.float16)


def batch_matmul_f16(a, b, transpose_a=False, transpose_b=False, bias=None, act=ACT_NONE):
    """a, b: [B,rows,cols] float16; bias: [N] float16 or None.  Returns float16 [B,M,N]."""
    a, b = _u16(a), _u16(b)
    assert a.ndim == 3 and b.ndim == 3
    m, n = matmul_out_shape(a.shape[1:], b.shape[1:], transpose_a, transpose_b)
    c = np.empty((a.shape[0], m, n), dtype=np.uint16)
    bb = None if bias is None else _u16(bias)
    if bb is not None:
        assert bb.shape == (n,)
    _check(_load().tfx_ref_batch_matmul_f16(_hp(a), _shape(a.shape), _hp(b), _shape(b.shape), int(transpose_a),
                                            int(transpose_b), None if bb is None else _hp(bb), int(act), _hp(c)))
    return c.view(np.float16)


def _conv_f16(fn_name, shape_fn, x, filt, bias, stride, pad, act):
    x, filt = _u16(x), _u16(filt)
    assert x.ndim == 4 and filt.ndim == 4
    sh, sw = (stride, stride) if np.isscalar(stride) else stride
    oshape, _ = shape_fn(x.shape, filt.shape, (sh, sw), pad)
    y = np.empty(oshape, dtype=np.uint16)
    b = None if bias is None else _u16(bias)
    if b is not None:
        assert b.shape == (oshape[3],)
    _check(getattr(_load(), fn_name)(_hp(x), _shape(x.shape), _hp(filt), _shape(filt.shape), None if b is None else _hp(b),
                                     int(sh), int(sw), int(pad), int(act), _hp(y)))
    return y.view(np.float16)


def conv2d_f16(x, filt, bias=None, stride=1, pad=PAD_SAME, act=ACT_NONE):
    return _conv_f16("tfx_ref_conv2d_f16", conv2d_out_shape, x, filt, bias, stride, pad, act)


def depthwise_conv2d_f16(x, filt, bias=None, stride=1, pad=PAD_SAME, act=ACT_NONE):
    return _conv_f16("tfx_ref_depthwise_conv2d_f16", depthwise_conv2d_out_shape, x, filt, bias, stride, pad, act)


def global_avg_pool_f16(x):
    x = _u16(x)
    assert x.ndim == 4
    y = np.empty((x.shape[0], x.shape[3]), dtype=np.uint16)
    _check(_load().tfx_ref_global_avg_pool_f16(_hp(x), _shape(x.shape), _hp(y)))
    return y.view(np.float16)


def softmax_f16(logits):
    logits = _u16(logits)
    assert logits.ndim == 2
    probs = np.empty(logits.shape, dtype=np.uint16)
    _check(_load().tfx_ref_softmax_f16(_hp(logits), ctypes.c_int64(logits.shape[0]), ctypes.c_int64(logits.shape[1]),
                                       _hp(probs)))
    return probs.view(np.float16)


def mobilenet_v1_forward_f16(image, weights, return_activations=False):
    """The MobileNet-v1 chain on 16-bit float storage: every tensor (image, weights, biases, feature
    maps, pooled vector, logits, probabilities) is float16 and every op rounds its result once."""
    acts = []
    a = conv2d_f16(image, weights["conv0_w"], weights["conv0_b"], stride=2, pad=PAD_SAME, act=ACT_RELU6)
    acts.append(a)
    for i in range(13):
        a = depthwise_conv2d_f16(a, weights["dw_w"][i], weights["dw_b"][i], stride=MOBILENET_V1_STRIDES[i],
                                 pad=PAD_SAME, act=ACT_RELU6)
        acts.append(a)
        a = conv2d_f16(a, weights["pw_w"][i], weights["pw_b"][i], stride=1, pad=PAD_SAME, act=ACT_RELU6)
        acts.append(a)
    pooled = global_avg_pool_f16(a)
    acts.append(pooled)
    n, c = pooled.shape
    fc_w = np.ascontiguousarray(weights["fc_w"])
    logits = conv2d_f16(pooled.reshape(n, 1, 1, c), fc_w.reshape(1, 1, fc_w.shape[0], fc_w.shape[1]),
                        weights["fc_b"], stride=1, pad=PAD_SAME, act=ACT_NONE).reshape(n, -1)
    probs = softmax_f16(logits)
    if return_activations:
        return probs, logits, acts
    return probs, logits


def mobilenet_v1_forward(image, weights, return_activations=False):
    """MobileNet-v1 1.0 forward as a chain of the single-op oracle functions.

    image: [N,224,224,3]; weights: dict with conv0_w [3,3,3,32], conv0_b [32],
    dw_w[i] [3,3,C,1], dw_b[i] [C], pw_w[i] [1,1,Cin,Cout], pw_b[i] [Cout]
    (i = 0..12), fc_w [1024,1000], fc_b [1000].  Returns (probs, logits) and,
    if asked, the list of the 27 post-activation feature maps plus the pooled
    vector, in execution order.
    """
    acts = []
    a = conv2d(image, weights["conv0_w"], weights["conv0_b"], stride=2, pad=PAD_SAME, act=ACT_RELU6)
    acts.append(a)
    for i in range(13):
        a = depthwise_conv2d(a, weights["dw_w"][i], weights["dw_b"][i], stride=MOBILENET_V1_STRIDES[i],
                             pad=PAD_SAME, act=ACT_RELU6)
        acts.append(a)
        a = conv2d(a, weights["pw_w"][i], weights["pw_b"][i], stride=1, pad=PAD_SAME, act=ACT_RELU6)
        acts.append(a)
    pooled = global_avg_pool(a)
    acts.append(pooled)
    n, c = pooled.shape
    fc_w = _f32(weights["fc_w"])
    # fully connected layer = 1x1 convolution over a 1x1 image: one rounding per logit
    logits = conv2d(pooled.reshape(n, 1, 1, c), fc_w.reshape(1, 1, fc_w.shape[0], fc_w.shape[1]),
                    weights["fc_b"], stride=1, pad=PAD_SAME, act=ACT_NONE).reshape(n, -1)
    probs = softmax(logits)
    if return_activations:
        return probs, logits, acts
    return probs, logits
