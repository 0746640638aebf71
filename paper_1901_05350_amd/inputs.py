"""Seeded synthetic inputs for the dense-op workloads.

This module only draws random numbers and shapes them; it contains none of the
ops' arithmetic.  It serves both the CPU oracle's tests and the GPU library's
tests/benchmark so that the two sides always see the same arrays.

All arrays are float32, C-contiguous, NHWC for images, HWIO for conv filters
and [fh,fw,C,mult] for depthwise filters.  Values come from
numpy.random.Generator(PCG64(seed)) in float64 and are cast to float32 on the
host.  Tensors are drawn in a fixed order: inputs first, then weights layer by
layer (filter before bias).

The workloads stand in for the trained MobileNet v1 1.0 / 224x224x3 image of
Section 3.9 (Table 1): same shapes, random values.  "He-normal" means an
untruncated normal with std = sqrt(2 / fan_in), fan_in being the number of
products summed per output value (fh*fw*Cin for conv2d, fh*fw for depthwise,
1024 for the fully connected layer); biases are N(0, 0.01^2).
"""
import numpy as np

MOBILENET_V1_CHANNELS = (64, 128, 128, 256, 256, 512, 512, 512, 512, 512, 512, 1024, 1024)
MOBILENET_V1_STRIDES = (1, 2, 1, 2, 1, 2, 1, 1, 1, 1, 1, 2, 1)
BIAS_STD = 0.01


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def uniform(rng, shape, lo=-1.0, hi=1.0):
    return rng.uniform(lo, hi, size=shape).astype(np.float32)


def normal(rng, shape, std=1.0):
    return (rng.standard_normal(size=shape) * std).astype(np.float32)


def he_normal(rng, shape, fan_in):
    return normal(rng, shape, np.sqrt(2.0 / fan_in))


def matmul_small(seed=0, m=64, k=128, n=64):
    """tf.matMul A[m,k] x B[k,n], entries uniform[-1,1)."""
    rng = _rng(seed)
    return {"a": uniform(rng, (m, k)), "b": uniform(rng, (k, n)), "transpose_a": False, "transpose_b": False}


def pointwise_conv(seed=1, n=1, h=56, w=56, cin=128, cout=128):
    """1x1 conv2d: x uniform[-1,1), filter He-normal, bias N(0,0.01^2); stride 1, same, ReLU6."""
    rng = _rng(seed)
    x = uniform(rng, (n, h, w, cin))
    f = he_normal(rng, (1, 1, cin, cout), cin)
    b = normal(rng, (cout,), BIAS_STD)
    return {"x": x, "filter": f, "bias": b, "stride": 1}


def depthwise_conv(seed=2, n=1, h=112, w=112, c=64, k=3, mult=1):
    """depthwiseConv2d kxk: x uniform[-1,1), filter He-normal (fan_in k*k), bias N(0,0.01^2)."""
    rng = _rng(seed)
    x = uniform(rng, (n, h, w, c))
    f = he_normal(rng, (k, k, c, mult), k * k)
    b = normal(rng, (c * mult,), BIAS_STD)
    return {"x": x, "filter": f, "bias": b}


def batch_matmul(seed=3, batch=8, m=1024, k=1024, n=1024):
    """batchMatMul with transposeB: A[batch,m,k], B stored [batch,n,k], entries N(0,1)."""
    rng = _rng(seed)
    return {"a": normal(rng, (batch, m, k)), "b": normal(rng, (batch, n, k)),
            "transpose_a": False, "transpose_b": True}


def batch_matmul_f16(seed=6, batch=8, m=1024, k=1024, n=1024, transpose_a=False, transpose_b=True, bias=False):
    """batchMatMul operands on 16-bit float storage: N(0,1) entries rounded to float16, stored
    [batch,k,m] / [batch,n,k] when transposed; optional bias N(0,1) of length n."""
    rng = _rng(seed)
    a = normal(rng, (batch, k, m) if transpose_a else (batch, m, k)).astype(np.float16)
    b = normal(rng, (batch, n, k) if transpose_b else (batch, k, n)).astype(np.float16)
    out = {"a": a, "b": b, "transpose_a": transpose_a, "transpose_b": transpose_b, "bias": None}
    if bias:
        out["bias"] = normal(rng, (n,)).astype(np.float16)
    return out


def add_operands(seed=8, n=1 << 20, dtype=np.float32):
    """Two vectors of n N(0,1) values spread over +-16 binades (so that sums round), in the storage type."""
    rng = _rng(seed)
    scale = lambda: np.exp2(rng.integers(-8, 9, n)).astype(np.float32)
    return {"a": (normal(rng, (n,)) * scale()).astype(dtype), "b": (normal(rng, (n,)) * scale()).astype(dtype)}


def conv_general(seed, n, h, w, cin, cout, fh, fw):
    rng = _rng(seed)
    x = uniform(rng, (n, h, w, cin))
    f = he_normal(rng, (fh, fw, cin, cout), fh * fw * cin)
    b = normal(rng, (cout,), BIAS_STD)
    return {"x": x, "filter": f, "bias": b}


def mobilenet_v1_weights(rng, width_quarters=4, classes=1000):
    """Random MobileNet-v1 weights (batch norm folded into the biases); every channel count of the
    1.0 network is scaled by width_quarters / 4."""
    q = int(width_quarters)
    w = {"dw_w": [], "dw_b": [], "pw_w": [], "pw_b": []}
    cin = 32 * q // 4
    w["conv0_w"] = he_normal(rng, (3, 3, 3, cin), 27)
    w["conv0_b"] = normal(rng, (cin,), BIAS_STD)
    for base in MOBILENET_V1_CHANNELS:
        cout = base * q // 4
        w["dw_w"].append(he_normal(rng, (3, 3, cin, 1), 9))
        w["dw_b"].append(normal(rng, (cin,), BIAS_STD))
        w["pw_w"].append(he_normal(rng, (1, 1, cin, cout), cin))
        w["pw_b"].append(normal(rng, (cout,), BIAS_STD))
        cin = cout
    w["fc_w"] = he_normal(rng, (cin, classes), cin)
    w["fc_b"] = normal(rng, (classes,), BIAS_STD)
    return w


def mobilenet_v1(seed=4, batch=1, image_size=224, width_quarters=4, classes=1000):
    """Image [batch,size,size,3] uniform[-1,1) and random MobileNet-v1 weights (1.0 / 224 by default)."""
    rng = _rng(seed)
    image = uniform(rng, (batch, image_size, image_size, 3))
    return {"image": image, "weights": mobilenet_v1_weights(rng, width_quarters, classes)}


def mobilenet_v1_f16(seed=4, batch=1, image_size=224, width_quarters=4, classes=1000):
    """The MobileNet-v1 workload on 16-bit float storage: the same draws as mobilenet_v1, rounded to float16."""
    d = mobilenet_v1(seed, batch, image_size, width_quarters, classes)
    h = lambda a: a.astype(np.float16)
    return {"image": h(d["image"]),
            "weights": {k: ([h(t) for t in v] if isinstance(v, list) else h(v)) for k, v in d["weights"].items()}}
