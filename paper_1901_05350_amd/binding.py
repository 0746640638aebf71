"""ctypes binding of libtfx.so: same names as the C ABI, torch tensors in and out."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libtfx.so")

PAD_VALID, PAD_SAME = 0, 1
ACT_NONE, ACT_RELU, ACT_RELU6 = 0, 1, 2

_I64P = ctypes.POINTER(ctypes.c_int64)
_VP = ctypes.c_void_p


class TfxWeights(ctypes.Structure):
    """Mirror of tfx_mobilenet_v1_weights (host struct of device pointers)."""
    _fields_ = [("conv0_w", _VP), ("conv0_b", _VP),
                ("dw_w", _VP * 13), ("dw_b", _VP * 13), ("pw_w", _VP * 13), ("pw_b", _VP * 13),
                ("fc_w", _VP), ("fc_b", _VP)]


class TfxWeightsF16(ctypes.Structure):
    """Mirror of tfx_mobilenet_v1_weights_f16 (same members, binary16 tensors)."""
    _fields_ = TfxWeights._fields_


class TfxVariant(ctypes.Structure):
    """Mirror of tfx_mobilenet_v1_variant."""
    _fields_ = [("image_size", ctypes.c_int64), ("width_quarters", ctypes.c_int64), ("classes", ctypes.c_int64)]


class TfxError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        try:
            msg = lib().tfx_status_string(status).decode()
        except Exception:
            msg = str(status)
        super().__init__("%s failed: %s" % (where, msg))


_lib = None

_SIGNATURES = {
    "tfx_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "tfx_matmul_out_shape": (ctypes.c_int, [_I64P, _I64P, ctypes.c_int, ctypes.c_int, _I64P]),
    "tfx_conv2d_out_shape": (ctypes.c_int, [_I64P, _I64P, ctypes.c_int, ctypes.c_int, ctypes.c_int, _I64P, _I64P]),
    "tfx_depthwise_conv2d_out_shape": (ctypes.c_int, [_I64P, _I64P, ctypes.c_int, ctypes.c_int, ctypes.c_int, _I64P, _I64P]),
    "tfx_matmul": (ctypes.c_int, [_VP, _I64P, _VP, _I64P, ctypes.c_int, ctypes.c_int, _VP, _VP]),
    "tfx_batch_matmul": (ctypes.c_int, [_VP, _I64P, _VP, _I64P, ctypes.c_int, ctypes.c_int, _VP, _VP]),
    "tfx_conv2d": (ctypes.c_int, [_VP, _I64P, _VP, _I64P, _VP, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                  ctypes.c_int, _VP, _VP]),
    "tfx_depthwise_conv2d": (ctypes.c_int, [_VP, _I64P, _VP, _I64P, _VP, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                            ctypes.c_int, _VP, _VP]),
    "tfx_add": (ctypes.c_int, [_VP, _VP, ctypes.c_int64, _VP, _VP]),
    "tfx_add_f16": (ctypes.c_int, [_VP, _VP, ctypes.c_int64, _VP, _VP]),
    "tfx_batch_matmul_f16": (ctypes.c_int, [_VP, _I64P, _VP, _I64P, ctypes.c_int, ctypes.c_int, _VP, ctypes.c_int,
                                            _VP, _VP]),
    "tfx_conv2d_f16": (ctypes.c_int, [_VP, _I64P, _VP, _I64P, _VP, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, _VP, _VP]),
    "tfx_depthwise_conv2d_f16": (ctypes.c_int, [_VP, _I64P, _VP, _I64P, _VP, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                ctypes.c_int, _VP, _VP]),
    "tfx_mobilenet_v1_workspace_bytes_f16": (ctypes.c_size_t, [ctypes.POINTER(TfxVariant), ctypes.c_int64]),
    "tfx_mobilenet_v1_forward_f16": (ctypes.c_int, [ctypes.POINTER(TfxVariant), _VP, ctypes.c_int64,
                                                    ctypes.POINTER(TfxWeightsF16), _VP, ctypes.c_size_t, _VP, _VP,
                                                    _VP]),
    "tfx_mobilenet_v1_features_f16": (ctypes.c_int, [ctypes.POINTER(TfxVariant), _VP, ctypes.c_int64,
                                                     ctypes.POINTER(TfxWeightsF16), _VP, ctypes.c_size_t, ctypes.c_int,
                                                     _VP, _VP]),
    "tfx_mobilenet_v1_workspace_bytes": (ctypes.c_size_t, [ctypes.c_int64]),
    "tfx_mobilenet_v1_forward": (ctypes.c_int, [_VP, ctypes.c_int64, ctypes.POINTER(TfxWeights), _VP,
                                                ctypes.c_size_t, _VP, _VP, _VP]),
    "tfx_mobilenet_v1_variant_workspace_bytes": (ctypes.c_size_t, [ctypes.POINTER(TfxVariant), ctypes.c_int64]),
    "tfx_mobilenet_v1_static_scratch_bytes": (ctypes.c_size_t, []),
    "tfx_mobilenet_v1_variant_forward_static": (ctypes.c_int, [ctypes.POINTER(TfxVariant), _VP, ctypes.c_int64,
                                                               ctypes.POINTER(TfxWeights), _VP, _VP, _VP]),
    "tfx_mobilenet_v1_variant_forward": (ctypes.c_int, [ctypes.POINTER(TfxVariant), _VP, ctypes.c_int64,
                                                        ctypes.POINTER(TfxWeights), _VP, ctypes.c_size_t, _VP, _VP,
                                                        _VP]),
    "tfx_mobilenet_v1_variant_features_shape": (ctypes.c_int, [ctypes.POINTER(TfxVariant), ctypes.c_int64, ctypes.c_int,
                                                               _I64P]),
    "tfx_mobilenet_v1_variant_features": (ctypes.c_int, [ctypes.POINTER(TfxVariant), _VP, ctypes.c_int64,
                                                         ctypes.POINTER(TfxWeights), _VP, ctypes.c_size_t, ctypes.c_int,
                                                         _VP, _VP]),
}


def library_path():
    return _LIB_PATH


def lib():
    """Load libtfx.so (once).  Raises if it has not been built: there is no fallback path."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libtfx.so is not built: run `python -m paper_1901_05350_amd.build`")
        handle = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)  # AttributeError if the symbol is missing
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _shape(dims):
    return (ctypes.c_int64 * len(dims))(*[int(d) for d in dims])


def _pair(stride):
    if isinstance(stride, (tuple, list)):
        return int(stride[0]), int(stride[1])
    return int(stride), int(stride)


def _check(status, where):
    if status != 0:
        raise TfxError(status, where)


def _dev(t, name, dtype=None):
    import torch
    dtype = torch.float32 if dtype is None else dtype
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a tensor in GPU memory" % name)
    if t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be contiguous %s" % (name, str(dtype).replace("torch.", "")))
    return t


def _rank(t, name, ranks):
    """Shape checks come before the pointer is handed to the library: the C side reads exactly `rank` entries of the
    host shape array and as many elements as the shapes say."""
    shape = getattr(t, "shape", None)
    if shape is None or len(shape) not in ranks:
        raise TypeError("%s must have rank %s" % (name, " or ".join(str(r) for r in ranks)))
    return tuple(int(d) for d in shape)


def _expect_shape(t, name, shape):
    if tuple(int(d) for d in getattr(t, "shape", ())) != tuple(int(d) for d in shape):
        raise TypeError("%s must have shape %s" % (name, list(shape)))


def _stream(t):
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream)


def tfx_status_string(status):
    return lib().tfx_status_string(int(status)).decode()


def tfx_matmul_out_shape(a_shape, b_shape, transpose_a=False, transpose_b=False):
    out = _shape((0, 0))
    _check(lib().tfx_matmul_out_shape(_shape(a_shape), _shape(b_shape), int(transpose_a), int(transpose_b), out),
           "tfx_matmul_out_shape")
    return tuple(out)


def tfx_conv2d_out_shape(x_shape, f_shape, stride, pad):
    sh, sw = _pair(stride)
    out, pads = _shape((0,) * 4), _shape((0,) * 4)
    _check(lib().tfx_conv2d_out_shape(_shape(x_shape), _shape(f_shape), sh, sw, int(pad), out, pads),
           "tfx_conv2d_out_shape")
    return tuple(out), tuple(pads)


def tfx_depthwise_conv2d_out_shape(x_shape, f_shape, stride, pad):
    sh, sw = _pair(stride)
    out, pads = _shape((0,) * 4), _shape((0,) * 4)
    _check(lib().tfx_depthwise_conv2d_out_shape(_shape(x_shape), _shape(f_shape), sh, sw, int(pad), out, pads),
           "tfx_depthwise_conv2d_out_shape")
    return tuple(out), tuple(pads)


def tfx_matmul(a, b, transpose_a=False, transpose_b=False, out=None):
    import torch
    _rank(a, "a", (2,)), _rank(b, "b", (2,))
    m, n = tfx_matmul_out_shape(a.shape, b.shape, transpose_a, transpose_b)
    if out is not None:
        _expect_shape(out, "out", (m, n))
    _dev(a, "a"), _dev(b, "b")
    c = torch.empty((m, n), dtype=torch.float32, device=a.device) if out is None else _dev(out, "out")
    _check(lib().tfx_matmul(a.data_ptr(), _shape(a.shape), b.data_ptr(), _shape(b.shape), int(transpose_a),
                            int(transpose_b), c.data_ptr(), _stream(a)), "tfx_matmul")
    return c


def tfx_batch_matmul(a, b, transpose_a=False, transpose_b=False, out=None):
    import torch
    _rank(a, "a", (3,)), _rank(b, "b", (3,))
    m, n = tfx_matmul_out_shape(a.shape[1:], b.shape[1:], transpose_a, transpose_b)
    if out is not None:
        _expect_shape(out, "out", (a.shape[0], m, n))
    _dev(a, "a"), _dev(b, "b")
    c = torch.empty((a.shape[0], m, n), dtype=torch.float32, device=a.device) if out is None else _dev(out, "out")
    _check(lib().tfx_batch_matmul(a.data_ptr(), _shape(a.shape), b.data_ptr(), _shape(b.shape), int(transpose_a),
                                  int(transpose_b), c.data_ptr(), _stream(a)), "tfx_batch_matmul")
    return c


def _add(fn_name, dtype, a, b, out):
    import torch
    _dev(a, "a", dtype), _dev(b, "b", dtype)
    if a.shape != b.shape:
        raise TypeError("add operands must have the same shape")
    c = torch.empty_like(a) if out is None else _dev(out, "out", dtype)
    if c.shape != a.shape:
        raise TypeError("out must have the operands' shape")
    _check(getattr(lib(), fn_name)(a.data_ptr(), b.data_ptr(), a.numel(), c.data_ptr(), _stream(a)), fn_name)
    return c


def tfx_add(a, b, out=None):
    """c = a + b element-wise, float32; out may be a or b."""
    import torch
    return _add("tfx_add", torch.float32, a, b, out)


def tfx_add_f16(a, b, out=None):
    """c = a + b element-wise on float16 storage; out may be a or b."""
    import torch
    return _add("tfx_add_f16", torch.float16, a, b, out)


def tfx_batch_matmul_f16(a, b, transpose_a=False, transpose_b=False, bias=None, act=ACT_NONE, out=None):
    """float16 [B,rows,cols] operands, float16 bias [N] or None, float16 result [B,M,N]."""
    import torch
    h = torch.float16
    _rank(a, "a", (3,)), _rank(b, "b", (3,))
    m, n = tfx_matmul_out_shape(a.shape[1:], b.shape[1:], transpose_a, transpose_b)
    if bias is not None:
        _expect_shape(bias, "bias", (n,))
    if out is not None:
        _expect_shape(out, "out", (a.shape[0], m, n))
    _dev(a, "a", h), _dev(b, "b", h)
    if bias is not None:
        _dev(bias, "bias", h)
    c = torch.empty((a.shape[0], m, n), dtype=h, device=a.device) if out is None else _dev(out, "out", h)
    _check(lib().tfx_batch_matmul_f16(a.data_ptr(), _shape(a.shape), b.data_ptr(), _shape(b.shape), int(transpose_a),
                                      int(transpose_b), None if bias is None else bias.data_ptr(), int(act),
                                      c.data_ptr(), _stream(a)), "tfx_batch_matmul_f16")
    return c


def _conv(fn_name, shape_fn, x, filt, bias, stride, pad, act, out, dtype=None):
    import torch
    dtype = torch.float32 if dtype is None else dtype
    _rank(x, "x", (4,)), _rank(filt, "filter", (4,))
    sh, sw = _pair(stride)
    oshape, _ = shape_fn(x.shape, filt.shape, (sh, sw), pad)
    if bias is not None:
        _expect_shape(bias, "bias", (oshape[3],))
    if out is not None:
        _expect_shape(out, "out", oshape)
    _dev(x, "x", dtype), _dev(filt, "filter", dtype)
    if bias is not None:
        _dev(bias, "bias", dtype)
    y = torch.empty(oshape, dtype=dtype, device=x.device) if out is None else _dev(out, "out", dtype)
    fn = getattr(lib(), fn_name)
    _check(fn(x.data_ptr(), _shape(x.shape), filt.data_ptr(), _shape(filt.shape),
              None if bias is None else bias.data_ptr(), sh, sw, int(pad), int(act), y.data_ptr(), _stream(x)),
           fn_name)
    return y


def tfx_conv2d(x, filt, bias=None, stride=1, pad=PAD_SAME, act=ACT_NONE, out=None):
    return _conv("tfx_conv2d", tfx_conv2d_out_shape, x, filt, bias, stride, pad, act, out)


def tfx_depthwise_conv2d(x, filt, bias=None, stride=1, pad=PAD_SAME, act=ACT_NONE, out=None):
    return _conv("tfx_depthwise_conv2d", tfx_depthwise_conv2d_out_shape, x, filt, bias, stride, pad, act, out)


def tfx_conv2d_f16(x, filt, bias=None, stride=1, pad=PAD_SAME, act=ACT_NONE, out=None):
    import torch
    return _conv("tfx_conv2d_f16", tfx_conv2d_out_shape, x, filt, bias, stride, pad, act, out, torch.float16)


def tfx_depthwise_conv2d_f16(x, filt, bias=None, stride=1, pad=PAD_SAME, act=ACT_NONE, out=None):
    import torch
    return _conv("tfx_depthwise_conv2d_f16", tfx_depthwise_conv2d_out_shape, x, filt, bias, stride, pad, act, out,
                 torch.float16)


def tfx_mobilenet_v1_workspace_bytes(batch):
    return int(lib().tfx_mobilenet_v1_workspace_bytes(int(batch)))


def tfx_mobilenet_v1_variant_workspace_bytes(variant, batch):
    return int(lib().tfx_mobilenet_v1_variant_workspace_bytes(ctypes.byref(variant), int(batch)))


_MOBILENET_CHANNELS = (64, 128, 128, 256, 256, 512, 512, 512, 512, 512, 512, 1024, 1024)


def _check_mobilenet_weights(weights, image_size, width_quarters):
    """Every weight tensor must have the shape the variant implies (include/tfx.h: channel counts are
    alpha = width_quarters / 4 times 32, 64, 128, ..., 1024): the library reads that many elements of each."""
    q = int(width_quarters)
    if q not in (1, 2, 3, 4) or not 32 <= int(image_size) <= 256:
        raise ValueError("unsupported MobileNet-v1 variant")
    for k in ("conv0_w", "conv0_b", "dw_w", "dw_b", "pw_w", "pw_b", "fc_w", "fc_b"):
        if k not in weights:
            raise TypeError("weights lack %r" % k)
    for k in ("dw_w", "dw_b", "pw_w", "pw_b"):
        if not isinstance(weights[k], (list, tuple)) or len(weights[k]) != 13:
            raise TypeError("weights[%r] must be a list of 13 tensors" % k)
    c = 32 * q // 4
    _expect_shape(weights["conv0_w"], "conv0_w", (3, 3, 3, c))
    _expect_shape(weights["conv0_b"], "conv0_b", (c,))
    for i, full in enumerate(_MOBILENET_CHANNELS):
        co = full * q // 4
        _expect_shape(weights["dw_w"][i], "dw_w[%d]" % i, (3, 3, c, 1))
        _expect_shape(weights["dw_b"][i], "dw_b[%d]" % i, (c,))
        _expect_shape(weights["pw_w"][i], "pw_w[%d]" % i, (1, 1, c, co))
        _expect_shape(weights["pw_b"][i], "pw_b[%d]" % i, (co,))
        c = co
    classes = _rank(weights["fc_w"], "fc_w", (2,))[1]
    _expect_shape(weights["fc_w"], "fc_w", (c, classes))
    _expect_shape(weights["fc_b"], "fc_b", (classes,))
    if not 1 <= classes <= 1024:
        raise ValueError("unsupported number of classes")
    return classes


def _check_forward_buffers(image, workspace, probs, logits, batch, size, classes, dtype):
    import torch
    _expect_shape(image, "image", (batch, size, size, 3))
    _expect_shape(probs, "probs", (batch, classes))
    if logits is not None:
        _expect_shape(logits, "logits", (batch, classes))
    _dev(image, "image", dtype), _dev(probs, "probs", dtype)
    if logits is not None:
        _dev(logits, "logits", dtype)
    if not isinstance(workspace, torch.Tensor) or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous tensor in GPU memory")


class MobileNetV1:
    """Device-resident MobileNet-v1 weights plus a workspace.

    With the defaults (224 pixels, width 4/4, 1000 classes) forward() calls tfx_mobilenet_v1_forward;
    any other member of the family goes through tfx_mobilenet_v1_variant_forward.
    """

    def __init__(self, weights, batch=1, device="cuda:0", image_size=224, width_quarters=4):
        import torch
        _check_mobilenet_weights(weights, image_size, width_quarters)
        self.device = torch.device(device)
        self.batch = int(batch)
        up = lambda a: torch.as_tensor(a, dtype=torch.float32).contiguous().to(self.device)
        self.tensors = {k: ([up(t) for t in v] if isinstance(v, (list, tuple)) else up(v)) for k, v in weights.items()}
        self.struct = TfxWeights()
        for k in ("conv0_w", "conv0_b", "fc_w", "fc_b"):
            setattr(self.struct, k, self.tensors[k].data_ptr())
        for k in ("dw_w", "dw_b", "pw_w", "pw_b"):
            arr = getattr(self.struct, k)
            for i in range(13):
                arr[i] = self.tensors[k][i].data_ptr()
        classes = int(self.tensors["fc_w"].shape[1])
        self.variant = TfxVariant(int(image_size), int(width_quarters), classes)
        self.is_base = (self.variant.image_size, self.variant.width_quarters, classes) == (224, 4, 1000)
        nbytes = (tfx_mobilenet_v1_workspace_bytes(self.batch) if self.is_base
                  else tfx_mobilenet_v1_variant_workspace_bytes(self.variant, self.batch))
        if nbytes == 0:
            raise ValueError("unsupported MobileNet-v1 variant or batch")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.probs = torch.empty((self.batch, classes), dtype=torch.float32, device=self.device)
        self.logits = torch.empty((self.batch, classes), dtype=torch.float32, device=self.device)

    def forward(self, image):
        """Enqueue one forward pass on the current stream; returns (probs, logits) device tensors."""
        _dev(image, "image")
        size = int(self.variant.image_size)
        if tuple(image.shape) != (self.batch, size, size, 3):
            raise TypeError("image must be [%d,%d,%d,3]" % (self.batch, size, size))
        if self.is_base:
            tfx_mobilenet_v1_forward(image, self.struct, self.workspace, self.probs, self.logits)
        else:
            tfx_mobilenet_v1_variant_forward(self.variant, image, self.struct, self.workspace, self.probs, self.logits)
        return self.probs, self.logits

    def features(self, image, end_block, out=None):
        """Enqueue the layers up to depthwise-separable block `end_block` (1 ... 13); returns its output [N,h,w,c]."""
        import torch
        if out is None:
            out = torch.empty(tfx_mobilenet_v1_variant_features_shape(self.variant, self.batch, end_block),
                              dtype=torch.float32, device=self.device)
        return tfx_mobilenet_v1_variant_features(self.variant, image, self.struct, self.workspace, end_block, out)


def tfx_mobilenet_v1_forward(image, weights_struct, workspace, probs, logits=None):
    import torch
    _check_forward_buffers(image, workspace, probs, logits, _rank(image, "image", (4,))[0], 224, 1000, torch.float32)
    _check(lib().tfx_mobilenet_v1_forward(image.data_ptr(), int(image.shape[0]), ctypes.byref(weights_struct),
                                          workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                          probs.data_ptr(), None if logits is None else logits.data_ptr(),
                                          _stream(image)), "tfx_mobilenet_v1_forward")
    return probs


def tfx_mobilenet_v1_variant_forward(variant, image, weights_struct, workspace, probs, logits=None):
    import torch
    _check_forward_buffers(image, workspace, probs, logits, _rank(image, "image", (4,))[0], int(variant.image_size),
                           int(variant.classes), torch.float32)
    _check(lib().tfx_mobilenet_v1_variant_forward(ctypes.byref(variant), image.data_ptr(), int(image.shape[0]),
                                                  ctypes.byref(weights_struct), workspace.data_ptr(),
                                                  workspace.numel() * workspace.element_size(), probs.data_ptr(),
                                                  None if logits is None else logits.data_ptr(), _stream(image)),
           "tfx_mobilenet_v1_variant_forward")
    return probs


def tfx_mobilenet_v1_variant_features_shape(variant, batch, end_block):
    out = (ctypes.c_int64 * 4)()
    _check(lib().tfx_mobilenet_v1_variant_features_shape(ctypes.byref(variant), int(batch), int(end_block), out),
           "tfx_mobilenet_v1_variant_features_shape")
    return tuple(int(v) for v in out)


def tfx_mobilenet_v1_variant_features(variant, image, weights_struct, workspace, end_block, features):
    """The output of depthwise-separable block `end_block` (1 ... 13) into `features`; nothing after it runs."""
    import torch
    batch = _rank(image, "image", (4,))[0]
    _expect_shape(image, "image", (batch, int(variant.image_size), int(variant.image_size), 3))
    _expect_shape(features, "features", tfx_mobilenet_v1_variant_features_shape(variant, batch, end_block))
    _dev(image, "image"), _dev(features, "features")
    if not isinstance(workspace, torch.Tensor) or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous tensor in GPU memory")
    _check(lib().tfx_mobilenet_v1_variant_features(ctypes.byref(variant), image.data_ptr(), batch,
                                                   ctypes.byref(weights_struct), workspace.data_ptr(),
                                                   workspace.numel() * workspace.element_size(), int(end_block),
                                                   features.data_ptr(), _stream(image)),
           "tfx_mobilenet_v1_variant_features")
    return features


def tfx_mobilenet_v1_static_scratch_bytes():
    return int(lib().tfx_mobilenet_v1_static_scratch_bytes())


def tfx_mobilenet_v1_variant_forward_static(variant, image, weights_struct, probs, logits=None):
    """The forward pass with the library's own fixed workspace: no allocation by the library or by this binding."""
    import torch
    batch = _rank(image, "image", (4,))[0]
    _expect_shape(image, "image", (batch, int(variant.image_size), int(variant.image_size), 3))
    _expect_shape(probs, "probs", (batch, int(variant.classes)))
    if logits is not None:
        _expect_shape(logits, "logits", (batch, int(variant.classes)))
        _dev(logits, "logits")
    _dev(image, "image"), _dev(probs, "probs")
    _check(lib().tfx_mobilenet_v1_variant_forward_static(ctypes.byref(variant), image.data_ptr(), batch,
                                                         ctypes.byref(weights_struct), probs.data_ptr(),
                                                         None if logits is None else logits.data_ptr(),
                                                         _stream(image)), "tfx_mobilenet_v1_variant_forward_static")
    return probs


class MobileNetV1F16:
    """Device-resident float16 MobileNet-v1 weights plus a workspace; calls tfx_mobilenet_v1_forward_f16."""

    def __init__(self, weights, batch=1, device="cuda:0", image_size=224, width_quarters=4):
        import torch
        _check_mobilenet_weights(weights, image_size, width_quarters)
        self.device = torch.device(device)
        self.batch = int(batch)
        up = lambda a: torch.as_tensor(a).to(torch.float16).contiguous().to(self.device)
        self.tensors = {k: ([up(t) for t in v] if isinstance(v, (list, tuple)) else up(v)) for k, v in weights.items()}
        self.struct = TfxWeightsF16()
        for k in ("conv0_w", "conv0_b", "fc_w", "fc_b"):
            setattr(self.struct, k, self.tensors[k].data_ptr())
        for k in ("dw_w", "dw_b", "pw_w", "pw_b"):
            arr = getattr(self.struct, k)
            for i in range(13):
                arr[i] = self.tensors[k][i].data_ptr()
        classes = int(self.tensors["fc_w"].shape[1])
        self.variant = TfxVariant(int(image_size), int(width_quarters), classes)
        nbytes = int(lib().tfx_mobilenet_v1_workspace_bytes_f16(ctypes.byref(self.variant), self.batch))
        if nbytes == 0:
            raise ValueError("unsupported MobileNet-v1 variant or batch")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.probs = torch.empty((self.batch, classes), dtype=torch.float16, device=self.device)
        self.logits = torch.empty((self.batch, classes), dtype=torch.float16, device=self.device)

    def forward(self, image):
        """Enqueue one forward pass on the current stream; returns (probs, logits) float16 device tensors."""
        import torch
        _check_forward_buffers(image, self.workspace, self.probs, self.logits, self.batch, int(self.variant.image_size),
                               int(self.variant.classes), torch.float16)
        _check(lib().tfx_mobilenet_v1_forward_f16(ctypes.byref(self.variant), image.data_ptr(), self.batch,
                                                  ctypes.byref(self.struct), self.workspace.data_ptr(),
                                                  self.workspace.numel(), self.probs.data_ptr(), self.logits.data_ptr(),
                                                  _stream(image)), "tfx_mobilenet_v1_forward_f16")
        return self.probs, self.logits

    def features(self, image, end_block, out=None):
        """Enqueue the layers up to depthwise-separable block `end_block` (1 ... 13); returns its output [N,h,w,c]."""
        import torch
        if out is None:
            out = torch.empty(tfx_mobilenet_v1_variant_features_shape(self.variant, self.batch, end_block),
                              dtype=torch.float16, device=self.device)
        return tfx_mobilenet_v1_features_f16(self.variant, image, self.struct, self.workspace, end_block, out)


def tfx_mobilenet_v1_features_f16(variant, image, weights_struct, workspace, end_block, features):
    """The float16 output of depthwise-separable block `end_block` (1 ... 13) into `features`; nothing after it runs."""
    import torch
    batch = _rank(image, "image", (4,))[0]
    _expect_shape(image, "image", (batch, int(variant.image_size), int(variant.image_size), 3))
    _expect_shape(features, "features", tfx_mobilenet_v1_variant_features_shape(variant, batch, end_block))
    _dev(image, "image", torch.float16), _dev(features, "features", torch.float16)
    if not isinstance(workspace, torch.Tensor) or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous tensor in GPU memory")
    _check(lib().tfx_mobilenet_v1_features_f16(ctypes.byref(variant), image.data_ptr(), batch,
                                               ctypes.byref(weights_struct), workspace.data_ptr(),
                                               workspace.numel() * workspace.element_size(), int(end_block),
                                               features.data_ptr(), _stream(image)),
           "tfx_mobilenet_v1_features_f16")
    return features
