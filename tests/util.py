"""Helpers shared by the GPU parity tests."""
import numpy as np

TOL = 1e-4  # |gpu - ref| <= TOL * (1 + |ref|), the fp32 parity bar


def assert_close(got, ref, what=""):
    got = np.asarray(got)
    ref = np.asarray(ref)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), what
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = TOL * (1.0 + np.abs(ref.astype(np.float64)))
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError("%s: %d of %d outside tolerance; worst at %s: got %r ref %r" %
                             (what, int(bad.sum()), bad.size, i, got[i], ref[i]))
    return float((err / (1.0 + np.abs(ref))).max())


def assert_close_f16(got, ref, what=""):
    """Parity bar for results stored as binary16: the kernel accumulates in fp32 and rounds once, the
    oracle accumulates in double and rounds once, so the two may land on neighbouring binary16 values
    when the sum is near a rounding boundary: |err| <= one binary16 step at ref + the fp32 bar.
    Infinities and NaNs must coincide."""
    got = np.asarray(got)
    ref = np.asarray(ref)
    assert got.dtype == np.float16 and ref.dtype == np.float16 and got.shape == ref.shape, (what, got.dtype, got.shape)
    special = ~np.isfinite(ref)
    assert np.array_equal(np.isnan(got), np.isnan(ref)), what
    assert np.array_equal(got[special & ~np.isnan(ref)], ref[special & ~np.isnan(ref)]), what
    g, r = got[~special].astype(np.float64), ref[~special].astype(np.float64)
    assert np.isfinite(g).all(), what
    step = np.spacing(np.abs(ref[~special])).astype(np.float64)
    err = np.abs(g - r)
    bound = step + TOL * (1.0 + np.abs(r))
    bad = err > bound
    if bad.any():
        i = int(np.argmax(err - bound))
        raise AssertionError("%s: %d of %d outside tolerance; worst: got %r ref %r" % (what, int(bad.sum()), bad.size, g[i], r[i]))
    return float((got.view(np.uint16) != ref.view(np.uint16)).mean())


def dev16(a):
    import torch
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16
    return torch.from_numpy(a).to("cuda:0")


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0")


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()
