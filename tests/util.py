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


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to("cuda:0")


def host(t):
    import torch
    torch.cuda.synchronize()
    return t.cpu().numpy()
