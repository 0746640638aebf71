"""GPU parity: tfx_matmul / tfx_batch_matmul against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
from paper_1901_05350_amd import inputs
from util import assert_close, dev, host

pytestmark = pytest.mark.gpu


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def run_matmul(a, b, ta, tb):
    import paper_1901_05350_amd as tfx
    return host(tfx.tfx_matmul(dev(a), dev(b), ta, tb))


def test_config_small_matmul():
    d = inputs.matmul_small(seed=0)
    got = run_matmul(d["a"], d["b"], False, False)
    assert got.shape == (64, 64)
    assert_close(got, oracle.matmul(d["a"], d["b"]), "matMul 64x128x64")


def test_one_hot_products_locate_every_register():
    # e_i e_k^T times e_k e_j^T = e_i e_j^T: a wrong lane / register mapping in the matrix-core
    # tile moves the single 1 somewhere else.
    m, k, n = 70, 40, 67
    r = rng(1)
    for _ in range(12):
        i, kk, j = int(r.integers(m)), int(r.integers(k)), int(r.integers(n))
        a = np.zeros((m, k), np.float32)
        b = np.zeros((k, n), np.float32)
        a[i, kk] = 1
        b[kk, j] = 1
        got = run_matmul(a, b, False, False)
        want = np.zeros((m, n), np.float32)
        want[i, j] = 1
        assert np.array_equal(got, want), (i, kk, j)


SIZES = [1, 2, 3, 31, 32, 33, 63, 64, 65, 127, 128, 129, 196]


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
def test_shape_sweep_all_transposes(ta, tb):
    r = rng(2 + 2 * ta + tb)
    # a spread of (m, k, n) that covers every size on every axis, aligned and ragged
    triples = [(SIZES[i % 13], SIZES[(5 * i + 3) % 13], SIZES[(7 * i + 1) % 13]) for i in range(26)]
    triples += [(784, 128, 256), (196, 512, 512), (49, 1024, 1024), (257, 36, 130), (1, 1, 1), (1, 1024, 1000)]
    for (m, k, n) in triples:
        a = r.uniform(-1, 1, (m, k)).astype(np.float32)
        b = r.uniform(-1, 1, (k, n)).astype(np.float32)
        ref = oracle.matmul(a, b)
        a_in = np.ascontiguousarray(a.T) if ta else a
        b_in = np.ascontiguousarray(b.T) if tb else b
        got = run_matmul(a_in, b_in, ta, tb)
        assert_close(got, ref, "matMul m=%d k=%d n=%d ta=%d tb=%d" % (m, k, n, ta, tb))


def test_small_m_untransposed_direct_operand_depths():
    """A [M,K] times B [K,N] with K one of 64, 96, 128, ..., 1024 and few output tiles: the 16-row kernel that loads its
    matrix-core operands straight from memory (no LDS staging; output columns interleaved between two column blocks).
    One-hot products pin the row / column / k mapping exactly; random operands, ragged M and N that are not
    multiples of the 32-column tile check the clamped loads and predicated stores; the pointwise-conv form adds
    bias and clamp."""
    import paper_1901_05350_amd as tfx
    from oracle import ACT_RELU6, PAD_SAME
    r = rng(77)
    for k in (64, 96, 128, 192, 256, 384, 512, 768, 1024):
        for (m, n) in ((196, 512), (49, 1024), (37, 130), (1, 2), (16, 34), (784, 256), (3136, 128), (200, 66)):
            for _ in range(3):
                i, kk, j = int(r.integers(m)), int(r.integers(k)), int(r.integers(n))
                a = np.zeros((m, k), np.float32)
                b = np.zeros((k, n), np.float32)
                a[i, kk] = 1
                b[kk, j] = 1
                want = np.zeros((m, n), np.float32)
                want[i, j] = 1
                assert np.array_equal(run_matmul(a, b, False, False), want), (m, k, n, i, kk, j)
            a = r.uniform(-1, 1, (m, k)).astype(np.float32)
            b = (r.standard_normal((k, n)) * np.sqrt(2.0 / k)).astype(np.float32)
            assert_close(run_matmul(a, b, False, False), oracle.matmul(a, b), "matMul m=%d k=%d n=%d" % (m, k, n))
            bias = (r.standard_normal(n) * 0.5).astype(np.float32)
            got = host(tfx.tfx_conv2d(dev(a.reshape(1, 1, m, k)), dev(b.reshape(1, 1, k, n)), dev(bias), 1, PAD_SAME, ACT_RELU6))
            ref = oracle.conv2d(a.reshape(1, 1, m, k), b.reshape(1, 1, k, n), bias, 1, PAD_SAME, ACT_RELU6)
            assert_close(got, ref, "pointwise m=%d k=%d n=%d" % (m, k, n))


def test_all_ones_counts_k_exactly():
    for k in [1, 5, 127, 129, 1000]:
        got = run_matmul(np.ones((37, k), np.float32), np.ones((k, 41), np.float32), False, False)
        assert np.array_equal(got, np.full((37, 41), k, np.float32))


def test_unaligned_base_pointers_take_the_scalar_path():
    import torch
    import paper_1901_05350_amd as tfx
    r = rng(9)
    a = r.uniform(-1, 1, (64, 128)).astype(np.float32)
    b = r.uniform(-1, 1, (128, 64)).astype(np.float32)
    buf_a = torch.empty(64 * 128 + 1, dtype=torch.float32, device="cuda:0")
    buf_b = torch.empty(128 * 64 + 3, dtype=torch.float32, device="cuda:0")
    av = buf_a[1:].view(64, 128)
    bv = buf_b[3:].view(128, 64)
    av.copy_(torch.from_numpy(a))
    bv.copy_(torch.from_numpy(b))
    assert av.data_ptr() % 16 != 0 and bv.data_ptr() % 16 != 0
    assert_close(host(tfx.tfx_matmul(av, bv)), oracle.matmul(a, b), "unaligned matMul")


def test_batch_matmul_small_and_no_leak():
    import paper_1901_05350_amd as tfx
    r = rng(10)
    a = r.standard_normal((5, 70, 33)).astype(np.float32)
    b = r.standard_normal((5, 45, 33)).astype(np.float32)
    got = host(tfx.tfx_batch_matmul(dev(a), dev(b), False, True))
    assert_close(got, oracle.batch_matmul(a, b, False, True), "batchMatMul 5x70x33x45")
    a[3] = 0
    got = host(tfx.tfx_batch_matmul(dev(a), dev(b), False, True))
    assert not got[3].any()


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
def test_batch_matmul_every_layout_with_batch_above_one(ta, tb):
    # the batch stride of each stored layout: ragged small tiles, 64 x 64 tiles, 128 x 128 tiles (XCD-remapped
    # order over batch x tiles) and the 16-row kernels; every batch differs, so a wrong stride shows
    r = rng(12 + 2 * ta + tb)
    for (bt, m, k, n) in [(5, 70, 33, 45), (3, 1, 1, 1), (7, 16, 64, 34), (6, 196, 128, 96), (12, 320, 96, 256),
                          (9, 512, 200, 640), (4, 129, 1024, 130)]:
        a = r.standard_normal((bt, m, k)).astype(np.float32)
        b = r.standard_normal((bt, k, n)).astype(np.float32)
        ref = np.stack([oracle.matmul(a[i], b[i]) for i in range(bt)])
        a_in = np.ascontiguousarray(a.transpose(0, 2, 1)) if ta else a
        b_in = np.ascontiguousarray(b.transpose(0, 2, 1)) if tb else b
        import paper_1901_05350_amd as tfx
        got = host(tfx.tfx_batch_matmul(dev(a_in), dev(b_in), ta, tb))
        assert_close(got, ref, "batchMatMul b=%d m=%d k=%d n=%d ta=%d tb=%d" % (bt, m, k, n, ta, tb))
        assert np.array_equal(oracle.batch_matmul(a_in, b_in, ta, tb), ref)


def test_config_batch_matmul_full_size():
    import paper_1901_05350_amd as tfx
    d = inputs.batch_matmul(seed=3)
    got = host(tfx.tfx_batch_matmul(dev(d["a"]), dev(d["b"]), False, True))
    assert got.shape == (8, 1024, 1024)
    ref = oracle.batch_matmul(d["a"], d["b"], False, True)
    assert_close(got, ref, "batchMatMul 8x1024^3 transposeB")


def test_nan_and_inf_propagate_without_activation():
    # ops are plain arithmetic when no activation is asked for: a NaN in A poisons exactly its row of C
    r = rng(11)
    a = r.uniform(-1, 1, (40, 24)).astype(np.float32)
    b = r.uniform(-1, 1, (24, 50)).astype(np.float32)
    a[7, 3] = np.nan
    a[9, 5] = np.inf
    got = run_matmul(a, b, False, False)
    ref = oracle.matmul(a, b)
    assert np.array_equal(np.isnan(got), np.isnan(ref))
    assert np.isnan(got[7]).all() and not np.isnan(got[8]).any()
    assert np.array_equal(np.isinf(got), np.isinf(ref)) and np.isinf(got[9]).all()
