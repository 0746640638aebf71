"""Pins for the oracle's matMul / batchMatMul (CPU only).

matMul is defined by Listing 2 (Section 4.1): C[r,c] = sum_i A[r,i] * B[i,c].
Each test fixes the result by something other than the oracle itself: identities,
one-hot products, exact integer cases worked by hand, numpy float64, pure-Python loops.
"""
import numpy as np
import pytest

import oracle


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def test_hand_worked_integers():
    a = np.array([[1, 2, 3], [4, 5, 6]], dtype=np.float32)
    b = np.array([[7, 8], [9, 10], [11, 12]], dtype=np.float32)
    # row 0: 1*7+2*9+3*11 = 58, 1*8+2*10+3*12 = 64; row 1: 4*7+5*9+6*11 = 139, 4*8+5*10+6*12 = 154
    assert oracle.matmul(a, b).tolist() == [[58, 64], [139, 154]]
    # a^T (3x2) times b^T (2x3):  [[1,4],[2,5],[3,6]] x [[7,9,11],[8,10,12]]
    want = [[1 * 7 + 4 * 8, 1 * 9 + 4 * 10, 1 * 11 + 4 * 12],
            [2 * 7 + 5 * 8, 2 * 9 + 5 * 10, 2 * 11 + 5 * 12],
            [3 * 7 + 6 * 8, 3 * 9 + 6 * 10, 3 * 11 + 6 * 12]]
    assert oracle.matmul(a, b, transpose_a=True, transpose_b=True).tolist() == want
    # non-square operands distinguish a transposed operand from a plain one:
    # a (2x3) times a^T given as transpose_b of a -> Gram matrix
    assert oracle.matmul(a, a, transpose_b=True).tolist() == [[14, 32], [32, 77]]
    assert oracle.matmul(a, a, transpose_a=True).tolist() == [[17, 22, 27], [22, 29, 36], [27, 36, 45]]


@pytest.mark.parametrize("m,k", [(5, 7), (64, 128), (33, 1)])
def test_identity_is_bit_exact(m, k):
    a = rng(1).standard_normal((m, k)).astype(np.float32)
    assert np.array_equal(oracle.matmul(a, np.eye(k, dtype=np.float32)), a)
    assert np.array_equal(oracle.matmul(np.eye(m, dtype=np.float32), a), a)


def test_one_hot_product():
    m, k, n = 6, 9, 7
    for (i, kk, j) in [(0, 0, 0), (5, 8, 6), (2, 3, 4)]:
        a = np.zeros((m, k), np.float32)
        b = np.zeros((k, n), np.float32)
        a[i, kk] = 1
        b[kk, j] = 1
        want = np.zeros((m, n), np.float32)
        want[i, j] = 1
        assert np.array_equal(oracle.matmul(a, b), want)
        b2 = np.zeros((k, n), np.float32)
        b2[(kk + 1) % k, j] = 1  # contraction index mismatch -> zero
        assert not oracle.matmul(a, b2).any()


@pytest.mark.parametrize("k", [1, 2, 3, 5, 127, 129, 1000])
def test_all_ones_counts_k(k):
    # shared dimensions that are not multiples of 4 (Listing 2 assumes a multiple of 4 only for brevity)
    c = oracle.matmul(np.ones((3, k), np.float32), np.ones((k, 4), np.float32))
    assert np.array_equal(c, np.full((3, 4), k, np.float32))


@pytest.mark.parametrize("ta", [False, True])
@pytest.mark.parametrize("tb", [False, True])
def test_transpose_flags_equal_explicit_transpose(ta, tb):
    r = rng(2)
    a = r.standard_normal((13, 17)).astype(np.float32)
    b = r.standard_normal((17, 11)).astype(np.float32)
    plain = oracle.matmul(a, b)
    a_in = np.ascontiguousarray(a.T) if ta else a
    b_in = np.ascontiguousarray(b.T) if tb else b
    assert np.array_equal(oracle.matmul(a_in, b_in, ta, tb), plain)
    # (AB)^T = B^T A^T
    assert np.array_equal(oracle.matmul(b, a, transpose_a=True, transpose_b=True), plain.T)


@pytest.mark.parametrize("m,k,n", [(64, 128, 64), (7, 129, 5), (1, 1, 1), (31, 2, 65)])
def test_against_numpy_float64(m, k, n):
    r = rng(3)
    a = r.uniform(-1, 1, (m, k)).astype(np.float32)
    b = r.uniform(-1, 1, (k, n)).astype(np.float32)
    want = a.astype(np.float64) @ b.astype(np.float64)
    got = oracle.matmul(a, b)
    # double accumulation + one rounding: at most half an ulp of float32 from the float64 product
    assert np.all(np.abs(got - want) <= 2.0 ** -24 * np.abs(want) + 1e-12 * k)


def test_against_pure_python_loops_exact_integers():
    r = rng(4)
    a = r.integers(-4, 5, (5, 6)).astype(np.float32)
    b = r.integers(-4, 5, (6, 3)).astype(np.float32)
    want = [[sum(int(a[i, k]) * int(b[k, j]) for k in range(6)) for j in range(3)] for i in range(5)]
    assert oracle.matmul(a, b).tolist() == want


def test_batch_equals_loop_and_batches_do_not_leak():
    r = rng(5)
    a = r.standard_normal((4, 9, 6)).astype(np.float32)
    b = r.standard_normal((4, 7, 6)).astype(np.float32)
    c = oracle.batch_matmul(a, b, transpose_b=True)
    assert c.shape == (4, 9, 7)
    for i in range(4):
        assert np.array_equal(c[i], oracle.matmul(a[i], b[i], transpose_b=True))
    a2 = a.copy()
    a2[2] = 0
    c2 = oracle.batch_matmul(a2, b, transpose_b=True)
    assert not c2[2].any()
    for i in (0, 1, 3):
        assert np.array_equal(c2[i], c[i])
    with pytest.raises(oracle.OracleError):
        oracle.batch_matmul(a[:3], b, transpose_b=True)
