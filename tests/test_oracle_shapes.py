"""Pins for the oracle's output-shape and padding rules (CPU only).

The expected values are hand-worked rows in tests/golden/same_valid_extents.txt.
"""
import os

import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "same_valid_extents.txt")


def golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            rows.append(line.split())
    return rows


@pytest.mark.parametrize("row", golden_rows(), ids=lambda r: "-".join(r))
def test_extent_matches_hand_worked_table(row):
    pad = oracle.PAD_SAME if row[0] == "same" else oracle.PAD_VALID
    n, k, s = int(row[1]), int(row[2]), int(row[3])
    if row[4] == "err":
        with pytest.raises(oracle.OracleError):
            oracle.out_extent(n, k, s, pad)
        return
    assert oracle.out_extent(n, k, s, pad) == (int(row[4]), int(row[5]), int(row[6]))


@pytest.mark.parametrize("n", range(1, 40))
@pytest.mark.parametrize("k", [1, 2, 3, 5, 7])
@pytest.mark.parametrize("s", [1, 2, 3, 4])
def test_extent_invariants(n, k, s):
    # SAME: every output position's window start lies inside the padded input, the window of the
    # last output ends inside it too, and the padded extent is the smallest that allows this.
    out, pb, pa = oracle.out_extent(n, k, s, oracle.PAD_SAME)
    assert out == -(-n // s)
    assert 0 <= pb <= pa <= pb + 1
    assert (out - 1) * s + k <= n + pb + pa
    if pb + pa > 0:
        assert (out - 1) * s + k == n + pb + pa
    if n >= k:
        out_v, pbv, pav = oracle.out_extent(n, k, s, oracle.PAD_VALID)
        assert (pbv, pav) == (0, 0)
        assert (out_v - 1) * s + k <= n < out_v * s + k  # last window fits, one more would not
    else:
        with pytest.raises(oracle.OracleError):
            oracle.out_extent(n, k, s, oracle.PAD_VALID)


def test_extent_rejects_bad_arguments():
    for bad in [(0, 3, 1), (5, 0, 1)]:
        with pytest.raises(oracle.OracleError) as e:
            oracle.out_extent(*bad, oracle.PAD_SAME)
        assert e.value.code == -2
    with pytest.raises(oracle.OracleError) as e:
        oracle.out_extent(5, 3, 0, oracle.PAD_SAME)
    assert e.value.code == -3
    with pytest.raises(oracle.OracleError) as e:
        oracle.out_extent(5, 3, 1, 7)
    assert e.value.code == -3


def test_matmul_shape_all_transpose_combos():
    assert oracle.matmul_out_shape((2, 3), (3, 5)) == (2, 5)
    assert oracle.matmul_out_shape((3, 2), (3, 5), transpose_a=True) == (2, 5)
    assert oracle.matmul_out_shape((2, 3), (5, 3), transpose_b=True) == (2, 5)
    assert oracle.matmul_out_shape((3, 2), (5, 3), transpose_a=True, transpose_b=True) == (2, 5)
    for args in [((2, 3), (4, 5), False, False), ((2, 3), (3, 5), True, False), ((2, 3), (3, 5), False, True)]:
        with pytest.raises(oracle.OracleError):
            oracle.matmul_out_shape(*args)


def test_conv_shapes():
    # MobileNet first layer and a stride-2 depthwise layer
    assert oracle.conv2d_out_shape((1, 224, 224, 3), (3, 3, 3, 32), 2, oracle.PAD_SAME) == \
        ((1, 112, 112, 32), (0, 1, 0, 1))
    assert oracle.depthwise_conv2d_out_shape((1, 112, 112, 64), (3, 3, 64, 1), 2, oracle.PAD_SAME) == \
        ((1, 56, 56, 64), (0, 1, 0, 1))
    assert oracle.depthwise_conv2d_out_shape((2, 7, 9, 5), (3, 2, 5, 3), (1, 2), oracle.PAD_SAME) == \
        ((2, 7, 5, 15), (1, 1, 0, 1))
    assert oracle.conv2d_out_shape((2, 7, 9, 5), (3, 2, 5, 4), (2, 1), oracle.PAD_VALID) == \
        ((2, 3, 8, 4), (0, 0, 0, 0))
    with pytest.raises(oracle.OracleError):  # channel mismatch
        oracle.conv2d_out_shape((1, 8, 8, 3), (3, 3, 4, 8), 1, oracle.PAD_SAME)
    with pytest.raises(oracle.OracleError):  # filter larger than image under VALID
        oracle.conv2d_out_shape((1, 2, 8, 3), (3, 3, 3, 8), 1, oracle.PAD_VALID)
