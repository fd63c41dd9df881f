"""Pins for the oracle's row form of the retained index set (16-bit in-row positions + row offsets):
a hand-made example, numpy's searchsorted / remainder as the independent statement, the round trip,
and the byte count it exists for."""
import numpy as np
import pytest

import oracle


def test_hand_made_example():
    # 4 rows of 4: retained flat indices 1, 2 | 7 | 8 | 15
    col, rowptr = oracle.rows_from_pairs(np.array([1, 2, 7, 8, 15], dtype=np.int32), (4, 4))
    assert col.tolist() == [1, 2, 3, 0, 3]
    assert rowptr.tolist() == [0, 2, 3, 4, 5]
    # empty rows in the middle and at both ends
    col, rowptr = oracle.rows_from_pairs(np.array([9, 10], dtype=np.int32), (2, 3, 3))
    assert col.tolist() == [0, 1] and rowptr.tolist() == [0, 0, 0, 0, 2, 2, 2]
    col, rowptr = oracle.rows_from_pairs(np.array([], dtype=np.int32), (3, 5))
    assert col.size == 0 and rowptr.tolist() == [0, 0, 0, 0]


@pytest.mark.parametrize("shape", [(7, 13), (64, 768), (3, 5, 7, 8), (1, 65536), (100,), (50, 1)])
@pytest.mark.parametrize("keep", [0.0, 0.1, 0.6, 1.0])
def test_against_searchsorted_and_round_trip(shape, keep):
    rng = np.random.default_rng(hash((shape, keep)) % (1 << 32))
    numel = int(np.prod(shape))
    idx = np.sort(rng.choice(numel, size=int(keep * numel), replace=False)).astype(np.int32)
    col, rowptr = oracle.rows_from_pairs(idx, shape)
    L = shape[-1]
    rows = numel // L
    assert np.array_equal(col, (idx % L).astype(np.uint16))
    assert np.array_equal(rowptr, np.searchsorted(idx, np.arange(rows + 1, dtype=np.int64) * L).astype(np.int32))
    assert np.array_equal(oracle.pairs_from_rows(col, rowptr, shape), idx)


def test_rejects_what_it_cannot_encode():
    with pytest.raises(ValueError):
        oracle.rows_from_pairs(np.array([0], dtype=np.int32), (2, 65537))          # position needs 17 bits
    with pytest.raises(ValueError):
        oracle.rows_from_pairs(np.array([5, 5], dtype=np.int32), (4, 4))           # not strictly ascending
    with pytest.raises(ValueError):
        oracle.rows_from_pairs(np.array([16], dtype=np.int32), (4, 4))             # outside the tensor


def test_index_bytes_shrink_for_the_benchmark_shapes():
    """int32 flat indices cost 4k bytes; the row form 2k + 4(rows+1): 0.50-0.51 of that for the
    transformer shapes, 0.59 for the 56-wide convolution rows, 0.66 for the 64-wide toy layer."""
    from dropit_inputs import WORKLOADS
    for w in WORKLOADS.values():
        numel = int(np.prod(w.x_shape))
        k = oracle.keep_count(numel, w.gamma)
        rows = numel // w.x_shape[-1]
        ratio = (2 * k + 4 * (rows + 1)) / (4 * k)
        assert ratio < (0.52 if w.x_shape[-1] >= 768 else 0.67), (w, ratio)
