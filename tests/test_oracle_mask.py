"""Pins for the oracle's bit-mask form of the retained index set (one bit per element + a block
offset table): a hand-made example, numpy's packbits / searchsorted as the independent statement,
the round trip, and the byte count it exists for."""
import numpy as np
import pytest

import oracle


def test_hand_made_example():
    # 70 elements, blocks of 32: retained 0, 5, 31 | 32, 40 | 69
    mask, blockptr = oracle.mask_from_pairs(np.array([0, 5, 31, 32, 40, 69], dtype=np.int32), 70, block=32)
    assert mask.tolist() == [(1 << 0) | (1 << 5) | (1 << 31), (1 << 0) | (1 << 8), 1 << 5]
    assert blockptr.tolist() == [0, 3, 5, 6]
    mask, blockptr = oracle.mask_from_pairs(np.array([], dtype=np.int32), 33, block=32)
    assert mask.tolist() == [0, 0] and blockptr.tolist() == [0, 0, 0]
    mask, blockptr = oracle.mask_from_pairs(np.arange(5, dtype=np.int32), 5, block=64)
    assert mask.tolist() == [0b11111] and blockptr.tolist() == [0, 5]


@pytest.mark.parametrize("numel", [1, 31, 32, 33, 1024, 1025, 5000, 100003])
@pytest.mark.parametrize("keep", [0.0, 0.1, 0.6, 1.0])
@pytest.mark.parametrize("block", [32, 1024])
def test_against_packbits_and_searchsorted_and_round_trip(numel, keep, block):
    rng = np.random.default_rng(numel * 7 + int(keep * 10) + block)
    idx = np.sort(rng.choice(numel, size=int(keep * numel), replace=False)).astype(np.int32)
    mask, blockptr = oracle.mask_from_pairs(idx, numel, block)
    dense = np.zeros((numel + 31) // 32 * 32, dtype=np.uint8)
    dense[idx] = 1
    assert np.array_equal(mask, np.packbits(dense, bitorder="little").view("<u4"))
    blocks = (numel + block - 1) // block
    assert np.array_equal(blockptr, np.searchsorted(idx, np.arange(blocks + 1, dtype=np.int64) * block).astype(np.int32))
    assert int(sum(bin(int(w)).count("1") for w in mask)) == idx.size == blockptr[-1]
    assert np.array_equal(oracle.pairs_from_mask(mask, blockptr, numel, block), idx)


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        oracle.mask_from_pairs(np.array([5, 5], dtype=np.int32), 16)               # not strictly ascending
    with pytest.raises(ValueError):
        oracle.mask_from_pairs(np.array([16], dtype=np.int32), 16)                 # outside the tensor
    with pytest.raises(ValueError):
        oracle.mask_from_pairs(np.array([1], dtype=np.int32), 16, block=48)        # block not a whole number of mask words
    mask, blockptr = oracle.mask_from_pairs(np.array([3, 40], dtype=np.int32), 64, block=32)
    blockptr[1] += 1
    with pytest.raises(ValueError):
        oracle.pairs_from_mask(mask, blockptr, 64, block=32)                       # offsets that contradict the mask


def test_mask_beats_int32_indices_when_more_than_one_in_32_is_kept():
    """numel/8 bytes of mask (+ 4 bytes per 1024 elements) against 4k bytes of int32 indices."""
    from dropit_inputs import WORKLOADS
    for w in WORKLOADS.values():
        numel = int(np.prod(w.x_shape))
        k = oracle.keep_count(numel, w.gamma)
        mask_bytes = 4 * ((numel + 31) // 32) + 4 * ((numel + 1023) // 1024 + 1)
        assert mask_bytes < 4 * k, w                      # every benchmark shape keeps 10-20 %
        assert mask_bytes / (4 * k) < 0.33 / (1 - w.gamma) / 10 + 0.01
    numel = 1 << 20
    for keep in (1 / 64, 1 / 40):                         # below 1/32 the indices are smaller
        assert 4 * int(keep * numel) < numel // 8
