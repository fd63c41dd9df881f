"""Pins for the oracle's random dropping (Sec. 3.3, Random Elements).

The generator is pinned by its published known-answer vectors; the selection by an O(n^2) rank count
with no sort, by the invariants of any k-subset, by independence from the tensor's values, and by the
statistics a uniform draw must show (every position kept with probability k/n; the draws themselves
uniform on 31 bits)."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    rows = 0
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if not line:
                continue
            w = [int(v, 16) for v in line]
            assert list(oracle.philox4x32_10(w[0:4], w[4:6])) == w[6:10]
            rows += 1
    assert rows == 3


def test_key_layout_counter_is_index_div_4_word_is_index_mod_4():
    for seed in (0, 1, 0xDEADBEEF, (0x12345678 << 32) | 0x9ABCDEF0):
        key = (seed & 0xFFFFFFFF, seed >> 32)
        for i in (0, 1, 2, 3, 4, 7, 1000, (1 << 31) - 1, (1 << 31) - 4):
            block = oracle.philox4x32_10((i >> 2, 0, 0, 0), key)
            assert oracle.random_key(i, seed) == int(block[i & 3]) >> 1


def _keys(n, seed):
    return np.array([oracle.random_key(i, seed) for i in range(n)], dtype=np.int64)


@pytest.mark.parametrize("n,seed", [(1, 3), (5, 0), (64, 1), (1000, 42), (1537, 1 << 40)])
def test_selection_equals_rank_count_definition(n, seed):
    x = np.random.default_rng(n).standard_normal(n).astype(np.float32)
    key = _keys(n, seed)
    order = np.arange(n)
    rank = (key[None, :] > key[:, None]).sum(1) + ((key[None, :] == key[:, None]) & (order[None, :] < order[:, None])).sum(1)
    for k in sorted({0, 1, n // 10, n // 2, n - 1, n} - {-1}):
        if k < 0 or k > n:
            continue
        vals, idx = oracle.compress_random(x, k, seed)
        want = np.nonzero(rank < k)[0]
        assert np.array_equal(idx, want.astype(np.int32))
        assert vals.tobytes() == x[want].tobytes()


def test_equal_draws_go_to_the_lowest_index():
    """Planted in the pin, not in the oracle: with 31-bit draws ties are rare, so find two equal keys among
    the first 200 000 by search and cut k between them."""
    seed, n = 7, 200000
    key = _keys(n, seed)
    dup = None
    seen = {}
    for i, v in enumerate(key):
        if v in seen:
            dup = (seen[v], i)
            break
        seen[int(v)] = i
    assert dup is not None, "no equal draws among 200000 keys (expected ~9 by the birthday bound)"
    lo, hi = dup
    above = int((key > key[lo]).sum())
    x = np.arange(n, dtype=np.float32)
    _, idx = oracle.compress_random(x, above + 1, seed)
    kept = set(idx.tolist())
    assert lo in kept and hi not in kept


def test_kept_set_does_not_depend_on_the_values():
    rng = np.random.default_rng(0)
    a = rng.standard_normal(5000).astype(np.float32)
    b = np.zeros(5000, dtype=np.float32)
    c = (rng.standard_normal(5000).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)   # bf16 bit patterns
    ia = oracle.compress_random(a, 500, 11)[1]
    assert np.array_equal(ia, oracle.compress_random(b, 500, 11)[1])
    vc, ic = oracle.compress_random(c, 500, 11)
    assert np.array_equal(ia, ic) and np.array_equal(vc, c[ic])
    assert not np.array_equal(ia, oracle.compress_random(a, 500, 12)[1])            # another seed, another set
    assert np.all(np.diff(ia) > 0) and ia[0] >= 0 and ia[-1] < 5000


def test_every_position_is_kept_with_probability_k_over_n():
    n, k, trials = 400, 100, 600
    x = np.zeros(n, dtype=np.float32)
    hits = np.zeros(n)
    for seed in range(trials):
        hits[oracle.compress_random(x, k, 1000 + seed)[1]] += 1
    p = k / n
    z = (hits - trials * p) / np.sqrt(trials * p * (1 - p))
    assert np.abs(z).max() < 4.5                    # 400 positions: P(|z| > 4.5 anywhere) ~ 3e-3
    assert abs(z.std() - 1.0) < 0.15                # too regular or too clumped both fail
    first_half = hits[: n // 2].sum() / (trials * k)
    assert abs(first_half - 0.5) < 0.01


def test_draws_are_uniform_on_31_bits():
    key = _keys(100000, 5)
    assert key.min() >= 0 and key.max() < (1 << 31)
    counts = np.bincount(key >> 27, minlength=16)     # 16 equal cells
    chi2 = ((counts - 6250.0) ** 2 / 6250.0).sum()
    assert chi2 < 45.0                                # 15 degrees of freedom: P(chi2 > 45) ~ 1e-4
    assert abs(key.mean() / (1 << 31) - 0.5) < 0.005
    assert abs(np.corrcoef(key[:-1], key[1:])[0, 1]) < 0.02
