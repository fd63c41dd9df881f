"""Pins for the oracle's keep count, min-k selection and recover.

The oracle (oracle/dropit_oracle.c) is checked here against things that are not
the oracle: an O(n^2) rank-count definition with no sort, invariants the paper
fixes, the CPU library top-k where ties cannot matter, closed-form Gaussian
quantiles, and the memory ratios the paper prints in Table 4.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from dropit_inputs import WORKLOADS, activation, bf16_bits_to_f32, f32_to_bf16_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                out.append(line.split())
    return out


# ---------------------------------------------------------------- keep count
def test_keep_count_literals():
    for numel, gamma, k in _rows("keep_counts.txt"):
        assert oracle.keep_count(int(numel), float(gamma)) == int(k)


def test_keep_count_workload_table():
    expect = {"tiny_fc": 1638, "vitb_fc1": 968294, "vitb_fc2": 3873177, "vitdet_fc1": 1258291,
              "vitdet_fc2": 5033164, "resnet_conv3x3": 2569011}
    for name, k in expect.items():
        w = WORKLOADS[name]
        assert oracle.keep_count(w.numel, w.gamma) == k


def test_keep_count_edges():
    assert oracle.keep_count(1000, 0.0) == 1000          # gamma=0 is the baseline: keep everything
    assert oracle.keep_count(1000, 1.0) == 0
    assert oracle.keep_count(0, 0.5) == 0
    assert oracle.keep_count(100, 0.9) == 10              # not 9: (1.0-0.9)*100 < 10 in binary
    assert oracle.keep_count(10, 0.25) == 7               # floor(7.5)
    assert oracle.keep_count(3, 0.5) == 1                 # floor(1.5)
    for bad in (-0.1, 1.0000001, float("nan"), float("inf")):
        assert oracle.keep_count(10, bad) == -1
    assert oracle.keep_count(-1, 0.5) == -1


def test_keep_count_is_floor_for_exact_gammas():
    # gammas exactly representable in binary: floor((1-g)*n) in rational arithmetic
    for g in (0.0, 0.125, 0.25, 0.5, 0.75, 0.875, 1.0):
        for n in (0, 1, 2, 3, 7, 10, 1000, 16384, 9682944, 2**31 - 1):
            exact = (Fraction(1) - Fraction(g)) * n
            assert oracle.keep_count(n, g) == exact.numerator // exact.denominator


def test_keep_count_never_exceeds_proportion_and_monotone():
    n = 12345
    prev = n + 1
    for g in np.linspace(0.0, 1.0, 101):
        k = oracle.keep_count(n, float(g))
        assert 0 <= k <= n
        assert k <= (1.0 - g) * n + 1e-6      # memory saving is at least gamma
        assert k > (1.0 - g) * n - 1 - 1e-6
        assert k <= prev
        prev = k


def test_keep_count_reproduces_table4_ratios():
    # DeiT-S FC inputs at batch 1024: memory scales as 1-gamma (Table 4).
    rows = [(int(g), float(m)) for g, m in _rows("table4_cached_memory.txt")]
    base = dict(rows)[0]
    numel = 1024 * 197 * 384
    for g, printed in rows:
        k = oracle.keep_count(numel, g / 100.0)
        assert abs(base * k / numel - printed) <= 0.006, (g, printed)


# ---------------------------------------------------------------- brute force
def _keys(x):
    if x.dtype == np.float32:
        return x.view(np.uint32) & np.uint32(0x7FFFFFFF)
    return (x & np.uint16(0x7FFF)).astype(np.uint32)


def brute_force_keep_mask(x, k):
    """rank_i = #{j: key_j > key_i} + #{j < i: key_j == key_i}; keep iff rank_i < k.  No sort."""
    key = _keys(x).astype(np.int64)
    n = key.size
    gt = (key[None, :] > key[:, None]).sum(axis=1)
    earlier_eq = np.tril(key[None, :] == key[:, None], k=-1).sum(axis=1)
    return (gt + earlier_eq) < k


def _adversarial_f32(n, rng):
    cases = {
        "normal": rng.standard_normal(n).astype(np.float32),
        "all_equal": np.full(n, 1.5, np.float32),
        "all_zero_mixed_sign": np.where(rng.random(n) < 0.5, np.float32(0.0), np.float32(-0.0)).astype(np.float32),
        "two_valued": np.where(rng.random(n) < 0.3, np.float32(2.0), np.float32(-0.5)).astype(np.float32),
        "pm_pairs": (rng.integers(1, 6, n) * rng.choice([-1.0, 1.0], n)).astype(np.float32),
        "denormal": (rng.integers(0, 8, n).astype(np.uint32)).view(np.float32),
        "relu": np.maximum(rng.standard_normal(n), 0).astype(np.float32),
    }
    special = rng.standard_normal(n).astype(np.float32)
    special[::7] = np.inf
    special[1::11] = -np.inf
    special[2::13] = np.nan
    special[3::17] = -np.float32(np.nan)
    cases["inf_nan"] = special
    return cases


@pytest.mark.parametrize("n", [1, 2, 33, 64])
def test_compress_matches_brute_force_every_k(n):
    rng = np.random.default_rng(7 + n)
    for name, x in _adversarial_f32(n, rng).items():
        for xx in (x, f32_to_bf16_bits(x)):
            for k in range(n + 1):
                vals, idx = oracle.compress(xx, k)
                mask = brute_force_keep_mask(xx, k)
                want = np.nonzero(mask)[0].astype(np.int32)
                assert np.array_equal(idx, want), (name, xx.dtype, k)
                assert vals.tobytes() == xx[want].tobytes(), (name, xx.dtype, k)


@pytest.mark.parametrize("n,ks", [(1000, (0, 1, 100, 499, 999, 1000)), (3000, (300, 1500, 2999))])
def test_compress_matches_brute_force_larger(n, ks):
    rng = np.random.default_rng(n)
    for name, x in _adversarial_f32(n, rng).items():
        for xx in (x, f32_to_bf16_bits(x)):
            for k in ks:
                vals, idx = oracle.compress(xx, k)
                want = np.nonzero(brute_force_keep_mask(xx, k))[0].astype(np.int32)
                assert np.array_equal(idx, want), (name, xx.dtype, k)
                assert vals.tobytes() == xx[want].tobytes()


# ---------------------------------------------------------------- invariants
def check_selection_invariants(x, k, vals, idx):
    """Properties that hold for the one correct answer at any size (also used by the GPU tests)."""
    x = x.reshape(-1)
    n = x.size
    assert idx.dtype == np.int32 and idx.shape == (k,) and vals.shape == (k,)
    if k == 0:
        return
    assert idx[0] >= 0 and idx[-1] < n
    assert np.all(np.diff(idx.astype(np.int64)) > 0)                  # strictly ascending, no duplicates
    assert vals.tobytes() == x[idx].tobytes()                          # exact bits, sign kept
    key = _keys(x)
    kept = np.zeros(n, dtype=bool)
    kept[idx] = True
    t = key[kept].min()
    if k < n:
        assert t >= key[~kept].max()                                   # every kept |x| >= every dropped |x|
    # ties at the threshold: the kept ones are exactly the first m by flat index
    tie_pos = np.nonzero(key == t)[0]
    m = int(kept[tie_pos].sum())
    assert m >= 1
    assert np.all(kept[tie_pos[:m]]) and not np.any(kept[tie_pos[m:]])


@pytest.mark.parametrize("name,shape,dist,gamma,dtype", [
    ("ln", (512, 768), "normal", 0.9, "bf16"),
    ("gelu", (256, 3072), "gelu", 0.9, "bf16"),
    ("relu", (4, 16, 56, 56), "relu", 0.8, "bf16"),
    ("relu_low_gamma", (4, 16, 56, 56), "relu", 0.3, "bf16"),      # threshold key is 0: ties among zeros
    ("f32", (256, 64), "normal", 0.9, "f32"),
])
def test_compress_invariants_on_workload_like_inputs(name, shape, dist, gamma, dtype):
    x = activation(shape, dist, 4242, dtype)
    k = oracle.keep_count(x.size, gamma)
    vals, idx = oracle.compress(x, k)
    check_selection_invariants(x, k, vals, idx)
    # E[alpha] >= 1-gamma (App. A.3): retained magnitude mass is at least the retained fraction
    mag = np.abs(oracle.widen(x).reshape(-1))
    assert mag[idx].sum() / mag.sum() >= k / x.size


def test_constant_tensor_keeps_first_k():
    x = np.full(1000, -3.0, np.float32)
    vals, idx = oracle.compress(x, 137)
    assert np.array_equal(idx, np.arange(137, dtype=np.int32))
    assert np.all(vals == np.float32(-3.0))


def test_two_level_tensor_cut_in_lower_level():
    # 10 large values, the rest equal small ones: k = 25 keeps all 10 large + the first 15 small
    x = np.full(200, 0.25, np.float32)
    big = np.array([3, 17, 40, 41, 77, 100, 150, 151, 198, 199])
    x[big] = -8.0
    vals, idx = oracle.compress(x, 25)
    small_first = [i for i in range(200) if i not in set(big)][:15]
    assert np.array_equal(idx, np.array(sorted(list(big) + small_first), dtype=np.int32))


def test_negative_zero_ties_with_positive_zero():
    x = np.array([0.0, -0.0, 0.0, -0.0, 1.0], np.float32)
    vals, idx = oracle.compress(x, 3)
    assert idx.tolist() == [0, 1, 4]
    assert vals.view(np.uint32).tolist() == [0x00000000, 0x80000000, 0x3F800000]   # sign of -0 preserved


def test_nan_ranks_above_inf_above_finite():
    x = np.array([1.0, np.inf, np.nan, -2.0, -np.inf], np.float32)
    assert oracle.compress(x, 1)[1].tolist() == [2]
    assert oracle.compress(x, 3)[1].tolist() == [1, 2, 4]
    assert oracle.compress(x, 4)[1].tolist() == [1, 2, 3, 4]


# ---------------------------------------------------------------- library special case
def test_compress_equals_torch_topk_when_no_ties():
    # config-1-like: fp32 N(0,1); no tie straddles the cut (checked) -> the kept set is unique
    x = activation((256, 64), "normal", 1001, "f32")
    mag = np.abs(x.reshape(-1))
    k = oracle.keep_count(x.size, 0.9)
    desc = np.sort(mag)[::-1]
    assert desc[k - 1] > desc[k]
    _, idx = oracle.compress(x, k)
    top = torch.topk(torch.from_numpy(mag), k).indices.numpy()
    assert np.array_equal(idx, np.sort(top).astype(np.int32))


# ---------------------------------------------------------------- closed-form thresholds
@pytest.mark.parametrize("dist,gamma,t_expected", [
    ("normal", 0.9, 1.6449),     # Phi^-1(0.95)
    ("gelu", 0.9, 1.1534),       # z*Phi(z) at z = Phi^-1(0.9) = 1.2816
    ("relu", 0.8, 0.8416),       # Phi^-1(0.8)
])
def test_threshold_lands_on_gaussian_quantile(dist, gamma, t_expected):
    x = activation((2048, 512), dist, 99, "bf16")            # ~1e6 samples
    k = oracle.keep_count(x.size, gamma)
    vals, _ = oracle.compress(x, k)
    t = np.abs(bf16_bits_to_f32(vals)).min()
    # quantile sampling error ~ sqrt(p(1-p)/n)/pdf ~ 2e-3; bf16 bin width 2^-7 in [1,2), 2^-8 in [.5,1)
    assert abs(t - t_expected) < 0.012, t


# ---------------------------------------------------------------- recover
def test_densify_roundtrip_gamma_zero_is_identity():
    for dtype in ("f32", "bf16"):
        x = activation((37, 19), "normal", 5, dtype)
        vals, idx = oracle.compress(x, x.size)
        assert np.array_equal(idx, np.arange(x.size, dtype=np.int32))
        xh = oracle.densify(vals, idx, x.shape)
        assert np.array_equal(xh, oracle.widen(x))


def test_densify_zero_fill_and_values():
    x = np.array([[0.5, -4.0, 0.0], [3.0, -0.25, 1.0]], np.float32)
    vals, idx = oracle.compress(x, 2)
    xh = oracle.densify(vals, idx, x.shape)
    assert np.array_equal(xh, np.array([[0, -4.0, 0], [3.0, 0, 0]], np.float64))
    with pytest.raises(ValueError):
        oracle.densify(vals, np.array([0, 6], np.int32), x.shape)


def test_widen_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x0001, 0x7F80, 0x4049], np.uint16)
    w = oracle.widen(bits)
    assert w[0] == 1.0 and w[1] == -1.0 and w[2] == 2.0 ** -133 and np.isinf(w[3]) and w[4] == 3.140625
