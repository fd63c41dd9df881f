"""GPU parity: dropit_compress_random (through the C ABI) vs the CPU oracle, bit for bit.

Both sides draw the same Philox4x32-10 keys from (seed, flat index), each with its own implementation;
the oracle's is pinned by the generator's published known-answer vectors."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_13808_amd as dropit
from paper_2202_13808_amd import nn as dnn
from dropit_inputs import WORKLOADS, activation, gradient
from gpu_util import to_device, to_host

pytestmark = pytest.mark.gpu

BIG_SEED = (0xC0FFEE12 << 32) | 0x3456789A


def run_and_compare(x, gamma, seed, tag=""):
    print("random", tag, x.dtype, x.size, gamma, hex(seed), flush=True)
    k = oracle.keep_count(x.size, gamma)
    want_v, want_i = oracle.compress_random(x, k, seed)
    vals, idx = dropit.compress_random(to_device(x), gamma, seed)
    torch.cuda.synchronize()
    got_v, got_i = to_host(vals), to_host(idx)
    assert got_i.shape == (k,) and got_v.shape == (k,)
    assert np.array_equal(got_i, want_i)
    assert got_v.tobytes() == want_v.tobytes()
    return got_v, got_i


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("numel", [1, 3, 4, 5, 8, 4095, 4097, 300003, (1 << 20) + 5])
def test_sizes_and_ragged_tails(dtype, numel):
    x = activation((numel,), "normal", 700 + numel % 89, dtype)
    for gamma, seed in ((0.9, 1), (0.5, BIG_SEED), (0.0, 2)):
        run_and_compare(x, gamma, seed)


@pytest.mark.parametrize("name", ["tiny_fc", "vitb_fc1", "resnet_conv3x3"])
def test_workload_shapes(name):
    w = WORKLOADS[name]
    x = activation(w.x_shape, w.x_dist, w.x_seed, w.dtype)
    run_and_compare(x, w.gamma, 20220228, name)


def test_kept_set_depends_on_the_seed_only():
    a = activation((50000,), "gelu", 1, "bf16")
    b = activation((50000,), "relu", 2, "bf16")
    ia = to_host(dropit.compress_random(to_device(a), 0.8, 5)[1])
    ib = to_host(dropit.compress_random(to_device(b), 0.8, 5)[1])
    ic = to_host(dropit.compress_random(to_device(a), 0.8, 6)[1])
    assert np.array_equal(ia, ib) and not np.array_equal(ia, ic)
    # about k/n of each half is kept
    assert abs((ia < 25000).mean() - 0.5) < 0.02


def test_separate_kernel_mode_and_everything_dropped():
    x = activation((70001,), "normal", 3, "f32")
    dropit.set_select_mode(1)
    try:
        run_and_compare(x, 0.7, 99, "separate kernels")
    finally:
        dropit.set_select_mode(0)
    vals, idx = dropit.compress_random(to_device(x), 1.0, 99)
    assert vals.numel() == 0 and idx.numel() == 0


def test_weight_grad_from_a_random_cache():
    """The pairs feed dropit_weight_grad unchanged (Sec. 3.2: the backward pass only sees R(a^))."""
    x = activation((1500, 256), "normal", 11, "bf16")
    dy = gradient((1500, 128), 0.02, 12, "bf16")
    vals, idx = dropit.compress_random(to_device(x), 0.9, 77)
    dW = dropit.weight_grad(vals, idx, x.shape, to_device(dy), 128)
    torch.cuda.synchronize()
    k = oracle.keep_count(x.size, 0.9)
    xhat = oracle.densify(*oracle.compress_random(x, k, 77), x.shape)
    ref = oracle.dw_fc(xhat, oracle.widen(dy))
    got = to_host(dW).astype(np.float64)
    assert np.abs(got - ref).max() <= 1e-3 * np.abs(ref).max()


def test_random_layer_draws_a_new_subset_each_call():
    layer = dnn.Linear(64, 32, gamma=0.9, strategy="random", seed=123, device="cuda:0", dtype=torch.bfloat16)
    x_h = activation((40, 64), "normal", 21, "bf16")
    dy_h = gradient((40, 32), 0.02, 22, "bf16")
    grads = []
    for call in range(2):
        layer.zero_grad(set_to_none=True)
        layer(to_device(x_h)).backward(to_device(dy_h))
        torch.cuda.synchronize()
        grads.append(layer.weight.grad.float().cpu().numpy().astype(np.float64))
        seed = (123 + call * 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
        k = oracle.keep_count(x_h.size, 0.9)
        ref = oracle.dw_fc(oracle.densify(*oracle.compress_random(x_h, k, seed), x_h.shape), oracle.widen(dy_h))
        assert np.abs(grads[-1] - ref).max() <= (1e-3 + 2.0 ** -8) * np.abs(ref).max()
    assert np.abs(grads[0] - grads[1]).max() > 0
