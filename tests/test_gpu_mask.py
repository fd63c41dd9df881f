"""GPU parity for the bit-mask form of the cache (one bit per element + block offsets): the encoding is
integer work and must match the oracle bit for bit; the weight gradient from it must match the oracle to
the same tolerance as from flat indices (and equals that result bit for bit, the kernels being the same)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_13808_amd as dropit
from dropit_inputs import WORKLOADS, activation, gradient
from gpu_util import to_device, to_host

pytestmark = pytest.mark.gpu


def _mask_host(mask: torch.Tensor) -> np.ndarray:
    return mask.cpu().numpy().view(np.uint32)


def run_and_compare(x, gamma, tag=""):
    print("mask", tag, x.dtype, x.shape, gamma, flush=True)
    k = oracle.keep_count(x.size, gamma)
    want_v, want_i = oracle.compress(x, k)
    want_m, want_b = oracle.mask_from_pairs(want_i, x.size)
    vals, mask, blockptr = dropit.compress_mask(to_device(x), gamma)
    torch.cuda.synchronize()
    assert to_host(vals).tobytes() == want_v.tobytes()
    assert np.array_equal(_mask_host(mask), want_m)
    assert np.array_equal(blockptr.cpu().numpy(), want_b)
    return vals, mask, blockptr


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(300, 100), (1, 8), (31,), (32,), (33,), (1024,), (1025,), (777, 257), (3, 16, 24, 24),
                                   (2049, 1)])
def test_shapes(dtype, shape):
    x = activation(shape, "relu", 940 + len(shape) + shape[-1] % 13, dtype)     # ~half zeros: empty blocks happen at gamma 0.9
    for gamma in (0.9, 0.5, 0.0, 1.0):
        run_and_compare(x, gamma)


def test_sparse_blocks_are_mostly_empty():
    """Nearly everything dropped: most blocks own no pair, runs of empty blocks at both ends."""
    x = np.zeros((5000, 16), dtype=np.float32)
    x[1234, 3] = 2.0
    x[1234, 9] = -3.0
    x[4000, 0] = 1.0
    vals, mask, blockptr = run_and_compare(x, 1.0 - 3.0 / x.size)
    assert vals.numel() == 3 and int(np.count_nonzero(_mask_host(mask))) == 2


@pytest.mark.parametrize("name", ["vitb_fc1", "resnet_conv3x3"])
def test_workload_shapes(name):
    w = WORKLOADS[name]
    run_and_compare(activation(w.x_shape, w.x_dist, w.x_seed, w.dtype), w.gamma, name)


@pytest.mark.parametrize("case", [
    dict(x=(1500, 256), dy=(1500, 128), dtype="bf16", conv=None),             # matrix-core FC path
    dict(x=(777, 257), dy=(777, 33), dtype="bf16", conv=None),                # odd shape
    dict(x=(300, 100), dy=(300, 70), dtype="f32", conv=None),                 # fp32 path
    dict(x=(4, 16, 24, 24), dy=(4, 32, 24, 24), dtype="bf16", conv=(3, 3, 1, 1, 1, 1, 1, 1)),   # matrix-core conv
    dict(x=(2, 8, 15, 15), dy=(2, 8, 8, 8), dtype="bf16", conv=(3, 3, 2, 2, 1, 1, 1, 1)),       # general conv
])
@pytest.mark.parametrize("gamma", [0.9, 0.0])
def test_weight_grad_from_mask(case, gamma):
    print("mask wgrad", case, gamma, flush=True)
    x = activation(case["x"], "gelu", 53, case["dtype"])
    dy = gradient(case["dy"], 0.02, 54, case["dtype"])
    c_out = case["dy"][-1] if case["conv"] is None else case["dy"][1]
    xd, dyd = to_device(x), to_device(dy)
    vals, mask, blockptr = dropit.compress_mask(xd, gamma)
    got = dropit.weight_grad_mask(vals, mask, blockptr, x.shape, dyd, c_out, conv=case["conv"])
    v2, i2 = dropit.compress(xd, gamma)
    flat = dropit.weight_grad(v2, i2, x.shape, dyd, c_out, conv=case["conv"])
    torch.cuda.synchronize()
    assert torch.equal(got, flat)
    k = oracle.keep_count(x.size, gamma)
    xhat = oracle.densify(*oracle.compress(x, k), x.shape)
    if case["conv"] is None:
        ref = oracle.dw_fc(xhat, oracle.widen(dy))
    else:
        c = case["conv"]
        ref = oracle.dw_conv(xhat, oracle.widen(dy), c[0], c[1], stride=c[2:4], pad=c[4:6], dil=c[6:8])
    tol = 1e-3 if case["dtype"] == "bf16" else 1e-5
    assert np.abs(to_host(got).astype(np.float64) - ref).max() <= tol * np.abs(ref).max()


def test_everything_dropped():
    x = activation((64, 32), "normal", 5, "bf16")
    vals, mask, blockptr = dropit.compress_mask(to_device(x), 1.0)
    assert vals.numel() == 0 and int(mask.abs().sum()) == 0 and blockptr.tolist() == [0, 0, 0]
    dW = dropit.weight_grad_mask(vals, mask, blockptr, x.shape, to_device(gradient((64, 16), 0.02, 6, "bf16")), 16)
    torch.cuda.synchronize()
    assert float(dW.abs().sum()) == 0.0


def test_autograd_layer_with_mask_cache():
    """The layers take index_format="mask": same gradients as with flat indices, a smaller cache."""
    from paper_2202_13808_amd import nn as dnn
    torch.manual_seed(3)
    a = dnn.Linear(256, 128, gamma=0.8, device="cuda:0", dtype=torch.bfloat16)
    b = dnn.Linear(256, 128, gamma=0.8, index_format="mask", device="cuda:0", dtype=torch.bfloat16)
    b.load_state_dict(a.state_dict())
    x = to_device(activation((512, 256), "gelu", 9, "bf16"))
    dy = to_device(gradient((512, 128), 0.02, 10, "bf16"))
    with dnn.cache_meter() as ma:
        ya = a(x)
    with dnn.cache_meter() as mb:
        yb = b(x)
    ya.backward(dy)
    yb.backward(dy)
    torch.cuda.synchronize()
    assert torch.equal(a.weight.grad, b.weight.grad)
    assert mb.index_bytes < ma.index_bytes / 2 and mb.value_bytes == ma.value_bytes
