"""GPU tests of the autograd wrappers: the layer's weight gradient against the fp64 CPU oracle
(same tolerance as the raw entry points), everything the method leaves untouched (forward output,
input gradient, bias gradient) against the plain torch layer, and the cached-bytes accounting
against the closed form k * element size."""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_13808_amd as dropit
from paper_2202_13808_amd import nn as dnn
from dropit_inputs import activation, gradient
from gpu_util import to_device, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-3}


def _oracle_xhat(x, gamma):
    k = oracle.keep_count(x.size, gamma)
    vals, idx = oracle.compress(x, k)
    return oracle.densify(vals, idx, x.shape)


def _same(a, b):
    """Two evaluations of the same dense torch expression: equal up to one rounding of the result dtype."""
    a, b = a.float(), b.float()
    assert float((a - b).abs().max()) <= 2.0 ** -7 * float(b.abs().max()) + 1e-30


def _close(got, ref, tol):
    scale = np.abs(ref).max()
    assert np.abs(got - ref).max() <= tol * scale, (np.abs(got - ref).max(), scale)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("gamma", [0.9, 0.6])
def test_linear_layer_gradients(dtype, gamma):
    print("autograd linear", dtype, gamma, flush=True)
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    x_h = activation((6, 50, 96), "gelu", 31, dtype)          # [batch, tokens, c_in]
    dy_h = gradient((6, 50, 40), 0.02, 32, dtype)
    torch.manual_seed(3)
    plain = torch.nn.Linear(96, 40, device="cuda:0", dtype=tdt)
    layer = dnn.Linear(96, 40, gamma=gamma, device="cuda:0", dtype=tdt)
    layer.load_state_dict(plain.state_dict())
    xa = to_device(x_h).requires_grad_(True)
    xb = to_device(x_h).requires_grad_(True)
    dy = to_device(dy_h)
    ya, yb = plain(xa), layer(xb)
    assert torch.equal(ya, yb)                                  # the forward pass is not affected (Sec. 3.5)
    ya.backward(dy)
    yb.backward(dy)
    torch.cuda.synchronize()
    _same(xa.grad, xb.grad)                                     # nor is the gradient that flows on (Sec. 3.2)
    _same(plain.bias.grad, layer.bias.grad)
    ref = oracle.dw_fc(_oracle_xhat(x_h, gamma).reshape(-1, 96), oracle.widen(dy_h).reshape(-1, 40))
    # the layer rounds the fp32 result to the parameter dtype: one more rounding for bf16 parameters
    tol = TOL[dtype] + (2.0 ** -8 if dtype == "bf16" else 0.0)
    _close(layer.weight.grad.float().cpu().numpy().astype(np.float64), ref, tol)


@pytest.mark.parametrize("geometry", [dict(k=3, s=1, p=1, d=1), dict(k=3, s=2, p=1, d=1), dict(k=1, s=1, p=0, d=1),
                                      dict(k=4, s=4, p=0, d=1)])
def test_conv_layer_gradients(geometry):
    print("autograd conv", geometry, flush=True)
    k, s, p, d = (geometry[n] for n in "kspd")
    x_h = activation((3, 16, 24, 24), "relu", 41, "bf16")
    torch.manual_seed(4)
    plain = torch.nn.Conv2d(16, 24, k, s, p, d, device="cuda:0", dtype=torch.bfloat16)
    layer = dnn.Conv2d(16, 24, k, s, p, d, gamma=0.8, device="cuda:0", dtype=torch.bfloat16)
    layer.load_state_dict(plain.state_dict())
    xa = to_device(x_h).requires_grad_(True)
    xb = to_device(x_h).requires_grad_(True)
    ya, yb = plain(xa), layer(xb)
    assert torch.equal(ya, yb)
    dy_h = gradient(tuple(ya.shape), 0.02, 42, "bf16")
    dy = to_device(dy_h)
    ya.backward(dy)
    yb.backward(dy)
    torch.cuda.synchronize()
    _same(xa.grad, xb.grad)
    _same(plain.bias.grad, layer.bias.grad)
    ref = oracle.dw_conv(_oracle_xhat(x_h, 0.8), oracle.widen(dy_h), k, k, stride=(s, s), pad=(p, p), dil=(d, d))
    _close(layer.weight.grad.float().cpu().numpy().astype(np.float64), ref, TOL["bf16"] + 2.0 ** -8)


def test_conv_layer_channels_last():
    """A channels-last model: the cache is taken from the NHWC memory, dW comes back channels-last."""
    print("autograd conv channels_last", flush=True)
    x_h = activation((3, 16, 24, 24), "relu", 43, "bf16")
    torch.manual_seed(5)
    layer = dnn.Conv2d(16, 24, 3, 1, 1, gamma=0.8, device="cuda:0", dtype=torch.bfloat16).to(memory_format=torch.channels_last)
    x = to_device(x_h).contiguous(memory_format=torch.channels_last).requires_grad_(True)
    with dnn.cache_meter() as meter:
        y = layer(x)
    assert meter.layers == 1
    dy_h = gradient(tuple(y.shape), 0.02, 44, "bf16")
    y.backward(to_device(dy_h))
    torch.cuda.synchronize()
    # the selection runs over the tensor as it lies in memory, [N, H, W, C]
    x_nhwc = np.ascontiguousarray(x_h.transpose(0, 2, 3, 1))
    xhat = np.ascontiguousarray(_oracle_xhat(x_nhwc, 0.8).transpose(0, 3, 1, 2))
    ref = oracle.dw_conv(xhat, oracle.widen(dy_h), 3, 3, stride=(1, 1), pad=(1, 1), dil=(1, 1))
    assert layer.weight.grad.shape == (24, 16, 3, 3)
    _close(layer.weight.grad.float().cpu().numpy().astype(np.float64), ref, TOL["bf16"] + 2.0 ** -8)


def test_gamma_zero_and_eval_run_the_plain_layer():
    layer = dnn.Linear(32, 16, gamma=0.0, device="cuda:0")
    x = torch.randn(8, 32, device="cuda:0", requires_grad=True)
    with dnn.cache_meter() as meter:
        layer(x).sum().backward()
        layer.gamma = 0.9
        layer.eval()
        layer(x)
        layer.train()
        with torch.no_grad():
            layer(x)
    assert meter.layers == 0


def _mlp_stack(depth, dim, hidden, dtype):
    """Blocks of LayerNorm -> FC1 -> GELU -> FC2 with a residual: the MLP half of a DeiT-S block (Sec. 3.5)."""
    class Block(torch.nn.Module):
        def __init__(self):
            super().__init__()
            self.norm = torch.nn.LayerNorm(dim)
            self.fc1 = torch.nn.Linear(dim, hidden)
            self.act = torch.nn.GELU()
            self.fc2 = torch.nn.Linear(hidden, dim)

        def forward(self, x):
            return x + self.fc2(self.act(self.fc1(self.norm(x))))

    model = torch.nn.Sequential(torch.nn.Linear(dim, dim), *[Block() for _ in range(depth)], torch.nn.Linear(dim, 10))
    return model.to(device="cuda:0", dtype=dtype)


@pytest.mark.parametrize("gamma", [0.6, 0.7, 0.8, 0.9])
def test_cached_value_bytes_fall_by_gamma(gamma):
    """Sec. 4.3, cached-tensor table: the retained values take (1 - gamma) of the dense cache (its four
    dropped columns are 0.4, 0.3, 0.2, 0.1 of the baseline to three figures); here exactly k * 2 bytes per
    layer with k = floor((1 - gamma) * numel).  The allocator's own count of live bytes after the forward
    pass must fall by the dense cache minus values and indices."""
    print("autograd cache bytes", gamma, flush=True)
    dim, hidden, depth, tokens = 384, 1536, 4, 64 * 197
    torch.manual_seed(5)
    model = _mlp_stack(depth, dim, hidden, torch.bfloat16)
    x = torch.randn(tokens, dim, device="cuda:0", dtype=torch.bfloat16)

    def live_after_forward():
        torch.cuda.synchronize()
        base = torch.cuda.memory_allocated()
        y = model(x)
        torch.cuda.synchronize()
        live = torch.cuda.memory_allocated() - base
        y.float().sum().backward()
        model.zero_grad(set_to_none=True)
        return live

    dense_live = live_after_forward()
    names = dnn.apply_dropit(model, gamma)
    assert len(names) == 2 * depth                                # every FC of the blocks, not the first / last layer
    with dnn.cache_meter() as meter:
        drop_live = live_after_forward()
    numels = [tokens * dim, tokens * hidden] * depth
    assert meter.layers == 2 * depth
    assert meter.dense_bytes == 2 * sum(numels)
    assert meter.value_bytes == 2 * sum(dropit.keep_count(n, gamma) for n in numels)
    assert meter.index_bytes == 2 * meter.value_bytes
    assert abs(meter.value_bytes / meter.dense_bytes - (1.0 - gamma)) < 1e-6
    # FC1's input (the LayerNorm output) is freed; FC2's input (the GELU output) is freed as well, since
    # GELU's own backward keeps its input, not its output
    saved = dense_live - drop_live
    expect = meter.dense_bytes - meter.value_bytes - meter.index_bytes
    assert abs(saved - expect) <= 0.02 * meter.dense_bytes, (saved, expect)


def test_row_index_format_gives_the_same_gradients_with_half_the_index_bytes():
    torch.manual_seed(8)
    x_h = activation((6, 50, 96), "gelu", 61, "bf16")
    dy = to_device(gradient((6, 50, 40), 0.02, 62, "bf16"))
    flat = dnn.Linear(96, 40, gamma=0.8, device="cuda:0", dtype=torch.bfloat16)
    rows = dnn.Linear(96, 40, gamma=0.8, index_format="rows", device="cuda:0", dtype=torch.bfloat16)
    rows.load_state_dict(flat.state_dict())
    with dnn.cache_meter() as mf:
        flat(to_device(x_h)).backward(dy)
    with dnn.cache_meter() as mr:
        rows(to_device(x_h)).backward(dy)
    torch.cuda.synchronize()
    assert torch.equal(flat.weight.grad, rows.weight.grad)
    k = dropit.keep_count(x_h.size, 0.8)
    assert mf.index_bytes == 4 * k and mr.index_bytes == 2 * k + 4 * (300 + 1)
    assert mf.value_bytes == mr.value_bytes == 2 * k
    conv = dnn.Conv2d(8, 8, 3, padding=1, gamma=0.8, index_format="rows", device="cuda:0", dtype=torch.bfloat16)
    xc = to_device(activation((2, 8, 16, 16), "relu", 63, "bf16"))
    conv(xc).float().sum().backward()
    ref = dnn.Conv2d(8, 8, 3, padding=1, gamma=0.8, device="cuda:0", dtype=torch.bfloat16)
    ref.load_state_dict(conv.state_dict())
    ref(xc).float().sum().backward()
    torch.cuda.synchronize()
    assert torch.equal(conv.weight.grad, ref.weight.grad)
    with pytest.raises(ValueError):
        dnn.Linear(8, 8, strategy="random", index_format="rows", device="cuda:0")(torch.randn(4, 8, device="cuda:0"))


def test_training_steps_reduce_the_loss():
    """A few SGD steps on a small regression problem with gamma = 0.9: the approximate weight gradient
    (Sec. 3.4: still a descent direction in expectation) must drive the loss down."""
    torch.manual_seed(6)
    model = torch.nn.Sequential(torch.nn.Linear(64, 256), torch.nn.GELU(), torch.nn.Linear(256, 256), torch.nn.GELU(),
                                torch.nn.Linear(256, 64), torch.nn.GELU(), torch.nn.Linear(64, 1)).to("cuda:0")
    assert dnn.apply_dropit(model, 0.9) == ["2", "4"]
    x = torch.randn(4096, 64, device="cuda:0")
    target = torch.sin(x[:, :1]) + 0.5 * x[:, 1:2]
    opt = torch.optim.SGD(model.parameters(), lr=0.05, momentum=0.9)
    losses = []
    for _ in range(60):
        opt.zero_grad(set_to_none=True)
        loss = torch.nn.functional.mse_loss(model(x), target)
        loss.backward()
        opt.step()
        losses.append(float(loss.detach()))
    assert losses[-1] < 0.25 * losses[0], (losses[0], losses[-1])


def test_linear_takes_a_contiguous_view_that_starts_inside_a_buffer():
    """x[1:] of a [tokens + 1, c] buffer with an odd row length is contiguous but not 16-byte aligned; the layer
    copies it to an aligned tensor instead of handing the library a pointer it rejects."""
    torch.manual_seed(3)
    buf = torch.randn(65, 100, device="cuda:0", dtype=torch.bfloat16)
    x = buf[1:]
    assert x.is_contiguous() and x.data_ptr() % 16 != 0
    lin = dnn.Linear(100, 24, gamma=0.8).to("cuda:0", torch.bfloat16)
    y = lin(x)
    gbuf = torch.randn(65, 24, device="cuda:0", dtype=torch.bfloat16)
    y.backward(gbuf[1:])                                   # the incoming gradient is an offset view too
    torch.cuda.synchronize()
    ref = dnn.Linear(100, 24, gamma=0.8).to("cuda:0", torch.bfloat16)
    ref.load_state_dict(lin.state_dict())
    ref(x.clone()).backward(gbuf[1:].clone())
    torch.cuda.synchronize()
    assert torch.equal(lin.weight.grad, ref.weight.grad)
