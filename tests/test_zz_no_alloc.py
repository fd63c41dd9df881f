"""dropit_compress_static (the entry point that allocates nothing: its exchange area is a static
device array of the library) against dropit_compress, through the C ABI, bit for bit."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2202_13808_amd as dropit
from paper_2202_13808_amd import binding
from dropit_inputs import activation
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def _shape(t):
    return (ctypes.c_int64 * t.dim())(*t.shape)


def _both(L, xd, gamma, stream):
    """One call of each entry point on raw pointers; outputs pre-allocated and poisoned."""
    k = dropit.keep_count(xd.numel(), gamma)
    code = binding.BF16 if xd.dtype == torch.bfloat16 else binding.F32
    out = []
    ws = torch.empty(dropit.compress_workspace_bytes(xd.numel(), xd.dtype), dtype=torch.uint8, device="cuda:0")
    for static in (False, True):
        vals = torch.full((k + 32,), 7.0, dtype=xd.dtype, device="cuda:0")
        idx = torch.full((k + 32,), -5, dtype=torch.int32, device="cuda:0")
        torch.cuda.synchronize()
        if static:
            rc = L.dropit_compress_static(xd.data_ptr(), _shape(xd), xd.dim(), code, gamma, vals.data_ptr(),
                                          idx.data_ptr(), stream)
        else:
            rc = L.dropit_compress(xd.data_ptr(), _shape(xd), xd.dim(), code, gamma, vals.data_ptr(), idx.data_ptr(),
                                   ws.data_ptr(), ws.numel(), stream)
        assert rc == binding.OK
        torch.cuda.synchronize()
        out.append((vals.cpu(), idx.cpu()))
    (v0, i0), (v1, i1) = out
    assert torch.equal(i0, i1)
    assert v0.view(torch.int16 if xd.dtype == torch.bfloat16 else torch.int32).equal(
        v1.view(torch.int16 if xd.dtype == torch.bfloat16 else torch.int32))
    assert bool((i1[k:] == -5).all()) and bool((i1[:k] >= 0).all())      # nothing past k, everything before it written
    assert bool((i1[1:k] > i1[:k - 1]).all())
    return k


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_entry_point_matches_the_workspace_one_on_two_calls_in_a_row(dtype):
    L = dropit.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # the second input is smaller and differently distributed: the array keeps the first call's contents
    first = to_device(activation((3001, 1031), "gelu", 41, dtype))            # 3.1 M elements: the sampled form for bf16
    second = to_device(activation((257, 129), "relu", 42, dtype))
    print("static compress", dtype, "first", tuple(first.shape), flush=True)
    k1 = _both(L, first, 0.9, stream)
    print("static compress", dtype, "second", tuple(second.shape), flush=True)
    k2 = _both(L, second, 0.8, stream)
    assert k2 < k1
    # and once more the large one, now after a smaller call
    _both(L, first, 0.5, stream)


def test_static_entry_point_rejects_bad_arguments():
    L = dropit.lib()
    x = torch.zeros(64, dtype=torch.bfloat16, device="cuda:0")
    vals = torch.zeros(64, dtype=torch.bfloat16, device="cuda:0")
    idx = torch.zeros(64, dtype=torch.int32, device="cuda:0")
    too_big = (ctypes.c_int64 * 2)(1 << 20, 1 << 12)                            # 2^32 elements: beyond the int32 index
    assert L.dropit_compress_static(x.data_ptr(), too_big, 2, binding.BF16, 0.5, vals.data_ptr(), idx.data_ptr(),
                                    None) == binding.EINVAL
    one = (ctypes.c_int64 * 1)(64)
    assert L.dropit_compress_static(x.data_ptr(), one, 1, binding.BF16, 1.5, vals.data_ptr(), idx.data_ptr(),
                                    None) == binding.EINVAL
    assert L.dropit_compress_static(None, one, 1, binding.BF16, 0.5, vals.data_ptr(), idx.data_ptr(),
                                    None) == binding.EINVAL
    assert L.dropit_compress_static(x.data_ptr(), one, 1, binding.BF16, 0.5, None, idx.data_ptr(), None) == binding.EINVAL
