"""The C-ABI library loads, exports every symbol include/dropit.h declares, and rejects
bad arguments before touching the GPU (no compute calls here)."""
import ctypes
import os
import re

import pytest
import torch

import paper_2202_13808_amd as dropit
from paper_2202_13808_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "dropit.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dropit_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    assert declared_symbols() == sorted([
        "dropit_status_string", "dropit_keep_count", "dropit_compress_workspace_bytes", "dropit_compress",
        "dropit_weight_grad_workspace_bytes", "dropit_weight_grad", "dropit_trace_events", "dropit_set_select_mode", "dropit_set_fc_recover",
        "dropit_weight_grad_path",
        "dropit_weight_grad_nhwc_path", "dropit_weight_grad_nhwc_workspace_bytes", "dropit_weight_grad_nhwc",
        "dropit_compress_random_workspace_bytes", "dropit_compress_random",
        "dropit_compress_rows_workspace_bytes", "dropit_compress_rows",
        "dropit_weight_grad_rows_workspace_bytes", "dropit_weight_grad_rows",
        "dropit_compress_mask_workspace_bytes", "dropit_compress_mask",
        "dropit_weight_grad_mask_workspace_bytes", "dropit_weight_grad_mask",
        "dropit_compress_static"])


def test_library_exports_every_declared_symbol():
    L = dropit.lib()
    for name in declared_symbols():
        assert hasattr(L, name), name


def test_keep_count_matches_the_stated_rule():
    assert dropit.keep_count(16384, 0.9) == 1638
    assert dropit.keep_count(9682944, 0.9) == 968294
    assert dropit.keep_count(38731776, 0.9) == 3873177
    assert dropit.keep_count(12582912, 0.9) == 1258291
    assert dropit.keep_count(50331648, 0.9) == 5033164
    assert dropit.keep_count(12845056, 0.8) == 2569011
    assert dropit.keep_count(100, 0.9) == 10
    assert dropit.keep_count(1000, 0.0) == 1000 and dropit.keep_count(1000, 1.0) == 0
    for bad in (-0.5, 1.5, float("nan")):
        assert dropit.keep_count(10, bad) == -1
    assert dropit.keep_count(2**31, 0.5) == -1 and dropit.keep_count(-3, 0.5) == -1


def test_status_strings():
    L = dropit.lib()
    for code in range(5):
        assert L.dropit_status_string(code).decode().startswith("DROPIT_")


def _shape(*dims):
    return (ctypes.c_int64 * len(dims))(*dims)


def test_compress_rejects_bad_arguments_without_a_gpu():
    L = dropit.lib()
    fake = ctypes.c_void_p(0x1000)           # never dereferenced: validation fails first
    ws = ctypes.c_void_p(0x10000)
    big = 1 << 30
    call = L.dropit_compress
    assert call(None, _shape(4, 4), 2, binding.BF16, 0.5, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, None, 2, binding.BF16, 0.5, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 0, binding.BF16, 0.5, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 0), 2, binding.BF16, 0.5, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(1 << 20, 1 << 12), 2, binding.BF16, 0.5, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, 7, 0.5, fake, fake, ws, big, None) == binding.EINVAL
    for g in (-0.1, 1.1, float("nan")):
        assert call(fake, _shape(4, 4), 2, binding.BF16, g, fake, fake, ws, big, None) == binding.EINVAL
    assert call(ctypes.c_void_p(0x1004), _shape(4, 4), 2, binding.BF16, 0.5, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 0.5, None, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 0.5, fake, None, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 0.5, fake, fake, None, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 0.5, fake, fake, ws, 16, None) == binding.EWORKSPACE
    # gamma = 1 keeps nothing: legal, nothing launched, outputs may be NULL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 1.0, None, None, None, 0, None) == binding.OK


def test_compress_random_rejects_bad_arguments_without_a_gpu():
    L = dropit.lib()
    fake = ctypes.c_void_p(0x1000)
    ws = ctypes.c_void_p(0x10000)
    big = 1 << 30
    call = L.dropit_compress_random
    assert call(None, _shape(4, 4), 2, binding.BF16, 0.5, 1, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 0), 2, binding.BF16, 0.5, 1, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, 7, 0.5, 1, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.F32, 1.5, 1, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.F32, 0.5, 1, None, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.F32, 0.5, 1, fake, fake, ctypes.c_void_p(0x10010), big, None) == binding.EINVAL
    need = L.dropit_compress_random_workspace_bytes(16, binding.F32)
    assert need > L.dropit_compress_workspace_bytes(16, binding.F32)
    assert call(fake, _shape(4, 4), 2, binding.F32, 0.5, 1, fake, fake, ws, need - 1, None) == binding.EWORKSPACE
    assert call(fake, _shape(4, 4), 2, binding.F32, 1.0, 1, None, None, None, 0, None) == binding.OK
    # one 32-bit draw per element, twice (keys and the select's copy of the kept ones)
    n = 1 << 20
    assert L.dropit_compress_random_workspace_bytes(n, binding.BF16) >= L.dropit_compress_workspace_bytes(n, binding.BF16) + 8 * n
    assert L.dropit_compress_random_workspace_bytes(0, binding.BF16) == 0
    assert L.dropit_compress_random_workspace_bytes(1 << 31, binding.BF16) == 0


def test_row_form_rejects_bad_arguments_without_a_gpu():
    L = dropit.lib()
    fake = ctypes.c_void_p(0x1000)
    ws = ctypes.c_void_p(0x10000)
    big = 1 << 30
    call = L.dropit_compress_rows
    assert call(fake, _shape(2, 65537), 2, binding.BF16, 0.5, fake, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 0.5, fake, fake, None, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 0.5, fake, None, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 2.0, fake, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 0.5, fake, fake, fake, ws, 64, None) == binding.EWORKSPACE
    assert L.dropit_compress_rows_workspace_bytes(1 << 20, 1 << 18, binding.BF16) >= \
        L.dropit_compress_workspace_bytes(1 << 20, binding.BF16) + 4 * (1 << 18)
    assert L.dropit_compress_rows_workspace_bytes(16, 17, binding.BF16) == 0
    wg = L.dropit_weight_grad_rows
    dw = ctypes.c_void_p(0x2000)
    assert wg(fake, fake, fake, 4, _shape(2, 65537), 2, binding.BF16, fake, 8, None, dw, ws, big, None) == binding.EINVAL
    assert wg(fake, None, fake, 4, _shape(4, 8), 2, binding.BF16, fake, 8, None, dw, ws, big, None) == binding.EINVAL
    assert wg(fake, fake, fake, 4, _shape(4, 8), 2, binding.BF16, fake, 8, None, dw, ws, 16, None) == binding.EWORKSPACE
    assert L.dropit_weight_grad_rows_workspace_bytes(_shape(4, 8), 2, binding.BF16, 4, 8, None) > \
        L.dropit_weight_grad_workspace_bytes(_shape(4, 8), 2, binding.BF16, 4, 8, None)


def test_weight_grad_path_of_the_benchmark_shapes():
    """Host-only query: which kernels a call would run.  The measured choice for the paper's layer
    shapes is part of the contract the benchmarks rely on."""
    c3 = (3, 3, 1, 1, 1, 1, 1, 1)
    bf, f32 = torch.bfloat16, torch.float32
    path = dropit.weight_grad_path
    assert path((64, 197, 768), bf, 1000, 3072) == "fc_mfma"
    assert path((64, 197, 3072), bf, 1000, 768) == "fc_mfma"
    assert path((64, 197, 768), f32, 1000, 3072) == "fma"
    assert path((64, 197, 768), bf, 1000, 3070) == "fma"               # c_out not a multiple of 8
    assert path((64, 64, 56, 56), bf, 1000, 64, conv=c3) == "conv_bands"
    assert path((64, 128, 28, 28), bf, 1000, 128, conv=c3) == "conv_bands"
    assert path((64, 256, 14, 14), bf, 1000, 256, conv=c3) == "conv_gemm"
    assert path((64, 512, 7, 7), bf, 1000, 512, conv=c3) == "conv_gemm"
    assert path((64, 64, 7, 7), bf, 1000, 64, conv=c3) == "conv_bands"  # few channels
    assert path((64, 516, 7, 7), bf, 1000, 512, conv=c3) == "conv_bands"  # channels not a multiple of 8
    assert path((64, 512, 7, 7), f32, 1000, 512, conv=c3) == "fma"
    assert path((2, 3, 20, 22), bf, 100, 8, conv=(7, 7, 2, 2, 3, 3, 1, 1)) == "conv_im2col"
    assert path((2, 3, 20, 22), bf, 100, 5, conv=(7, 7, 2, 2, 3, 3, 1, 1)) == "fma"   # c_out not a multiple of 8
    assert path((2, 3, 20, 22), f32, 100, 8, conv=(7, 7, 2, 2, 3, 3, 1, 1)) == "fma"
    assert path((64, 3, 224, 224), bf, 1000, 768, conv=(16, 16, 16, 16, 0, 0, 1, 1)) == "conv_im2col"   # patch embedding
    assert path((64, 256, 56, 56), bf, 1000, 64, conv=(1, 1, 1, 1, 0, 0, 1, 1)) == "conv_im2col"
    assert path((64, 4096, 7, 7), bf, 1000, 64, conv=(3, 3, 2, 2, 1, 1, 1, 1)) == "fma"   # C*kh*kw > 32768
    assert path((64, 56, 56, 64), bf, 1000, 64, conv=c3, layout="nhwc") == "conv_im2col"
    assert path((64, 56, 56, 64), f32, 1000, 64, conv=c3, layout="nhwc") == "fma"
    assert path((64, 56, 56, 256), bf, 1000, 64, conv=(1, 1, 1, 1, 0, 0, 1, 1), layout="nhwc") == "fc_mfma"
    assert path((64, 56, 56, 256), bf, 1000, 64, conv=(1, 1, 2, 2, 0, 0, 1, 1), layout="nhwc") == "conv_im2col"
    assert path((64, 56, 56, 64), bf, -1, 64, conv=c3, layout="nhwc") == "none"
    assert path((3, 16, 9, 1), bf, 10, 8, conv=c3) == "conv_im2col"     # a single column: not the row-band kernel
    assert path((64, 512, 7, 7), bf, -1, 512, conv=c3) == "none"
    assert path((1, 2, 4, 4), bf, 4, 2, conv=(7, 7, 1, 1, 0, 0, 1, 1)) == "none"


def test_mask_entry_points_validate_arguments():
    L = dropit.lib()
    fake = ctypes.c_void_p(0x1000)
    ws = ctypes.c_void_p(0x4000)
    dw = ctypes.c_void_p(0x2000)
    big = 1 << 30
    call = L.dropit_compress_mask
    assert call(fake, _shape(4, 4), 2, binding.BF16, 0.5, fake, None, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 0.5, fake, fake, None, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 2.0, fake, fake, fake, ws, big, None) == binding.EINVAL
    assert call(fake, _shape(4, 4), 2, binding.BF16, 0.5, fake, fake, fake, ws, 64, None) == binding.EWORKSPACE
    assert L.dropit_compress_mask_workspace_bytes(1 << 20, 1 << 18, binding.BF16) >= \
        L.dropit_compress_workspace_bytes(1 << 20, binding.BF16) + 4 * (1 << 18)
    assert L.dropit_compress_mask_workspace_bytes(16, 17, binding.BF16) == 0
    wg = L.dropit_weight_grad_mask
    assert wg(fake, None, fake, 4, _shape(4, 8), 2, binding.BF16, fake, 8, None, dw, ws, big, None) == binding.EINVAL
    assert wg(fake, fake, fake, 33, _shape(4, 8), 2, binding.BF16, fake, 8, None, dw, ws, big, None) == binding.EINVAL
    assert wg(fake, fake, fake, 4, _shape(4, 8), 2, binding.BF16, fake, 8, None, dw, ws, 16, None) == binding.EWORKSPACE
    assert L.dropit_weight_grad_mask_workspace_bytes(_shape(4, 8), 2, binding.BF16, 4, 8, None) > \
        L.dropit_weight_grad_workspace_bytes(_shape(4, 8), 2, binding.BF16, 4, 8, None)


def test_nhwc_entry_points_validate_arguments():
    L = dropit.lib()
    fake = ctypes.c_void_p(0x1000)
    dw = ctypes.c_void_p(0x2000)
    ws = ctypes.c_void_p(0x4000)
    geom = binding.Conv2d(3, 3, 1, 1, 1, 1, 1, 1)
    g = ctypes.byref(geom)
    call = L.dropit_weight_grad_nhwc
    shape = _shape(2, 8, 8, 16)
    assert L.dropit_weight_grad_nhwc_workspace_bytes(shape, binding.BF16, 4, 8, g) > 0
    assert L.dropit_weight_grad_nhwc_workspace_bytes(shape, binding.BF16, 4, 8, None) == 0
    assert L.dropit_weight_grad_nhwc_workspace_bytes(shape, binding.BF16, 2 * 8 * 8 * 16 + 1, 8, g) == 0
    assert call(fake, fake, 4, shape, binding.BF16, fake, 8, None, dw, ws, 1 << 30, None) == binding.EINVAL
    assert call(fake, fake, 4, None, binding.BF16, fake, 8, g, dw, ws, 1 << 30, None) == binding.EINVAL
    assert call(fake, None, 4, shape, binding.BF16, fake, 8, g, dw, ws, 1 << 30, None) == binding.EINVAL
    assert call(fake, fake, 4, shape, binding.BF16, None, 8, g, dw, ws, 1 << 30, None) == binding.EINVAL
    assert call(fake, fake, 4, shape, binding.BF16, fake, 8, g, dw, ws, 16, None) == binding.EWORKSPACE
    big = binding.Conv2d(17, 3, 1, 1, 0, 0, 1, 1)                      # window taller than the input
    assert call(fake, fake, 4, shape, binding.BF16, fake, 8, ctypes.byref(big), dw, ws, 1 << 30, None) == binding.EINVAL


def test_select_mode_switch_validates():
    L = dropit.lib()
    assert L.dropit_set_select_mode(1) == binding.OK
    assert L.dropit_set_select_mode(0) == binding.OK
    assert L.dropit_set_select_mode(2) == binding.OK
    assert L.dropit_set_select_mode(3) == binding.OK
    assert L.dropit_set_select_mode(4) == binding.EINVAL
    assert L.dropit_set_select_mode(-1) == binding.EINVAL
    assert L.dropit_set_select_mode(0) == binding.OK                  # leave the default for whatever runs next


def test_fc_recover_switch_validates_and_changes_the_answers():
    L = dropit.lib()
    shape, k, c_out = (12608, 768), 968294, 3072
    dense_form = dropit.weight_grad_workspace_bytes(shape, torch.bfloat16, k, c_out)
    assert dropit.weight_grad_path(shape, torch.bfloat16, k, c_out) == "fc_mfma"
    assert L.dropit_set_fc_recover(2) == binding.EINVAL and L.dropit_set_fc_recover(-1) == binding.EINVAL
    assert L.dropit_set_fc_recover(1) == binding.OK
    try:
        assert dropit.weight_grad_path(shape, torch.bfloat16, k, c_out) == "fc_fused"
        in_lds = dropit.weight_grad_workspace_bytes(shape, torch.bfloat16, k, c_out)
        # the dense operand (2 bytes per element of x) gives way to a word per pair and two small tables
        assert dense_form - in_lds > 12608 * 768 * 2 - 4 * k - (1 << 16)
        assert dropit.weight_grad_path(shape, torch.bfloat16, k, 128) == "fc_mfma"      # not covered: unchanged
        assert dropit.weight_grad_path(shape, torch.float32, k, c_out) == "fma"
    finally:
        assert L.dropit_set_fc_recover(0) == binding.OK
    assert dropit.weight_grad_path(shape, torch.bfloat16, k, c_out) == "fc_mfma"


def test_workspace_queries():
    assert dropit.compress_workspace_bytes(16384, __import__("torch").float32) > 0
    L = dropit.lib()
    assert L.dropit_compress_workspace_bytes(0, binding.BF16) == 0
    assert L.dropit_compress_workspace_bytes(1 << 31, binding.BF16) == 0
    assert L.dropit_compress_workspace_bytes(100, 9) == 0
