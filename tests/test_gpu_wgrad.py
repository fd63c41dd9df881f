"""GPU parity: dropit_weight_grad (through the C ABI) vs the fp64 CPU oracle.

Tolerance (max |dW_gpu - dW_ref| / max |dW_ref|): 1e-3 for bf16 inputs with fp32
accumulation, 1e-5 for fp32 inputs.  bf16 products are exact in fp32, so the only
error is fp32 accumulation order; integer-valued cases must match exactly.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2202_13808_amd as dropit
from dropit_inputs import WORKLOADS, activation, f32_to_bf16_bits, gradient, make
from gpu_util import to_device, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-3}
CONV3 = (3, 3, 1, 1, 1, 1, 1, 1)


def gpu_dw(x, dy, gamma, c_out, conv=None):
    xd, dyd = to_device(x), to_device(dy)
    vals, idx = dropit.compress(xd, gamma)
    dW = dropit.weight_grad(vals, idx, x.shape, dyd, c_out, conv=conv)
    torch.cuda.synchronize()
    return to_host(dW).astype(np.float64), to_host(vals), to_host(idx)


def ref_xhat(x, gamma):
    k = oracle.keep_count(x.size, gamma)
    vals, idx = oracle.compress(x, k)
    return oracle.densify(vals, idx, x.shape)


def assert_close(got, ref, tol, scale=None):
    scale = np.abs(ref).max() if scale is None else scale
    err = np.abs(got - ref).max()
    assert err <= tol * scale, (err, scale, err / max(scale, 1e-300))


def test_config1_tiny_fc_fp32():
    w = WORKLOADS["tiny_fc"]
    x, dy = make(w)
    print("wgrad tiny_fc", flush=True)
    got, _, _ = gpu_dw(x, dy, w.gamma, w.c_out)
    ref = oracle.dw_fc(ref_xhat(x, w.gamma), oracle.widen(dy))
    assert got.shape == (128, 64)
    assert_close(got, ref, TOL["f32"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ntok,cin,cout", [(300, 100, 70), (1, 8, 8), (1000, 64, 128), (777, 257, 33),
                                           (2048, 768, 256), (1500, 256, 768)])
@pytest.mark.parametrize("gamma", [0.9, 0.0])
def test_fc_shapes(dtype, ntok, cin, cout, gamma):
    print("wgrad fc", dtype, ntok, cin, cout, gamma, flush=True)
    x = activation((ntok, cin), "normal", 100 + ntok, dtype)
    dy = gradient((ntok, cout), 0.02, 200 + ntok, dtype)
    got, _, _ = gpu_dw(x, dy, gamma, cout)
    ref = oracle.dw_fc(ref_xhat(x, gamma), oracle.widen(dy))
    assert_close(got, ref, TOL[dtype])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ntok,cin,cout,gamma", [(256, 64, 128, 0.9), (1024, 16, 40, 0.5), (5, 24, 16, 0.5), (1, 4, 1, 0.0),
                                                 (33, 496, 3, 0.9), (64, 256, 4096, 0.9), (100, 132, 17, 0.7)])
def test_fc_small_layers_take_one_launch(dtype, ntok, cin, cout, gamma):
    """At most 16384 input elements (c_in a multiple of 4): recover in LDS + exact fp32 multiply-adds, one kernel."""
    print("wgrad fc small", dtype, ntok, cin, cout, gamma, flush=True)
    x = activation((ntok, cin), "normal", 600 + ntok, dtype)
    dy = gradient((ntok, cout), 0.02, 700 + ntok, dtype)
    k = oracle.keep_count(x.size, gamma)
    assert dropit.weight_grad_path(x.shape, torch.float32 if dtype == "f32" else torch.bfloat16, k, cout) == "fc_small"
    got, _, _ = gpu_dw(x, dy, gamma, cout)
    ref = oracle.dw_fc(ref_xhat(x, gamma), oracle.widen(dy))
    assert_close(got, ref, 1e-5)            # fp32 accumulation of exact products in token order, for either input type


@pytest.mark.parametrize("ntok,cin,cout,gamma", [
    (777, 257, 40, 0.9),      # c_in not a multiple of 8: padded row pitch of the recovered matrix
    (5, 24, 16, 0.5),         # fewer tokens than one token block
    (33, 520, 264, 0.9),      # ragged tiles in both output dimensions, ragged last token block
    (4100, 8, 3080, 0.8),     # many row tiles, one narrow column tile
    (2000, 3000, 8, 0.95),    # many column tiles, one narrow row tile
    (9000, 512, 512, 0.9),    # several K-slices per tile
    (640, 40000, 8, 0.9),     # c_in beyond what the recover kernel holds in LDS: generic path
    (20000, 200, 64, 0.9),    # the whole result is one 128-row tile: 31 K-slices, added by the many-slice kernel
    (70000, 64, 8, 0.8),      # ... 109 slices of a nearly empty tile
    (6000, 300, 136, 0.9),    # just over 128 output channels: the wide tile, two column tiles
    (20, 1024, 264, 0.9),     # the wide tile with a single (partial) token block: the pipeline's prologue is the whole loop
    (70, 520, 392, 0.5),      # ... three token blocks, as many as are loaded ahead
])
def test_fc_bf16_tile_edges(ntok, cin, cout, gamma):
    print("wgrad fc edges", ntok, cin, cout, gamma, flush=True)
    x = activation((ntok, cin), "normal", 300 + ntok, "bf16")
    dy = gradient((ntok, cout), 0.02, 400 + ntok, "bf16")
    got, _, _ = gpu_dw(x, dy, gamma, cout)
    ref = oracle.dw_fc(ref_xhat(x, gamma), oracle.widen(dy))
    assert_close(got, ref, TOL["bf16"])


@pytest.mark.parametrize("case", [
    # where the kept pairs sit in the index-sorted arrays is first guessed from an even spread; these inputs are not evenly spread
    dict(ntok=3000, cin=256, cout=32, gamma=0.9, layout="tail"),      # everything kept lies in the last rows: the guess fails, exact search
    dict(ntok=3000, cin=256, cout=32, gamma=0.9, layout="head"),      # ... in the first rows
    dict(ntok=3000, cin=256, cout=32, gamma=0.9, layout="stripes"),   # dense and empty stretches alternate
    dict(ntok=4000, cin=768, cout=64, gamma=0.3, layout="even"),      # large k: one search per workgroup, forward walk, several batches per tile
    dict(ntok=4000, cin=768, cout=64, gamma=0.3, layout="tail"),      # large k with empty tiles in front
    dict(ntok=5003, cin=520, cout=40, gamma=0.5, layout="stripes"),   # large k, padded rows (c_in not a multiple of the tile pitch), ragged last tile
])
def test_fc_bf16_uneven_density(case):
    print("wgrad fc density", case, flush=True)
    ntok, cin, cout, gamma = case["ntok"], case["cin"], case["cout"], case["gamma"]
    rng = np.random.default_rng(ntok + cin)
    xf = rng.standard_normal((ntok, cin), dtype=np.float32)
    rows = np.arange(ntok)
    if case["layout"] == "tail":
        xf[rows < int(0.7 * ntok)] *= 1e-3
    elif case["layout"] == "head":
        xf[rows >= int(0.3 * ntok)] *= 1e-3
    elif case["layout"] == "stripes":
        xf[(rows // 200) % 2 == 0] *= 1e-3
    x = f32_to_bf16_bits(xf)
    dy = gradient((ntok, cout), 0.02, 500 + ntok, "bf16")
    got, _, _ = gpu_dw(x, dy, gamma, cout)
    ref = oracle.dw_fc(ref_xhat(x, gamma), oracle.widen(dy))
    assert_close(got, ref, TOL["bf16"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("conv", [None, CONV3])
def test_everything_dropped_gives_zero(dtype, conv):
    print("wgrad all dropped", dtype, conv, flush=True)
    shape = (2, 16, 8, 8) if conv else (96, 64)
    dy_shape = (2, 24, 8, 8) if conv else (96, 24)
    x = activation(shape, "normal", 7, dtype)
    dy = gradient(dy_shape, 0.02, 8, dtype)
    got, vals, idx = gpu_dw(x, dy, 1.0, 24, conv=conv)
    assert vals.size == 0 and idx.size == 0
    assert got.shape == ((24, 16, 3, 3) if conv else (24, 64))
    assert not got.any()


def test_fc_leading_dims_are_tokens():
    x = activation((4, 50, 96), "gelu", 3, "bf16")
    dy = gradient((4, 50, 40), 0.02, 4, "bf16")
    got, _, _ = gpu_dw(x, dy, 0.8, 40)
    ref = oracle.dw_fc(ref_xhat(x, 0.8), oracle.widen(dy))
    assert_close(got, ref, TOL["bf16"])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_fc_integer_values_are_exact(dtype):
    rng = np.random.default_rng(5)
    xf = rng.integers(-4, 5, (640, 192)).astype(np.float32)
    dyf = rng.integers(-3, 4, (640, 160)).astype(np.float32)
    x, dy = (xf, dyf) if dtype == "f32" else (f32_to_bf16_bits(xf), f32_to_bf16_bits(dyf))
    got, _, _ = gpu_dw(x, dy, 0.7, 160)
    ref = oracle.dw_fc(ref_xhat(x, 0.7), oracle.widen(dy))
    assert np.array_equal(got, ref)


def test_k_zero_gives_zero_gradient():
    x = activation((64, 32), "normal", 1, "bf16")
    dy = gradient((64, 16), 0.02, 2, "bf16")
    got, vals, idx = gpu_dw(x, dy, 1.0, 16)
    assert vals.size == 0 and idx.size == 0
    assert np.array_equal(got, np.zeros((16, 32)))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,C,H,W,J", [(2, 5, 9, 11, 7), (1, 1, 3, 3, 1), (3, 16, 14, 14, 32), (2, 64, 56, 56, 64),
                                       (2, 8, 7, 30, 8),
                                       # shapes the matrix-core path takes (W % 8 == 0): ragged channel blocks,
                                       # odd and single rows, several (j, c) blocks, several row bands
                                       (2, 5, 9, 16, 7), (1, 70, 6, 8, 130), (3, 64, 1, 24, 64), (2, 16, 28, 32, 24),
                                       (1, 130, 5, 40, 66), (300, 8, 3, 8, 8), (1, 3, 61, 120, 5)])
def test_conv3x3_shapes(dtype, N, C, H, W, J):
    print("wgrad conv", dtype, N, C, H, W, J, flush=True)
    x = activation((N, C, H, W), "relu", 300 + H, dtype)
    dy = gradient((N, J, H, W), 0.02, 400 + H, dtype)
    got, _, _ = gpu_dw(x, dy, 0.8, J, conv=CONV3)
    ref = oracle.dw_conv(ref_xhat(x, 0.8), oracle.widen(dy), 3, 3, (1, 1), (1, 1))
    assert got.shape == (J, C, 3, 3)
    assert_close(got, ref, TOL[dtype])


@pytest.mark.parametrize("N,C,H,W,J,path", [
    (4, 64, 28, 28, 64, "conv_bands"),     # ResNet stage 2 plane: rows of 28 go through the zero-padded copy of dY (rows of 32)
    (6, 128, 14, 14, 96, "conv_bands"),    # stage 3 plane, two channel blocks, a ragged filter block; too small for the GEMM form
    (32, 256, 7, 7, 256, "conv_gemm"),     # stage 4 plane, many channels: one GEMM over im2col rows
    (40, 192, 7, 7, 128, "conv_gemm"),     # ... with zero pad rows after the last token block
    (24, 128, 14, 14, 264, "conv_gemm"),   # ... 16-channel im2col tiles, c_out not a multiple of 64
    (48, 136, 5, 9, 72, "conv_gemm"),      # ... a non-square plane, a ragged last channel block (136 = 64 + 64 + 8)
    (128, 128, 1, 16, 64, "conv_gemm"),    # ... a single row
    (128, 128, 16, 1, 64, "conv_gemm"),    # ... a single column
    (600, 64, 7, 7, 64, "conv_bands"),     # few channels: more (image, block) units than compute units
                                           # -> several images per workgroup
    (778, 64, 7, 7, 64, "conv_bands"),     # ... with a ragged last image group
    (3, 16, 9, 1, 8, "conv_im2col"),       # a single column with few channels: the general im2col form
    (3, 16, 9, 2, 8, "conv_bands"),        # two columns: the narrowest plane of the row-band kernel
    (2, 24, 10, 119, 16, "conv_bands"),    # the widest padded row (120)
])
def test_conv3x3_matrix_core_paths_widths_and_image_groups(N, C, H, W, J, path):
    print("wgrad conv3x3 widths", N, C, H, W, J, path, flush=True)
    x = activation((N, C, H, W), "relu", 310 + W, "bf16")
    dy = gradient((N, J, H, W), 0.02, 410 + W, "bf16")
    k = oracle.keep_count(x.size, 0.8)
    assert dropit.weight_grad_path(x.shape, torch.bfloat16, k, J, conv=CONV3) == path
    got, _, _ = gpu_dw(x, dy, 0.8, J, conv=CONV3)
    ref = oracle.dw_conv(ref_xhat(x, 0.8), oracle.widen(dy), 3, 3, (1, 1), (1, 1))
    assert_close(got, ref, TOL["bf16"])


@pytest.mark.parametrize("layout", ["dead_channels", "late_images", "one_image"])
def test_conv3x3_gemm_form_uneven_density(layout):
    """The im2col kernel guesses where a block's pairs sit from an even spread and verifies the guess:
    tensors whose kept elements bunch up (dead channels, a few bright images) take its search instead."""
    N, C, H, W, J = 32, 256, 7, 7, 128
    print("wgrad conv gemm density", layout, flush=True)
    rng = np.random.default_rng(len(layout))
    xf = np.maximum(rng.standard_normal((N, C, H, W), dtype=np.float32), 0)
    if layout == "dead_channels":
        xf[:, (np.arange(C) // 24) % 2 == 0] *= 1e-3
    elif layout == "late_images":
        xf[: int(0.7 * N)] *= 1e-3
    else:
        xf[np.arange(N) != 5] *= 1e-3
    x = f32_to_bf16_bits(xf)
    dy = gradient((N, J, H, W), 0.02, 77, "bf16")
    k = oracle.keep_count(x.size, 0.9)
    assert dropit.weight_grad_path(x.shape, torch.bfloat16, k, J, conv=CONV3) == "conv_gemm"
    got, _, _ = gpu_dw(x, dy, 0.9, J, conv=CONV3)
    ref = oracle.dw_conv(ref_xhat(x, 0.9), oracle.widen(dy), 3, 3, (1, 1), (1, 1))
    assert_close(got, ref, TOL["bf16"])


@pytest.mark.parametrize("conv", [CONV3, (3, 3, 2, 2, 1, 1, 1, 1)])
def test_conv_pairs_at_a_4_byte_aligned_address_only(conv):
    """The pair arrays need only their natural alignment: views one element into a buffer give the same dW."""
    x = activation((3, 16, 21, 24), "relu", 61, "bf16")
    OH, OW = (21, 24) if conv == CONV3 else (11, 12)
    dy = gradient((3, 16, OH, OW), 0.02, 62, "bf16")
    xd, dyd = to_device(x), to_device(dy)
    vals, idx = dropit.compress(xd, 0.7)
    want = dropit.weight_grad(vals, idx, x.shape, dyd, 16, conv=conv)
    vbuf = torch.empty(vals.numel() + 1, dtype=vals.dtype, device=vals.device)
    ibuf = torch.empty(idx.numel() + 1, dtype=idx.dtype, device=idx.device)
    vbuf[1:] = vals
    ibuf[1:] = idx
    assert ibuf[1:].data_ptr() % 16 == 4
    got = dropit.weight_grad(vbuf[1:], ibuf[1:], x.shape, dyd, 16, conv=conv)
    torch.cuda.synchronize()
    assert torch.equal(got, want)


def test_conv3x3_integer_values_are_exact():
    rng = np.random.default_rng(6)
    x = f32_to_bf16_bits(rng.integers(-3, 4, (2, 16, 28, 28)).astype(np.float32))
    dy = f32_to_bf16_bits(rng.integers(-2, 3, (2, 24, 28, 28)).astype(np.float32))
    got, _, _ = gpu_dw(x, dy, 0.6, 24, conv=CONV3)
    ref = oracle.dw_conv(ref_xhat(x, 0.6), oracle.widen(dy), 3, 3, (1, 1), (1, 1))
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,C,H,W,J,geom", [
    (2, 6, 9, 11, 5, (1, 1, 1, 1, 0, 0, 1, 1)),        # 1x1
    (2, 3, 20, 22, 8, (7, 7, 2, 2, 3, 3, 1, 1)),       # 7x7 / stride 2 / pad 3 (first ResNet layer's geometry)
    (3, 8, 15, 14, 4, (3, 3, 2, 2, 1, 1, 1, 1)),       # 3x3 / stride 2
    (2, 3, 32, 48, 6, (16, 16, 16, 16, 0, 0, 1, 1)),   # 16x16 / stride 16 (ViT patch embedding)
    (1, 4, 13, 17, 3, (3, 2, 1, 2, 2, 0, 2, 3)),       # asymmetric kernel, stride, pad, dilation
    (2, 5, 12, 10, 7, (3, 3, 1, 1, 1, 1, 2, 2)),       # dilated 3x3: not the matrix-core geometry
])
def test_conv_general_geometries(dtype, N, C, H, W, J, geom):
    """Every geometry other than 3x3/s1/p1 takes the exact fp32 kernel; same oracle (it is general)."""
    kh, kw, sh, sw, ph, pw, dh, dw = geom
    OH = (H + 2 * ph - dh * (kh - 1) - 1) // sh + 1
    OW = (W + 2 * pw - dw * (kw - 1) - 1) // sw + 1
    print("wgrad conv general", dtype, N, C, H, W, J, geom, flush=True)
    x = activation((N, C, H, W), "relu", 900 + H + kh, dtype)
    dy = gradient((N, J, OH, OW), 0.02, 950 + W + kw, dtype)
    got, _, _ = gpu_dw(x, dy, 0.6, J, conv=geom)
    ref = oracle.dw_conv(ref_xhat(x, 0.6), oracle.widen(dy), kh, kw, (sh, sw), (ph, pw), (dh, dw))
    assert got.shape == (J, C, kh, kw)
    assert_close(got, ref, TOL[dtype])


GEOMETRIES = [
    ((2, 16, 9, 11), 24, (1, 1, 1, 1, 0, 0, 1, 1)),        # 1x1 (most of a ResNet-50's convolutions)
    ((3, 40, 7, 9), 16, (1, 1, 2, 2, 0, 0, 1, 1)),         # 1x1 / stride 2 (a ResNet downsampling shortcut)
    ((2, 3, 40, 44), 16, (7, 7, 2, 2, 3, 3, 1, 1)),        # 7x7 / stride 2 / pad 3 (first ResNet layer's geometry)
    ((3, 8, 15, 14), 8, (3, 3, 2, 2, 1, 1, 1, 1)),         # 3x3 / stride 2
    ((2, 3, 32, 48), 40, (16, 16, 16, 16, 0, 0, 1, 1)),    # 16x16 / stride 16 (ViT patch embedding)
    ((1, 4, 13, 17), 8, (3, 2, 1, 2, 2, 0, 2, 3)),         # asymmetric kernel, stride, pad, dilation
    ((2, 5, 12, 10), 16, (3, 3, 1, 1, 1, 1, 2, 2)),        # dilated 3x3
    ((5, 24, 20, 20), 72, (3, 3, 1, 1, 1, 1, 1, 1)),       # 3x3 / stride 1 / pad 1 (channels-last only: NCHW has kernels of its own)
    ((3, 20, 37, 23), 136, (5, 5, 3, 2, 2, 1, 1, 1)),      # more than 256 output positions per image, three filter blocks
    ((2, 8, 6, 6), 8, (3, 3, 1, 1, 4, 4, 1, 1)),           # padding wider than the window: whole rows of taps see only zeros
    ((128, 8, 18, 18), 8, (3, 3, 1, 1, 0, 0, 1, 1)),       # many images: bands of several output rows per im2col tile
    ((2, 256, 9, 32), 16, (3, 3, 2, 2, 1, 1, 1, 1)),       # a row of tokens beyond one tile: blocks of channels (NCHW) / taps (NHWC), ragged last block
    ((2, 20, 9, 300), 8, (5, 5, 1, 1, 2, 2, 1, 1)),        # ... with channels not a multiple of 8: zero fill + scatter instead of tiles
]


def _out_extent(n, k, s, p, d):
    return (n + 2 * p - d * (k - 1) - 1) // s + 1


@pytest.mark.parametrize("x_shape,J,geom", GEOMETRIES)
def test_conv_general_geometries_on_the_matrix_cores(x_shape, J, geom):
    """bf16 with c_out a multiple of 8: im2col rows written from the pairs + the fully-connected GEMM."""
    kh, kw, sh, sw, ph, pw, dh, dw = geom
    N, C, H, W = x_shape
    if geom == CONV3:
        pytest.skip("NCHW 3x3/s1/p1 has kernels of its own")
    OH, OW = _out_extent(H, kh, sh, ph, dh), _out_extent(W, kw, sw, pw, dw)
    print("wgrad conv im2col nchw", x_shape, J, geom, flush=True)
    x = activation(x_shape, "relu", 700 + H + kh, "bf16")
    dy = gradient((N, J, OH, OW), 0.02, 750 + W + kw, "bf16")
    k = oracle.keep_count(x.size, 0.6)
    assert dropit.weight_grad_path(x_shape, torch.bfloat16, k, J, conv=geom) == "conv_im2col"
    got, _, _ = gpu_dw(x, dy, 0.6, J, conv=geom)
    ref = oracle.dw_conv(ref_xhat(x, 0.6), oracle.widen(dy), kh, kw, (sh, sw), (ph, pw), (dh, dw))
    assert got.shape == (J, C, kh, kw)
    assert_close(got, ref, TOL["bf16"])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("x_shape,J,geom", GEOMETRIES)
def test_conv_channels_last(dtype, x_shape, J, geom):
    """x [N,H,W,C], dY [N,OH,OW,J] -> dW [J,kh,kw,C]; the oracle (NCHW) sees the same tensors permuted."""
    kh, kw, sh, sw, ph, pw, dh, dw = geom
    N, C, H, W = x_shape
    OH, OW = _out_extent(H, kh, sh, ph, dh), _out_extent(W, kw, sw, pw, dw)
    print("wgrad conv nhwc", dtype, x_shape, J, geom, flush=True)
    x = activation((N, H, W, C), "relu", 800 + H + kh, dtype)
    dy = gradient((N, OH, OW, J), 0.02, 850 + W + kw, dtype)
    k = oracle.keep_count(x.size, 0.6)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    pointwise = geom[:6] == (1, 1, 1, 1, 0, 0)         # a fully-connected layer over the positions in this layout
    small = pointwise and x.size <= 16384 and N * H * W <= 1024 and C % 4 == 0      # ... and a small one takes the one-launch form
    assert dropit.weight_grad_path(x.shape, tdt, k, J, conv=geom, layout="nhwc") == \
        ("fc_small" if small else "fma" if dtype == "f32" else "fc_mfma" if pointwise else "conv_im2col")
    xd, dyd = to_device(x), to_device(dy)
    vals, idx = dropit.compress(xd, 0.6)
    dW = dropit.weight_grad(vals, idx, x.shape, dyd, J, conv=geom, layout="nhwc")
    torch.cuda.synchronize()
    got = to_host(dW).astype(np.float64)
    assert got.shape == (J, kh, kw, C)
    xhat = np.ascontiguousarray(ref_xhat(x, 0.6).transpose(0, 3, 1, 2))          # selection on the NHWC tensor, then NCHW
    dy_nchw = np.ascontiguousarray(oracle.widen(dy).transpose(0, 3, 1, 2))
    ref = oracle.dw_conv(xhat, dy_nchw, kh, kw, (sh, sw), (ph, pw), (dh, dw)).transpose(0, 2, 3, 1)
    assert_close(got, ref, TOL[dtype])


def test_conv_channels_last_everything_dropped_and_bad_layout():
    x = activation((2, 6, 6, 8), "relu", 1, "bf16")
    dy = gradient((2, 6, 6, 8), 0.02, 2, "bf16")
    xd, dyd = to_device(x), to_device(dy)
    vals, idx = dropit.compress(xd, 1.0)
    dW = dropit.weight_grad(vals, idx, x.shape, dyd, 8, conv=CONV3, layout="nhwc")
    torch.cuda.synchronize()
    assert dW.shape == (8, 3, 3, 8) and not dW.any()
    with pytest.raises(ValueError):
        dropit.weight_grad(vals, idx, x.shape, dyd, 8, conv=None, layout="nhwc")
    with pytest.raises(ValueError):
        dropit.weight_grad(vals, idx, x.shape, dyd, 8, conv=CONV3, layout="chwn")


def test_conv_window_larger_than_input_is_rejected():
    x = activation((1, 2, 4, 4), "relu", 1, "bf16")
    dy = gradient((1, 2, 1, 1), 0.02, 2, "bf16")
    xd, dyd = to_device(x), to_device(dy)
    vals, idx = dropit.compress(xd, 0.5)
    with pytest.raises(dropit.DropitError) as e:
        dropit.weight_grad(vals, idx, x.shape, dyd, 2, conv=(7, 7, 1, 1, 0, 0, 1, 1))
    assert e.value.status == 1


@pytest.fixture
def recover_in_lds():
    """The FC recover step inside the product (dropit_set_fc_recover(1)) for the test, the default form after it."""
    dropit.set_fc_recover(1)
    try:
        yield
    finally:
        dropit.set_fc_recover(0)


def _dw_both_forms(x, dy, gamma, cout):
    """dW of one layer by the dense-operand form and by the in-LDS form, each in a workspace of exactly its size
    filled with NaN bits; also the two workspace sizes."""
    xd, dyd = to_device(x), to_device(dy)
    vals, idx = dropit.compress(xd, gamma)
    out, need = {}, {}
    for form in (0, 1):
        dropit.set_fc_recover(form)
        try:
            assert dropit.weight_grad_path(x.shape, xd.dtype, vals.numel(), cout) == ("fc_fused" if form else "fc_mfma")
            need[form] = dropit.weight_grad_workspace_bytes(x.shape, xd.dtype, vals.numel(), cout)
            ws, check_ws = _guarded(need[form], torch.uint8, pattern=0xFF)
            dwf, check_dw = _guarded(cout * x.shape[-1] * 4, torch.float32, pattern=0xFF)
            out[form] = dropit.weight_grad(vals, idx, x.shape, dyd, cout, dW=dwf.view(cout, x.shape[-1]), workspace=ws)
            torch.cuda.synchronize()
            check_ws()
            check_dw()
        finally:
            dropit.set_fc_recover(0)
    return out, need


@pytest.mark.parametrize("ntok,cin,cout,gamma", [
    (200, 264, 512, 0.9),      # ragged token block, ragged column tile, two row tiles, a single K-slice
    (33, 520, 264, 0.9),       # two token blocks only: fewer tiles than the pipeline is deep
    (20, 1024, 264, 0.9),      # a single token block
    (1000, 520, 264, 0.9),
    (4100, 768, 768, 0.8),     # ~1640 pairs per tile: every tile takes the path for more words than the staging slot holds
    (2500, 768, 1536, 0.0),    # nothing dropped: 8192 words per tile
    (3000, 1000, 520, 0.5),
    (700, 2048, 256, 0.97),    # eight column blocks per token block
    (9000, 512, 512, 0.9),     # several K-slices per tile
    (6000, 300, 136, 0.9),     # just over 128 output channels: the smallest layer the form covers
    (3000, 777, 200, 0.9),     # c_in not a multiple of 8
    (5000, 768, 768, 0.999),   # 24 pairs per token block: most tiles hold a handful of pairs, some none
])
def test_fc_recover_inside_the_product_is_bit_identical(ntok, cin, cout, gamma):
    """Sec. 3.2: R(a^) built tile by tile in LDS gives the dW of the dense-operand form bit for bit, in a smaller
    workspace; and the dense-operand form is the one compared with the oracle element by element above."""
    print("wgrad fc in-LDS recover", ntok, cin, cout, gamma, flush=True)
    x = activation((ntok, cin), "normal", 700 + ntok, "bf16")
    dy = gradient((ntok, cout), 0.02, 800 + ntok, "bf16")
    out, need = _dw_both_forms(x, dy, gamma, cout)
    assert torch.equal(out[0], out[1])
    if gamma >= 0.5:
        assert need[1] < need[0]
    ref = oracle.dw_fc(ref_xhat(x, gamma), oracle.widen(dy))
    assert_close(to_host(out[1]).astype(np.float64), ref, TOL["bf16"])


@pytest.mark.parametrize("layout", ["one_column_block", "tail_rows", "stripes", "single_row"])
def test_fc_recover_inside_the_product_uneven_density(layout):
    """Kept elements that bunch up: tiles of thousands of words beside empty ones, empty token blocks."""
    print("wgrad fc in-LDS recover density", layout, flush=True)
    ntok, cin, cout, gamma = 3000, 768, 264, 0.9
    rng = np.random.default_rng(17)
    xf = rng.standard_normal((ntok, cin), dtype=np.float32)
    rows = np.arange(ntok)
    if layout == "one_column_block":
        xf[:, :256] *= 1e-3
        xf[:, 512:] *= 1e-3
    elif layout == "tail_rows":
        xf[rows < int(0.8 * ntok)] *= 1e-3
    elif layout == "stripes":
        xf[(rows // 100) % 2 == 0] *= 1e-3
    else:
        xf *= 1e-3
        xf[1234] = rng.standard_normal(cin, dtype=np.float32) + 3.0
    x = f32_to_bf16_bits(xf)
    dy = gradient((ntok, cout), 0.02, 501, "bf16")
    out, _ = _dw_both_forms(x, dy, gamma, cout)
    assert torch.equal(out[0], out[1])
    ref = oracle.dw_fc(ref_xhat(x, gamma), oracle.widen(dy))
    assert_close(to_host(out[1]).astype(np.float64), ref, TOL["bf16"])


def test_fc_recover_form_falls_back_where_it_does_not_exist(recover_in_lds):
    """Layers the in-LDS form does not cover keep their path; the setting is per call, not sticky state in the result."""
    bf16 = torch.bfloat16
    assert dropit.weight_grad_path((4000, 768), bf16, 1000, 128) == "fc_mfma"          # the 128-row tile
    assert dropit.weight_grad_path((256, 64), bf16, 100, 128) == "fc_small"
    assert dropit.weight_grad_path((4000, 768), torch.float32, 1000, 256) == "fma"
    assert dropit.weight_grad_path((4000, 768), bf16, 0, 256) == "fc_mfma"             # k == 0: dW = 0 either way
    assert dropit.weight_grad_path((4, 64, 28, 28), bf16, 1000, 64, conv=CONV3) == "conv_bands"
    assert dropit.weight_grad_path((4000, 768), bf16, 1000, 256) == "fc_fused"
    with pytest.raises(dropit.DropitError):
        dropit.set_fc_recover(2)
    # a narrow layer still computes, through the dense operand
    x = activation((700, 520), "normal", 5, "bf16")
    dy = gradient((700, 64), 0.02, 6, "bf16")
    got, _, _ = gpu_dw(x, dy, 0.9, 64)
    assert_close(got, oracle.dw_fc(ref_xhat(x, 0.9), oracle.widen(dy)), TOL["bf16"])


def test_fc_recover_inside_the_product_in_a_hip_graph(recover_in_lds):
    print("wgrad fc in-LDS recover graph", flush=True)
    x = activation((3000, 520), "normal", 31, "bf16")
    dy = gradient((3000, 264), 0.02, 32, "bf16")
    xd, dyd = to_device(x), to_device(dy)
    vals, idx = dropit.compress(xd, 0.9)
    assert dropit.weight_grad_path(x.shape, xd.dtype, vals.numel(), 264) == "fc_fused"
    ws = torch.empty(dropit.weight_grad_workspace_bytes(x.shape, xd.dtype, vals.numel(), 264), dtype=torch.uint8, device="cuda:0")
    dW = dropit.weight_grad(vals, idx, x.shape, dyd, 264, workspace=ws)        # warm-up outside capture
    torch.cuda.synchronize()
    want = to_host(dW).copy()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dropit.weight_grad(vals, idx, x.shape, dyd, 264, dW=dW, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        dropit.weight_grad(vals, idx, x.shape, dyd, 264, dW=dW, workspace=ws)
    for replay in range(3):
        dW.zero_()
        ws.fill_(replay * 41 + 1)                                         # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert to_host(dW).tobytes() == want.tobytes(), replay


def report_elementwise(name, got, ref, cond):
    """Printed, not gated (the gate is the max-normalised error): the worst element-wise error relative to
    the sum of the magnitudes of the element's terms, sum_n |dY[n][j] * R(a^)[n][c]|, which is what bounds
    the rounding of a sum; and the worst plain relative error over the entries of at least 1 % of max|dW|."""
    delta = np.abs(got - ref)
    ratio = (delta / np.maximum(cond, 1e-300)).max()
    big = np.abs(ref) >= 1e-2 * np.abs(ref).max()
    rel = (delta[big] / np.abs(ref[big])).max()
    print("%s: all %d entries compared; max|d|/max|ref| %.3e, worst |d|/sum|terms| %.3e, worst relative error "
          "over entries >= 1%% of the maximum %.3e" % (name, ref.size, delta.max() / np.abs(ref).max(), ratio, rel),
          flush=True)
    return ratio


@pytest.mark.parametrize("name", ["vitb_fc1", "vitb_fc2", "vitdet_fc1", "vitdet_fc2"])
def test_full_size_fc_every_element(name):
    """Full benchmark shape, every entry of dW against the fp64 oracle (Sec. 3.2, Eq. fc_backward_elem_save)."""
    w = WORKLOADS[name]
    print("wgrad full", name, flush=True)
    x, dy = make(w)
    got, vals, idx = gpu_dw(x, dy, w.gamma, w.c_out)
    k = oracle.keep_count(x.size, w.gamma)
    ov, oi = oracle.compress(x, k)
    assert np.array_equal(idx, oi) and vals.tobytes() == ov.tobytes()
    xh = oracle.densify(ov, oi, x.shape)
    dyw = oracle.widen(dy)
    ref = oracle.dw_fc(xh, dyw)
    assert got.shape == ref.shape == (w.c_out, x.shape[-1])
    assert_close(got, ref, TOL["bf16"])
    # fp32 accumulation of exact products: an entry is off by at most (terms) * 2^-24 of the sum of its terms' magnitudes
    ratio = report_elementwise(name, got, ref, oracle.dw_fc(np.abs(xh), np.abs(dyw)))
    assert ratio <= x.shape[0] * 2.0 ** -24


def test_full_size_conv_every_element():
    """Full benchmark shape, every entry of dW against the fp64 oracle (Sec. 3.2, Eq. conv_backward_elem)."""
    w = WORKLOADS["resnet_conv3x3"]
    print("wgrad full conv", flush=True)
    x, dy = make(w)
    got, vals, idx = gpu_dw(x, dy, w.gamma, w.c_out, conv=CONV3)
    k = oracle.keep_count(x.size, w.gamma)
    ov, oi = oracle.compress(x, k)
    assert np.array_equal(idx, oi) and vals.tobytes() == ov.tobytes()
    xh = oracle.densify(ov, oi, x.shape)
    dyw = oracle.widen(dy)
    ref = oracle.dw_conv(xh, dyw, 3, 3, (1, 1), (1, 1))
    assert got.shape == ref.shape == (w.c_out, x.shape[1], 3, 3)
    assert_close(got, ref, TOL["bf16"])
    ratio = report_elementwise("resnet_conv3x3", got, ref, oracle.dw_conv(np.abs(xh), np.abs(dyw), 3, 3, (1, 1), (1, 1)))
    assert ratio <= x.shape[0] * x.shape[2] * x.shape[3] * 2.0 ** -24


@pytest.mark.parametrize("conv", [None, CONV3])
def test_weight_grad_is_bit_reproducible_and_ignores_workspace_contents(conv):
    """Fixed summation order: the same inputs give the same dW bytes, whatever the workspace held before."""
    print("wgrad determinism", conv, flush=True)
    if conv is None:
        x = activation((3000, 520), "normal", 21, "bf16")
        dy = gradient((3000, 264), 0.02, 22, "bf16")
        c_out = 264
    else:
        x = activation((3, 64, 28, 24), "relu", 23, "bf16")
        dy = gradient((3, 40, 28, 24), 0.02, 24, "bf16")
        c_out = 40
    xd, dyd = to_device(x), to_device(dy)
    vals, idx = dropit.compress(xd, 0.85)
    nbytes = dropit.weight_grad_workspace_bytes(x.shape, xd.dtype, vals.numel(), c_out, conv)
    outs = []
    for fill in (0, 255, 0x5A):
        ws = torch.full((max(nbytes, 1),), fill, dtype=torch.uint8, device="cuda:0")
        outs.append(to_host(dropit.weight_grad(vals, idx, x.shape, dyd, c_out, conv=conv, workspace=ws)).copy())
    torch.cuda.synchronize()
    assert outs[0].tobytes() == outs[1].tobytes() == outs[2].tobytes()


@pytest.mark.parametrize("conv", [None, CONV3])
def test_weight_grad_in_a_hip_graph(conv):
    """dropit_weight_grad is ordinary kernel launches only: a captured graph replays it correctly."""
    print("wgrad graph", conv, flush=True)
    if conv is None:
        x = activation((1500, 256), "gelu", 31, "bf16")
        dy = gradient((1500, 136), 0.02, 32, "bf16")
        c_out = 136
    else:
        x = activation((2, 32, 16, 16), "relu", 33, "bf16")
        dy = gradient((2, 24, 16, 16), 0.02, 34, "bf16")
        c_out = 24
    xd, dyd = to_device(x), to_device(dy)
    vals, idx = dropit.compress(xd, 0.9)
    ws = torch.empty(max(1, dropit.weight_grad_workspace_bytes(x.shape, xd.dtype, vals.numel(), c_out, conv)),
                     dtype=torch.uint8, device="cuda:0")
    dW = dropit.weight_grad(vals, idx, x.shape, dyd, c_out, conv=conv, workspace=ws)     # warm-up outside capture
    torch.cuda.synchronize()
    want = to_host(dW).copy()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        dropit.weight_grad(vals, idx, x.shape, dyd, c_out, conv=conv, dW=dW, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        dropit.weight_grad(vals, idx, x.shape, dyd, c_out, conv=conv, dW=dW, workspace=ws)
    for replay in range(3):
        dW.zero_()
        ws.fill_(replay * 41)                                             # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert to_host(dW).tobytes() == want.tobytes(), replay


def _guarded(nbytes, dtype, pattern=0xC3, guard=4096):
    """A tensor of `nbytes` bytes viewed as `dtype`, carved out of the middle of a larger poisoned buffer
    (256-byte aligned); returns (tensor, check) where check() asserts the guard zones on both sides are intact."""
    nbytes = max(int(nbytes), 16)
    size = (nbytes + 255) // 256 * 256
    whole = torch.full((guard + size + guard,), pattern, dtype=torch.uint8, device="cuda:0")
    base = (-whole.data_ptr()) % 256
    lo = base + (guard // 2) // 256 * 256
    inner = whole[lo:lo + nbytes]

    def check():
        assert bool((whole[:lo] == pattern).all()), "bytes before the buffer were written"
        assert bool((whole[lo + nbytes:] == pattern).all()), "bytes after the buffer were written"
    return inner.view(dtype), check


@pytest.mark.parametrize("case", [
    dict(x=(3000, 520), gamma=0.85, c_out=264, conv=None, dist="normal"),              # FC on the matrix cores: recover + GEMM + slice sum
    dict(x=(256, 64), gamma=0.9, c_out=128, conv=None, dist="normal"),                 # small FC: one launch
    dict(x=(640, 40000), gamma=0.9, c_out=8, conv=None, dist="normal"),                # FC, generic path
    dict(x=(3, 64, 28, 24), gamma=0.8, c_out=40, conv=CONV3, dist="relu"),             # conv row bands
    dict(x=(32, 256, 7, 7), gamma=0.8, c_out=256, conv=CONV3, dist="relu"),            # conv as one GEMM over im2col rows
    dict(x=(3, 8, 15, 14), gamma=0.6, c_out=8, conv=(3, 3, 2, 2, 1, 1, 1, 1), dist="relu"),   # general im2col
])
def test_nothing_is_written_outside_dW_and_the_workspace(case):
    """Canaries: dW and the workspace sit inside poisoned buffers exactly as large as the library asks for."""
    print("wgrad canary", case, flush=True)
    x = activation(case["x"], case["dist"], 91, "bf16")
    conv, c_out = case["conv"], case["c_out"]
    if conv is None:
        dy_shape = (x.shape[0], c_out)
        dw_shape = (c_out, x.shape[1])
    else:
        kh, kw, sh, sw, ph, pw, dh, dw_ = conv
        oh = (x.shape[2] + 2 * ph - dh * (kh - 1) - 1) // sh + 1
        ow = (x.shape[3] + 2 * pw - dw_ * (kw - 1) - 1) // sw + 1
        dy_shape = (x.shape[0], c_out, oh, ow)
        dw_shape = (c_out, x.shape[1], kh, kw)
    dy = gradient(dy_shape, 0.02, 92, "bf16")
    xd, dyd = to_device(x), to_device(dy)
    vals, idx = dropit.compress(xd, case["gamma"])
    need = dropit.weight_grad_workspace_bytes(x.shape, xd.dtype, vals.numel(), c_out, conv)
    ws, check_ws = _guarded(need, torch.uint8)
    dwf, check_dw = _guarded(int(np.prod(dw_shape)) * 4, torch.float32)
    dW = dwf.view(dw_shape)
    want = dropit.weight_grad(vals, idx, x.shape, dyd, c_out, conv=conv)
    got = dropit.weight_grad(vals, idx, x.shape, dyd, c_out, conv=conv, dW=dW, workspace=ws)
    torch.cuda.synchronize()
    check_ws()
    check_dw()
    assert torch.equal(got, want)
