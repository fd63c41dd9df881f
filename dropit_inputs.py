"""Seeded synthetic inputs for the DropIT hot path.

This module holds input generation only: shapes, seeds, value distributions
and the fp32 -> bf16 storage rounding.  None of the method's arithmetic
(selection, recover, weight gradient) lives here, so both the CPU oracle's
tests and the GPU path's tests/benchmark can draw identical bytes from it.

The tensors stand in for the workloads the paper trains on (DeiT / ViT FC
inputs after LayerNorm and GELU, ResNet conv inputs after ReLU; Sec. 3.2,
Fig. 3, Sec. 3.5; ViTDet-B at 1024x1024 from the introduction): same shapes
and value distributions, no dataset.

bf16 tensors are returned as ``np.uint16`` bit patterns, fp32 tensors as
``np.float32``.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    out = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = (b & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    if nan.any():
        out[nan] = ((b[nan] >> np.uint32(16)) | np.uint32(0x0040)).astype(np.uint16)
    return out


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    """Exact bf16 (uint16 bit patterns) -> fp32."""
    return (np.ascontiguousarray(a, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                      # "f32" | "bf16"
    x_shape: Tuple[int, ...]
    x_dist: str                     # "normal" | "gelu" | "relu"
    gamma: float
    c_out: int
    dy_std: float
    x_seed: int
    dy_seed: int
    conv: Optional[Tuple[int, int, int, int]] = None   # (kh, kw, stride, pad); None = FC

    @property
    def numel(self) -> int:
        return int(np.prod(self.x_shape, dtype=np.int64))

    @property
    def dy_shape(self) -> Tuple[int, ...]:
        if self.conv is None:
            return tuple(self.x_shape[:-1]) + (self.c_out,)
        kh, kw, s, p = self.conv
        n, _, h, w = self.x_shape
        oh = (h + 2 * p - kh) // s + 1
        ow = (w + 2 * p - kw) // s + 1
        return (n, self.c_out, oh, ow)

    @property
    def dw_shape(self) -> Tuple[int, ...]:
        if self.conv is None:
            return (self.c_out, self.x_shape[-1])
        return (self.c_out, self.x_shape[1], self.conv[0], self.conv[1])

    @property
    def dense_flops(self) -> int:
        """Dense-equivalent flops of the weight gradient (the paper keeps the dense GEMM, Sec. 3.2)."""
        if self.conv is None:
            ntok = self.numel // self.x_shape[-1]
            return 2 * self.c_out * self.x_shape[-1] * ntok
        n, c, _, _ = self.x_shape
        _, _, oh, ow = self.dy_shape
        return 2 * self.c_out * c * self.conv[0] * self.conv[1] * n * oh * ow


# The five benchmark configurations (4 has two tensors).
WORKLOADS = {
    "tiny_fc": Workload("tiny_fc", "f32", (256, 64), "normal", 0.9, 128, 1.0, 1001, 2001),
    "vitb_fc1": Workload("vitb_fc1", "bf16", (12608, 768), "normal", 0.9, 3072, 0.02, 1002, 2002),
    "vitb_fc2": Workload("vitb_fc2", "bf16", (12608, 3072), "gelu", 0.9, 768, 0.02, 1003, 2003),
    "vitdet_fc1": Workload("vitdet_fc1", "bf16", (16384, 768), "normal", 0.9, 3072, 0.02, 1004, 2004),
    "vitdet_fc2": Workload("vitdet_fc2", "bf16", (16384, 3072), "gelu", 0.9, 768, 0.02, 1005, 2005),
    "resnet_conv3x3": Workload("resnet_conv3x3", "bf16", (64, 64, 56, 56), "relu", 0.8, 64, 0.02,
                               1006, 2006, conv=(3, 3, 1, 1)),
}

# Further shapes the benchmark can run (`bench.py --workload NAME`); not part of the five configurations above.
# The 3x3 convolutions of the later ResNet-50 stages at batch 64: planes of 28, 14 and 7.
EXTRA_WORKLOADS = {
    "resnet_conv3x3_28": Workload("resnet_conv3x3_28", "bf16", (64, 128, 28, 28), "relu", 0.8, 128, 0.02,
                                  1007, 2007, conv=(3, 3, 1, 1)),
    "resnet_conv3x3_14": Workload("resnet_conv3x3_14", "bf16", (64, 256, 14, 14), "relu", 0.8, 256, 0.02,
                                  1008, 2008, conv=(3, 3, 1, 1)),
    "resnet_conv3x3_7": Workload("resnet_conv3x3_7", "bf16", (64, 512, 7, 7), "relu", 0.8, 512, 0.02,
                                 1009, 2009, conv=(3, 3, 1, 1)),
    # other geometries of the same networks: a bottleneck's 1x1, the strided 3x3 that opens a stage,
    # ResNet's first layer (on the normalised image), ViT's patch embedding
    "resnet_conv1x1": Workload("resnet_conv1x1", "bf16", (64, 256, 56, 56), "relu", 0.8, 64, 0.02,
                               1010, 2010, conv=(1, 1, 1, 0)),
    "resnet_conv3x3_s2": Workload("resnet_conv3x3_s2", "bf16", (64, 128, 56, 56), "relu", 0.8, 128, 0.02,
                                  1011, 2011, conv=(3, 3, 2, 1)),
    "resnet_conv7x7_s2": Workload("resnet_conv7x7_s2", "bf16", (64, 3, 224, 224), "normal", 0.8, 64, 0.02,
                                  1012, 2012, conv=(7, 7, 2, 3)),
    "vit_patch_embed": Workload("vit_patch_embed", "bf16", (64, 3, 224, 224), "normal", 0.8, 768, 0.02,
                                1013, 2013, conv=(16, 16, 16, 0)),
}


def _normal(shape, seed: int) -> np.ndarray:
    return np.random.default_rng(seed).standard_normal(size=shape, dtype=np.float32)


def activation(shape, dist: str, seed: int, dtype: str) -> np.ndarray:
    """Layer-input-like tensor: N(0,1) (post-LayerNorm), GELU(N(0,1)) or ReLU(N(0,1))."""
    z = _normal(shape, seed)
    if dist == "normal":
        a = z
    elif dist == "relu":
        a = np.maximum(z, np.float32(0.0))
    elif dist == "gelu":
        from scipy.special import erf
        z64 = z.astype(np.float64)
        a = (0.5 * z64 * (1.0 + erf(z64 / np.sqrt(2.0)))).astype(np.float32)
    else:
        raise ValueError(dist)
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(a)
    raise ValueError(dtype)


def gradient(shape, std: float, seed: int, dtype: str) -> np.ndarray:
    """Output-gradient-like tensor ~ N(0, std^2)."""
    g = _normal(shape, seed) * np.float32(std)
    return np.ascontiguousarray(g, dtype=np.float32) if dtype == "f32" else f32_to_bf16_bits(g)


def make(w: Workload, ntok_limit: Optional[int] = None):
    """(x, dY) host arrays for a workload.  ``ntok_limit`` (FC only) keeps the
    first tokens only -- same generator stream, truncated -- for bounded CPU timing."""
    x = activation(w.x_shape, w.x_dist, w.x_seed, w.dtype)
    dy = gradient(w.dy_shape, w.dy_std, w.dy_seed, w.dtype)
    if ntok_limit is not None and w.conv is None:
        x = np.ascontiguousarray(x.reshape(-1, w.x_shape[-1])[:ntok_limit])
        dy = np.ascontiguousarray(dy.reshape(-1, w.c_out)[:ntok_limit])
    return x, dy
