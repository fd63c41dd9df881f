"""torch.autograd integration of the DropIT hot path.

The paper's implementation note (Sec. 4, implementation paragraph) describes the layer-level mechanism: in
the forward pass the layer's input is converted to (value, index) form and the dense input is left
to be released; in the backward pass the sparse form is recovered for the weight gradient only
(Sec. 3.2, 3.3).  The forward output and the gradient with respect to the input never touch the
cache (Sec. 3.5: dropping happens only where the gradient flows to the parameters), so they are
computed here by the ordinary torch operators; the two steps the method adds -- the min-k
compression and the weight gradient from the sparse cache -- are the library's HIP kernels behind
``dropit_compress`` / ``dropit_weight_grad``.  There is no CPU path: training-mode calls need
device tensors and the built library.

Layer policy (Sec. 3.5 and the appendix on first and final layers): fully-connected and
convolutional layers are applicable, normalisation and activation layers are not, and the first
and the last applicable layer of a network are left alone because dropping there cannot lower the
peak.  Inference is unchanged.
"""
from __future__ import annotations

import contextlib
import threading
from typing import Iterator, List, Optional, Sequence, Tuple, Union

import torch
import torch.nn.functional as F

from . import binding

_Int2 = Union[int, Sequence[int]]


def _check_format(index_format: str) -> str:
    if index_format not in ("flat", "rows", "mask"):
        raise ValueError("index_format must be 'flat', 'rows' or 'mask'")
    return index_format


def _pair(v: _Int2) -> Tuple[int, int]:
    if isinstance(v, int):
        return (v, v)
    a, b = v
    return (int(a), int(b))


# ---------------------------------------------------------------------------------------------
# cache accounting (Sec. 4.3, table of cached-tensor memory: value bytes fall by exactly gamma;
# the indices are the method's own extra cost)
# ---------------------------------------------------------------------------------------------
class CacheMeter:
    """Bytes the DropIT layers cached during the forward passes run under ``cache_meter()``."""

    def __init__(self) -> None:
        self.dense_bytes = 0     # what the same layers would have kept without dropping
        self.value_bytes = 0     # retained values
        self.index_bytes = 0     # their indices (int32 flat, or 16-bit in-row positions + row offsets)
        self.layers = 0

    def _add(self, x: torch.Tensor, cache: Sequence[torch.Tensor]) -> None:
        self.dense_bytes += x.numel() * x.element_size()
        self.value_bytes += cache[0].numel() * cache[0].element_size()
        self.index_bytes += sum(t.numel() * t.element_size() for t in cache[1:])
        self.layers += 1


_meters = threading.local()


@contextlib.contextmanager
def cache_meter() -> Iterator[CacheMeter]:
    meter = CacheMeter()
    stack = getattr(_meters, "stack", None)
    if stack is None:
        stack = _meters.stack = []
    stack.append(meter)
    try:
        yield meter
    finally:
        stack.pop()


def _account(x: torch.Tensor, cache: Sequence[torch.Tensor]) -> None:
    for meter in getattr(_meters, "stack", ()):
        meter._add(x, cache)


def _compress_input(x: torch.Tensor, gamma: float, seed: Optional[int], fmt: str) -> Tuple[torch.Tensor, ...]:
    """Min-k dropping, or (seed given) the random strategy of Sec. 3.3 with that seed.  Returns the
    cache: (vals, idx), or one of the cheaper index forms: "rows" (vals, col, rowptr), "mask"
    (vals, mask, blockptr)."""
    if not x.is_cuda:
        raise RuntimeError("DropIT layers train on device tensors only: there is no CPU path")
    xc = x.detach()
    if not xc.is_contiguous() or xc.data_ptr() % 16:      # the library reads 16-byte vectors: a contiguous view that
        xc = xc.clone(memory_format=torch.contiguous_format)   # starts inside a buffer (x[1:]) is copied to an aligned one
    if fmt != "flat":
        if seed is not None:
            raise ValueError("the random strategy keeps flat indices (index_format='flat')")
        cache = binding.compress_rows(xc, gamma) if fmt == "rows" else binding.compress_mask(xc, gamma)
    elif seed is None:
        cache = binding.compress(xc, gamma)
    else:
        cache = binding.compress_random(xc, gamma, seed)
    _account(xc, cache)
    return tuple(cache)


def _weight_grad(cache: Sequence[torch.Tensor], fmt: str, x_shape, dy: torch.Tensor, c_out: int, conv=None) -> torch.Tensor:
    dy = _match_dtype(dy, cache[0])
    if fmt == "rows":
        return binding.weight_grad_rows(cache[0], cache[1], cache[2], x_shape, dy, c_out, conv=conv)
    if fmt == "mask":
        return binding.weight_grad_mask(cache[0], cache[1], cache[2], x_shape, dy, c_out, conv=conv)
    return binding.weight_grad(cache[0], cache[1], x_shape, dy, c_out, conv=conv)


def _match_dtype(dy: torch.Tensor, vals: torch.Tensor) -> torch.Tensor:
    dy = dy if dy.dtype == vals.dtype else dy.to(vals.dtype)
    if not dy.is_contiguous() or dy.data_ptr() % 16:       # 16-byte vector loads, as for the input
        dy = dy.clone(memory_format=torch.contiguous_format)
    return dy


# ---------------------------------------------------------------------------------------------
# fully-connected layer (Sec. 3.2, Eq. fc_backward_elem_save, weight gradient of a fully-connected layer from the retained elements)
# ---------------------------------------------------------------------------------------------
class _LinearFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, gamma, seed, fmt):
        y = F.linear(x, weight, bias)
        ctx.save_for_backward(weight, *_compress_input(x, gamma, seed, fmt))
        ctx.fmt = fmt
        ctx.x_shape = tuple(x.shape)
        ctx.has_bias = bias is not None
        return y

    @staticmethod
    def backward(ctx, dy):
        weight, *cache = ctx.saved_tensors
        c_out, c_in = weight.shape
        dx = dw = db = None
        dy2 = dy.reshape(-1, c_out)
        if ctx.needs_input_grad[0]:
            dx = (dy2 @ weight.to(dy.dtype)).reshape(ctx.x_shape)
        if ctx.needs_input_grad[1]:
            dw = _weight_grad(cache, ctx.fmt, ctx.x_shape, dy2, c_out).to(weight.dtype)
        if ctx.has_bias and ctx.needs_input_grad[2]:
            db = dy2.sum(0)
        return dx, dw, db, None, None, None


def linear(x: torch.Tensor, weight: torch.Tensor, bias: Optional[torch.Tensor] = None,
           gamma: float = 0.9, seed: Optional[int] = None, index_format: str = "flat") -> torch.Tensor:
    """``F.linear`` whose backward computes the weight gradient from the min-k cache of ``x``
    (from a random cache drawn with ``seed`` when one is given).  ``index_format`` "rows" caches
    16-bit in-row positions and row offsets instead of int32 flat indices, "mask" one bit per
    element and block offsets."""
    return _LinearFn.apply(x, weight, bias, float(gamma), seed, _check_format(index_format))


# ---------------------------------------------------------------------------------------------
# convolution (Sec. 3.2, Eq. conv_backward_elem, weight gradient of a convolutional layer from the retained elements)
# ---------------------------------------------------------------------------------------------
class _Conv2dFn(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, weight, bias, stride, padding, dilation, gamma, seed, fmt):
        y = F.conv2d(x, weight, bias, stride, padding, dilation, 1)
        # a channels-last input is cached as it lies in memory ([N, H, W, C]) instead of being copied to NCHW
        ctx.fmt = fmt
        ctx.nhwc = (fmt == "flat" and x.dim() == 4 and not x.is_contiguous()
                    and x.is_contiguous(memory_format=torch.channels_last))
        ctx.save_for_backward(weight, *_compress_input(x.permute(0, 2, 3, 1) if ctx.nhwc else x, gamma, seed, fmt))
        ctx.x_shape = tuple(x.shape)
        ctx.geometry = (stride, padding, dilation)
        ctx.has_bias = bias is not None
        return y

    @staticmethod
    def backward(ctx, dy):
        weight, *cache = ctx.saved_tensors
        stride, padding, dilation = ctx.geometry
        c_out, _, kh, kw = weight.shape
        dx = dw = db = None
        if ctx.needs_input_grad[0]:
            dx = torch.nn.grad.conv2d_input(ctx.x_shape, weight.to(dy.dtype), dy, stride, padding, dilation, 1)
        if ctx.needs_input_grad[1]:
            conv = (kh, kw, stride[0], stride[1], padding[0], padding[1], dilation[0], dilation[1])
            if ctx.nhwc:
                n, c, h, w = ctx.x_shape
                dyl = _match_dtype(dy.permute(0, 2, 3, 1), cache[0])
                dw = binding.weight_grad(cache[0], cache[1], (n, h, w, c), dyl, c_out, conv=conv, layout="nhwc")
                dw = dw.permute(0, 3, 1, 2).to(weight.dtype)        # [J, C, kh, kw] with channels-last strides
            else:
                dw = _weight_grad(cache, ctx.fmt, ctx.x_shape, dy, c_out, conv=conv).to(weight.dtype)
        if ctx.has_bias and ctx.needs_input_grad[2]:
            db = dy.sum((0, 2, 3))
        return dx, dw, db, None, None, None, None, None, None


def conv2d(x: torch.Tensor, weight: torch.Tensor, bias: Optional[torch.Tensor] = None,
           stride: _Int2 = 1, padding: _Int2 = 0, dilation: _Int2 = 1, gamma: float = 0.9,
           seed: Optional[int] = None, index_format: str = "flat") -> torch.Tensor:
    """``F.conv2d`` (groups = 1, zero padding) whose backward computes the weight gradient
    from the min-k cache of ``x`` (from a random cache drawn with ``seed`` when one is given);
    ``index_format`` as for ``linear``.  A channels-last ``x`` is cached and multiplied in that
    layout (flat index format)."""
    return _Conv2dFn.apply(x, weight, bias, _pair(stride), _pair(padding), _pair(dilation), float(gamma), seed,
                           _check_format(index_format))


# ---------------------------------------------------------------------------------------------
# modules and the layer policy
# ---------------------------------------------------------------------------------------------
_SEED_STRIDE = 0x9E3779B97F4A7C15      # odd: successive calls of a layer walk through all 2^64 seeds


def _next_seed(module: torch.nn.Module) -> Optional[int]:
    """None for min-k; for the random strategy a fresh seed per forward call, so that every
    iteration drops a different subset (Sec. 3.3: dropped at random within each mini-batch)."""
    if getattr(module, "strategy", "mink") != "random":
        return None
    calls = getattr(module, "_dropit_calls", 0)
    module._dropit_calls = calls + 1
    return (int(getattr(module, "seed", 0)) + calls * _SEED_STRIDE) & 0xFFFFFFFFFFFFFFFF


def _check_strategy(strategy: str) -> str:
    if strategy not in ("mink", "random"):
        raise ValueError("strategy must be 'mink' or 'random'")
    return strategy


def _dropping(module: torch.nn.Module) -> bool:
    """Inference, no-grad regions, frozen weights and gamma = 0 (the baseline column) run the plain operator."""
    return (module.training and torch.is_grad_enabled() and module.gamma > 0.0
            and module.weight.requires_grad)


class Linear(torch.nn.Linear):
    def __init__(self, in_features: int, out_features: int, bias: bool = True, gamma: float = 0.9,
                 strategy: str = "mink", seed: int = 0, index_format: str = "flat", device=None,
                 dtype=None) -> None:
        super().__init__(in_features, out_features, bias, device=device, dtype=dtype)
        self.gamma = float(gamma)
        self.strategy = _check_strategy(strategy)
        self.seed = int(seed)
        self.index_format = _check_format(index_format)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        if not _dropping(self):
            return F.linear(x, self.weight, self.bias)
        return linear(x, self.weight, self.bias, self.gamma, _next_seed(self),
                      getattr(self, "index_format", "flat"))

    def extra_repr(self) -> str:
        return super().extra_repr() + ", gamma=%g" % self.gamma


def _conv_applicable(m: torch.nn.Conv2d) -> bool:
    return m.groups == 1 and m.padding_mode == "zeros" and not isinstance(m.padding, str)


class Conv2d(torch.nn.Conv2d):
    def __init__(self, *args, gamma: float = 0.9, strategy: str = "mink", seed: int = 0,
                 index_format: str = "flat", **kwargs) -> None:
        super().__init__(*args, **kwargs)
        if not _conv_applicable(self):
            raise ValueError("DropIT Conv2d supports groups=1, zero padding given as integers")
        self.gamma = float(gamma)
        self.strategy = _check_strategy(strategy)
        self.seed = int(seed)
        self.index_format = _check_format(index_format)

    def forward(self, x: torch.Tensor) -> torch.Tensor:
        if not _dropping(self):
            return self._conv_forward(x, self.weight, self.bias)
        return conv2d(x, self.weight, self.bias, self.stride, self.padding, self.dilation, self.gamma,
                      _next_seed(self), getattr(self, "index_format", "flat"))

    def extra_repr(self) -> str:
        return super().extra_repr() + ", gamma=%g" % self.gamma


def apply_dropit(model: torch.nn.Module, gamma: float, skip_first: bool = True,
                 skip_last: bool = True, strategy: str = "mink", seed: int = 0,
                 index_format: str = "flat") -> List[str]:
    """Switch the applicable layers of ``model`` to DropIT in place and return their names.

    Applicable: ``nn.Linear`` and ``nn.Conv2d`` (groups = 1, zero padding); the modules keep their
    parameters, buffers, hooks and state-dict keys (only their class changes).  The first and the
    last applicable layer, in module registration order, are left as they are unless asked
    otherwise: their inputs stay alive (or are created last) whatever the layer caches, so
    dropping there adds the sparse copy to the peak instead of lowering it.  ``strategy`` is
    "mink" (Sec. 3.3 Min-K Elements) or "random" (Sec. 3.3 Random Elements, seeded per layer
    and per call from ``seed``).  ``index_format`` "rows" caches 16-bit in-row positions and row
    offsets instead of int32 flat indices (min-k only)."""
    found: List[Tuple[str, torch.nn.Module]] = []
    for name, m in model.named_modules():
        if type(m) is torch.nn.Linear or (type(m) is torch.nn.Conv2d and _conv_applicable(m)):
            found.append((name, m))
    if skip_first and found:
        found = found[1:]
    if skip_last and found:
        found = found[:-1]
    _check_strategy(strategy)
    _check_format(index_format)
    for number, (_, m) in enumerate(found):
        m.index_format = index_format
        m.__class__ = Linear if isinstance(m, torch.nn.Linear) else Conv2d
        m.gamma = float(gamma)
        m.strategy = strategy
        m.seed = (int(seed) + (number << 48)) & 0xFFFFFFFFFFFFFFFF     # layers draw from disjoint seed ranges
    return [name for name, _ in found]
