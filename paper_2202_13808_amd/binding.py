"""ctypes binding of the C ABI in ``include/dropit.h`` -- marshalling only.

Every function here has the name of the C entry point without the ``dropit_``
prefix and does nothing but turn torch tensors into pointers and sizes.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libdropit.so")

F32, BF16 = 0, 1
OK, EINVAL, EWORKSPACE, EUNSUPPORTED, EHIP = range(5)


class DropitError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(message)
        self.status = status


class Conv2d(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in
                ("kh", "kw", "stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w")]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_2202_13808_amd.build` "
                "(there is no CPU fallback)" % _LIB_PATH)
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32, dbl, sz = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_double,
                                 ctypes.c_size_t)
        p64 = ctypes.POINTER(ctypes.c_int64)
        pconv = ctypes.POINTER(Conv2d)
        L.dropit_status_string.restype = ctypes.c_char_p
        L.dropit_status_string.argtypes = [i32]
        L.dropit_keep_count.restype = i64
        L.dropit_keep_count.argtypes = [i64, dbl]
        L.dropit_compress_workspace_bytes.restype = sz
        L.dropit_compress_workspace_bytes.argtypes = [i64, i32]
        L.dropit_compress.restype = i32
        L.dropit_compress.argtypes = [vp, p64, i32, i32, dbl, vp, vp, vp, sz, vp]
        L.dropit_compress_static.restype = i32
        L.dropit_compress_static.argtypes = [vp, p64, i32, i32, dbl, vp, vp, vp]
        L.dropit_compress_random_workspace_bytes.restype = sz
        L.dropit_compress_random_workspace_bytes.argtypes = [i64, i32]
        L.dropit_compress_random.restype = i32
        L.dropit_compress_random.argtypes = [vp, p64, i32, i32, dbl, ctypes.c_uint64, vp, vp, vp, sz, vp]
        L.dropit_compress_rows_workspace_bytes.restype = sz
        L.dropit_compress_rows_workspace_bytes.argtypes = [i64, i64, i32]
        L.dropit_compress_rows.restype = i32
        L.dropit_compress_rows.argtypes = [vp, p64, i32, i32, dbl, vp, vp, vp, vp, sz, vp]
        L.dropit_weight_grad_rows_workspace_bytes.restype = sz
        L.dropit_weight_grad_rows_workspace_bytes.argtypes = [p64, i32, i32, i64, i64, pconv]
        L.dropit_weight_grad_rows.restype = i32
        L.dropit_weight_grad_rows.argtypes = [vp, vp, vp, i64, p64, i32, i32, vp, i64, pconv, vp, vp, sz, vp]
        L.dropit_compress_mask_workspace_bytes.restype = sz
        L.dropit_compress_mask_workspace_bytes.argtypes = [i64, i64, i32]
        L.dropit_compress_mask.restype = i32
        L.dropit_compress_mask.argtypes = [vp, p64, i32, i32, ctypes.c_double, vp, vp, vp, vp, sz, vp]
        L.dropit_weight_grad_mask_workspace_bytes.restype = sz
        L.dropit_weight_grad_mask_workspace_bytes.argtypes = [p64, i32, i32, i64, i64, pconv]
        L.dropit_weight_grad_mask.restype = i32
        L.dropit_weight_grad_mask.argtypes = [vp, vp, vp, i64, p64, i32, i32, vp, i64, pconv, vp, vp, sz, vp]
        L.dropit_weight_grad_workspace_bytes.restype = sz
        L.dropit_weight_grad_workspace_bytes.argtypes = [p64, i32, i32, i64, i64, pconv]
        L.dropit_weight_grad_path.restype = i32
        L.dropit_weight_grad_path.argtypes = [p64, i32, i32, i64, i64, pconv]
        L.dropit_weight_grad_nhwc_path.restype = i32
        L.dropit_weight_grad_nhwc_path.argtypes = [p64, i32, i64, i64, pconv]
        L.dropit_weight_grad_nhwc_workspace_bytes.restype = sz
        L.dropit_weight_grad_nhwc_workspace_bytes.argtypes = [p64, i32, i64, i64, pconv]
        L.dropit_weight_grad_nhwc.restype = i32
        L.dropit_weight_grad_nhwc.argtypes = [vp, vp, i64, p64, i32, vp, i64, pconv, vp, vp, sz, vp]
        L.dropit_set_select_mode.restype = i32
        L.dropit_set_select_mode.argtypes = [i32]
        L.dropit_set_fc_recover.restype = i32
        L.dropit_set_fc_recover.argtypes = [i32]
        L.dropit_trace_events.restype = None
        L.dropit_trace_events.argtypes = [ctypes.POINTER(vp), i32]
        L.dropit_weight_grad.restype = i32
        L.dropit_weight_grad.argtypes = [vp, vp, i64, p64, i32, i32, vp, i64, pconv, vp, vp, sz, vp]
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != OK:
        raise DropitError(status, lib().dropit_status_string(status).decode())


def _dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return F32
    if t == torch.bfloat16:
        return BF16
    raise TypeError("dropit supports float32 and bfloat16 tensors, got %s" % t)


def _shape_array(shape: Sequence[int]):
    return (ctypes.c_int64 * len(shape))(*[int(s) for s in shape])


def _conv_struct(conv) -> Optional[Conv2d]:
    if conv is None:
        return None
    if isinstance(conv, Conv2d):
        return conv
    return Conv2d(*[int(v) for v in conv])


def _stream_ptr(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


class _on:
    """Makes `device` the current one for the duration of a call, and costs nothing when it already is
    (the library launches on the current device; torch's own context manager takes several microseconds,
    which a launch-bound layer notices)."""
    __slots__ = ("index", "previous")

    def __init__(self, device):
        self.index = device.index
        self.previous = None

    def __enter__(self):
        if self.index is not None:
            current = torch.cuda.current_device()
            if current != self.index:
                self.previous = current
                torch.cuda.set_device(self.index)
        return self

    def __exit__(self, *exc):
        if self.previous is not None:
            torch.cuda.set_device(self.previous)
        return False


def _require_device(*tensors) -> None:
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("dropit operates on device tensors only (no CPU path)")
        if t is not None and not t.is_contiguous():
            raise ValueError("dropit tensors must be contiguous")


def keep_count(numel: int, gamma: float) -> int:
    """dropit_keep_count: k = floor((1-gamma)*numel); -1 if the arguments are invalid."""
    return int(lib().dropit_keep_count(int(numel), float(gamma)))


def compress_workspace_bytes(numel: int, dtype: torch.dtype) -> int:
    return int(lib().dropit_compress_workspace_bytes(int(numel), _dtype_code(dtype)))


def compress(x: torch.Tensor, gamma: float, vals: Optional[torch.Tensor] = None,
             idx: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
             stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """dropit_compress: returns (vals[k] of x.dtype, idx[k] int32).  Output and workspace
    tensors are allocated with torch when not passed in."""
    _require_device(x, vals, idx, workspace)
    code = _dtype_code(x.dtype)
    k = keep_count(x.numel(), gamma)
    if k < 0:
        _check(EINVAL)
    if vals is None:
        vals = torch.empty(k, dtype=x.dtype, device=x.device)
    if idx is None:
        idx = torch.empty(k, dtype=torch.int32, device=x.device)
    if vals.numel() < k or idx.numel() < k or vals.dtype != x.dtype or idx.dtype != torch.int32:
        raise ValueError("vals/idx must hold k=%d elements of %s / int32" % (k, x.dtype))
    if workspace is None:
        workspace = torch.empty(max(compress_workspace_bytes(x.numel(), x.dtype), 1),
                                dtype=torch.uint8, device=x.device)
    shape = _shape_array(x.shape)
    with _on(x.device):
        _check(lib().dropit_compress(x.data_ptr(), shape, x.dim(), code, float(gamma),
                                     vals.data_ptr() if k else None, idx.data_ptr() if k else None,
                                     workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return vals[:k], idx[:k]


def compress_static(x: torch.Tensor, gamma: float, vals: torch.Tensor, idx: torch.Tensor, stream=None
                    ) -> Tuple[torch.Tensor, torch.Tensor]:
    """dropit_compress_static: dropit_compress on the library's own static exchange area.  Nothing is
    allocated, here or in the library: the caller passes the outputs (at least k elements each)."""
    _require_device(x, vals, idx)
    code = _dtype_code(x.dtype)
    k = keep_count(x.numel(), gamma)
    if k < 0:
        _check(EINVAL)
    if vals.numel() < k or idx.numel() < k or vals.dtype != x.dtype or idx.dtype != torch.int32:
        raise ValueError("vals/idx must hold k=%d elements of %s / int32" % (k, x.dtype))
    shape = _shape_array(x.shape)
    with _on(x.device):
        _check(lib().dropit_compress_static(x.data_ptr(), shape, x.dim(), code, float(gamma),
                                            vals.data_ptr() if k else None, idx.data_ptr() if k else None,
                                            _stream_ptr(stream)))
    return vals[:k], idx[:k]


def compress_random_workspace_bytes(numel: int, dtype: torch.dtype) -> int:
    return int(lib().dropit_compress_random_workspace_bytes(int(numel), _dtype_code(dtype)))


def compress_random(x: torch.Tensor, gamma: float, seed: int, vals: Optional[torch.Tensor] = None,
                    idx: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                    stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """dropit_compress_random: like ``compress`` with a uniformly random retained set fixed by ``seed``."""
    _require_device(x, vals, idx, workspace)
    code = _dtype_code(x.dtype)
    k = keep_count(x.numel(), gamma)
    if k < 0 or not 0 <= int(seed) < (1 << 64):
        _check(EINVAL)
    if vals is None:
        vals = torch.empty(k, dtype=x.dtype, device=x.device)
    if idx is None:
        idx = torch.empty(k, dtype=torch.int32, device=x.device)
    if vals.numel() < k or idx.numel() < k or vals.dtype != x.dtype or idx.dtype != torch.int32:
        raise ValueError("vals/idx must hold k=%d elements of %s / int32" % (k, x.dtype))
    if workspace is None:
        workspace = torch.empty(max(compress_random_workspace_bytes(x.numel(), x.dtype), 1),
                                dtype=torch.uint8, device=x.device)
    shape = _shape_array(x.shape)
    with _on(x.device):
        _check(lib().dropit_compress_random(x.data_ptr(), shape, x.dim(), code, float(gamma), int(seed),
                                            vals.data_ptr() if k else None, idx.data_ptr() if k else None,
                                            workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return vals[:k], idx[:k]


def _nhwc(layout: str, x_shape, cs) -> bool:
    if layout not in ("nchw", "nhwc"):
        raise ValueError("layout must be 'nchw' or 'nhwc'")
    if layout == "nhwc" and (cs is None or len(x_shape) != 4):
        raise ValueError("the channels-last layout is for convolutions: 4-d x_shape and conv=...")
    return layout == "nhwc"


def weight_grad_workspace_bytes(x_shape: Sequence[int], dtype: torch.dtype, k: int, c_out: int,
                                conv=None, layout: str = "nchw") -> int:
    cs = _conv_struct(conv)
    pc = ctypes.byref(cs) if cs is not None else None
    if _nhwc(layout, x_shape, cs):
        return int(lib().dropit_weight_grad_nhwc_workspace_bytes(
            _shape_array(x_shape), _dtype_code(dtype), int(k), int(c_out), pc))
    return int(lib().dropit_weight_grad_workspace_bytes(
        _shape_array(x_shape), len(x_shape), _dtype_code(dtype), int(k), int(c_out), pc))


WGRAD_PATHS = {0: "none", 1: "fc_mfma", 2: "conv_bands", 3: "conv_gemm", 4: "fma", 5: "conv_im2col", 6: "fc_small",
               7: "fc_fused"}


def weight_grad_path(x_shape: Sequence[int], dtype: torch.dtype, k: int, c_out: int, conv=None,
                     layout: str = "nchw") -> str:
    """dropit_weight_grad_path: which kernels ``weight_grad`` runs for these arguments."""
    cs = _conv_struct(conv)
    pc = ctypes.byref(cs) if cs is not None else None
    if _nhwc(layout, x_shape, cs):
        return WGRAD_PATHS[int(lib().dropit_weight_grad_nhwc_path(
            _shape_array(x_shape), _dtype_code(dtype), int(k), int(c_out), pc))]
    return WGRAD_PATHS[int(lib().dropit_weight_grad_path(
        _shape_array(x_shape), len(x_shape), _dtype_code(dtype), int(k), int(c_out), pc))]


def weight_grad(vals: torch.Tensor, idx: torch.Tensor, x_shape: Sequence[int], dY: torch.Tensor,
                c_out: int, conv=None, dW: Optional[torch.Tensor] = None,
                workspace: Optional[torch.Tensor] = None, stream=None, layout: str = "nchw") -> torch.Tensor:
    """dropit_weight_grad: dW (fp32) from the (vals, idx) pair of a tensor of ``x_shape``.
    ``conv`` is None for a fully-connected layer, else (kh, kw, stride_h, stride_w, pad_h,
    pad_w, dil_h, dil_w).  ``layout="nhwc"`` (dropit_weight_grad_nhwc): x_shape = [N, H, W, C],
    dY [N, OH, OW, c_out], dW [c_out, kh, kw, C]."""
    _require_device(vals, idx, dY, dW, workspace)
    code = _dtype_code(dY.dtype)
    if vals.dtype != dY.dtype or idx.dtype != torch.int32:
        raise ValueError("vals must have dY's dtype and idx must be int32")
    cs = _conv_struct(conv)
    x_shape = [int(s) for s in x_shape]
    nhwc = _nhwc(layout, x_shape, cs)
    if dW is None:
        if cs is None:
            dw_shape = (int(c_out), x_shape[-1])
        elif nhwc:
            dw_shape = (int(c_out), cs.kh, cs.kw, x_shape[3])
        else:
            dw_shape = (int(c_out), x_shape[1], cs.kh, cs.kw)
        dW = torch.empty(dw_shape, dtype=torch.float32, device=dY.device)
    k = int(vals.numel())
    if workspace is None:
        workspace = torch.empty(max(weight_grad_workspace_bytes(x_shape, dY.dtype, k, c_out, cs, layout), 1),
                                dtype=torch.uint8, device=dY.device)
    pc = ctypes.byref(cs) if cs is not None else None
    with _on(dY.device):
        if nhwc:
            _check(lib().dropit_weight_grad_nhwc(
                vals.data_ptr() if k else None, idx.data_ptr() if k else None, k,
                _shape_array(x_shape), code, dY.data_ptr(), int(c_out), pc, dW.data_ptr(),
                workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
        else:
            _check(lib().dropit_weight_grad(
                vals.data_ptr() if k else None, idx.data_ptr() if k else None, k,
                _shape_array(x_shape), len(x_shape), code, dY.data_ptr(), int(c_out), pc, dW.data_ptr(),
                workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return dW


def compress_rows(x: torch.Tensor, gamma: float, workspace: Optional[torch.Tensor] = None,
                  stream=None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """dropit_compress_rows: (vals[k], col[k] int16 holding the uint16 in-row positions,
    rowptr[rows+1] int32), rows being the last dimension of ``x``."""
    _require_device(x, workspace)
    code = _dtype_code(x.dtype)
    k = keep_count(x.numel(), gamma)
    if k < 0:
        _check(EINVAL)
    rows = x.numel() // x.shape[-1]
    vals = torch.empty(k, dtype=x.dtype, device=x.device)
    col = torch.empty(k, dtype=torch.int16, device=x.device)        # torch has no uint16 arithmetic; bits are uint16
    rowptr = torch.empty(rows + 1, dtype=torch.int32, device=x.device)
    if workspace is None:
        need = int(lib().dropit_compress_rows_workspace_bytes(x.numel(), k, code))
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=x.device)
    with _on(x.device):
        _check(lib().dropit_compress_rows(x.data_ptr(), _shape_array(x.shape), x.dim(), code, float(gamma),
                                          vals.data_ptr() if k else None, col.data_ptr() if k else None,
                                          rowptr.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                          _stream_ptr(stream)))
    return vals, col, rowptr


def weight_grad_rows(vals: torch.Tensor, col: torch.Tensor, rowptr: torch.Tensor, x_shape: Sequence[int],
                     dY: torch.Tensor, c_out: int, conv=None, dW: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """dropit_weight_grad_rows: ``weight_grad`` from the row form of the cache."""
    _require_device(vals, col, rowptr, dY, dW, workspace)
    code = _dtype_code(dY.dtype)
    if vals.dtype != dY.dtype or col.dtype != torch.int16 or rowptr.dtype != torch.int32:
        raise ValueError("vals must have dY's dtype, col int16 (uint16 bits), rowptr int32")
    cs = _conv_struct(conv)
    x_shape = [int(s) for s in x_shape]
    if dW is None:
        dw_shape = (int(c_out), x_shape[-1]) if cs is None else (int(c_out), x_shape[1], cs.kh, cs.kw)
        dW = torch.empty(dw_shape, dtype=torch.float32, device=dY.device)
    k = int(vals.numel())
    shape = _shape_array(x_shape)
    ref = ctypes.byref(cs) if cs is not None else None
    if workspace is None:
        need = int(lib().dropit_weight_grad_rows_workspace_bytes(shape, len(x_shape), code, k, int(c_out), ref))
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=dY.device)
    with _on(dY.device):
        _check(lib().dropit_weight_grad_rows(
            vals.data_ptr() if k else None, col.data_ptr() if k else None, rowptr.data_ptr(), k,
            shape, len(x_shape), code, dY.data_ptr(), int(c_out), ref, dW.data_ptr(),
            workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return dW


MASK_BLOCK = 1024      # DROPIT_MASK_BLOCK: elements per entry of the block-offset table


def compress_mask(x: torch.Tensor, gamma: float, workspace: Optional[torch.Tensor] = None,
                  stream=None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """dropit_compress_mask: (vals[k], mask[ceil(numel/32)] int32 holding the uint32 words,
    blockptr[ceil(numel/1024)+1] int32)."""
    _require_device(x, workspace)
    code = _dtype_code(x.dtype)
    numel = x.numel()
    k = keep_count(numel, gamma)
    if k < 0:
        _check(EINVAL)
    vals = torch.empty(k, dtype=x.dtype, device=x.device)
    mask = torch.empty((numel + 31) // 32, dtype=torch.int32, device=x.device)      # bits are uint32
    blockptr = torch.empty((numel + MASK_BLOCK - 1) // MASK_BLOCK + 1, dtype=torch.int32, device=x.device)
    if workspace is None:
        need = int(lib().dropit_compress_mask_workspace_bytes(numel, k, code))
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=x.device)
    with _on(x.device):
        _check(lib().dropit_compress_mask(x.data_ptr(), _shape_array(x.shape), x.dim(), code, float(gamma),
                                          vals.data_ptr() if k else None, mask.data_ptr(), blockptr.data_ptr(),
                                          workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return vals, mask, blockptr


def weight_grad_mask(vals: torch.Tensor, mask: torch.Tensor, blockptr: torch.Tensor, x_shape: Sequence[int],
                     dY: torch.Tensor, c_out: int, conv=None, dW: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """dropit_weight_grad_mask: ``weight_grad`` from the bit-mask form of the cache."""
    _require_device(vals, mask, blockptr, dY, dW, workspace)
    code = _dtype_code(dY.dtype)
    if vals.dtype != dY.dtype or mask.dtype != torch.int32 or blockptr.dtype != torch.int32:
        raise ValueError("vals must have dY's dtype, mask int32 (uint32 bits), blockptr int32")
    cs = _conv_struct(conv)
    x_shape = [int(s) for s in x_shape]
    if dW is None:
        dw_shape = (int(c_out), x_shape[-1]) if cs is None else (int(c_out), x_shape[1], cs.kh, cs.kw)
        dW = torch.empty(dw_shape, dtype=torch.float32, device=dY.device)
    k = int(vals.numel())
    shape = _shape_array(x_shape)
    ref = ctypes.byref(cs) if cs is not None else None
    if workspace is None:
        need = int(lib().dropit_weight_grad_mask_workspace_bytes(shape, len(x_shape), code, k, int(c_out), ref))
        workspace = torch.empty(max(need, 1), dtype=torch.uint8, device=dY.device)
    with _on(dY.device):
        _check(lib().dropit_weight_grad_mask(
            vals.data_ptr() if k else None, mask.data_ptr(), blockptr.data_ptr(), k,
            shape, len(x_shape), code, dY.data_ptr(), int(c_out), ref, dW.data_ptr(),
            workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)))
    return dW


def set_select_mode(mode: int) -> None:
    """dropit_set_select_mode: 0 = one persistent kernel (default), 1 = separate ordinary
    kernels, 2 = the persistent kernel through a cooperative launch, 3 = test hook that forces
    the persistent kernel's serial redo path."""
    _check(lib().dropit_set_select_mode(int(mode)))


def set_fc_recover(form: int) -> None:
    """dropit_set_fc_recover: 0 = the recover step writes a dense operand into the workspace (default),
    1 = it happens inside the product, in LDS (smaller workspace, same dW, slower)."""
    _check(lib().dropit_set_fc_recover(int(form)))


def trace_events(events: Optional[Sequence[torch.cuda.Event]]) -> None:
    """dropit_trace_events: record the given (already created, timing-enabled) events around
    the kernels of the next compress / weight_grad call from this thread; None switches it off."""
    if not events:
        lib().dropit_trace_events(None, 0)
        return
    handles = (ctypes.c_void_p * len(events))(*[int(e.cuda_event) for e in events])
    trace_events._keepalive = handles          # the library reads this array during the next call
    lib().dropit_trace_events(handles, len(events))
