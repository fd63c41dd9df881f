"""CPU oracle for the DropIT hot path -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes front end over ``dropit_oracle.c`` (plain C, gcc, fp64).
Nothing in the product package may import this module; it is for the tests,
the smoke check and the benchmark's cpu_baseline leg.  It shares no code with
the HIP path and never imports it.

Array conventions: fp32 tensors are ``np.float32`` arrays; bf16 tensors are
``np.uint16`` arrays holding the raw bit patterns.  Indices are ``np.int32``.

Paper passages each function follows are cited in ``dropit_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dropit_oracle.c")
_LIB = os.path.join(_HERE, "libdropit_oracle.so")

F32, BF16 = 0, 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, dbl, vp, i32 = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        lib.oracle_keep_count.restype = i64
        lib.oracle_keep_count.argtypes = [i64, dbl]
        lib.oracle_compress.restype = i32
        lib.oracle_compress.argtypes = [vp, i64, i32, i64, vp, vp]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        lib.oracle_random_key.restype = ctypes.c_uint32
        lib.oracle_random_key.argtypes = [i64, ctypes.c_uint64]
        lib.oracle_compress_random.restype = i32
        lib.oracle_compress_random.argtypes = [vp, i64, i32, i64, ctypes.c_uint64, vp, vp]
        lib.oracle_rows_from_pairs.restype = i32
        lib.oracle_rows_from_pairs.argtypes = [vp, i64, i64, i64, vp, vp]
        lib.oracle_pairs_from_rows.restype = i32
        lib.oracle_pairs_from_rows.argtypes = [vp, vp, i64, i64, vp]
        lib.oracle_mask_from_pairs.restype = i32
        lib.oracle_mask_from_pairs.argtypes = [vp, i64, i64, i64, vp, vp]
        lib.oracle_pairs_from_mask.restype = i64
        lib.oracle_pairs_from_mask.argtypes = [vp, vp, i64, i64, vp]
        lib.oracle_widen.restype = None
        lib.oracle_widen.argtypes = [vp, i64, i32, vp]
        lib.oracle_densify.restype = i32
        lib.oracle_densify.argtypes = [vp, vp, i64, i32, i64, vp]
        lib.oracle_dw_fc.restype = None
        lib.oracle_dw_fc.argtypes = [vp, vp, i64, i64, i64, i64, i64, vp]
        lib.oracle_dw_conv.restype = None
        lib.oracle_dw_conv.argtypes = [vp, vp] + [i64] * 17 + [vp]
        lib.oracle_num_threads.restype = i32
        lib.oracle_num_threads.argtypes = []
        _lib = lib
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle takes float32 arrays or uint16 (bf16 bit pattern) arrays, got %s" % a.dtype)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def keep_count(numel: int, gamma: float) -> int:
    """k = floor((1-gamma)*numel)  [Sec. 4.1 / Sec. 3.3 Min-K]."""
    return int(_load().oracle_keep_count(int(numel), float(gamma)))


def compress(x: np.ndarray, k: int):
    """D(a) = {a_Xr, Xr} by full sort  [Sec. 3.2, Sec. 3.3 Min-K, Sec. 4.1].

    Returns (vals, idx): vals has x's dtype (exact bit copies), idx int32
    ascending flat indices.
    """
    x = np.ascontiguousarray(x).reshape(-1)
    code = _dtype_code(x)
    vals = np.empty(k, dtype=x.dtype)
    idx = np.empty(k, dtype=np.int32)
    rc = _load().oracle_compress(_ptr(x), x.size, code, int(k), _ptr(vals), _ptr(idx))
    if rc != 0:
        raise ValueError("oracle_compress rejected its arguments")
    return vals, idx


def philox4x32_10(ctr, key):
    """One block of Philox4x32-10 (Salmon et al., SC'11): 4 counter words, 2 key words -> 4 words."""
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def random_key(i: int, seed: int) -> int:
    """31-bit selection key of flat index i under `seed`  [Sec. 3.3 Random Elements; reading in the C header]."""
    return int(_load().oracle_random_key(int(i), int(seed)))


def compress_random(x: np.ndarray, k: int, seed: int):
    """D(a) with a uniformly random retained set of k elements  [Sec. 3.3 Random Elements]."""
    x = np.ascontiguousarray(x).reshape(-1)
    code = _dtype_code(x)
    vals = np.empty(k, dtype=x.dtype)
    idx = np.empty(k, dtype=np.int32)
    rc = _load().oracle_compress_random(_ptr(x), x.size, code, int(k), int(seed), _ptr(vals), _ptr(idx))
    if rc != 0:
        raise ValueError("oracle_compress_random rejected its arguments")
    return vals, idx


def rows_from_pairs(idx: np.ndarray, shape):
    """Row form of a retained index set: (col uint16 [k], rowptr int32 [rows+1]); rows are the last
    dimension of `shape`  [Sec. 4.3, index memory]."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    row_len = int(shape[-1])
    rows = int(np.prod(shape[:-1], dtype=np.int64)) if len(shape) > 1 else 1
    col = np.empty(idx.size, dtype=np.uint16)
    rowptr = np.empty(rows + 1, dtype=np.int32)
    if _load().oracle_rows_from_pairs(_ptr(idx), idx.size, rows, row_len, _ptr(col), _ptr(rowptr)) != 0:
        raise ValueError("oracle_rows_from_pairs rejected its arguments")
    return col, rowptr


def pairs_from_rows(col: np.ndarray, rowptr: np.ndarray, shape) -> np.ndarray:
    """Inverse of rows_from_pairs: the int32 flat indices."""
    col = np.ascontiguousarray(col, dtype=np.uint16)
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    idx = np.empty(col.size, dtype=np.int32)
    if _load().oracle_pairs_from_rows(_ptr(col), _ptr(rowptr), rowptr.size - 1, int(shape[-1]), _ptr(idx)) != 0:
        raise ValueError("oracle_pairs_from_rows rejected its arguments")
    return idx


MASK_BLOCK = 1024      # elements per entry of the block-offset table of the bit-mask form


def mask_from_pairs(idx: np.ndarray, numel: int, block: int = MASK_BLOCK):
    """Bit-mask form of a retained index set: (mask uint32 [ceil(numel/32)], blockptr int32
    [ceil(numel/block)+1])  [Sec. 4.3, index memory]."""
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    mask = np.empty((numel + 31) // 32, dtype=np.uint32)
    blockptr = np.empty((numel + block - 1) // block + 1, dtype=np.int32)
    if _load().oracle_mask_from_pairs(_ptr(idx), idx.size, int(numel), int(block), _ptr(mask), _ptr(blockptr)) != 0:
        raise ValueError("oracle_mask_from_pairs rejected its arguments")
    return mask, blockptr


def pairs_from_mask(mask: np.ndarray, blockptr: np.ndarray, numel: int, block: int = MASK_BLOCK) -> np.ndarray:
    """Inverse of mask_from_pairs: the ascending int32 flat indices."""
    mask = np.ascontiguousarray(mask, dtype=np.uint32)
    blockptr = np.ascontiguousarray(blockptr, dtype=np.int32)
    idx = np.empty(int(numel), dtype=np.int32)
    n = _load().oracle_pairs_from_mask(_ptr(mask), _ptr(blockptr), int(numel), int(block), _ptr(idx))
    if n < 0:
        raise ValueError("oracle_pairs_from_mask: the block offsets do not match the mask")
    return idx[:n].copy()


def widen(a: np.ndarray) -> np.ndarray:
    """Exact fp32/bf16 -> fp64 widening, same shape."""
    a = np.ascontiguousarray(a)
    out = np.empty(a.shape, dtype=np.float64)
    _load().oracle_widen(_ptr(a), a.size, _dtype_code(a), _ptr(out))
    return out


def densify(vals: np.ndarray, idx: np.ndarray, shape) -> np.ndarray:
    """R(a^): fp64 dense tensor of ``shape`` with zeros at dropped positions  [Sec. 3.2]."""
    vals = np.ascontiguousarray(vals)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    numel = int(np.prod(shape, dtype=np.int64))
    out = np.empty(numel, dtype=np.float64)
    rc = _load().oracle_densify(_ptr(vals), _ptr(idx), vals.size, _dtype_code(vals), numel, _ptr(out))
    if rc != 0:
        raise ValueError("oracle_densify: index out of range")
    return out.reshape(shape)


def dw_fc(xhat: np.ndarray, dY: np.ndarray, j0: int = 0, j1: int | None = None) -> np.ndarray:
    """dW[j][c] = sum_n dY[n][j] * xhat[n][c], fp64  [Sec. 3.2, Eq. fc_backward_elem_save].

    xhat: fp64 [..., cin] (leading dims are tokens); dY: fp64 [..., cout].
    Returns the rows j0:j1 of dW, shape [j1-j0, cin].
    """
    cin = xhat.shape[-1]
    cout = dY.shape[-1]
    xh = np.ascontiguousarray(xhat, dtype=np.float64).reshape(-1, cin)
    dy = np.ascontiguousarray(dY, dtype=np.float64).reshape(-1, cout)
    if xh.shape[0] != dy.shape[0]:
        raise ValueError("token counts differ")
    j1 = cout if j1 is None else j1
    dW = np.zeros((cout, cin), dtype=np.float64)
    _load().oracle_dw_fc(_ptr(xh), _ptr(dy), xh.shape[0], cin, cout, int(j0), int(j1), _ptr(dW))
    return dW[j0:j1].copy()


def dw_conv(xhat: np.ndarray, dY: np.ndarray, kh: int, kw: int, stride=(1, 1), pad=(0, 0),
            dil=(1, 1), j0: int = 0, j1: int | None = None) -> np.ndarray:
    """Conv weight gradient, fp64 direct loops  [Sec. 3.2, Eq. conv_backward_elem].

    xhat: fp64 NCHW [N,C,H,W]; dY: fp64 [N,cout,OH,OW].  Returns dW[j0:j1] of
    shape [j1-j0, C, kh, kw].
    """
    xh = np.ascontiguousarray(xhat, dtype=np.float64)
    dy = np.ascontiguousarray(dY, dtype=np.float64)
    N, C, H, W = xh.shape
    N2, cout, OH, OW = dy.shape
    if N != N2:
        raise ValueError("batch sizes differ")
    j1 = cout if j1 is None else j1
    dW = np.zeros((cout, C, kh, kw), dtype=np.float64)
    _load().oracle_dw_conv(_ptr(xh), _ptr(dy), N, C, H, W, cout, OH, OW, kh, kw,
                           stride[0], stride[1], pad[0], pad[1], dil[0], dil[1],
                           int(j0), int(j1), _ptr(dW))
    return dW[j0:j1].copy()
