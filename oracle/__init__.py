"""ctypes front end of the CPU oracle (``conv_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  It never imports the GPU
package and the GPU package never imports it.

The functions mirror the C entry points one to one; all arithmetic is in the C
file (fp64).  Arrays are numpy, C-contiguous; inputs float32 (bf16 workloads
pass bf16-representable float32 values), outputs float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        f32p, f64p, i64p = (ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_double),
                            ctypes.POINTER(ctypes.c_int64))
        i = ctypes.c_int
        lib.oracle_conv2d_fused.restype = i
        lib.oracle_conv2d_fused.argtypes = [f32p] * 6 + [f64p] + [i] * 12
        lib.oracle_conv2d_fused_at.restype = i
        lib.oracle_conv2d_fused_at.argtypes = [f32p] * 6 + [i64p, ctypes.c_int64, f64p] + [i] * 12
        lib.oracle_dwconv2d_fused.restype = i
        lib.oracle_dwconv2d_fused.argtypes = [f32p] * 6 + [f64p] + [i] * 11
        lib.oracle_maxpool2d.restype = i
        lib.oracle_maxpool2d.argtypes = [f32p, f64p] + [i] * 7
        lib.oracle_round_to_bf16.restype = None
        lib.oracle_round_to_bf16.argtypes = [f64p, f32p, ctypes.c_int64]
        lib.oracle_num_threads.restype = i
        lib.oracle_set_num_threads.argtypes = [i]
        _lib = lib
    return _lib


def _f32(a, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _ptr(a: Optional[np.ndarray], ctype):
    if a is None:
        return ctypes.cast(None, ctypes.POINTER(ctype))
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def out_extent(size: int, pad: int, k: int, stride: int) -> int:
    span = size + 2 * pad - k
    return span // stride + 1 if span >= 0 else 0


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def conv2d_fused(x, w, scale, shift, bias=None, residual=None, *, stride=(1, 1), pad=(0, 0),
                 relu=False) -> np.ndarray:
    """Dense fused conv2d (Table 2 operator + Section 3 fused element-wise tail), fp64."""
    lib = _load()
    x = _f32(x)
    w = _f32(w)
    N, IC, H, W = x.shape
    OC, IC2, R, S = w.shape
    if IC2 != IC:
        raise ValueError("weight input channels do not match x")
    OH, OW = out_extent(H, pad[0], R, stride[0]), out_extent(W, pad[1], S, stride[1])
    if OH < 1 or OW < 1:
        raise ValueError("empty output")
    scale, shift = _f32(scale, (OC,)), _f32(shift, (OC,))
    bias = None if bias is None else _f32(bias, (OC,))
    residual = None if residual is None else _f32(residual, (N, OC, OH, OW))
    y = np.empty((N, OC, OH, OW), dtype=np.float64)
    rc = lib.oracle_conv2d_fused(_ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float),
                                 _ptr(scale, ctypes.c_float), _ptr(shift, ctypes.c_float),
                                 _ptr(bias, ctypes.c_float), _ptr(residual, ctypes.c_float),
                                 _ptr(y, ctypes.c_double), N, IC, H, W, OC, R, S,
                                 stride[0], stride[1], pad[0], pad[1], int(bool(relu)))
    if rc != 0:
        raise RuntimeError(f"oracle_conv2d_fused failed ({rc})")
    return y


def conv2d_fused_at(x, w, scale, shift, bias=None, residual=None, *, idx, stride=(1, 1),
                    pad=(0, 0), relu=False) -> np.ndarray:
    """The same operator at the flat NCHW output indices ``idx`` only."""
    lib = _load()
    x = _f32(x)
    w = _f32(w)
    N, IC, H, W = x.shape
    OC, IC2, R, S = w.shape
    if IC2 != IC:
        raise ValueError("weight input channels do not match x")
    OH, OW = out_extent(H, pad[0], R, stride[0]), out_extent(W, pad[1], S, stride[1])
    scale, shift = _f32(scale, (OC,)), _f32(shift, (OC,))
    bias = None if bias is None else _f32(bias, (OC,))
    residual = None if residual is None else _f32(residual, (N, OC, OH, OW))
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float64)
    rc = lib.oracle_conv2d_fused_at(_ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float),
                                    _ptr(scale, ctypes.c_float), _ptr(shift, ctypes.c_float),
                                    _ptr(bias, ctypes.c_float), _ptr(residual, ctypes.c_float),
                                    _ptr(idx, ctypes.c_int64), idx.size, _ptr(out, ctypes.c_double),
                                    N, IC, H, W, OC, R, S,
                                    stride[0], stride[1], pad[0], pad[1], int(bool(relu)))
    if rc != 0:
        raise RuntimeError(f"oracle_conv2d_fused_at failed ({rc})")
    return out


def dwconv2d_fused(x, w, scale, shift, bias=None, residual=None, *, stride=(1, 1), pad=(1, 1),
                   relu=False) -> np.ndarray:
    """Depthwise fused conv2d, channel multiplier 1 (Table 2, D rows), fp64."""
    lib = _load()
    x = _f32(x)
    w = _f32(w)
    N, C, H, W = x.shape
    C2, one, R, S = w.shape
    if C2 != C or one != 1:
        raise ValueError("depthwise weights must be [C][1][R][S]")
    OH, OW = out_extent(H, pad[0], R, stride[0]), out_extent(W, pad[1], S, stride[1])
    if OH < 1 or OW < 1:
        raise ValueError("empty output")
    scale, shift = _f32(scale, (C,)), _f32(shift, (C,))
    bias = None if bias is None else _f32(bias, (C,))
    residual = None if residual is None else _f32(residual, (N, C, OH, OW))
    y = np.empty((N, C, OH, OW), dtype=np.float64)
    rc = lib.oracle_dwconv2d_fused(_ptr(x, ctypes.c_float), _ptr(w, ctypes.c_float),
                                   _ptr(scale, ctypes.c_float), _ptr(shift, ctypes.c_float),
                                   _ptr(bias, ctypes.c_float), _ptr(residual, ctypes.c_float),
                                   _ptr(y, ctypes.c_double), N, C, H, W, R, S,
                                   stride[0], stride[1], pad[0], pad[1], int(bool(relu)))
    if rc != 0:
        raise RuntimeError(f"oracle_dwconv2d_fused failed ({rc})")
    return y


def dwpw_fused(x, w_dw, scale_dw, shift_dw, w_pw, scale_pw, shift_pw, bias_pw=None,
               residual=None, *, stride=1, relu_dw=True, relu_pw=True, store="bf16") -> np.ndarray:
    """Depthwise 3x3 (pad 1) + tail, then 1x1 conv + tail: the MobileNet block that the fused
    GPU operator evaluates in one launch (Section 3, operator fusion; Table 2 rows D).

    This is the definition, two oracle calls: the depthwise result is rounded to the storage
    type between them (``store`` = "bf16": nearest bfloat16; "f32": nearest float32), because
    the operator's second stage reads values of that type.  fp64 output.
    """
    t = dwconv2d_fused(x, w_dw, scale_dw, shift_dw, None, None, stride=(stride, stride),
                       pad=(1, 1), relu=relu_dw)
    if store == "bf16":
        t = round_to_bf16(t)
    elif store == "f32":
        t = t.astype(np.float32)
    else:
        raise ValueError(store)
    return conv2d_fused(t, w_pw, scale_pw, shift_pw, bias_pw, residual, stride=(1, 1), pad=(0, 0),
                        relu=relu_pw)


def maxpool2d(x, *, k=3, stride=2, pad=1) -> np.ndarray:
    """Max-pool with padded taps ignored, fp64 output."""
    lib = _load()
    x = _f32(x)
    N, C, H, W = x.shape
    OH, OW = out_extent(H, pad, k, stride), out_extent(W, pad, k, stride)
    if OH < 1 or OW < 1:
        raise ValueError("empty output")
    y = np.empty((N, C, OH, OW), dtype=np.float64)
    rc = lib.oracle_maxpool2d(_ptr(x, ctypes.c_float), _ptr(y, ctypes.c_double),
                              N, C, H, W, k, stride, pad)
    if rc != 0:
        raise RuntimeError(f"oracle_maxpool2d failed ({rc})")
    return y


def round_to_bf16(y64) -> np.ndarray:
    """fp64 -> nearest bfloat16 (ties to even), returned as float32 values."""
    lib = _load()
    y64 = np.ascontiguousarray(y64, dtype=np.float64)
    out = np.empty(y64.shape, dtype=np.float32)
    lib.oracle_round_to_bf16(_ptr(y64, ctypes.c_double), _ptr(out, ctypes.c_float), y64.size)
    return out
