"""numpy front end of the C operator oracle (``tt_oracle.c``).

TEST INFRASTRUCTURE ONLY: the product package never imports this module.  It
compiles the C file with gcc on first use (or through ``build()``), loads it
with ctypes and marshals numpy float32 arrays.  Every function computes the
plain definition of one kernel class of the paper (Algorithm 2 for
conv+bias+ReLU, Table 1 for the other ResNet18 classes, Algorithm 1's
unscheduled loop nest for GEMM); see the header of ``tt_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tt_oracle.c")
_LIB = os.path.join(_HERE, "libtt_oracle.so")

ACT_NONE, ACT_RELU, ACT_RELU6, ACT_GELU = 0, 1, 2, 3

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc -O2, OpenMP over the outermost output axis)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        i = ctypes.c_int
        lib.tt_oracle_conv2d.argtypes = [fp, fp, fp, fp, fp] + [i] * 13
        lib.tt_oracle_conv2d.restype = None
        lib.tt_oracle_conv2d_points.argtypes = [fp, fp, fp, fp, ctypes.POINTER(ctypes.c_int), fp, ctypes.c_longlong] + \
            [i] * 12
        lib.tt_oracle_conv2d_points.restype = None
        lib.tt_oracle_dense.argtypes = [fp, fp, fp, fp] + [i] * 5
        lib.tt_oracle_dense.restype = None
        lib.tt_oracle_batch_matmul.argtypes = [fp, fp, fp] + [i] * 6
        lib.tt_oracle_batch_matmul.restype = None
        lib.tt_oracle_dwconv.argtypes = [fp, fp, fp, fp] + [i] * 12
        lib.tt_oracle_dwconv.restype = None
        lib.tt_oracle_conv_out_extent.argtypes = [i] * 4
        lib.tt_oracle_conv_out_extent.restype = i
        lib.tt_oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        lib.tt_oracle_f32_to_bf16.restype = ctypes.c_uint16
        lib.tt_oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        lib.tt_oracle_bf16_to_f32.restype = ctypes.c_float
        lib.tt_oracle_round_to_bf16.argtypes = [fp, fp, ctypes.c_size_t]
        lib.tt_oracle_round_to_bf16.restype = None
        _lib = lib
    return _lib


def _f32(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _ptr(a):
    if a is None:
        return ctypes.cast(None, ctypes.POINTER(ctypes.c_float))
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def set_threads(n: int) -> None:
    """OpenMP thread count for subsequent calls (through the OMP runtime the oracle links)."""
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(n))


def max_threads() -> int:
    omp = ctypes.CDLL("libgomp.so.1")
    return int(omp.omp_get_max_threads())


def conv_out_extent(size: int, filt: int, stride: int, pad: int) -> int:
    return int(_load().tt_oracle_conv_out_extent(size, filt, stride, pad))


def conv2d(x, w, bias=None, res=None, stride=(1, 1), pad=(0, 0), act=ACT_NONE, acc64=True):
    """Conv2d (+bias) (+residual) (+activation), NCHW / KCRS; paper Algorithm 2 and Table 1."""
    lib = _load()
    x = _f32(x)
    w = _f32(w)
    n, c, h, wd = x.shape
    k, c2, r, s = w.shape
    if c2 != c:
        raise ValueError("channel mismatch")
    ho = conv_out_extent(h, r, stride[0], pad[0])
    wo = conv_out_extent(wd, s, stride[1], pad[1])
    bias = None if bias is None else _f32(bias, (k,))
    res = None if res is None else _f32(res, (n, k, ho, wo))
    y = np.empty((n, k, ho, wo), dtype=np.float32)
    lib.tt_oracle_conv2d(_ptr(x), _ptr(w), _ptr(bias), _ptr(res), _ptr(y), n, c, h, wd, k, r, s,
                         stride[0], stride[1], pad[0], pad[1], act, int(acc64))
    return y


def conv2d_points(x, w, coords, bias=None, res=None, stride=(1, 1), pad=(0, 0), act=ACT_NONE):
    """conv2d (+bias) (+residual) (+activation) at the output coordinates coords[:, (n, k, p, q)] only."""
    lib = _load()
    x = _f32(x)
    w = _f32(w)
    n, c, h, wd = x.shape
    k, c2, r, s = w.shape
    if c2 != c:
        raise ValueError("channel mismatch")
    coords = np.ascontiguousarray(coords, dtype=np.int32)
    if coords.ndim != 2 or coords.shape[1] != 4:
        raise ValueError("coords must be [npts, 4]")
    ho = conv_out_extent(h, r, stride[0], pad[0])
    wo = conv_out_extent(wd, s, stride[1], pad[1])
    if coords.size and (coords.min() < 0 or (coords.max(axis=0) >= np.array([n, k, ho, wo])).any()):
        raise ValueError("coordinate out of range")
    bias = None if bias is None else _f32(bias, (k,))
    res = None if res is None else _f32(res, (n, k, ho, wo))
    out = np.empty(coords.shape[0], dtype=np.float32)
    lib.tt_oracle_conv2d_points(_ptr(x), _ptr(w), _ptr(bias), _ptr(res),
                                coords.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), _ptr(out), coords.shape[0], n, c,
                                h, wd, k, r, s, stride[0], stride[1], pad[0], pad[1], act)
    return out


def dense(x, w, bias=None, act=ACT_NONE, acc64=True):
    """y = act(x @ w.T + bias); w is [out, in] (paper Table 1, dense_add)."""
    lib = _load()
    x = _f32(x)
    w = _f32(w)
    m, i = x.shape
    o, i2 = w.shape
    if i2 != i:
        raise ValueError("inner dimension mismatch")
    bias = None if bias is None else _f32(bias, (o,))
    y = np.empty((m, o), dtype=np.float32)
    lib.tt_oracle_dense(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), m, o, i, act, int(acc64))
    return y


def batch_matmul(a, b, trans_b=False, acc64=True):
    """c[b] = a[b] @ b[b] (b stored [B,K,N]) or a[b] @ b[b].T (b stored [B,N,K], trans_b)."""
    lib = _load()
    a = _f32(a)
    b = _f32(b)
    bt, m, k = a.shape
    if trans_b:
        bt2, n, k2 = b.shape
    else:
        bt2, k2, n = b.shape
    if bt2 != bt or k2 != k:
        raise ValueError("operand mismatch")
    c = np.empty((bt, m, n), dtype=np.float32)
    lib.tt_oracle_batch_matmul(_ptr(a), _ptr(b), _ptr(c), bt, m, n, k, int(bool(trans_b)), int(acc64))
    return c


def dwconv(x, w, bias=None, stride=(1, 1), pad=(1, 1), act=ACT_RELU6, acc64=True):
    """Depthwise conv (+bias) (+activation); w is [C,1,R,S]."""
    lib = _load()
    x = _f32(x)
    w = _f32(w)
    n, c, h, wd = x.shape
    c2, one, r, s = w.shape
    if c2 != c or one != 1:
        raise ValueError("depthwise weights must be [C,1,R,S]")
    ho = conv_out_extent(h, r, stride[0], pad[0])
    wo = conv_out_extent(wd, s, stride[1], pad[1])
    bias = None if bias is None else _f32(bias, (c,))
    y = np.empty((n, c, ho, wo), dtype=np.float32)
    lib.tt_oracle_dwconv(_ptr(x), _ptr(w), _ptr(bias), _ptr(y), n, c, h, wd, r, s, stride[0], stride[1],
                         pad[0], pad[1], act, int(acc64))
    return y


def f32_to_bf16_bits(v: float) -> int:
    return int(_load().tt_oracle_f32_to_bf16(ctypes.c_float(v)))


def bf16_bits_to_f32(h: int) -> float:
    return float(_load().tt_oracle_bf16_to_f32(ctypes.c_uint16(h)))


def round_to_bf16(a):
    """Round float32 values to the nearest bf16 (ties to even), returned as float32."""
    lib = _load()
    a = _f32(a)
    out = np.empty_like(a)
    lib.tt_oracle_round_to_bf16(_ptr(a), _ptr(out), a.size)
    return out
