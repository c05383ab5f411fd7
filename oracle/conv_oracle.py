"""ctypes marshalling for ``conv_oracle.c`` -- TEST INFRASTRUCTURE ONLY.

No arithmetic of the method is done here: arrays are made contiguous fp32 and
handed to the C functions, which follow the paper's Section II definition of
the convolution (window at (oy*stride, ox*stride), element-wise product, sum,
optional ReLU) with zero padding, a per-channel bias and double accumulation.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_f32p = ctypes.POINTER(ctypes.c_float)
_i32p = ctypes.POINTER(ctypes.c_int)


def build(force=False):
    """Compile conv_oracle.c into liboracle.so with gcc (-O2 -fopenmp)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.run(
        ["gcc", "-O2", "-fopenmp", "-std=c11", "-Wall", "-Wextra", "-shared",
         "-fPIC", "-o", tmp, _SRC],
        check=True)
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_conv_out_dims.argtypes = [ctypes.c_int] * 6 + [_i32p, _i32p]
        lib.oracle_conv_out_dims.restype = ctypes.c_int
        lib.oracle_conv_fwd.argtypes = ([_f32p, _f32p, _f32p, _f32p]
                                        + [ctypes.c_int] * 10)
        lib.oracle_conv_fwd.restype = ctypes.c_int
        lib.oracle_conv_fwd_exact.argtypes = ([_f32p, _f32p, _f32p, ctypes.POINTER(ctypes.c_double)]
                                              + [ctypes.c_int] * 10)
        lib.oracle_conv_fwd_exact.restype = ctypes.c_int
        lib.oracle_maxpool_fwd.argtypes = [_f32p, _f32p] + [ctypes.c_int] * 6
        lib.oracle_maxpool_fwd.restype = ctypes.c_int
        lib.oracle_sgemm.argtypes = [_f32p] * 3 + [ctypes.c_int] * 3
        lib.oracle_sgemm.restype = ctypes.c_int
        lib.oracle_num_threads.argtypes = []
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _as_f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a):
    return a.ctypes.data_as(_f32p)


def conv_out_dims(H, W, R, S, stride, pad):
    """(P, Q) of the output; ValueError if no output point exists."""
    P, Q = ctypes.c_int(0), ctypes.c_int(0)
    rc = _load().oracle_conv_out_dims(H, W, R, S, stride, pad,
                                      ctypes.byref(P), ctypes.byref(Q))
    if rc != 0:
        raise ValueError("no valid output for H=%d W=%d R=%d S=%d stride=%d pad=%d"
                         % (H, W, R, S, stride, pad))
    return P.value, Q.value


def conv_fwd(inp, filt, bias=None, stride=1, pad=0, relu=False):
    """out[N,K,P,Q] (fp32) of in[N,C,H,W] with filt[K,C,R,S] (+bias[K]) (+ReLU)."""
    inp, filt = _as_f32(inp), _as_f32(filt)
    if inp.ndim != 4 or filt.ndim != 4 or inp.shape[1] != filt.shape[1]:
        raise ValueError("expected in[N,C,H,W] and filt[K,C,R,S] with equal C")
    N, C, H, W = inp.shape
    K, _, R, S = filt.shape
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    if bias is not None:
        bias = _as_f32(bias)
        if bias.shape != (K,):
            raise ValueError("bias must have shape (K,)")
    out = np.empty((N, K, P, Q), dtype=np.float32)
    rc = _load().oracle_conv_fwd(_ptr(inp), _ptr(filt),
                                 _ptr(bias) if bias is not None else None,
                                 _ptr(out), N, C, H, W, K, R, S, stride, pad,
                                 1 if relu else 0)
    if rc != 0:
        raise ValueError("oracle_conv_fwd rejected its arguments")
    return out


def conv_fwd_f16(inp, filt, bias=None, stride=1, pad=0, relu=False):
    """Half-precision storage: in[N,C,H,W] and filt[K,C,R,S] are fp16, bias fp32; the
    exact result (double accumulation, bias, ReLU) is rounded to fp16 once."""
    inp, filt = np.asarray(inp), np.asarray(filt)
    if inp.dtype != np.float16 or filt.dtype != np.float16:
        raise ValueError("expected fp16 input and filters")
    inp, filt = _as_f32(inp), _as_f32(filt)      # widening is exact
    if inp.ndim != 4 or filt.ndim != 4 or inp.shape[1] != filt.shape[1]:
        raise ValueError("expected in[N,C,H,W] and filt[K,C,R,S] with equal C")
    N, C, H, W = inp.shape
    K, _, R, S = filt.shape
    P, Q = conv_out_dims(H, W, R, S, stride, pad)
    if bias is not None:
        bias = _as_f32(bias)
        if bias.shape != (K,):
            raise ValueError("bias must have shape (K,)")
    out = np.empty((N, K, P, Q), dtype=np.float64)
    rc = _load().oracle_conv_fwd_exact(_ptr(inp), _ptr(filt),
                                       _ptr(bias) if bias is not None else None,
                                       out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                       N, C, H, W, K, R, S, stride, pad, 1 if relu else 0)
    if rc != 0:
        raise ValueError("oracle_conv_fwd_exact rejected its arguments")
    return out.astype(np.float16)    # one rounding, to nearest even


def maxpool_fwd(inp, ksz=3, stride=2):
    """Max over ksz x ksz windows stepped by `stride`, no padding, floor extents."""
    inp = _as_f32(inp)
    N, C, H, W = inp.shape
    if H < ksz or W < ksz:
        raise ValueError("window larger than input")
    P, Q = (H - ksz) // stride + 1, (W - ksz) // stride + 1
    out = np.empty((N, C, P, Q), dtype=np.float32)
    rc = _load().oracle_maxpool_fwd(_ptr(inp), _ptr(out), N, C, H, W, ksz, stride)
    if rc != 0:
        raise ValueError("oracle_maxpool_fwd rejected its arguments")
    return out


def sgemm(a, b):
    """C = A * B by definition (row-major, double accumulation, one rounding)."""
    a, b = _as_f32(a), _as_f32(b)
    M, K = a.shape
    K2, N = b.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    c = np.empty((M, N), dtype=np.float32)
    if _load().oracle_sgemm(_ptr(a), _ptr(b), _ptr(c), M, N, K) != 0:
        raise ValueError("oracle_sgemm rejected its arguments")
    return c


def num_threads():
    """Threads the oracle's OpenMP loops use."""
    return int(_load().oracle_num_threads())
