"""Python face of the direct-loop conv / inner-product oracle (test infrastructure only).

The arithmetic lives in `csrc/twn_oracle.c` (plain C, double accumulation, one
loop nest per output element; Eq. 2 and Alg. 1 steps 8-10).  This module builds
that file with gcc on first use and marshals numpy arrays to it.  Activations
are NHWC float32 arrays (bf16-valued inputs widened exactly), codes are int8
[O][C][R][S], alpha is one scalar or one value per filter, results are float64.
"""

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csrc", "twn_oracle.c")
_SO = os.path.join(_HERE, "libtwn_oracle.so")
_lib = None


def build(force=False):
    """Compile the C oracle (gcc -O2 -fopenmp, no intrinsics, no BLAS)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _SO, _SRC])
    return _SO


class _Conv(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("N", "H", "W", "C", "O", "R", "S", "sh", "sw", "ph", "pw", "dh", "dw", "P", "Q")]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_SO)
        _lib.twn_oracle_max_threads.restype = ctypes.c_int
    return _lib


def max_threads():
    return int(_load().twn_oracle_max_threads())


def out_size(h, r, stride, pad, dil):
    return (h + 2 * pad - dil * (r - 1) - 1) // stride + 1


def geometry(x_shape, w_shape, stride=(1, 1), pad=(0, 0), dil=(1, 1)):
    n, h, w, c = x_shape
    o, c2, r, s = w_shape
    if c != c2:
        raise ValueError("channel mismatch")
    g = _Conv(n, h, w, c, o, r, s, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1],
              out_size(h, r, stride[0], pad[0], dil[0]), out_size(w, s, stride[1], pad[1], dil[1]))
    if g.P <= 0 or g.Q <= 0:
        raise ValueError("empty output")
    return g


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i8(a):
    return np.ascontiguousarray(a, dtype=np.int8)


def _alpha_vec(alpha, o):
    a = np.asarray(alpha, dtype=np.float64).ravel()
    if a.size == 1:
        return np.full(o, float(a[0]), dtype=np.float64)
    if o % a.size != 0:
        raise ValueError("alpha groups must divide the number of filters")
    return np.ascontiguousarray(np.repeat(a, o // a.size))


def _p(a, t):
    return a.ctypes.data_as(ctypes.POINTER(t)) if a is not None else None


def conv2d_fwd(x, codes, alpha, stride=(1, 1), pad=(0, 0), dil=(1, 1), bias=None, addsub=False):
    x, codes = _f32(x), _i8(codes)
    g = geometry(x.shape, codes.shape, stride, pad, dil)
    av = _alpha_vec(alpha, g.O)
    y = np.empty((g.N, g.P, g.Q, g.O), dtype=np.float64)
    lib = _load()
    if addsub:
        lib.twn_oracle_conv2d_fwd_addsub(ctypes.byref(g), _p(x, ctypes.c_float), _p(codes, ctypes.c_int8),
                                         _p(av, ctypes.c_double), _p(y, ctypes.c_double))
        if bias is not None:
            y += np.asarray(bias, dtype=np.float64)
    else:
        b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
        lib.twn_oracle_conv2d_fwd(ctypes.byref(g), _p(x, ctypes.c_float), _p(codes, ctypes.c_int8),
                                  _p(av, ctypes.c_double), _p(b, ctypes.c_double), _p(y, ctypes.c_double))
    return y


def conv2d_fwd_at(x, codes, alpha, flat_idx, stride=(1, 1), pad=(0, 0), dil=(1, 1), bias=None):
    x, codes = _f32(x), _i8(codes)
    g = geometry(x.shape, codes.shape, stride, pad, dil)
    av = _alpha_vec(alpha, g.O)
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
    out = np.empty(idx.size, dtype=np.float64)
    _load().twn_oracle_conv2d_fwd_at(ctypes.byref(g), _p(x, ctypes.c_float), _p(codes, ctypes.c_int8),
                                     _p(av, ctypes.c_double), _p(b, ctypes.c_double),
                                     _p(idx, ctypes.c_int64), ctypes.c_int64(idx.size),
                                     _p(out, ctypes.c_double))
    return out


def conv2d_bwd_data(dy, codes, alpha, x_shape, stride=(1, 1), pad=(0, 0), dil=(1, 1)):
    dy, codes = _f32(dy), _i8(codes)
    g = geometry(x_shape, codes.shape, stride, pad, dil)
    if dy.shape != (g.N, g.P, g.Q, g.O):
        raise ValueError("dY shape mismatch")
    av = _alpha_vec(alpha, g.O)
    dx = np.empty(tuple(x_shape), dtype=np.float64)
    _load().twn_oracle_conv2d_bwd_data(ctypes.byref(g), _p(dy, ctypes.c_float), _p(codes, ctypes.c_int8),
                                       _p(av, ctypes.c_double), _p(dx, ctypes.c_double))
    return dx


def conv2d_bwd_data_at(dy, codes, alpha, x_shape, flat_idx, stride=(1, 1), pad=(0, 0), dil=(1, 1)):
    dy, codes = _f32(dy), _i8(codes)
    g = geometry(x_shape, codes.shape, stride, pad, dil)
    if dy.shape != (g.N, g.P, g.Q, g.O):
        raise ValueError("dY shape mismatch")
    av = _alpha_vec(alpha, g.O)
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    out = np.empty(idx.size, dtype=np.float64)
    _load().twn_oracle_conv2d_bwd_data_at(ctypes.byref(g), _p(dy, ctypes.c_float), _p(codes, ctypes.c_int8),
                                          _p(av, ctypes.c_double), _p(idx, ctypes.c_int64),
                                          ctypes.c_int64(idx.size), _p(out, ctypes.c_double))
    return out


def conv2d_bwd_weight(x, dy, w_shape, stride=(1, 1), pad=(0, 0), dil=(1, 1)):
    x, dy = _f32(x), _f32(dy)
    g = geometry(x.shape, w_shape, stride, pad, dil)
    if dy.shape != (g.N, g.P, g.Q, g.O):
        raise ValueError("dY shape mismatch")
    dw = np.empty(tuple(w_shape), dtype=np.float64)
    _load().twn_oracle_conv2d_bwd_weight(ctypes.byref(g), _p(x, ctypes.c_float), _p(dy, ctypes.c_float),
                                         _p(dw, ctypes.c_double))
    return dw


def conv2d_bwd_weight_at(x, dy, w_shape, flat_idx, stride=(1, 1), pad=(0, 0), dil=(1, 1)):
    x, dy = _f32(x), _f32(dy)
    g = geometry(x.shape, w_shape, stride, pad, dil)
    if dy.shape != (g.N, g.P, g.Q, g.O):
        raise ValueError("dY shape mismatch")
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    out = np.empty(idx.size, dtype=np.float64)
    _load().twn_oracle_conv2d_bwd_weight_at(ctypes.byref(g), _p(x, ctypes.c_float), _p(dy, ctypes.c_float),
                                            _p(idx, ctypes.c_int64), ctypes.c_int64(idx.size),
                                            _p(out, ctypes.c_double))
    return out


def bias_grad(dy):
    """db[o] = sum over n,p,q of dY[n,p,q,o]."""
    d = np.asarray(dy, dtype=np.float64)
    return d.reshape(-1, d.shape[-1]).sum(axis=0)


def gemm_fwd(x, codes, alpha, bias=None):
    x, codes = _f32(x), _i8(codes)
    m, k = x.shape
    n, k2 = codes.shape
    if k != k2:
        raise ValueError("K mismatch")
    av = _alpha_vec(alpha, n)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
    y = np.empty((m, n), dtype=np.float64)
    _load().twn_oracle_gemm_fwd(_p(x, ctypes.c_float), _p(codes, ctypes.c_int8), _p(av, ctypes.c_double),
                                _p(b, ctypes.c_double), ctypes.c_int64(m), ctypes.c_int64(n),
                                ctypes.c_int64(k), _p(y, ctypes.c_double))
    return y


def gemm_fwd_at(x, codes, alpha, flat_idx, bias=None):
    x, codes = _f32(x), _i8(codes)
    m, k = x.shape
    n, k2 = codes.shape
    if k != k2:
        raise ValueError("K mismatch")
    av = _alpha_vec(alpha, n)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float64)
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    out = np.empty(idx.size, dtype=np.float64)
    _load().twn_oracle_gemm_fwd_at(_p(x, ctypes.c_float), _p(codes, ctypes.c_int8), _p(av, ctypes.c_double),
                                   _p(b, ctypes.c_double), ctypes.c_int64(m), ctypes.c_int64(n),
                                   ctypes.c_int64(k), _p(idx, ctypes.c_int64), ctypes.c_int64(idx.size),
                                   _p(out, ctypes.c_double))
    return out


def epilogue(z, scale=None, shift=None, residual=None, relu=False):
    """Per-channel affine, residual add and ReLU applied to a block output:
    X_next = g(Z) of Eq. 2 with g = ReLU, preceded by the folded batch-norm
    affine of the ternary block (Sec. 2.4)."""
    y = np.asarray(z, dtype=np.float64).copy()
    if scale is not None:
        y *= np.asarray(scale, dtype=np.float64)
    if shift is not None:
        y += np.asarray(shift, dtype=np.float64)
    if residual is not None:
        y += np.asarray(residual, dtype=np.float64)
    if relu:
        y = np.maximum(y, 0.0)
    return y
