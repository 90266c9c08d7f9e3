"""ctypes loader for conv2d_oracle.c (the plain CPU convolution).

TEST INFRASTRUCTURE ONLY: the arithmetic lives in conv2d_oracle.c; this file
marshals numpy arrays into it.  `build()` compiles the C file with gcc.
"""
import ctypes
import os
import subprocess

import numpy as np

PAD_VALID = 0
PAD_SAME = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "conv2d_oracle.c")
_LIB = os.path.join(_HERE, "libconv2d_oracle.so")
_lib = None


class _Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "in_rows", "in_cols", "channels", "features",
        "window_rows", "window_cols", "stride_rows", "stride_cols", "padding")]


class _Geometry(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "out_rows", "out_cols", "pad_top", "pad_bottom", "pad_left", "pad_right")]


def build(force=False):
    """Compile the oracle with gcc (-O3 -march=native -fopenmp)."""
    global _lib
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    tmp = _LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["gcc", "-O3", "-march=native", "-fopenmp", "-fPIC", "-shared",
                           "-std=c11", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
    os.replace(tmp, _LIB)
    _lib = None
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        pp, gp = ctypes.POINTER(_Params), ctypes.POINTER(_Geometry)
        lib.conv2d_oracle_get_geometry.argtypes = [pp, gp]
        lib.conv2d_oracle_forward_f32.argtypes = [pp, ctypes.c_void_p, ctypes.c_void_p,
                                                  ctypes.c_void_p, ctypes.c_int]
        lib.conv2d_oracle_forward_f64.argtypes = lib.conv2d_oracle_forward_f32.argtypes
        lib.conv2d_oracle_points_f32.argtypes = [pp, ctypes.c_void_p, ctypes.c_void_p,
                                                 ctypes.c_void_p, ctypes.c_int64,
                                                 ctypes.c_void_p, ctypes.c_int]
        lib.conv2d_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _params(batch, in_rows, in_cols, channels, features, window_rows, window_cols,
            stride_rows, stride_cols, padding):
    return _Params(batch, in_rows, in_cols, channels, features, window_rows, window_cols,
                   stride_rows, stride_cols, padding)


def max_threads():
    return int(_load().conv2d_oracle_max_threads())


def geometry(in_rows, in_cols, window_rows, window_cols, stride_rows, stride_cols, padding):
    """(out_rows, out_cols, pad_top, pad_bottom, pad_left, pad_right) or ValueError."""
    p = _params(1, in_rows, in_cols, 1, 1, window_rows, window_cols, stride_rows, stride_cols,
                padding)
    g = _Geometry()
    if _load().conv2d_oracle_get_geometry(ctypes.byref(p), ctypes.byref(g)):
        raise ValueError("no valid output for these convolution parameters")
    return (g.out_rows, g.out_cols, g.pad_top, g.pad_bottom, g.pad_left, g.pad_right)


def _forward(x, f, stride, padding, dtype, fn_name, num_threads):
    x = np.ascontiguousarray(x, dtype=dtype)
    f = np.ascontiguousarray(f, dtype=dtype)
    if x.ndim != 4 or f.ndim != 4 or x.shape[3] != f.shape[2]:
        raise ValueError("expected NHWC input and HWCF filter with matching channels")
    n, h, w, c = x.shape
    r, s, _, k = f.shape
    sr, sc = (stride, stride) if isinstance(stride, int) else stride
    p = _params(n, h, w, c, k, r, s, sr, sc, padding)
    g = _Geometry()
    lib = _load()
    if lib.conv2d_oracle_get_geometry(ctypes.byref(p), ctypes.byref(g)):
        raise ValueError("no valid output for these convolution parameters")
    out = np.empty((n, g.out_rows, g.out_cols, k), dtype=dtype)
    rc = getattr(lib, fn_name)(ctypes.byref(p), x.ctypes.data, f.ctypes.data, out.ctypes.data,
                               int(num_threads))
    if rc:
        raise RuntimeError("%s failed with status %d" % (fn_name, rc))
    return out


def forward_f32(x, f, stride=1, padding=PAD_SAME, num_threads=0):
    """NHWC x (float32), HWCF f (float32) -> NHWC float32 (fp64 accumulate)."""
    return _forward(x, f, stride, padding, np.float32, "conv2d_oracle_forward_f32", num_threads)


def forward_f64(x, f, stride=1, padding=PAD_SAME, num_threads=0):
    """Same definition on float64 data with float64 output."""
    return _forward(x, f, stride, padding, np.float64, "conv2d_oracle_forward_f64", num_threads)


def points_f32(x, f, flat_index, stride=1, padding=PAD_SAME, num_threads=0):
    """fp64 sums at selected flat NHWC output indices (float32 data)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    f = np.ascontiguousarray(f, dtype=np.float32)
    idx = np.ascontiguousarray(flat_index, dtype=np.int64)
    n, h, w, c = x.shape
    r, s, _, k = f.shape
    sr, sc = (stride, stride) if isinstance(stride, int) else stride
    p = _params(n, h, w, c, k, r, s, sr, sc, padding)
    vals = np.empty(idx.shape, dtype=np.float64)
    rc = _load().conv2d_oracle_points_f32(ctypes.byref(p), x.ctypes.data, f.ctypes.data,
                                          idx.ctypes.data, idx.size, vals.ctypes.data,
                                          int(num_threads))
    if rc:
        raise RuntimeError("conv2d_oracle_points_f32 failed with status %d" % rc)
    return vals


def forward_bias_act_f32(x, f, bias=None, relu=False, stride=1, padding=PAD_SAME, num_threads=0):
    """The fused epilogue written out from its definition:
    out = act(conv(x, f) + bias[k]), conv in fp64 on the float32 data, bias added in fp64,
    act = max(., 0) if `relu`, one rounding to float32 at the end.  (Section 3 of the paper
    names the layers between the convolutions only in passing; bias and ReLU are the usual
    ones, and this is their plain definition.)"""
    y = forward_f64(np.asarray(x, dtype=np.float32).astype(np.float64),
                    np.asarray(f, dtype=np.float32).astype(np.float64), stride, padding,
                    num_threads)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float32).astype(np.float64)
        if b.shape != (y.shape[3],):
            raise ValueError("bias must have one value per output feature")
        y = y + b
    if relu:
        y = np.maximum(y, 0.0)
    return y.astype(np.float32)


def max_pool_2x2(y):
    """2x2 max pooling with stride 2 and no padding over an NHWC array, written out as loops
    over the four window positions: out[n, i, j, k] = max over a, b in {0, 1} of
    y[n, 2 i + a, 2 j + b, k]; a trailing odd row or column is dropped.  (The pooling layer
    that section 3 of the paper names next to the convolutions, in its usual VGG form.)"""
    y = np.asarray(y)
    n, h, w, k = y.shape
    ph, pw = h // 2, w // 2
    out = np.full((n, ph, pw, k), -np.inf, dtype=y.dtype)
    for a in range(2):
        for b in range(2):
            out = np.maximum(out, y[:, a:2 * ph:2, b:2 * pw:2, :])
    return out


def forward_bias_act_pool_f32(x, f, bias=None, relu=False, stride=1, padding=PAD_SAME,
                              num_threads=0):
    """Convolution, bias, activation, then 2x2 max pooling: the plain composition
    max_pool_2x2(act(conv(x, f) + bias)), everything in fp64 on the float32 data, one rounding
    to float32 at the end."""
    y = forward_f64(np.asarray(x, dtype=np.float32).astype(np.float64),
                    np.asarray(f, dtype=np.float32).astype(np.float64), stride, padding,
                    num_threads)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float32).astype(np.float64)
        if b.shape != (y.shape[3],):
            raise ValueError("bias must have one value per output feature")
        y = y + b
    if relu:
        y = np.maximum(y, 0.0)
    return max_pool_2x2(y).astype(np.float32)

