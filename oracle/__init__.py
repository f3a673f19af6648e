"""ctypes front end of the CPU oracle (test infrastructure, not product code).

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It never imports the HIP package and
shares nothing with it.

The shared object is built from ``mdnn_oracle.c`` by :func:`build` (gcc, -O2,
OpenMP over the output-filter loop only).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mdnn_oracle.c")
_LIB = os.path.join(_HERE, "libmdnn_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  Returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    lib = ctypes.CDLL(_LIB)
    i, f = ctypes.c_int, ctypes.c_float
    p = ctypes.c_void_p
    lib.mdnn_oracle_out_dims.argtypes = [i, i, i, i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
    lib.mdnn_oracle_out_dims.restype = i
    lib.mdnn_oracle_flops.argtypes = [i] * 6
    lib.mdnn_oracle_flops.restype = ctypes.c_uint64
    lib.mdnn_oracle_max_threads.argtypes = []
    lib.mdnn_oracle_max_threads.restype = i
    lib.mdnn_oracle_conv_fprop.argtypes = [p, p, p, p, i, i, i, i, i, i, i, i, f, i]
    lib.mdnn_oracle_conv_fprop.restype = i
    lib.mdnn_oracle_conv_bprop_data.argtypes = [p, p, p, p, i, i, i, i, i, i, i, i, f, i]
    lib.mdnn_oracle_conv_bprop_data.restype = i
    lib.mdnn_oracle_conv_bprop_filter.argtypes = [p, p, p, p, i, i, i, i, i, i, i, i, f, i]
    lib.mdnn_oracle_conv_bprop_filter.restype = i
    lib.mdnn_oracle_conv_bprop_filter_points.argtypes = [p, p, p, ctypes.c_int64, p, p,
                                                         i, i, i, i, i, i, i, i, f]
    lib.mdnn_oracle_conv_bprop_filter_points.restype = i
    lib.mdnn_oracle_conv_bprop_data_points.argtypes = [p, p, p, ctypes.c_int64, p, p,
                                                       i, i, i, i, i, i, i, i, f]
    lib.mdnn_oracle_conv_bprop_data_points.restype = i
    lib.mdnn_oracle_sgemm_tn.argtypes = [p, p, p, p, i, i, i, f, i]
    lib.mdnn_oracle_sgemm_tn.restype = i
    lib.mdnn_oracle_conv_fprop_points.argtypes = [p, p, p, ctypes.c_int64, p, p,
                                                  i, i, i, i, i, i, i, i, f]
    lib.mdnn_oracle_conv_fprop_points.restype = i
    _lib = lib
    return lib


def out_dims(Wi, Hi, Sk, stride, pad):
    """(Wo, Ho) by the floor formula; raises ValueError when no output exists."""
    wo, ho = ctypes.c_int(), ctypes.c_int()
    if _load().mdnn_oracle_out_dims(Wi, Hi, Sk, stride, pad, ctypes.byref(wo), ctypes.byref(ho)):
        raise ValueError("invalid convolution geometry")
    return wo.value, ho.value


def flops(Nb, Wo, Ho, Nc, No, Sk) -> int:
    """Complexity formula of Section 2."""
    return int(_load().mdnn_oracle_flops(Nb, Wo, Ho, Nc, No, Sk))


def max_threads() -> int:
    return int(_load().mdnn_oracle_max_threads())


def _check(a, shape, name):
    if a.dtype != np.float32 or not a.flags["C_CONTIGUOUS"] or tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name}: want C-contiguous float32 of shape {tuple(shape)}, "
                         f"got {a.dtype} {a.shape}")


def conv_fprop(inp, filt, stride, pad, alpha, want_abs=True, nthreads=0):
    """inp (Nc,Hi,Wi,Nb) f32, filt (Nc,Sk,Sk,No) f32 -> out (No,Ho,Wo,Nb) f32
    and, when ``want_abs``, the per-output sum of |products| in float64."""
    Nc, Hi, Wi, Nb = inp.shape
    Nc2, Sk, Sk2, No = filt.shape
    if Nc2 != Nc or Sk2 != Sk:
        raise ValueError("filter shape does not match input")
    _check(inp, inp.shape, "inp")
    _check(filt, filt.shape, "filt")
    Wo, Ho = out_dims(Wi, Hi, Sk, stride, pad)
    out = np.empty((No, Ho, Wo, Nb), dtype=np.float32)
    ab = np.empty((No, Ho, Wo, Nb), dtype=np.float64) if want_abs else None
    rc = _load().mdnn_oracle_conv_fprop(
        inp.ctypes.data, filt.ctypes.data, out.ctypes.data,
        ab.ctypes.data if ab is not None else None,
        Nb, Wi, Hi, Nc, No, Sk, stride, pad, float(alpha), int(nthreads))
    if rc:
        raise ValueError("oracle rejected the arguments")
    return (out, ab) if want_abs else out


def conv_fprop_points(inp, filt, idx, stride, pad, alpha):
    """Evaluate the definition at the (o,y,x,n) rows of ``idx`` only.
    Returns (values float32[npts], abs_sums float64[npts])."""
    Nc, Hi, Wi, Nb = inp.shape
    _, Sk, _, No = filt.shape
    _check(inp, inp.shape, "inp")
    _check(filt, filt.shape, "filt")
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.ndim != 2 or idx.shape[1] != 4:
        raise ValueError("idx must be (npts, 4)")
    vals = np.empty(idx.shape[0], dtype=np.float32)
    ab = np.empty(idx.shape[0], dtype=np.float64)
    rc = _load().mdnn_oracle_conv_fprop_points(
        inp.ctypes.data, filt.ctypes.data, idx.ctypes.data, idx.shape[0],
        vals.ctypes.data, ab.ctypes.data,
        Nb, Wi, Hi, Nc, No, Sk, stride, pad, float(alpha))
    if rc:
        raise ValueError("oracle rejected the arguments (index out of range?)")
    return vals, ab


def conv_bprop_data(dout, filt, in_hw, stride, pad, alpha, want_abs=True, nthreads=0):
    """dout (No,Ho,Wo,Nb) f32, filt (Nc,Sk,Sk,No) f32, in_hw = (Hi, Wi) of the forward input
    -> din (Nc,Hi,Wi,Nb) f32 and, when ``want_abs``, the per-element sum of |products|."""
    No, Ho, Wo, Nb = dout.shape
    Nc, Sk, Sk2, No2 = filt.shape
    Hi, Wi = in_hw
    if No2 != No or Sk2 != Sk:
        raise ValueError("filter shape does not match dout")
    _check(dout, dout.shape, "dout")
    _check(filt, filt.shape, "filt")
    if out_dims(Wi, Hi, Sk, stride, pad) != (Wo, Ho):
        raise ValueError("dout spatial size does not match the forward geometry")
    din = np.empty((Nc, Hi, Wi, Nb), dtype=np.float32)
    ab = np.empty((Nc, Hi, Wi, Nb), dtype=np.float64) if want_abs else None
    rc = _load().mdnn_oracle_conv_bprop_data(
        dout.ctypes.data, filt.ctypes.data, din.ctypes.data,
        ab.ctypes.data if ab is not None else None,
        Nb, Wi, Hi, Nc, No, Sk, stride, pad, float(alpha), int(nthreads))
    if rc:
        raise ValueError("oracle rejected the arguments")
    return (din, ab) if want_abs else din


def conv_bprop_filter(inp, dout, Sk, stride, pad, alpha, want_abs=True, nthreads=0):
    """inp (Nc,Hi,Wi,Nb) f32, dout (No,Ho,Wo,Nb) f32 -> dfilt (Nc,Sk,Sk,No) f32 and, when
    ``want_abs``, the per-element sum of |products| in float64."""
    Nc, Hi, Wi, Nb = inp.shape
    No, Ho, Wo, Nb2 = dout.shape
    if Nb2 != Nb:
        raise ValueError("batch sizes differ")
    _check(inp, inp.shape, "inp")
    _check(dout, dout.shape, "dout")
    if out_dims(Wi, Hi, Sk, stride, pad) != (Wo, Ho):
        raise ValueError("dout spatial size does not match the forward geometry")
    dfilt = np.empty((Nc, Sk, Sk, No), dtype=np.float32)
    ab = np.empty((Nc, Sk, Sk, No), dtype=np.float64) if want_abs else None
    rc = _load().mdnn_oracle_conv_bprop_filter(
        inp.ctypes.data, dout.ctypes.data, dfilt.ctypes.data,
        ab.ctypes.data if ab is not None else None,
        Nb, Wi, Hi, Nc, No, Sk, stride, pad, float(alpha), int(nthreads))
    if rc:
        raise ValueError("oracle rejected the arguments")
    return (dfilt, ab) if want_abs else dfilt


def conv_bprop_filter_points(inp, dout, idx, Sk, stride, pad, alpha):
    """The filter gradient at the (c,ky,kx,o) rows of ``idx`` only.
    Returns (values float32[npts], abs_sums float64[npts])."""
    Nc, Hi, Wi, Nb = inp.shape
    No = dout.shape[0]
    _check(inp, inp.shape, "inp")
    _check(dout, dout.shape, "dout")
    if out_dims(Wi, Hi, Sk, stride, pad) != (dout.shape[2], dout.shape[1]) or dout.shape[3] != Nb:
        raise ValueError("dout does not match the forward geometry")
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.ndim != 2 or idx.shape[1] != 4:
        raise ValueError("idx must be (npts, 4)")
    vals = np.empty(idx.shape[0], dtype=np.float32)
    ab = np.empty(idx.shape[0], dtype=np.float64)
    rc = _load().mdnn_oracle_conv_bprop_filter_points(
        inp.ctypes.data, dout.ctypes.data, idx.ctypes.data, idx.shape[0],
        vals.ctypes.data, ab.ctypes.data,
        Nb, Wi, Hi, Nc, No, Sk, stride, pad, float(alpha))
    if rc:
        raise ValueError("oracle rejected the arguments (index out of range?)")
    return vals, ab


def conv_bprop_data_points(dout, filt, idx, in_hw, stride, pad, alpha):
    """The data gradient at the (c,iy,ix,n) rows of ``idx`` only.
    Returns (values float32[npts], abs_sums float64[npts])."""
    No, Ho, Wo, Nb = dout.shape
    Nc, Sk, Sk2, No2 = filt.shape
    Hi, Wi = in_hw
    if No2 != No or Sk2 != Sk:
        raise ValueError("filter shape does not match dout")
    _check(dout, dout.shape, "dout")
    _check(filt, filt.shape, "filt")
    if out_dims(Wi, Hi, Sk, stride, pad) != (Wo, Ho):
        raise ValueError("dout spatial size does not match the forward geometry")
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.ndim != 2 or idx.shape[1] != 4:
        raise ValueError("idx must be (npts, 4)")
    vals = np.empty(idx.shape[0], dtype=np.float32)
    ab = np.empty(idx.shape[0], dtype=np.float64)
    rc = _load().mdnn_oracle_conv_bprop_data_points(
        dout.ctypes.data, filt.ctypes.data, idx.ctypes.data, idx.shape[0],
        vals.ctypes.data, ab.ctypes.data,
        Nb, Wi, Hi, Nc, No, Sk, stride, pad, float(alpha))
    if rc:
        raise ValueError("oracle rejected the arguments (index out of range?)")
    return vals, ab


def sgemm_tn(a, b, alpha, want_abs=True, nthreads=0):
    """a (K,N) f32, b (K,M) f32 -> c (N,M) f32 = alpha * a^T b and, when
    ``want_abs``, the per-element sum of |products| in float64."""
    K, N = a.shape
    K2, M = b.shape
    if K2 != K:
        raise ValueError("a and b must have the same number of rows")
    _check(a, a.shape, "a")
    _check(b, b.shape, "b")
    c = np.empty((N, M), dtype=np.float32)
    ab = np.empty((N, M), dtype=np.float64) if want_abs else None
    rc = _load().mdnn_oracle_sgemm_tn(
        a.ctypes.data, b.ctypes.data, c.ctypes.data,
        ab.ctypes.data if ab is not None else None,
        N, M, K, float(alpha), int(nthreads))
    if rc:
        raise ValueError("oracle rejected the arguments")
    return (c, ab) if want_abs else c
