"""CPU oracle for the mixed-precision convolution path -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It is independent of the HIP library: it neither imports the product
package nor shares any code with it.

The arithmetic lives in ``oracle_conv.c`` (plain fp64 nested sums over inputs
given as binary16 bit patterns; section 2.2 "Mixed Precision Training" of the
paper fixes half-precision inputs and loss scaling, the sums are the textbook
definitions of convolution forward, data gradient and weight gradient).  This
module only marshals numpy arrays into that C code.

Pins: see ``tests/test_oracle_pins.py`` -- every function here is pinned
(nothing is "parity unpinned").
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle_conv.c")
_LIB = os.path.join(_HERE, "liboracle.so")


class ConvDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "N", "H", "W", "C", "K", "R", "S",
        "stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w")]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc + OpenMP into ``liboracle.so`` beside the source."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        p = ctypes.c_void_p
        for name in ("oracle_conv2d_fwd", "oracle_conv2d_dgrad", "oracle_conv2d_wgrad",
                     "oracle_conv2d_fwd_f32", "oracle_conv2d_dgrad_f32", "oracle_conv2d_wgrad_f32"):
            fn = getattr(lib, name)
            fn.argtypes = [ctypes.POINTER(ConvDesc), p, p, p, ctypes.c_int64, p]
            fn.restype = ctypes.c_int
        lib.oracle_conv2d_out_shape.argtypes = [ctypes.POINTER(ConvDesc),
                                                ctypes.POINTER(ctypes.c_int32),
                                                ctypes.POINTER(ctypes.c_int32)]
        lib.oracle_conv2d_out_shape.restype = ctypes.c_int
        lib.oracle_unscale_check.argtypes = [p, ctypes.c_int64, ctypes.c_float, p,
                                             ctypes.POINTER(ctypes.c_int32)]
        lib.oracle_unscale_check.restype = ctypes.c_int
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def make_desc(N, H, W, C, K, R, S, stride=(1, 1), pad=(0, 0), dil=(1, 1)) -> ConvDesc:
    return ConvDesc(N, H, W, C, K, R, S, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])


def out_shape(d: ConvDesc):
    ho, wo = ctypes.c_int32(), ctypes.c_int32()
    if _load().oracle_conv2d_out_shape(ctypes.byref(d), ctypes.byref(ho), ctypes.byref(wo)):
        raise ValueError("invalid convolution descriptor")
    return ho.value, wo.value


def num_threads() -> int:
    return _load().oracle_num_threads()


def _half_bits(a: np.ndarray, shape: Sequence[int]) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float16:
        raise TypeError("oracle inputs are binary16 arrays (the values both sides see)")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a.view(np.uint16)


def _run(fn, d, a, b, full_shape, idx: Optional[np.ndarray]):
    if idx is None:
        out = np.empty(full_shape, dtype=np.float64)
        rc = fn(ctypes.byref(d), a.ctypes.data, b.ctypes.data, None, 0, out.ctypes.data)
    else:
        idx = np.ascontiguousarray(idx, dtype=np.int64)
        total = int(np.prod(full_shape))
        if idx.size and (idx.min() < 0 or idx.max() >= total):
            raise IndexError("sample index outside the output tensor")
        out = np.empty(idx.shape, dtype=np.float64)
        rc = fn(ctypes.byref(d), a.ctypes.data, b.ctypes.data, idx.ctypes.data, idx.size,
                out.ctypes.data)
    if rc:
        raise RuntimeError(f"oracle call failed with code {rc}")
    return out


def conv2d_fwd(d: ConvDesc, x: np.ndarray, w: np.ndarray, idx=None) -> np.ndarray:
    """y[N,Ho,Wo,K] in fp64 (or the flat elements ``idx`` of it)."""
    ho, wo = out_shape(d)
    xb = _half_bits(x, (d.N, d.H, d.W, d.C))
    wb = _half_bits(w, (d.K, d.R, d.S, d.C))
    return _run(_load().oracle_conv2d_fwd, d, xb, wb, (d.N, ho, wo, d.K), idx)


def conv2d_dgrad(d: ConvDesc, dy: np.ndarray, w: np.ndarray, idx=None) -> np.ndarray:
    """dx[N,H,W,C] in fp64 (or the flat elements ``idx`` of it)."""
    ho, wo = out_shape(d)
    gb = _half_bits(dy, (d.N, ho, wo, d.K))
    wb = _half_bits(w, (d.K, d.R, d.S, d.C))
    return _run(_load().oracle_conv2d_dgrad, d, gb, wb, (d.N, d.H, d.W, d.C), idx)


def conv2d_wgrad(d: ConvDesc, x: np.ndarray, dy: np.ndarray, idx=None) -> np.ndarray:
    """dw[K,R,S,C] in fp64 (or the flat elements ``idx`` of it)."""
    ho, wo = out_shape(d)
    xb = _half_bits(x, (d.N, d.H, d.W, d.C))
    gb = _half_bits(dy, (d.N, ho, wo, d.K))
    return _run(_load().oracle_conv2d_wgrad, d, xb, gb, (d.K, d.R, d.S, d.C), idx)


def _f32(a: np.ndarray, shape: Sequence[int]) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32:
        raise TypeError("inputs of the single-precision path are binary32 arrays")
    if tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def conv2d_fwd_f32(d: ConvDesc, x: np.ndarray, w: np.ndarray, idx=None) -> np.ndarray:
    """conv2d_fwd on binary32 inputs (the full-precision training section 2.2 compares against)."""
    ho, wo = out_shape(d)
    return _run(_load().oracle_conv2d_fwd_f32, d, _f32(x, (d.N, d.H, d.W, d.C)), _f32(w, (d.K, d.R, d.S, d.C)),
                (d.N, ho, wo, d.K), idx)


def conv2d_dgrad_f32(d: ConvDesc, dy: np.ndarray, w: np.ndarray, idx=None) -> np.ndarray:
    ho, wo = out_shape(d)
    return _run(_load().oracle_conv2d_dgrad_f32, d, _f32(dy, (d.N, ho, wo, d.K)), _f32(w, (d.K, d.R, d.S, d.C)),
                (d.N, d.H, d.W, d.C), idx)


def conv2d_wgrad_f32(d: ConvDesc, x: np.ndarray, dy: np.ndarray, idx=None) -> np.ndarray:
    ho, wo = out_shape(d)
    return _run(_load().oracle_conv2d_wgrad_f32, d, _f32(x, (d.N, d.H, d.W, d.C)), _f32(dy, (d.N, ho, wo, d.K)),
                (d.K, d.R, d.S, d.C), idx)


def unscale_check(g: np.ndarray, inv_scale: float):
    """Returns (g * inv_scale rounded once to fp32, flag) with flag = any non-finite input."""
    g = np.ascontiguousarray(g)
    if g.dtype != np.float32:
        raise TypeError("gradient buffer is fp32")
    out = np.empty_like(g)
    flag = ctypes.c_int32(-1)
    rc = _load().oracle_unscale_check(g.ctypes.data, g.size, ctypes.c_float(inv_scale),
                                      out.ctypes.data, ctypes.byref(flag))
    if rc:
        raise RuntimeError(f"oracle call failed with code {rc}")
    return out, flag.value
