"""CPU oracle for the fused convolution epilogues -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module.  It
shares nothing with the HIP library.

Section 2.3 of the paper recalls that detectors are trained with the batch-normalisation
parameters frozen: such a layer is a fixed per-channel affine map of the convolution output,
followed in a residual network by the shortcut addition and the ReLU.  What is computed here
is that composition written out on top of the plain convolution definitions of this package,
in fp64, on the binary16 tensors and binary32 per-channel vectors both sides receive:

  forward        y[n,h,w,k]  = act( scale[k] * conv(x, w)[n,h,w,k] + bias[k] + residual[n,h,w,k] )
                 act(v) = v if v > 0 else 0 when relu is set, else v
  data gradient  dx[n,h,w,c] = scale[c] * dgrad(dy, w)[n,h,w,c]  if relu_mask[n,h,w,c] > 0 else 0
                 (the chain rule through a = relu(scale*z + bias) that feeds the convolution:
                 relu_mask is that activation a, scale the affine map's factor; dx is dL/dz)

Every part is optional (None / False leaves it out).  Readings taken where the paper is
silent: the ReLU gradient is 0 at 0, the comparison is strict, and a NaN passes neither test.

Pins: tests/test_oracle_epilogue_pins.py (nothing here is "parity unpinned").
"""
from __future__ import annotations

import numpy as np

from . import conv2d_dgrad, conv2d_fwd, out_shape


def _vec(v, n, name):
    v = np.ascontiguousarray(v)
    if v.dtype != np.float32 or v.shape != (n,):
        raise TypeError(f"{name} is a binary32 vector of {n} channels")
    return v.astype(np.float64)


def _act(t, shape, name):
    t = np.ascontiguousarray(t)
    if t.dtype != np.float16 or tuple(t.shape) != tuple(shape):
        raise TypeError(f"{name} is a binary16 tensor of shape {tuple(shape)}")
    return t.astype(np.float64)


def frozen_bn_affine(gamma, beta, mean, var, eps):
    """(scale, bias) in fp64 of a batch normalisation whose statistics and parameters are fixed:
    gamma * (z - mean) / sqrt(var + eps) + beta  ==  scale * z + bias."""
    gamma, beta, mean, var = (np.asarray(a, dtype=np.float64) for a in (gamma, beta, mean, var))
    scale = gamma / np.sqrt(var + np.float64(eps))
    return scale, beta - mean * scale


def _at(t: np.ndarray, idx):
    """The whole tensor, or its flat elements idx."""
    return t if idx is None else t.ravel()[np.asarray(idx, dtype=np.int64)]


def fwd_tail(y, d, scale=None, bias=None, residual=None, relu=False, idx=None) -> np.ndarray:
    """The elementwise part of the fused forward pass, applied to y = conv2d_fwd(d, x, w) in
    fp64: y is the whole tensor [N,Ho,Wo,K], or its flat elements idx (then idx must be given,
    so that the per-channel vectors and the shortcut are taken at the same positions)."""
    ho, wo = out_shape(d)
    k = slice(None) if idx is None else np.asarray(idx, dtype=np.int64) % d.K
    y = np.asarray(y, dtype=np.float64)
    if idx is None and tuple(y.shape) != (d.N, ho, wo, d.K):
        raise ValueError("y is the whole forward result")
    if scale is not None:
        y = y * _vec(scale, d.K, "scale")[k]
    if bias is not None:
        y = y + _vec(bias, d.K, "bias")[k]
    if residual is not None:
        y = y + _at(_act(residual, (d.N, ho, wo, d.K), "residual"), idx)
    if relu:
        y = np.where(y > 0, y, 0.0)
    return y


def dgrad_tail(dx, d, scale=None, relu_mask=None, idx=None) -> np.ndarray:
    """The elementwise part of the fused data gradient, applied to dx = conv2d_dgrad(d, dy, w)
    in fp64 (whole tensor [N,H,W,C], or its flat elements idx)."""
    c = slice(None) if idx is None else np.asarray(idx, dtype=np.int64) % d.C
    dx = np.asarray(dx, dtype=np.float64)
    if idx is None and tuple(dx.shape) != (d.N, d.H, d.W, d.C):
        raise ValueError("dx is the whole data gradient")
    if scale is not None:
        dx = dx * _vec(scale, d.C, "scale")[c]
    if relu_mask is not None:
        dx = np.where(_at(_act(relu_mask, (d.N, d.H, d.W, d.C), "relu_mask"), idx) > 0, dx, 0.0)
    return dx


def conv2d_fwd_fused(d, x, w, scale=None, bias=None, residual=None, relu=False, idx=None) -> np.ndarray:
    """y[N,Ho,Wo,K] in fp64 (or the flat elements ``idx`` of it)."""
    return fwd_tail(conv2d_fwd(d, x, w, idx=idx), d, scale, bias, residual, relu, idx)


def conv2d_dgrad_fused(d, dy, w, scale=None, relu_mask=None, idx=None) -> np.ndarray:
    """dx[N,H,W,C] in fp64 (or the flat elements ``idx`` of it)."""
    return dgrad_tail(conv2d_dgrad(d, dy, w, idx=idx), d, scale, relu_mask, idx)
