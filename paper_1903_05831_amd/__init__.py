"""Thin ctypes binding over libsdconv.so -- argument marshalling only.

Every step of the path (convolution forward, data gradient, weight gradient, loss-scale
removal with overflow check; the mixed-precision training compute of section 2.2 of the
paper) runs in the hand-written HIP kernels behind the C ABI declared in
``include/sdconv.h``.  PyTorch is used by callers for device memory and streams only.
There is no CPU fallback: if the library is missing, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsdconv.so")

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP = 0, -1, -2, -3, -4
FWD, DGRAD, WGRAD = 0, 1, 2

EXPORTS = (
    "conv2d_out_shape", "conv2d_workspace_bytes", "conv2d_fwd", "conv2d_dgrad", "conv2d_wgrad",
    "grad_unscale_check", "sdconv_status_string", "sdconv_last_hip_error", "sdconv_kernel_name",
    "sdconv_mfma_ceiling", "grad_unscale_check_dynamic", "sgd_momentum_update",
    "conv2d_fwd_fused", "conv2d_dgrad_fused", "sdconv_tail_pass",
    "conv2d_workspace_bytes_f32", "conv2d_fwd_f32", "conv2d_dgrad_f32", "conv2d_wgrad_f32",
    "conv2d_wgrad_static_scratch",
)


class conv2d_desc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "N", "H", "W", "C", "K", "R", "S",
        "stride_h", "stride_w", "pad_h", "pad_w", "dil_h", "dil_w")]


class conv2d_fwd_epilogue(ctypes.Structure):
    _fields_ = [("scale", ctypes.c_void_p), ("bias", ctypes.c_void_p), ("residual", ctypes.c_void_p),
                ("relu", ctypes.c_int32)]


class conv2d_dgrad_epilogue(ctypes.Structure):
    _fields_ = [("scale", ctypes.c_void_p), ("relu_mask", ctypes.c_void_p)]


class SdconvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status}, hip error {last_hip_error()})")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads libsdconv.so (built in-tree by ``build.py``); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1903_05831_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, i32p = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(ctypes.c_int32)
        dp = ctypes.POINTER(conv2d_desc)
        L.conv2d_out_shape.argtypes = [dp, i32p, i32p]
        L.conv2d_out_shape.restype = ctypes.c_int
        L.conv2d_workspace_bytes.argtypes = [dp, ctypes.c_int]
        L.conv2d_workspace_bytes.restype = sz
        for name in ("conv2d_fwd", "conv2d_dgrad", "conv2d_wgrad"):
            fn = getattr(L, name)
            fn.argtypes = [dp, vp, vp, vp, vp, sz, vp]
            fn.restype = ctypes.c_int
        L.grad_unscale_check.argtypes = [vp, sz, ctypes.c_float, vp, vp]
        L.grad_unscale_check.restype = ctypes.c_int
        L.sdconv_status_string.argtypes = [ctypes.c_int]
        L.sdconv_status_string.restype = ctypes.c_char_p
        L.sdconv_last_hip_error.restype = ctypes.c_int
        L.sdconv_kernel_name.argtypes = [dp, ctypes.c_int]
        L.sdconv_kernel_name.restype = ctypes.c_char_p
        L.grad_unscale_check_dynamic.argtypes = [vp, sz, vp, vp, vp]
        L.grad_unscale_check_dynamic.restype = ctypes.c_int
        f32 = ctypes.c_float
        L.sgd_momentum_update.argtypes = [vp, vp, vp, vp, sz, f32, f32, f32, vp, vp, f32, f32, ctypes.c_int32, vp]
        L.sgd_momentum_update.restype = ctypes.c_int
        L.conv2d_fwd_fused.argtypes = [dp, vp, vp, ctypes.POINTER(conv2d_fwd_epilogue), vp, vp, sz, vp]
        L.conv2d_fwd_fused.restype = ctypes.c_int
        L.conv2d_dgrad_fused.argtypes = [dp, vp, vp, ctypes.POINTER(conv2d_dgrad_epilogue), vp, vp, sz, vp]
        L.conv2d_dgrad_fused.restype = ctypes.c_int
        L.conv2d_workspace_bytes_f32.argtypes = [dp, ctypes.c_int]
        L.conv2d_workspace_bytes_f32.restype = sz
        for name in ("conv2d_fwd_f32", "conv2d_dgrad_f32", "conv2d_wgrad_f32"):
            fn = getattr(L, name)
            fn.argtypes = [dp, vp, vp, vp, vp, sz, vp]
            fn.restype = ctypes.c_int
        L.conv2d_wgrad_static_scratch.argtypes = [dp, vp, vp, vp, vp]
        L.conv2d_wgrad_static_scratch.restype = ctypes.c_int
        L.sdconv_tail_pass.argtypes = [vp, sz, ctypes.c_int32, vp, vp, vp, vp, ctypes.c_int32, vp]
        L.sdconv_tail_pass.restype = ctypes.c_int
        L.sdconv_mfma_ceiling.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp]
        L.sdconv_mfma_ceiling.restype = ctypes.c_int
        _lib = L
    return _lib


def make_desc(N, H, W, C, K, R, S, stride=(1, 1), pad=(0, 0), dil=(1, 1)) -> conv2d_desc:
    return conv2d_desc(N, H, W, C, K, R, S, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1])


def desc_of(layer) -> conv2d_desc:
    """Descriptor for a ``workloads.ConvLayer``."""
    return make_desc(layer.N, layer.H, layer.W, layer.C, layer.K, layer.R, layer.S,
                     (layer.stride, layer.stride), (layer.pad, layer.pad), (layer.dil, layer.dil))


def status_string(status: int) -> str:
    return lib().sdconv_status_string(status).decode()


def last_hip_error() -> int:
    return lib().sdconv_last_hip_error()


def kernel_name(desc: conv2d_desc, pass_id: int) -> str:
    return lib().sdconv_kernel_name(ctypes.byref(desc), pass_id).decode()


def conv2d_out_shape(desc: conv2d_desc) -> Tuple[int, int]:
    ho, wo = ctypes.c_int32(), ctypes.c_int32()
    rc = lib().conv2d_out_shape(ctypes.byref(desc), ctypes.byref(ho), ctypes.byref(wo))
    if rc:
        raise SdconvError(rc, "conv2d_out_shape")
    return ho.value, wo.value


def conv2d_workspace_bytes(desc: conv2d_desc, pass_id: int) -> int:
    return int(lib().conv2d_workspace_bytes(ctypes.byref(desc), pass_id))


def _ptr(t) -> int:
    """Device address of a torch tensor (or a raw integer address, or None)."""
    if t is None:
        return 0
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensors must be dense and contiguous")
    return t.data_ptr()


def _ws(workspace) -> Tuple[int, int]:
    if workspace is None:
        return 0, 0
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def _call(name, desc, a, b, out, workspace, stream) -> None:
    wp, wb = _ws(workspace)
    rc = getattr(lib(), name)(ctypes.byref(desc), _ptr(a), _ptr(b), _ptr(out), wp, wb, stream or 0)
    if rc:
        raise SdconvError(rc, name)


def conv2d_fwd(desc, x, w, y, workspace=None, stream: int = 0) -> None:
    _call("conv2d_fwd", desc, x, w, y, workspace, stream)


def conv2d_dgrad(desc, dy, w, dx, workspace=None, stream: int = 0) -> None:
    _call("conv2d_dgrad", desc, dy, w, dx, workspace, stream)


def conv2d_fwd_fused(desc, x, w, y, workspace=None, stream: int = 0, *, scale=None, bias=None, residual=None,
                     relu: bool = False) -> None:
    """y = act(scale[k] * conv(x, w) + bias[k] + residual); scale, bias: fp32 [K] device tensors."""
    ep = conv2d_fwd_epilogue(_ptr(scale) or None, _ptr(bias) or None, _ptr(residual) or None, 1 if relu else 0)
    wp, wb = _ws(workspace)
    rc = lib().conv2d_fwd_fused(ctypes.byref(desc), _ptr(x), _ptr(w), ctypes.byref(ep), _ptr(y), wp, wb, stream or 0)
    if rc:
        raise SdconvError(rc, "conv2d_fwd_fused")


def conv2d_dgrad_fused(desc, dy, w, dx, workspace=None, stream: int = 0, *, scale=None, relu_mask=None) -> None:
    """dx = relu_mask > 0 ? scale[c] * dgrad(dy, w) : 0; scale: fp32 [C], relu_mask: fp16 like dx."""
    ep = conv2d_dgrad_epilogue(_ptr(scale) or None, _ptr(relu_mask) or None)
    wp, wb = _ws(workspace)
    rc = lib().conv2d_dgrad_fused(ctypes.byref(desc), _ptr(dy), _ptr(w), ctypes.byref(ep), _ptr(dx), wp, wb,
                                  stream or 0)
    if rc:
        raise SdconvError(rc, "conv2d_dgrad_fused")


def conv2d_workspace_bytes_f32(desc: conv2d_desc, pass_id: int) -> int:
    return int(lib().conv2d_workspace_bytes_f32(ctypes.byref(desc), pass_id))


def conv2d_fwd_f32(desc, x, w, y, workspace=None, stream: int = 0) -> None:
    """Single-precision companion of conv2d_fwd: every tensor fp32."""
    _call("conv2d_fwd_f32", desc, x, w, y, workspace, stream)


def conv2d_dgrad_f32(desc, dy, w, dx, workspace=None, stream: int = 0) -> None:
    _call("conv2d_dgrad_f32", desc, dy, w, dx, workspace, stream)


def conv2d_wgrad_f32(desc, x, dy, dw, workspace=None, stream: int = 0) -> None:
    _call("conv2d_wgrad_f32", desc, x, dy, dw, workspace, stream)


def sdconv_tail_pass(t, pixels: int, channels: int, stream: int = 0, *, scale=None, bias=None, residual=None,
                     relu_mask=None, relu: bool = False) -> None:
    """Measurement aid: the elementwise tail as a separate in-place pass over t [pixels][channels] fp16."""
    rc = lib().sdconv_tail_pass(_ptr(t), pixels, channels, _ptr(scale) or None, _ptr(bias) or None,
                                _ptr(residual) or None, _ptr(relu_mask) or None, 1 if relu else 0, stream or 0)
    if rc:
        raise SdconvError(rc, "sdconv_tail_pass")


def conv2d_wgrad(desc, x, dy, dw, workspace=None, stream: int = 0) -> None:
    _call("conv2d_wgrad", desc, x, dy, dw, workspace, stream)


STATIC_SCRATCH_BYTES = 64 << 20


def conv2d_wgrad_static_scratch(desc, x, dy, dw, stream: int = 0) -> None:
    """conv2d_wgrad on the library's own fixed device scratch: allocates nothing."""
    rc = lib().conv2d_wgrad_static_scratch(ctypes.byref(desc), _ptr(x), _ptr(dy), _ptr(dw), stream or 0)
    if rc:
        raise SdconvError(rc, "conv2d_wgrad_static_scratch")


def grad_unscale_check_dynamic(grad, n: int, state, found_nonfinite, stream: int = 0) -> None:
    """state: device tensor holding a loss_scale_state {float scale; int32 good_steps}."""
    rc = lib().grad_unscale_check_dynamic(_ptr(grad), n, _ptr(state), _ptr(found_nonfinite), stream or 0)
    if rc:
        raise SdconvError(rc, "grad_unscale_check_dynamic")


def sgd_momentum_update(master_w, momentum_buf, grad, w_half, n: int, lr: float, momentum: float,
                        weight_decay: float, found_nonfinite, state, growth: float, backoff: float,
                        interval: int, stream: int = 0) -> None:
    rc = lib().sgd_momentum_update(_ptr(master_w), _ptr(momentum_buf), _ptr(grad), _ptr(w_half), n,
                                   lr, momentum, weight_decay, _ptr(found_nonfinite), _ptr(state),
                                   growth, backoff, interval, stream or 0)
    if rc:
        raise SdconvError(rc, "sgd_momentum_update")


def sdconv_mfma_ceiling(scratch, blocks: int, iters: int, stream: int = 0) -> None:
    rc = lib().sdconv_mfma_ceiling(_ptr(scratch), blocks, iters, stream or 0)
    if rc:
        raise SdconvError(rc, "sdconv_mfma_ceiling")


def grad_unscale_check(grad, n: int, inv_scale: float, found_nonfinite, stream: int = 0) -> None:
    rc = lib().grad_unscale_check(_ptr(grad), n, ctypes.c_float(inv_scale), _ptr(found_nonfinite),
                                  stream or 0)
    if rc:
        raise SdconvError(rc, "grad_unscale_check")
