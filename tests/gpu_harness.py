"""Helpers for the GPU parity tests: run one pass through the C ABI on torch-owned device
memory (with red zones around the output) and compare against the CPU oracle."""
from __future__ import annotations

import sys

import numpy as np
import torch

import oracle
import paper_1903_05831_amd as sd

ELEM_TOL = 2e-2      # |gpu - ref| <= ELEM_TOL * (1 + |ref|) per element
FRO_TOL = 1e-3       # ||gpu - ref||_F / ||ref||_F
GUARD = 1024         # red-zone elements on each side of every output
_SENTINEL16 = 0x7BCD  # a large finite half bit pattern
_SENTINEL32 = 0x7F7FABCD


def say(msg: str) -> None:
    print(msg, flush=True)
    sys.stdout.flush()


def oracle_desc(d: sd.conv2d_desc):
    return oracle.make_desc(d.N, d.H, d.W, d.C, d.K, d.R, d.S, (d.stride_h, d.stride_w),
                            (d.pad_h, d.pad_w), (d.dil_h, d.dil_w))


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class GuardedOut:
    """Output buffer with sentinel-filled red zones before and after it."""

    def __init__(self, shape, dtype):
        n = int(np.prod(shape))
        self.shape, self.n, self.dtype = shape, n, dtype
        # keep the payload 256-byte aligned: GUARD elements * elsize is a multiple of 256
        self.buf = torch.empty(n + 2 * GUARD, dtype=dtype, device="cuda")
        ibuf = self.buf.view(torch.int16 if dtype == torch.float16 else torch.int32)
        sent = _SENTINEL16 if dtype == torch.float16 else _SENTINEL32
        ibuf.fill_(sent)
        self._ibuf, self._sent = ibuf, sent
        self.view = self.buf[GUARD:GUARD + n].view(shape)

    def check_guards(self) -> None:
        i = self._ibuf
        assert bool((i[:GUARD] == self._sent).all()), "write before the output buffer"
        assert bool((i[GUARD + self.n:] == self._sent).all()), "write past the output buffer"

    def all_written(self) -> bool:
        """Heuristic: no element still holds the sentinel pattern."""
        return not bool((self._ibuf[GUARD:GUARD + self.n] == self._sent).any())

    def numpy(self) -> np.ndarray:
        return self.view.cpu().numpy()


def workspace_for(d, pass_id):
    need = sd.conv2d_workspace_bytes(d, pass_id)
    if need == 0:
        return None
    return torch.empty(need, dtype=torch.uint8, device="cuda")


def run_pass(d: sd.conv2d_desc, pass_id: int, a: torch.Tensor, b: torch.Tensor) -> GuardedOut:
    ho, wo = sd.conv2d_out_shape(d)
    stream = torch.cuda.current_stream().cuda_stream
    ws = workspace_for(d, pass_id)
    if pass_id == sd.FWD:
        out = GuardedOut((d.N, ho, wo, d.K), torch.float16)
        sd.conv2d_fwd(d, a, b, out.view, ws, stream)
    elif pass_id == sd.DGRAD:
        out = GuardedOut((d.N, d.H, d.W, d.C), torch.float16)
        sd.conv2d_dgrad(d, a, b, out.view, ws, stream)
    else:
        out = GuardedOut((d.K, d.R, d.S, d.C), torch.float32)
        sd.conv2d_wgrad(d, a, b, out.view, ws, stream)
    torch.cuda.synchronize()
    out.check_guards()
    return out


def compare(gpu: np.ndarray, ref: np.ndarray, what: str) -> None:
    """The parity bar: per-element and Frobenius, both against the fp64 oracle."""
    g = gpu.astype(np.float64).ravel()
    r = ref.ravel()
    assert g.shape == r.shape, what
    assert np.all(np.isfinite(g)), f"{what}: non-finite GPU output"
    err = np.abs(g - r)
    bound = ELEM_TOL * (1.0 + np.abs(r))
    worst = int(np.argmax(err - bound))
    assert err[worst] <= bound[worst], (
        f"{what}: element {worst} gpu={g[worst]!r} ref={r[worst]!r} err={err[worst]:.3e} bound={bound[worst]:.3e}")
    rn = np.linalg.norm(r)
    fro = np.linalg.norm(g - r) / rn if rn > 0 else np.linalg.norm(g - r)
    assert fro <= FRO_TOL, f"{what}: relative Frobenius error {fro:.3e} > {FRO_TOL}"


PASS_NAMES = {sd.FWD: "fwd", sd.DGRAD: "dgrad", sd.WGRAD: "wgrad"}


def check_all_passes(d, x: np.ndarray, w: np.ndarray, g: np.ndarray, tag: str, sample=None, seed=0, extra=None):
    """Runs fwd, dgrad, wgrad on the GPU and checks each against the oracle: the whole
    tensor when `sample` is None, else `sample` seeded output elements per pass plus the flat
    indices listed in extra[pass_id]."""
    from paper_1903_05831_amd import workloads
    od = oracle_desc(d)
    xd, wd, gd = to_dev(x), to_dev(w), to_dev(g)
    jobs = [(sd.FWD, xd, wd, oracle.conv2d_fwd, x, w),
            (sd.DGRAD, gd, wd, oracle.conv2d_dgrad, g, w),
            (sd.WGRAD, xd, gd, oracle.conv2d_wgrad, x, g)]
    for pass_id, a_dev, b_dev, ofn, a_np, b_np in jobs:
        what = f"{tag} {PASS_NAMES[pass_id]} [{sd.kernel_name(d, pass_id)}]"
        say(f"  run {what}")
        out = run_pass(d, pass_id, a_dev, b_dev)
        got = out.numpy()
        assert out.all_written(), f"{what}: some output elements were never written"
        if sample is None:
            compare(got, ofn(od, a_np, b_np), what)
        else:
            idx = workloads.sample_indices(got.size, sample, seed + pass_id)
            if extra and extra.get(pass_id):
                idx = np.unique(np.concatenate([idx, np.asarray(extra[pass_id], dtype=idx.dtype)]))
            compare(got.ravel()[idx], ofn(od, a_np, b_np, idx=idx), what + f" ({idx.size} samples)")


def check_fused(d, x: np.ndarray, w: np.ndarray, g: np.ndarray, tag: str, seed=0, fwd_opts=None, dgrad_opts=None):
    """Runs conv2d_fwd_fused and conv2d_dgrad_fused with seeded tails and checks the whole
    tensors against the fused-epilogue oracle (same bar as the plain passes).

    fwd_opts: subset of {"scale", "bias", "residual", "relu"}; dgrad_opts: subset of
    {"scale", "relu_mask"}; None = everything."""
    from oracle import epilogue as oep
    fwd_opts = {"scale", "bias", "residual", "relu"} if fwd_opts is None else set(fwd_opts)
    dgrad_opts = {"scale", "relu_mask"} if dgrad_opts is None else set(dgrad_opts)
    od = oracle_desc(d)
    ho, wo = sd.conv2d_out_shape(d)
    rng = np.random.default_rng(seed + 12345)
    stream = torch.cuda.current_stream().cuda_stream
    xd, wd, gd = to_dev(x), to_dev(w), to_dev(g)

    # forward: factors around 1 with both signs, a shortcut of the size of the output
    scale = (rng.standard_normal(d.K) * 0.5 + 1.0).astype(np.float32) if "scale" in fwd_opts else None
    bias = rng.standard_normal(d.K).astype(np.float32) if "bias" in fwd_opts else None
    res = rng.standard_normal((d.N, ho, wo, d.K)).astype(np.float16) if "residual" in fwd_opts else None
    relu = "relu" in fwd_opts
    what = f"{tag} fwd_fused{sorted(fwd_opts)} [{sd.kernel_name(d, sd.FWD)}]"
    say(f"  run {what}")
    out = GuardedOut((d.N, ho, wo, d.K), torch.float16)
    sd.conv2d_fwd_fused(d, xd, wd, out.view, workspace_for(d, sd.FWD), stream,
                        scale=None if scale is None else to_dev(scale), bias=None if bias is None else to_dev(bias),
                        residual=None if res is None else to_dev(res), relu=relu)
    torch.cuda.synchronize()
    out.check_guards()
    assert out.all_written(), f"{what}: some output elements were never written"
    compare(out.numpy(), oep.conv2d_fwd_fused(od, x, w, scale, bias, res, relu), what)

    # data gradient: the mask is an activation tensor, about half of it positive, some exact zeros
    dscale = (rng.standard_normal(d.C) * 0.5 + 1.0).astype(np.float32) if "scale" in dgrad_opts else None
    mask = None
    if "relu_mask" in dgrad_opts:
        mask = np.maximum(rng.standard_normal((d.N, d.H, d.W, d.C)), 0.0).astype(np.float16)
    what = f"{tag} dgrad_fused{sorted(dgrad_opts)} [{sd.kernel_name(d, sd.DGRAD)}]"
    say(f"  run {what}")
    out = GuardedOut((d.N, d.H, d.W, d.C), torch.float16)
    sd.conv2d_dgrad_fused(d, gd, wd, out.view, workspace_for(d, sd.DGRAD), stream,
                          scale=None if dscale is None else to_dev(dscale),
                          relu_mask=None if mask is None else to_dev(mask))
    torch.cuda.synchronize()
    out.check_guards()
    assert out.all_written(), f"{what}: some output elements were never written"
    got = out.numpy()
    compare(got, oep.conv2d_dgrad_fused(od, g, w, dscale, mask), what)
    if mask is not None:
        # the masked positions are decided on binary16 inputs: exact zeros, bit for bit
        assert not got[mask <= 0].view(np.uint16).any(), f"{what}: masked elements must be +0"
