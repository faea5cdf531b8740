"""Full-size parity on the benchmark configurations, in the launch configuration bench.py times
(tuned table on, default dispatch).

Whole tensors: every layer of configs 2-4 and the first instance of every layer shape that
config 5 adds (stem, the first res2 block, res3 blocks 1-3, the res5 head): all three passes
element by element against the fp64 oracle (dw of the six res5 shapes on 150 000 stratified
elements, see WGRAD_WHOLE_MAX_FLOP), then conv2d_fwd_fused / conv2d_dgrad_fused with
seeded tails against the oracle's tails applied to the same fp64 convolution results.

Stratified samples (at least 1e5 outputs per pass, see workloads.stratified_indices: one pixel
out of every 8 consecutive pixels of every stride-parity class, first / last / spread channels,
first and last pixel whole, every 8 x tap x 8 cell of dw; each sampled output is an independent
sum that the oracle computes exactly): the other layers of config 5 (same shapes as a layer
checked in full, other seeds) and every layer of the FPN / RPN shape set (6), plain passes and,
once per distinct shape of config 6, the fused calls."""
import time

import numpy as np
import pytest
import torch

import oracle
from oracle import epilogue as oep
import paper_1903_05831_amd as sd
from paper_1903_05831_amd import workloads

from gpu_harness import (GuardedOut, PASS_NAMES, compare, oracle_desc, run_pass, say, to_dev, workspace_for)

pytestmark = pytest.mark.gpu

# The oracle's weight gradient walks both operands with a stride per output element and runs at
# about 1 GFLOP/s on the 16 host threads of the GPU machine (the other two passes: 4-13): the six
# layers of the RoI head (53-118 GFLOP per pass) would take five minutes for dw alone, so their
# dw is checked on 150 000 stratified elements (6-29 % of the tensor, every 8 x tap x 8 cell
# hit); y and dx of those layers, and all three tensors of every other layer, are checked whole.
WGRAD_WHOLE_MAX_FLOP = 30e9


def _key(l):
    return (l.N, l.H, l.W, l.C, l.K, l.R, l.stride, l.pad)


def _plan():
    """(full, sampled, sampled_with_fused): lists of (cfg, layer index)."""
    full, sampled, fused = [], [], []
    seen = set()
    for cfg in (2, 3, 4):
        for li, l in enumerate(workloads.CONFIGS[cfg]):
            full.append((cfg, li))
            seen.add(_key(l))
    for li, l in enumerate(workloads.CONFIGS[5]):
        if _key(l) in seen:
            sampled.append((5, li))
        else:
            seen.add(_key(l))
            full.append((5, li))
    seen6 = set()
    for li, l in enumerate(workloads.CONFIGS[6]):
        (sampled if _key(l) in seen6 else fused).append((6, li))
        seen6.add(_key(l))
    return full, sampled, fused


FULL, SAMPLED, SAMPLED_FUSED = _plan()


def _tails(l, seed):
    """Seeded fused-tail operands of a layer: (scale[K], bias[K], residual like y, scale[C], mask like x)."""
    rng = np.random.default_rng(np.random.SeedSequence([workloads.BASE_SEED, 79, seed]))
    scale = (rng.standard_normal(l.K, dtype=np.float32) * np.float32(0.5) + np.float32(1.0))
    bias = rng.standard_normal(l.K, dtype=np.float32)
    res = rng.standard_normal(l.y_shape, dtype=np.float32).astype(np.float16)
    dscale = (rng.standard_normal(l.C, dtype=np.float32) * np.float32(0.5) + np.float32(1.0))
    mask = np.maximum(rng.standard_normal(l.x_shape, dtype=np.float32), np.float32(0)).astype(np.float16)
    return scale, bias, res, dscale, mask


def _run_fused(d, l, xd, wd, gd, tails):
    scale, bias, res, dscale, mask = tails
    st = torch.cuda.current_stream().cuda_stream
    y = GuardedOut(l.y_shape, torch.float16)
    sd.conv2d_fwd_fused(d, xd, wd, y.view, workspace_for(d, sd.FWD), st, scale=to_dev(scale), bias=to_dev(bias),
                        residual=to_dev(res), relu=True)
    dx = GuardedOut(l.x_shape, torch.float16)
    sd.conv2d_dgrad_fused(d, gd, wd, dx.view, workspace_for(d, sd.DGRAD), st, scale=to_dev(dscale),
                          relu_mask=to_dev(mask))
    torch.cuda.synchronize()
    for o in (y, dx):
        o.check_guards()
        assert o.all_written()
    return y.numpy(), dx.numpy()


def _layer(cfg, li):
    l = workloads.CONFIGS[cfg][li]
    d = sd.desc_of(l)
    say(f"config {cfg} layer {li} {l.name} {l.x_shape} -> {l.y_shape} R={l.R} s={l.stride}: "
        + ", ".join(sd.kernel_name(d, p) for p in (sd.FWD, sd.DGRAD, sd.WGRAD)))
    x, w, g = workloads.make_x(l, cfg, li), workloads.make_w(l, cfg, li), workloads.make_g(l, cfg, li)
    return l, d, x, w, g


@pytest.mark.parametrize("cfg,li", FULL, ids=lambda v: str(v))
def test_layer_whole_tensors_plain_and_fused(cfg, li):
    l, d, x, w, g = _layer(cfg, li)
    od = oracle_desc(d)
    xd, wd, gd = to_dev(x), to_dev(w), to_dev(g)
    tag = f"cfg{cfg}.{l.name}"
    tails = _tails(l, cfg * 100 + li)
    t_or = 0.0
    # GPU first (all five calls), then the oracle pass by pass, so that only one fp64 result is alive
    got = {p: run_pass(d, p, a, b) for p, a, b in ((sd.FWD, xd, wd), (sd.DGRAD, gd, wd), (sd.WGRAD, xd, gd))}
    for o in got.values():
        assert o.all_written(), f"{tag}: some output elements were never written"
    yf, dxf = _run_fused(d, l, xd, wd, gd, tails)
    del xd, wd, gd
    torch.cuda.empty_cache()
    scale, bias, res, dscale, mask = tails

    t0 = time.time(); ref = oracle.conv2d_fwd(od, x, w); t_or += time.time() - t0
    compare(got[sd.FWD].numpy(), ref, f"{tag} fwd")
    compare(yf, oep.fwd_tail(ref, od, scale, bias, res, True), f"{tag} fwd_fused")
    t0 = time.time(); ref = oracle.conv2d_dgrad(od, g, w); t_or += time.time() - t0
    compare(got[sd.DGRAD].numpy(), ref, f"{tag} dgrad")
    compare(dxf, oep.dgrad_tail(ref, od, dscale, mask), f"{tag} dgrad_fused")
    assert not dxf[mask <= 0].view(np.uint16).any(), f"{tag}: masked elements must be +0"
    dw = got[sd.WGRAD].numpy()
    if l.flops <= WGRAD_WHOLE_MAX_FLOP:
        t0 = time.time(); ref = oracle.conv2d_wgrad(od, x, g); t_or += time.time() - t0
        compare(dw, ref, f"{tag} wgrad")
        say(f"  whole tensors ok, oracle {t_or:.1f} s for {3 * l.flops / 1e9:.1f} GFLOP")
    else:
        idx = workloads.stratified_indices(l, sd.WGRAD, cfg * 100 + li, min_count=150_000)
        t0 = time.time(); ref = oracle.conv2d_wgrad(od, x, g, idx=idx); t_wg = time.time() - t0
        compare(dw.ravel()[idx], ref, f"{tag} wgrad ({idx.size} of {dw.size} elements)")
        say(f"  whole y and dx ok, oracle {t_or:.1f} s for {2 * l.flops / 1e9:.1f} GFLOP; "
            f"dw on {idx.size} of {dw.size} elements, oracle {t_wg:.1f} s")


def _sampled(cfg, li, fused):
    l, d, x, w, g = _layer(cfg, li)
    od = oracle_desc(d)
    xd, wd, gd = to_dev(x), to_dev(w), to_dev(g)
    tag = f"cfg{cfg}.{l.name}"
    seed = cfg * 100 + li
    jobs = [(sd.FWD, xd, wd, oracle.conv2d_fwd, x, w), (sd.DGRAD, gd, wd, oracle.conv2d_dgrad, g, w),
            (sd.WGRAD, xd, gd, oracle.conv2d_wgrad, x, g)]
    idxs = {}
    for p, a, b, ofn, an, bn in jobs:
        out = run_pass(d, p, a, b)
        assert out.all_written(), f"{tag}: some output elements were never written"
        idx = workloads.stratified_indices(l, p, seed)
        idxs[p] = idx
        compare(out.numpy().ravel()[idx], ofn(od, an, bn, idx=idx), f"{tag} {PASS_NAMES[p]} ({idx.size} samples)")
    if fused:
        tails = _tails(l, seed)
        scale, bias, res, dscale, mask = tails
        yf, dxf = _run_fused(d, l, xd, wd, gd, tails)
        i = idxs[sd.FWD]
        compare(yf.ravel()[i], oep.conv2d_fwd_fused(od, x, w, scale, bias, res, True, idx=i), f"{tag} fwd_fused")
        i = idxs[sd.DGRAD]
        compare(dxf.ravel()[i], oep.conv2d_dgrad_fused(od, g, w, dscale, mask, idx=i), f"{tag} dgrad_fused")
        assert not dxf[mask <= 0].view(np.uint16).any(), f"{tag}: masked elements must be +0"
    say(f"  samples ok: {', '.join(str(v.size) for v in idxs.values())}")
    torch.cuda.empty_cache()


@pytest.mark.parametrize("cfg,li", SAMPLED, ids=lambda v: str(v))
def test_repeated_layer_stratified_samples(cfg, li):
    _sampled(cfg, li, fused=False)


@pytest.mark.parametrize("cfg,li", SAMPLED_FUSED, ids=lambda v: str(v))
def test_second_shape_set_stratified_samples_plain_and_fused(cfg, li):
    _sampled(cfg, li, fused=True)


@pytest.mark.parametrize("batch", [1, 4])
@pytest.mark.parametrize("name", ["res2.0c", "res3.0b", "res3.1b", "res4.1a", "res4.1b", "res4.0p"])
def test_other_batch_sizes(name, batch):
    """The tuned table was measured at N = 2; N = 1 and N = 4 take the same entries (tile variant,
    pixel ranges of the weight gradient scaled with the batch): stratified samples, all passes."""
    import dataclasses
    li, l2 = next((i, l) for i, l in enumerate(workloads.CONFIGS[5]) if l.name == name)
    l = dataclasses.replace(l2, N=batch)
    d = sd.desc_of(l)
    assert sd.kernel_name(d, sd.FWD) == sd.kernel_name(sd.desc_of(l2), sd.FWD)
    say(f"{name} at N={batch}: " + ", ".join(sd.kernel_name(d, p) for p in (sd.FWD, sd.DGRAD, sd.WGRAD)))
    cfg = 70 + batch
    x, w, g = workloads.make_x(l, cfg, li), workloads.make_w(l, cfg, li), workloads.make_g(l, cfg, li)
    od = oracle_desc(d)
    xd, wd, gd = to_dev(x), to_dev(w), to_dev(g)
    for p, a, b, ofn, an, bn in ((sd.FWD, xd, wd, oracle.conv2d_fwd, x, w), (sd.DGRAD, gd, wd, oracle.conv2d_dgrad, g, w),
                                 (sd.WGRAD, xd, gd, oracle.conv2d_wgrad, x, g)):
        out = run_pass(d, p, a, b)
        assert out.all_written()
        idx = workloads.stratified_indices(l, p, cfg * 100 + li, min_count=50_000)
        compare(out.numpy().ravel()[idx], ofn(od, an, bn, idx=idx), f"{name} N={batch} {PASS_NAMES[p]}")
    torch.cuda.empty_cache()


def test_dgrad_zero_fill_and_determinism_res3_projection():
    """1x1 stride-2 projection (256->512 from 200x336): dx is +0 at every pixel no tap reaches,
    and two runs give identical bits for all three passes."""
    cfg, li = 3, 3
    l = workloads.CONFIGS[cfg][li]
    d = sd.desc_of(l)
    dev = torch.device("cuda")
    w = torch.from_numpy(workloads.make_w(l, cfg, li)).to(dev)
    g = torch.from_numpy(workloads.make_g(l, cfg, li)).to(dev)
    x = torch.from_numpy(workloads.make_x(l, cfg, li)).to(dev)
    st = torch.cuda.current_stream().cuda_stream
    need = max(sd.conv2d_workspace_bytes(d, p) for p in (sd.FWD, sd.DGRAD, sd.WGRAD))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    outs = []
    for rep in range(2):
        dx = torch.full(l.x_shape, float("nan"), dtype=torch.float16, device=dev)
        dw = torch.full(l.w_shape, float("nan"), dtype=torch.float32, device=dev)
        y = torch.full(l.y_shape, float("nan"), dtype=torch.float16, device=dev)
        sd.conv2d_fwd(d, x, w, y, ws, st)
        sd.conv2d_dgrad(d, g, w, dx, ws, st)
        sd.conv2d_wgrad(d, x, g, dw, ws, st)
        torch.cuda.synchronize()
        outs.append((y, dx, dw))
    dx = outs[0][1]
    mask = torch.ones(l.H, l.W, dtype=torch.bool, device=dev)
    mask[::2, ::2] = False
    untouched = dx[:, mask, :].view(torch.int16)
    assert bool((untouched == 0).all()), "positions without a tap must be +0"
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a.view(torch.int16 if a.dtype == torch.float16 else torch.int32),
                           b.view(torch.int16 if b.dtype == torch.float16 else torch.int32))
