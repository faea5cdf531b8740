#!/usr/bin/env python3
"""Benchmark of the mixed-precision convolution hot path on one MI355X.

One step = one pass of the whole path over the full ResNet-50-C4 Faster R-CNN conv
workload (N=2 images of 800x1344 plus 512 RoIs; 53 conv layers), in the order of a training
step: conv2d_fwd for every layer first to last, then last to first conv2d_dgrad and
conv2d_wgrad of each layer, then grad_unscale_check over all 23 454 912 fp32 weight-gradient
elements.  The two gradients of a layer depend only on the incoming gradient, not on each
other, and the weight gradients of different layers do not depend on one another: with
--streams 3 (default) the weight gradients are dealt in turn to two side HIP streams (default
priority, a workspace each; the projection shortcuts go to the first of them), each gated by
an event so that it starts only when the gradient it consumes exists; --streams 2 uses one
side stream, --streams 1 keeps everything on one stream.  Inputs are synthetic (N(0,1) activations and gradients, He-normal weights), generated
on the device before the timed region.

Prints ONE JSON line.  `value` is algorithmic TFLOP/s of the whole step (2*N*Ho*Wo*K*R*S*C
per pass and layer).  `roofline` is for the kernel with the largest share of the step,
timed with HIP events on the launch stream in a second, single-stream pass over the same calls.  `cpu_baseline` times the fp64 CPU oracle on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_F16_TFLOPS = 2516.6     # 256 CUs x 4096 FLOP/clk x 2.4 GHz, dense fp16 MFMA
PEAK_HBM_GBS = 8000.0
CONFIG_ID = 5
LOSS_SCALE = 1024.0


KERNEL_SOURCES = ("igemm_ws.hip", "igemm_epilogue.h", "dma.h", "lds_tr.h", "igemm.h", "common.h")


def kernel_source_hash() -> str:
    """sha256 over the sources of the dominant (split-role implicit-GEMM) kernel: measured HBM
    traffic in profiles/ is only quoted while it belongs to the code that is being timed."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_1903_05831_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def device_clock_mhz() -> float:
    """Peak engine clock the HIP runtime reports for device 0 (hipDeviceAttributeClockRate, kHz)."""
    import ctypes
    try:
        hip = ctypes.CDLL("libamdhip64.so")
        v = ctypes.c_int(0)
        if hip.hipDeviceGetAttribute(ctypes.byref(v), 5, 0) != 0:      # 5 = hipDeviceAttributeClockRate
            return 0.0
        return v.value / 1e3
    except OSError:
        return 0.0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--streams", type=int, default=3, choices=(1, 2, 3, 4),
                    help="2: weight gradients on a second stream, overlapping the data gradients; "
                         "3, 4: weight gradients dealt in turn to two or three side streams")
    ap.add_argument("--core-only", action="store_true",
                    help="only the timed step and its per-kernel pass (for profiler runs): skip the fused-epilogue, "
                         "second-workload and FP32 sections, whose launches would mix into the kernel statistics")
    ap.add_argument("--layer", type=str, default="",
                    help="run only this layer of the workload (with --passes), 20 times, and print its time: for "
                         "per-kernel hardware-counter runs")
    ap.add_argument("--passes", type=str, default="fwd", help="with --layer: comma-separated fwd,dgrad,wgrad")
    ap.add_argument("--detail", type=str, default="", help="write per-layer timings (JSON) to this file")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="run one plain streaming kernel over this many MiB first (a known-size reference "
                         "dispatch for scaling FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--traffic-file", type=str, default=os.path.join(ROOT, "profiles", "dominant_kernel_traffic.json"),
                    help="measured HBM traffic per launch of the dominant kernel (from the pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        return 2

    import torch
    import paper_1903_05831_amd as sd
    from paper_1903_05831_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    sd.lib()   # fail loudly when the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    main_stream = torch.cuda.current_stream()
    stream = main_stream.cuda_stream
    side_streams = [torch.cuda.Stream() for _ in range(args.streams - 1)]      # default priority
    side_stream = side_streams[0] if side_streams else None
    stream2 = side_stream.cuda_stream if side_stream is not None else stream
    layers = workloads.CONFIGS[CONFIG_ID]

    if args.calib_copy_mib > 0:
        src = torch.ones(args.calib_copy_mib << 18, dtype=torch.float32, device=dev)   # MiB / 4 B
        dst = torch.empty_like(src)
        torch.neg(src, out=dst)      # an elementwise kernel: reads N MiB, writes N MiB (copy_ would use a DMA engine)
        torch.cuda.synchronize()
        del src, dst

    # ---- device-resident synthetic inputs --------------------------------------------------
    gen = torch.Generator(device=dev)
    gen.manual_seed(workloads.BASE_SEED)
    dw_total = sum(l.dw_numel for l in layers)
    dw_flat = torch.empty(dw_total, dtype=torch.float32, device=dev)
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    ws_bytes = 256
    jobs = []
    off = 0
    for l in layers:
        d = sd.desc_of(l)
        x = torch.randn(l.x_shape, generator=gen, device=dev, dtype=torch.float32).half()
        w = (torch.randn(l.w_shape, generator=gen, device=dev, dtype=torch.float32)
             * (2.0 / (l.R * l.S * l.C)) ** 0.5).half()
        g = torch.randn(l.y_shape, generator=gen, device=dev, dtype=torch.float32).half()
        y = torch.empty(l.y_shape, dtype=torch.float16, device=dev)
        dx = torch.empty(l.x_shape, dtype=torch.float16, device=dev)
        dw = dw_flat[off:off + l.dw_numel]
        off += l.dw_numel
        for pid in (sd.FWD, sd.DGRAD, sd.WGRAD):
            ws_bytes = max(ws_bytes, sd.conv2d_workspace_bytes(d, pid))
        jobs.append((l, d, x, w, g, y, dx, dw))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    side_ws = [torch.empty(ws_bytes, dtype=torch.uint8, device=dev) for _ in side_streams]   # one workspace per stream
    ws2 = side_ws[0] if side_ws else ws
    inv_scale = 1.0 / LOSS_SCALE

    # (layer, pass name, kernel name, flops, closure(workspace, stream)) in training order:
    # forward first to last, then backward last to first
    calls = []
    for (l, d, x, w, g, y, dx, dw) in jobs:
        calls.append((l, "fwd", sd.kernel_name(d, sd.FWD), l.flops,
                      lambda wsp, st, d=d, x=x, w=w, y=y: sd.conv2d_fwd(d, x, w, y, wsp, st)))
    for (l, d, x, w, g, y, dx, dw) in reversed(jobs):
        calls.append((l, "dgrad", sd.kernel_name(d, sd.DGRAD), l.flops,
                      lambda wsp, st, d=d, g=g, w=w, dx=dx: sd.conv2d_dgrad(d, g, w, dx, wsp, st)))
        calls.append((l, "wgrad", sd.kernel_name(d, sd.WGRAD), l.flops,
                      lambda wsp, st, d=d, x=x, g=g, dw=dw: sd.conv2d_wgrad(d, x, g, dw, wsp, st)))

    def unscale():
        sd.grad_unscale_check(dw_flat, dw_total, inv_scale, flag, stream)

    if args.layer:
        sel = [c for c in calls if c[0].name == args.layer and c[1] in args.passes.split(",")]
        if not sel:
            print("bench.py: no such layer / pass", file=sys.stderr)
            return 2
        out = []
        for c in sel:
            for _ in range(3):
                c[4](ws, stream)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                c[4](ws, stream)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 20
            out.append({"layer": c[0].name, "pass": c[1], "kernel": c[2], "us": ms * 1e3, "tflops": c[3] / ms / 1e9})
        print(json.dumps({"single_layer": out}))
        return 0

    # Schedule of one step on the main and the side streams, with the dependencies a training step has:
    #  - forward: the projection shortcut (".0p") of a stage's first block only needs the block
    #    input, so it runs on the side stream next to the 0a-0b-0c branch; the next block waits
    #    for both;
    #  - backward: a layer's weight gradient needs the gradient of the layer's output, which the
    #    data gradient issued just before it on the main stream produces: an event recorded
    #    there gates the side stream that takes it (they take turns), so wgrad(l) runs beside
    #    dgrad(l) and the weight gradients of its neighbours, and never before its input exists.  The shortcut's two gradients run on the side stream; the layer before
    #    the block waits for both branches.
    n_l = len(jobs)
    fwd_calls = calls[:n_l]
    bwd_calls = calls[n_l:]             # dgrad, wgrad pairs, last layer first
    ev_pool = [torch.cuda.Event() for _ in range(2 * n_l + 16)] if side_stream is not None else []

    def step():
        if side_stream is None:
            for c in calls:
                c[4](ws, stream)
            unscale()
            return
        ei = 0
        pending_p = None                # event of a shortcut conv still running on the side stream
        e_in = None
        for c in fwd_calls:
            name = c[0].name
            if name.endswith(".0a"):
                e_in = ev_pool[ei]; ei += 1
                e_in.record(main_stream)                    # block input is ready
            if name.endswith(".0p"):
                side_stream.wait_event(e_in)
                c[4](ws2, stream2)
                pending_p = ev_pool[ei]; ei += 1
                pending_p.record(side_stream)
                continue
            if pending_p is not None:                       # first layer after the block: needs both branches
                main_stream.wait_event(pending_p)
                pending_p = None
            c[4](ws, stream)
        e_dy = ev_pool[ei]; ei += 1
        e_dy.record(main_stream)                            # "the gradient the next layer consumes is ready"
        turn = 0
        for i in range(0, len(bwd_calls), 2):
            cd, cw = bwd_calls[i], bwd_calls[i + 1]
            name = cd[0].name
            if name.endswith(".0p"):
                side_stream.wait_event(e_dy)
                cd[4](ws2, stream2)
                cw[4](ws2, stream2)
                pending_p = ev_pool[ei]; ei += 1
                pending_p.record(side_stream)
                continue
            wst = side_streams[turn % len(side_streams)]    # weight gradients take the side streams in turn
            wst.wait_event(e_dy)
            cw[4](side_ws[turn % len(side_streams)], wst.cuda_stream)
            turn += 1
            cd[4](ws, stream)
            if name.endswith(".0a") and pending_p is not None:
                main_stream.wait_event(pending_p)           # block-input gradient = branch + shortcut
                pending_p = None
            e_dy = ev_pool[ei]; ei += 1
            e_dy.record(main_stream)
        for st in side_streams:
            main_stream.wait_stream(st)                     # all weight gradients done before the unscale
        unscale()
        for st in side_streams:
            st.wait_stream(main_stream)                     # the next step follows this unscale

    flops_per_step = 3 * sum(l.flops for l in layers)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = flops_per_step / (ms_per_step * 1e-3) / 1e12

    # ---- per-call HIP-event timing (second pass over the same steps) ---------------------------
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(len(calls) + 1)] for _ in range(args.steps)]
    for s in range(args.steps):
        for i, c in enumerate(calls):
            ev[s][i][0].record()
            c[4](ws, stream)
            ev[s][i][1].record()
        ev[s][-1][0].record()
        unscale()
        ev[s][-1][1].record()
    torch.cuda.synchronize()
    groups = {}
    per_call = []
    for i, c in enumerate(calls):
        ms = sum(ev[s][i][0].elapsed_time(ev[s][i][1]) for s in range(args.steps)) / args.steps
        # the layer's own roofline: min(matrix peak, arithmetic intensity x HBM peak) on the bytes
        # every tensor moves once
        cbytes = c[0].compulsory_bytes(c[1])
        roof = min(PEAK_F16_TFLOPS, c[3] / cbytes * PEAK_HBM_GBS / 1e3)
        per_call.append({"layer": c[0].name, "pass": c[1], "kernel": c[2], "us": ms * 1e3,
                         "tflops": c[3] / ms / 1e9, "pct_peak": 100 * c[3] / ms / 1e9 / PEAK_F16_TFLOPS,
                         "flop_per_byte": c[3] / cbytes, "roof_tflops": roof,
                         "pct_of_roof": 100 * c[3] / ms / 1e9 / roof, "GBps": cbytes / ms / 1e6})
        gk = groups.setdefault(c[2], {"ms": 0.0, "flops": 0.0, "launches": 0, "pass": c[1], "bytes": 0.0})
        gk["ms"] += ms
        gk["flops"] += c[3]
        gk["bytes"] += c[0].compulsory_bytes(c[1])
        gk["launches"] += 1
    unscale_ms = sum(ev[s][-1][0].elapsed_time(ev[s][-1][1]) for s in range(args.steps)) / args.steps
    instrumented_ms = sum(g["ms"] for g in groups.values()) + unscale_ms

    # dominant kernel: largest share of the step among the calls that are exactly one kernel per
    # event pair: every forward call but the stem's, and the data-gradient calls of the split-role
    # and patch kernels (the older data-gradient path and the weight gradient launch a filter copy
    # or a reduction beside their main kernel)
    def single_kernel(name, g):
        if g["pass"] == "fwd":
            return not name.startswith(("thin", "padk"))
        return g["pass"] == "dgrad" and ("_ws_" in name or "patch" in name) and not name.startswith("padk")
    try:
        with open(args.traffic_file) as f:
            traffic_entries = json.load(f)
        if isinstance(traffic_entries, dict):
            traffic_entries = [traffic_entries]
    except (OSError, ValueError):
        traffic_entries = []

    src_hash = kernel_source_hash()

    def roofline_of(name, g):
        avg_ms = g["ms"] / g["launches"]
        fl = g["flops"] / g["launches"]
        r = {"kernel": name, "bound": "mfma", "achieved": fl / avg_ms / 1e9, "peak": PEAK_F16_TFLOPS,
             "unit": "TFLOP/s", "frac": fl / avg_ms / 1e9 / PEAK_F16_TFLOPS, "traffic": None,
             "avg_launch_us": avg_ms * 1e3, "launches_per_step": g["launches"], "ms_per_step": g["ms"],
             "flop_per_launch": fl, "algorithmic_bytes_per_launch": g["bytes"] / g["launches"]}
        for tr in traffic_entries:
            if tr.get("kernel") == name:
                if tr.get("source_hash") == src_hash:
                    r["traffic"] = tr.get("hbm_bytes_per_launch")
                    r["traffic_note"] = tr.get("note")
                else:
                    r["traffic_note"] = ("measured traffic on file belongs to kernel sources %s, the library is built "
                                         "from %s: not quoted" % (tr.get("source_hash"), src_hash))
        return r
    ranked = sorted(((k, g) for k, g in groups.items() if single_kernel(k, g)), key=lambda kv: -kv[1]["ms"])
    roofline = roofline_of(*ranked[0])
    roofline["next_kernels"] = [roofline_of(k, g) for k, g in ranked[1:3]]
    unscale_gbs = 8.0 * dw_total / unscale_ms / 1e6

    # every call against its own roofline min(matrix peak, arithmetic intensity x 8 TB/s), summed by
    # which of the two bounds it: time the calls would take at their rooflines / time they took
    own_roof = {}
    for kind, sel in (("hbm_bound", lambda p: p["roof_tflops"] < PEAK_F16_TFLOPS),
                      ("mfma_bound", lambda p: p["roof_tflops"] >= PEAK_F16_TFLOPS)):
        ps = [p for p in per_call if sel(p)]
        t_us = sum(p["us"] for p in ps)
        t_roof_us = sum(p["us"] * p["pct_of_roof"] / 100 for p in ps)
        own_roof[kind] = {"calls": len(ps), "ms": t_us / 1e3, "ms_at_roofline": t_roof_us / 1e3,
                          "pct_of_own_roof": 100 * t_roof_us / t_us if t_us else None,
                          "GBps": sum(p["GBps"] * p["us"] for p in ps) / t_us if t_us else None,
                          "tflops": sum(p["tflops"] * p["us"] for p in ps) / t_us if t_us else None}
    own_roof["what"] = ("one-stream pass with an event pair per call (each pair adds ~3 us); roofline of a call = "
                        "min(2516.6 TFLOP/s, FLOP / bytes of each tensor once x 8 TB/s); time-weighted")

    # ---- side figures ---------------------------------------------------------------------------
    # the nominal "~25M" gradient buffer of the workload description (24 * 2^20 elements)
    # cold: six distinct buffers in rotation (604 MB, more than the 256 MB Infinity Cache holds);
    # hot: one buffer over and over (it fits that cache, so the rate can exceed the HBM's)
    n_nom = 24 << 20
    g_noms = [torch.randn(n_nom, dtype=torch.float32, device=dev) for _ in range(6)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for b in g_noms:
        sd.grad_unscale_check(b, n_nom, inv_scale, flag, stream)
    e0.record()
    for _ in range(2):
        for b in g_noms:
            sd.grad_unscale_check(b, n_nom, inv_scale, flag, stream)
    e1.record()
    torch.cuda.synchronize()
    nom_ms = e0.elapsed_time(e1) / 12
    e0.record()
    for _ in range(6):
        sd.grad_unscale_check(g_noms[0], n_nom, inv_scale, flag, stream)
    e1.record()
    torch.cuda.synchronize()
    nom_hot_ms = e0.elapsed_time(e1) / 6
    del g_noms
    # the optimizer tail that follows the check (not part of `value`): dynamic unscale, then the
    # SGD-momentum update with the fp16 weight cast and the loss-scale transition, on the
    # workload's 23 454 912 weights
    mw = torch.randn(dw_total, dtype=torch.float32, device=dev) * 0.05
    mbuf = torch.zeros(dw_total, dtype=torch.float32, device=dev)
    w16 = torch.empty(dw_total, dtype=torch.float16, device=dev)
    ls_state = torch.tensor([1149239296, 0], dtype=torch.int32, device=dev)     # {scale = 1024.0f, good_steps = 0}

    def tail():
        sd.grad_unscale_check_dynamic(dw_flat, dw_total, ls_state, flag, stream)
        sd.sgd_momentum_update(mw, mbuf, dw_flat, w16, dw_total, 0.02, 0.9, 1e-4, flag, ls_state,
                               2.0, 0.5, 2000, stream)
    dw_flat.normal_()
    for _ in range(2):
        tail()
    e0.record()
    for _ in range(5):
        tail()
    e1.record()
    torch.cuda.synchronize()
    tail_ms = e0.elapsed_time(e1) / 5
    del mw, mbuf, w16
    fused_ms = second = None
    second_ms = second_flops = f32_ms = f16_ms = f32_flops = 0
    tail_bytes_fwd = tail_bytes_dg = 0
    if not args.core_only:
        # ---- fused epilogues: forward and data-gradient chains of the whole network, one stream -----
        # every layer gets the tail it has in a residual network with frozen batch normalisation:
        # affine + ReLU (stem, a, b), affine + shortcut + ReLU (c), affine only (projection p); the
        # data gradients get the scale and ReLU mask of the activation that feeds the layer.
        # Three ways: the plain pass, the fused call, the plain pass followed by a separate tail pass.
        def tail_of(l):
            if l.name.endswith("c"):
                return dict(residual=True, relu=True)
            if l.name.endswith("p"):
                return dict(residual=False, relu=False)
            return dict(residual=False, relu=True)
        vecs = {}
        for (l, d, x, w, g, y, dx, dw) in jobs:
            for n in (l.K, l.C):
                if n not in vecs and n % 8 == 0:
                    vecs[n] = (torch.rand(n, device=dev) + 0.5, torch.randn(n, device=dev))
        fwd_modes = {"plain": [], "fused": [], "separate": []}
        dg_modes = {"plain": [], "fused": [], "separate": []}
        tail_bytes_fwd = tail_bytes_dg = 0
        for (l, d, x, w, g, y, dx, dw) in jobs:
            t = tail_of(l)
            sc, bi = vecs[l.K]
            res = g if t["residual"] else None          # a tensor of y's shape stands in for the shortcut
            npix = l.N * l.Ho * l.Wo
            fwd_modes["plain"].append(lambda d=d, x=x, w=w, y=y: sd.conv2d_fwd(d, x, w, y, ws, stream))
            fwd_modes["fused"].append(lambda d=d, x=x, w=w, y=y, sc=sc, bi=bi, res=res, r=t["relu"]:
                                      sd.conv2d_fwd_fused(d, x, w, y, ws, stream, scale=sc, bias=bi, residual=res, relu=r))
            fwd_modes["separate"].append(lambda d=d, x=x, w=w, y=y, sc=sc, bi=bi, res=res, r=t["relu"], npix=npix, K=l.K:
                                         (sd.conv2d_fwd(d, x, w, y, ws, stream),
                                          sd.sdconv_tail_pass(y, npix, K, stream, scale=sc, bias=bi, residual=res, relu=r)))
            tail_bytes_fwd += 2 * y.numel() * (3 if t["residual"] else 2)
            if l.C % 8:
                continue                                 # the stem: no gradient with respect to the image
            scc = vecs[l.C][0]
            nin = l.N * l.H * l.W
            dg_modes["plain"].append(lambda d=d, g=g, w=w, dx=dx: sd.conv2d_dgrad(d, g, w, dx, ws, stream))
            dg_modes["fused"].append(lambda d=d, g=g, w=w, dx=dx, scc=scc, x=x:
                                     sd.conv2d_dgrad_fused(d, g, w, dx, ws, stream, scale=scc, relu_mask=x))
            dg_modes["separate"].append(lambda d=d, g=g, w=w, dx=dx, scc=scc, x=x, nin=nin, C=l.C:
                                        (sd.conv2d_dgrad(d, g, w, dx, ws, stream),
                                         sd.sdconv_tail_pass(dx, nin, C, stream, scale=scc, relu_mask=x)))
            tail_bytes_dg += 2 * dx.numel() * 3

        def time_chain(fns, reps=3):
            for f in fns:
                f()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                for f in fns:
                    f()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        fused_ms = {"fwd": {k: time_chain(v) for k, v in fwd_modes.items()},
                    "dgrad": {k: time_chain(v) for k, v in dg_modes.items()}}
        # ---- second shape set: what a ResNet-50-FPN Faster R-CNN adds (Table 1 of the paper quotes its
        # speed on that model): res5 on the image, FPN, RPN heads on P2-P6, box-head FCs, C4 RPN --------
        del fwd_modes, dg_modes
        torch.cuda.empty_cache()
        second = {}
        fns2, flops2 = {}, {}
        for l in workloads.CONFIGS[6]:
            d2 = sd.desc_of(l)
            x2 = torch.randn(l.x_shape, device=dev, dtype=torch.float32).half()
            w2 = (torch.randn(l.w_shape, device=dev, dtype=torch.float32) * (2.0 / (l.R * l.S * l.C)) ** 0.5).half()
            g2 = torch.randn(l.y_shape, device=dev, dtype=torch.float32).half()
            y2 = torch.empty(l.y_shape, dtype=torch.float16, device=dev)
            dx2 = torch.empty(l.x_shape, dtype=torch.float16, device=dev)
            dw2 = torch.empty(l.w_shape, dtype=torch.float32, device=dev)
            need = max(sd.conv2d_workspace_bytes(d2, pid) for pid in (sd.FWD, sd.DGRAD, sd.WGRAD))
            wsl = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
            grp = l.name.split(".")[0]
            fns2.setdefault(grp, []).extend([
                lambda d2=d2, x2=x2, w2=w2, y2=y2, wsl=wsl: sd.conv2d_fwd(d2, x2, w2, y2, wsl, stream),
                lambda d2=d2, g2=g2, w2=w2, dx2=dx2, wsl=wsl: sd.conv2d_dgrad(d2, g2, w2, dx2, wsl, stream),
                lambda d2=d2, x2=x2, g2=g2, dw2=dw2, wsl=wsl: sd.conv2d_wgrad(d2, x2, g2, dw2, wsl, stream)])
            flops2[grp] = flops2.get(grp, 0) + 3 * l.flops
        for grp, fns in fns2.items():
            ms = time_chain(fns)
            second[grp] = {"ms": ms, "gflop": flops2[grp] / 1e9, "tflops": flops2[grp] / ms / 1e9}
        second_ms = sum(v["ms"] for v in second.values())
        second_flops = sum(flops2.values())
        del fns2
        torch.cuda.empty_cache()
        # ---- FP32 -> FP16 on this hardware (the form of Figure 1(b) of the paper): the same layers,
        # all three passes, through the single-precision companion path and through the mixed-
        # precision path, layer by layer on one stream (the C = 3 stem is left out: the companion
        # path takes channel counts in multiples of 4) -------------------------------------------------
        f32_ms = f16_ms = 0.0
        f32_flops = 0
        for (l, d, x, w, g, y, dx, dw) in jobs:
            if l.C % 4 or l.K % 4:
                continue
            need = max(sd.conv2d_workspace_bytes_f32(d, pid) for pid in (sd.FWD, sd.DGRAD, sd.WGRAD))
            ws32 = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
            x32, w32, g32 = x.float(), w.float(), g.float()
            y32, dx32, dw32 = torch.empty_like(g32), torch.empty_like(x32), torch.empty(l.w_shape, dtype=torch.float32, device=dev)
            f32_ms += time_chain([lambda: sd.conv2d_fwd_f32(d, x32, w32, y32, ws32, stream),
                                  lambda: sd.conv2d_dgrad_f32(d, g32, w32, dx32, ws32, stream),
                                  lambda: sd.conv2d_wgrad_f32(d, x32, g32, dw32, ws32, stream)], reps=2)
            f16_ms += time_chain([lambda: sd.conv2d_fwd(d, x, w, y, ws, stream),
                                  lambda: sd.conv2d_dgrad(d, g, w, dx, ws, stream),
                                  lambda: sd.conv2d_wgrad(d, x, g, dw, ws, stream)], reps=2)
            f32_flops += 3 * l.flops
            del x32, w32, g32, y32, dx32, dw32, ws32
        torch.cuda.empty_cache()

    # what the matrix pipes sustain with nothing else in the way (see sdconv_mfma_ceiling)
    props = torch.cuda.get_device_properties(dev)
    cus = props.multi_processor_count
    blocks, iters = 4 * cus, 4000
    scratch = torch.empty(blocks * 512, dtype=torch.float32, device=dev)
    sd.sdconv_mfma_ceiling(scratch, blocks, 50, stream)
    e0.record()
    sd.sdconv_mfma_ceiling(scratch, blocks, iters, stream)
    e1.record()
    torch.cuda.synchronize()
    ceiling_tflops = blocks * 8 * iters * 16 * 32768.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12
    del scratch
    # the stem's data gradient is never needed in training (there is no gradient w.r.t. the image)
    stem_dgrad_ms = sum(p["us"] for p in per_call if p["layer"] == "stem" and p["pass"] == "dgrad") / 1e3
    stem_flops = next(l.flops for l in layers if l.name == "stem")

    # ---- the named target layers: 3x3 convs of res3/res4 ----------------------------------------
    targets = [p for p in per_call if p["layer"].endswith("b") and p["layer"].startswith(("res3", "res4"))]
    tgt_flops = sum(next(l.flops for l in layers if l.name == p["layer"]) for p in targets)
    tgt_ms = sum(p["us"] for p in targets) / 1e3
    target_pct = 100 * tgt_flops / tgt_ms / 1e9 / PEAK_F16_TFLOPS if tgt_ms > 0 else None

    # One layer, each pass back to back between two events over `nc` copies of its tensors in
    # rotation: nc = 1 is cache-hot (the tensors of most layers fit the 256 MB Infinity Cache), a
    # footprint of 600 MB is cold (every call finds its inputs in HBM, as in a training step).
    def time_layer(l, cold):
        d = sd.desc_of(l)
        foot = 2 * (2 * l.N * l.H * l.W * l.C + 2 * l.N * l.Ho * l.Wo * l.K) + 2 * l.dw_numel
        nc = max(2, min(64, -(-(600 << 20) // foot))) if cold else 1
        xs = [torch.randn(l.x_shape, generator=gen, device=dev, dtype=torch.float32).half() for _ in range(nc)]
        gs = [torch.randn(l.y_shape, generator=gen, device=dev, dtype=torch.float32).half() for _ in range(nc)]
        wts = [(torch.randn(l.w_shape, generator=gen, device=dev, dtype=torch.float32)
                * (2.0 / (l.R * l.S * l.C)) ** 0.5).half() for _ in range(nc)]
        y = torch.empty(l.y_shape, dtype=torch.float16, device=dev)
        dx = torch.empty(l.x_shape, dtype=torch.float16, device=dev)
        dw = torch.empty(l.w_shape, dtype=torch.float32, device=dev)
        need = max(sd.conv2d_workspace_bytes(d, pid) for pid in (sd.FWD, sd.DGRAD, sd.WGRAD))
        wsl = ws if need <= ws.numel() else torch.empty(need, dtype=torch.uint8, device=dev)
        fns = {"fwd": lambda i: sd.conv2d_fwd(d, xs[i], wts[i], y, wsl, stream),
               "dgrad": lambda i: sd.conv2d_dgrad(d, gs[i], wts[i], dx, wsl, stream),
               "wgrad": lambda i: sd.conv2d_wgrad(d, xs[i], gs[i], dw, wsl, stream)}
        t = {}
        for pname, fn in fns.items():
            for i in range(max(nc, 3)):
                fn(i % nc)
            torch.cuda.synchronize()
            ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = max(3 * nc, 10)
            ea.record()
            for i in range(reps):
                fn(i % nc)
            eb.record()
            torch.cuda.synchronize()
            t[pname] = ea.elapsed_time(eb) / reps
        del xs, gs, wts, y, dx, dw
        torch.cuda.empty_cache()
        return t, nc

    # ---- configs 1-4 of the workload description, each as a whole: the three passes of its layers,
    # cold, summed (config 1 is one 0.23 GFLOP layer: a launch-latency figure, not a throughput one) ---
    per_config = []
    shape_times = {}
    if not args.core_only:
        for cfg in (1, 2, 3, 4):
            ms = fl = 0.0
            for l in workloads.CONFIGS[cfg]:
                key = (l.N, l.H, l.W, l.C, l.K, l.R, l.stride, l.pad)
                if key not in shape_times:
                    shape_times[key] = time_layer(l, cold=True)[0]
                ms += sum(shape_times[key].values())
                fl += 3 * l.flops
            per_config.append({"config": cfg, "workload": workloads.CONFIG_NAMES[cfg], "layers": len(workloads.CONFIGS[cfg]),
                               "gflop": fl / 1e9, "ms": ms, "tflops": fl / ms / 1e9,
                               "pct_fp16_mfma_peak": 100 * fl / ms / 1e9 / PEAK_F16_TFLOPS})

    # ---- hot and cold, side by side, for the layers whose arithmetic intensity puts them under the
    # HBM roofline (below 315 FLOP/B): one instance of every such shape of the workload ---------------
    hot_cold = []
    if not args.core_only:
        seen_hc = set()
        for l in layers:
            key = (l.N, l.H, l.W, l.C, l.K, l.R, l.stride, l.pad)
            if key in seen_hc or l.flops / l.compulsory_bytes("fwd") >= PEAK_F16_TFLOPS * 1e3 / PEAK_HBM_GBS:
                continue
            seen_hc.add(key)
            cold_t = shape_times.get(key) or time_layer(l, cold=True)[0]
            hot_t = time_layer(l, cold=False)[0]
            row = {"layer": l.name, "flop_per_byte": l.flops / l.compulsory_bytes("fwd")}
            for pname in ("fwd", "dgrad", "wgrad"):
                b = l.compulsory_bytes(pname)
                row[pname] = {"cold_us": cold_t[pname] * 1e3, "hot_us": hot_t[pname] * 1e3,
                              "cold_GBps": b / cold_t[pname] / 1e6, "hot_GBps": b / hot_t[pname] / 1e6,
                              "cold_pct_of_hbm_roof": 100 * b / cold_t[pname] / 1e6 / PEAK_HBM_GBS}
            hot_cold.append(row)

    # The target layers one by one, back to back between two events (no per-call event, which adds
    # ~3 us to a 15-30 us kernel), rotating over enough copies of the tensors that every call finds
    # its inputs in HBM.
    iso = {"fwd": [0.0, 0.0], "dgrad": [0.0, 0.0], "wgrad": [0.0, 0.0]}       # pass -> [ms, flops]
    iso_layers = []
    seen_geo = {}
    for l in layers:
        if not (l.name.endswith("b") and l.name.startswith(("res3", "res4"))):
            continue
        key = (l.N, l.H, l.W, l.C, l.K, l.R, l.stride)
        if key not in seen_geo:
            t, nc = time_layer(l, cold=True)
            seen_geo[key] = t
            iso_layers.append({"layer": l.name, "fwd_us": t["fwd"] * 1e3, "dgrad_us": t["dgrad"] * 1e3,
                               "wgrad_us": t["wgrad"] * 1e3, "copies": nc})
        for pname in iso:
            iso[pname][0] += seen_geo[key][pname]
            iso[pname][1] += l.flops
    iso_all_ms = sum(v[0] for v in iso.values())
    iso_all_fl = sum(v[1] for v in iso.values())
    isolated = {"what": "the ten 3x3 layers of res3 / res4, each pass timed back to back on rotating cold copies "
                        "(no event per call); % of the fp16 dense peak over fwd, dgrad, wgrad (incl. its reduction)",
                "pct_peak": {p: 100 * v[1] / v[0] / 1e9 / PEAK_F16_TFLOPS for p, v in iso.items()},
                "pct_peak_all": 100 * iso_all_fl / iso_all_ms / 1e9 / PEAK_F16_TFLOPS,
                "distinct_layers": iso_layers}

    out = {
        "metric": "conv TFLOP/s (fwd+dgrad+wgrad) on ResNet-50-C4 shapes; % fp16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "configs[4]: " + workloads.CONFIG_NAMES[CONFIG_ID],
                   "layers": len(layers), "gflop_per_step": flops_per_step / 1e9,
                   "passes": "fwd of all layers, then dgrad+wgrad last to first, then grad_unscale_check "
                             "on %d fp32" % dw_total,
                   "streams": args.streams, "loss_scale": LOSS_SCALE},
        "pct_fp16_mfma_peak": 100 * value / PEAK_F16_TFLOPS,
        "pct_peak_res3_res4_3x3": target_pct,
        "res3_res4_3x3_isolated": isolated,
        "roofline": roofline,
        "own_roofline": own_roof,
        "per_config": per_config or None,
        "hbm_bound_layers_hot_cold": hot_cold or None,
        "unscale": {"us": unscale_ms * 1e3, "GBps": unscale_gbs, "frac_hbm": unscale_gbs / PEAK_HBM_GBS,
                    "bytes": 8 * dw_total},
        "unscale_nominal_25M": {"elements": n_nom, "us": nom_ms * 1e3, "GBps": 8.0 * n_nom / nom_ms / 1e6,
                                "what": "cold: six buffers in rotation (604 MB); hot: one buffer repeated",
                                "hot_us": nom_hot_ms * 1e3, "hot_GBps": 8.0 * n_nom / nom_hot_ms / 1e6},
        "optimizer_tail": {"what": "grad_unscale_check_dynamic + sgd_momentum_update on %d weights" % dw_total,
                           "us": tail_ms * 1e3, "bytes": 30 * dw_total,
                           "GBps": 30.0 * dw_total / tail_ms / 1e6,
                           "frac_hbm": 30.0 * dw_total / tail_ms / 1e6 / PEAK_HBM_GBS},
        "fused_epilogue": None if args.core_only else {
            "what": "forward / data-gradient chains of all layers on one stream: plain pass, fused tail "
                    "(frozen-BN affine, shortcut on the c layers, ReLU; scale + ReLU mask in the data gradient), "
                    "plain pass + separate in-place tail pass",
            "fwd_ms": fused_ms["fwd"], "dgrad_ms": fused_ms["dgrad"],
            "separate_pass_algorithmic_bytes": {"fwd": tail_bytes_fwd, "dgrad": tail_bytes_dg}},
        "second_workload": None if args.core_only else {
            "workload": "config 6: " + workloads.CONFIG_NAMES[6],
            "what": "fwd + dgrad + wgrad of each layer, one stream, per group of layers",
            "layers": len(workloads.CONFIGS[6]), "ms": second_ms, "gflop": second_flops / 1e9,
            "tflops": second_flops / second_ms / 1e9, "groups": second},
        "fp32_vs_fp16": None if args.core_only else {
            "what": "fwd + dgrad + wgrad of the 52 layers after the stem, layer by layer on one stream: "
                    "conv2d_*_f32 (fp32 MFMA) against conv2d_* (fp16 MFMA, fp32 accumulation)",
            "fp32_ms": f32_ms, "fp16_ms": f16_ms, "speedup": f32_ms / f16_ms,
            "fp32_tflops": f32_flops / f32_ms / 1e9, "fp32_frac_of_peak": f32_flops / f32_ms / 1e9 / 157.3,
            "fp16_tflops": f32_flops / f16_ms / 1e9,
            "paper": "Fig. 1(b): 2.0x end to end (whole training step, hardware not stated)"},
        "device": {"name": props.name, "arch": getattr(props, "gcnArchName", ""), "compute_units": cus,
                   "clock_mhz": device_clock_mhz(), "rocm": torch.version.hip,
                   "mfma_only_tflops": ceiling_tflops, "mfma_only_frac_of_peak": ceiling_tflops / PEAK_F16_TFLOPS},
        "ms_per_step_with_events": instrumented_ms,
        "one_stream_events": {"tflops": flops_per_step / instrumented_ms / 1e9,
                              "tflops_without_stem_dgrad": (flops_per_step - stem_flops)
                              / (instrumented_ms - stem_dgrad_ms) / 1e9},
        "kernels": {k: {"ms_per_step": g["ms"], "launches": g["launches"],
                        "tflops": g["flops"] / g["ms"] / 1e9} for k, g in sorted(groups.items())},
        "paper_context": "Fig. 1(b): 2.0x FP32->FP16 end-to-end training speedup, hardware not stated",
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
        # GPU / oracle per config, on the part of each config the oracle was timed on
        by_cfg = {c["config"]: c for c in out["cpu_baseline"]["per_config"]}
        for c in per_config:
            o = by_cfg.get(c["config"])
            if o:
                c["oracle_gflops"] = o["gflops"]
                c["oracle_sample"] = o["sample"]
                c["gpu_over_oracle"] = c["tflops"] * 1e3 / o["gflops"]
        out["cpu_baseline"]["gpu_over_oracle_full_workload"] = value / out["cpu_baseline"]["value"]
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump(per_call, f, indent=1)
    print(json.dumps(out))
    return 0


def cpu_baseline() -> dict:
    """The CPU oracle as it stands, timed on a bounded sample of the workload: all three passes of
    every layer of the res4 trunk (configs[3]: 19 layers, 376.5 GFLOP, whole tensors, fp64) is the
    headline figure; configs[0] in full and the forward passes of configs[1] and [2] give a rate
    per configuration.  (configs[4] by distinct layer shape takes the oracle about five minutes,
    mostly in the weight gradients of the RoI head: tests/test_gpu_configs.py does that, not the
    benchmark.)"""
    import oracle
    from paper_1903_05831_amd import workloads

    def leg(cfg, passes):
        flops = 0
        seconds = 0.0
        for li, l in enumerate(workloads.CONFIGS[cfg]):
            x, w, g = workloads.make_x(l, cfg, li), workloads.make_w(l, cfg, li), workloads.make_g(l, cfg, li)
            d = oracle.make_desc(l.N, l.H, l.W, l.C, l.K, l.R, l.S, (l.stride,) * 2, (l.pad,) * 2, (l.dil,) * 2)
            t0 = time.perf_counter()
            if "fwd" in passes:
                oracle.conv2d_fwd(d, x, w)
            if "dgrad" in passes:
                oracle.conv2d_dgrad(d, g, w)
            if "wgrad" in passes:
                oracle.conv2d_wgrad(d, x, g)
            seconds += time.perf_counter() - t0
            flops += len(passes) * l.flops
        return flops, seconds

    all3 = ("fwd", "dgrad", "wgrad")
    per_config = []
    for cfg, passes, what in ((1, all3, "all three passes in full"), (2, ("fwd",), "forward passes in full"),
                              (3, ("fwd",), "forward passes in full"), (4, all3, "all three passes in full")):
        fl, sec = leg(cfg, passes)
        per_config.append({"config": cfg, "gflops": fl / sec / 1e9, "seconds": sec, "gflop": fl / 1e9, "sample": what})
    flops, seconds = per_config[-1]["gflop"] * 1e9, per_config[-1]["seconds"]
    return {"value": flops / seconds / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": seconds,
            "sample": "configs[3] (res4 trunk, 19 conv layers, N=2): fwd+dgrad+wgrad of every layer in full, "
                      "fp64, %.1f GFLOP" % (flops / 1e9),
            "per_config": per_config}


if __name__ == "__main__":
    sys.exit(main())
