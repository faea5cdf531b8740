"""Measures every kernel variant on every distinct layer of the benchmark workloads on the
GPU at hand and writes the winners to csrc/tuned_table.inc (rebuild the library afterwards).

    python -m paper_1903_05831_amd.tune [--configs 5] [--ms 10]

With SDCONV_TUNE=1 in the environment before the library's first call (set below) the dispatcher
reads SDCONV_IGEMM_VARIANT / SDCONV_WGRAD_VARIANT / SDCONV_WGRAD_SPLITS on every call, which is
how this script forces a variant.  Unlisted geometries keep using the built-in heuristics.

In a training step every layer finds its inputs in HBM, not in the 256 MB Infinity Cache: the
timed calls therefore rotate over enough copies of the layer's tensors (--cold-mib of
footprint, default 640) that no call sees data a recent call touched.  --cold-mib 0 times the
same tensors over and over (cache-warm).
"""
from __future__ import annotations

import argparse
import dataclasses
import os
import sys

import torch

os.environ["SDCONV_TUNE"] = "1"      # before the first library call: enables the override hooks

import paper_1903_05831_amd as sd
from paper_1903_05831_amd import workloads

FWD_DGRAD_VARIANTS = [101, 105, 107, 112, 113, 300, 303, 306, 310, 311, 312, 313, 314, 316, 317, 318, 319, 320, 321, 322, 323, 324, 401, 403, 404, 408, 411, 412, 414, 415, 416, 417, 418, 419, 420, 421, 422, 423, 424, 425, 426, 427, 428, 429, 430, 431, 432, 433, 434, 435]
# patch variants with a single patch buffer (the dispatcher hands them layers with 64 contraction channels only)
ONE_SLAB_VARIANTS = {422, 423, 424, 425, 426, 427, 433, 434}
WGRAD_VARIANTS = [100, 102, 104, 105, 107, 108, 109, 110, 112, 113, 114, 115, 116, 117, 118, 119, 120]
WGRAD_SPLITS = [1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16, 24, 32, 48, 64, 96, 128, 192, 256]
HERE = os.path.dirname(os.path.abspath(__file__))


def time_call(fn, ms_budget: float, ncopies: int = 1) -> float:
    """fn(i) runs the call on copy i of the inputs; returns milliseconds per call."""
    for i in range(2):
        fn(i % ncopies)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(); fn(0); e1.record(); torch.cuda.synchronize()
    t1 = max(e0.elapsed_time(e1), 1e-3)
    iters = max(3, min(500, int(ms_budget / t1)))
    iters = max(iters, min(ncopies, 64))
    best = 1e30
    k = 0
    for _ in range(2):
        e0.record()
        for _ in range(iters):
            fn(k % ncopies)
            k += 1
        e1.record(); torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / iters)
    return best


def time_pair(fn_a, fn_b, side, ms_budget: float, ncopies: int = 1) -> float:
    """Milliseconds per iteration of fn_a(i) on the current stream running beside fn_b(i) on the
    stream `side`, both free-running, joined at the end."""
    main = torch.cuda.current_stream()
    def run(iters, k0):
        for j in range(iters):
            fn_a((k0 + j) % ncopies)
            fn_b((k0 + j) % ncopies)
        main.wait_stream(side)
    side.wait_stream(main)
    run(2, 0)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(); run(2, 0); e1.record(); torch.cuda.synchronize()
    t1 = max(e0.elapsed_time(e1) / 2, 1e-3)
    iters = max(3, min(300, int(ms_budget / t1)))
    iters = max(iters, min(ncopies, 48))
    best = 1e30
    k = 0
    for _ in range(2):
        side.wait_stream(main)
        e0.record()
        run(iters, k)
        k += iters
        e1.record(); torch.cuda.synchronize()
        best = min(best, e0.elapsed_time(e1) / iters)
    return best


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", type=str, default="1,2,3,4,5")
    ap.add_argument("--ms", type=float, default=8.0)
    ap.add_argument("--layers", type=str, default="",
                    help="comma-separated name fragments: tune only matching layers (a partial table, for experiments)")
    ap.add_argument("--fwd-dgrad-only", action="store_true", help="skip the weight-gradient search")
    ap.add_argument("--wgrad-only", action="store_true",
                    help="search the weight gradient only; the data gradient beside it runs the variant of the "
                         "table built into the library (use with --keep)")
    ap.add_argument("--out", type=str, default=os.path.join(HERE, "csrc", "tuned_table.inc"))
    ap.add_argument("--wgrad-solo", action="store_true",
                    help="pick the weight-gradient variant by its time alone instead of beside the data gradient")
    ap.add_argument("--keep", type=str, default="",
                    help="an existing table: its entries for geometries not tuned in this run are kept in the output")
    ap.add_argument("--cold-mib", type=int, default=640,
                    help="rotate over copies of the inputs with this total footprint (0: one copy, cache-warm)")
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    st = torch.cuda.current_stream().cuda_stream
    side = torch.cuda.Stream()
    st2 = side.cuda_stream
    if not args.wgrad_only:
        os.environ["SDCONV_NO_TUNED_TABLE"] = "1"
    seen = set()
    lines = []
    for cfg in [int(c) for c in args.configs.split(",")]:
        for l in workloads.CONFIGS[cfg]:
            key = (l.N, l.H, l.W, l.C, l.K, l.R, l.S, l.stride, l.pad, l.dil)
            if l.C % 8 == 0 and l.K % 8:
                # such a layer runs as one with the filter count rounded up to a multiple of 8 (the
                # padded-filter-count route of the dispatcher): that inner layer is what gets tuned
                l = dataclasses.replace(l, name=l.name + "+pad", K=(l.K + 7) // 8 * 8)
                key = (l.N, l.H, l.W, l.C, l.K, l.R, l.S, l.stride, l.pad, l.dil)
            if key in seen or l.C % 8 or l.K % 8:
                continue
            if args.layers and not any(f in l.name for f in args.layers.split(",")):
                continue
            seen.add(key)
            d = sd.desc_of(l)
            foot = 2 * (l.N * l.H * l.W * l.C + l.K * l.R * l.S * l.C + l.N * l.Ho * l.Wo * l.K)
            nc = 1 if args.cold_mib <= 0 else max(1, min(48, -(-(args.cold_mib << 20) // foot)))
            xs = [torch.randn(l.x_shape, device=dev, dtype=torch.float16) for _ in range(nc)]
            wts = [torch.randn(l.w_shape, device=dev, dtype=torch.float16) * 0.05 for _ in range(nc)]
            gs = [torch.randn(l.y_shape, device=dev, dtype=torch.float16) for _ in range(nc)]
            y = torch.empty(l.y_shape, device=dev, dtype=torch.float16)
            dx = torch.empty(l.x_shape, device=dev, dtype=torch.float16)
            dw = torch.empty(l.w_shape, device=dev, dtype=torch.float32)
            geom = f"{l.N},{l.H},{l.W},{l.C},{l.K},{l.R},{l.S},{l.stride},{l.stride},{l.pad},{l.pad},{l.dil},{l.dil}"
            best_dgrad = None
            for pid, pname in (() if args.wgrad_only else ((sd.FWD, "fwd"), (sd.DGRAD, "dgrad"))):
                results = []
                for v in FWD_DGRAD_VARIANTS:
                    os.environ["SDCONV_IGEMM_VARIANT"] = str(v)
                    if v >= 400 and "patch" not in sd.kernel_name(d, pid):
                        continue        # the patch kernels take stride-1 3x3-class layers only
                    if v in ONE_SLAB_VARIANTS and (l.C if pid == sd.FWD else l.K) != 64:
                        continue        # one patch buffer: a single 64-channel slab on the contraction side
                    ws = torch.empty(max(sd.conv2d_workspace_bytes(d, pid), 256), dtype=torch.uint8, device=dev)
                    if pid == sd.FWD:
                        fn = lambda i: sd.conv2d_fwd(d, xs[i], wts[i], y, ws, st)
                    else:
                        fn = lambda i: sd.conv2d_dgrad(d, gs[i], wts[i], dx, ws, st)
                    results.append((time_call(fn, args.ms, nc), v))
                os.environ.pop("SDCONV_IGEMM_VARIANT")
                t, v = min(results)
                if pid == sd.DGRAD:
                    best_dgrad = v
                print(f"{l.name:9s} {pname:5s} best variant {v} {t*1e3:8.1f} us {l.flops/t/1e9:7.1f} TF/s   "
                      + " ".join(f"{vv}:{tt*1e3:.0f}" for tt, vv in results), flush=True)
                lines.append(f"    {{{geom}, {pid}, {v}, 0}},  // {l.name} {pname} {t*1e3:.1f} us")
            if args.fwd_dgrad_only:
                continue
            # The weight gradient of a layer runs beside its data gradient on a second stream in a
            # training step: what counts is how long the pair takes, which favours variants that
            # leave compute units and bandwidth to the other kernel.
            results = []
            if best_dgrad is not None:
                os.environ["SDCONV_IGEMM_VARIANT"] = str(best_dgrad)
            ws_d = torch.empty(max(sd.conv2d_workspace_bytes(d, sd.DGRAD), 256), dtype=torch.uint8, device=dev)
            fn_d = lambda i: sd.conv2d_dgrad(d, gs[i], wts[i], dx, ws_d, st)
            for wv in WGRAD_VARIANTS:
                os.environ["SDCONV_WGRAD_VARIANT"] = str(wv)
                best_t, worse = 1e30, 0
                for sp in WGRAD_SPLITS:
                    os.environ["SDCONV_WGRAD_SPLITS"] = str(sp)
                    need = sd.conv2d_workspace_bytes(d, sd.WGRAD)
                    if need > (1 << 30):
                        break
                    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
                    if args.wgrad_solo:
                        t = time_call(lambda i: sd.conv2d_wgrad(d, xs[i], gs[i], dw, ws, st), args.ms, nc)
                    else:
                        t = time_pair(fn_d, lambda i: sd.conv2d_wgrad(d, xs[i], gs[i], dw, ws, st2), side, args.ms, nc)
                    results.append((t, wv, sp))
                    if t < best_t:
                        best_t, worse = t, 0
                    else:
                        worse += 1
                        if worse >= 4:
                            break
            os.environ.pop("SDCONV_IGEMM_VARIANT", None)
            os.environ.pop("SDCONV_WGRAD_SPLITS", None)
            os.environ.pop("SDCONV_WGRAD_VARIANT", None)
            t, wv, sp = min(results)
            per_variant = {}
            for tt, vv, ss in results:
                if vv not in per_variant or tt < per_variant[vv][0]:
                    per_variant[vv] = (tt, ss)
            what = "alone" if args.wgrad_solo else "dgrad+wgrad pair"
            print(f"{l.name:9s} wgrad best variant {wv} splits {sp} {t*1e3:8.1f} us ({what})   "
                  + " ".join(f"{vv}:{tt*1e3:.0f}@{ss}" for vv, (tt, ss) in sorted(per_variant.items())), flush=True)
            lines.append(f"    {{{geom}, {sd.WGRAD}, {wv}, {sp}}},  // {l.name} wgrad {t*1e3:.1f} us {what}")
            del xs, wts, gs, y, dx, dw
            torch.cuda.empty_cache()
    if args.keep:
        def geom_and_pass(ln):      # "{N,...,dw, pass, variant, splits}, // ..." -> "{N,...,dw, pass"
            return ln.split("},")[0].rsplit(",", 2)[0].strip()
        fresh = {geom_and_pass(ln) for ln in lines}
        kept = []
        for ln in open(args.keep):
            if not ln.lstrip().startswith("{"):
                continue
            if geom_and_pass(ln) not in fresh:
                kept.append(ln.rstrip("\n"))
        lines = kept + lines
    with open(args.out, "w") as f:
        f.write("// Written by tune.py on %s: {N,H,W,C,K,R,S,sh,sw,ph,pw,dh,dw, pass, variant, splits}\n"
                % torch.cuda.get_device_name(0))
        f.write("\n".join(lines) + "\n")
    print("wrote", args.out, len(lines), "entries")
    return 0


if __name__ == "__main__":
    sys.exit(main())
