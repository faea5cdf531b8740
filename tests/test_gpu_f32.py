"""GPU parity of the single-precision companion path (conv2d_*_f32) against the fp64 oracle on
the same binary32 inputs.

Tolerance: binary32 products are accumulated in binary32 in an order the kernel is free to
choose.  A sum of n terms of rms size t that is accumulated one term after the other has partial
sums of size sqrt(i) * t, each rounded with a relative error of up to 2^-24, so its error has an
rms of about 2^-24 * n * t / sqrt(2) -- and it does not shrink when the terms cancel, so it cannot
be bounded by a multiple of |ref|.  The bar per element is therefore
    2e-4 * (1 + |ref|) + 2^-23 * n * t
(n = contraction length of the pass: up to 4608 forward, 134 400 pixels in the weight gradient),
and 2e-5 in the Frobenius norm.  Every comparison prints the largest |err| / bound it saw, and
the largest |err| relative to the second term alone, so that the slack in the bar is visible."""
import numpy as np
import pytest
import torch

import oracle
import paper_1903_05831_amd as sd
from paper_1903_05831_amd import workloads

from gpu_harness import GuardedOut, oracle_desc, say, to_dev

pytestmark = pytest.mark.gpu

ELEM_TOL_F32 = 2e-4
FRO_TOL_F32 = 2e-5


def _compare(got, ref, what, nterms, term_rms):
    g, r = got.astype(np.float64).ravel(), ref.ravel()
    assert np.all(np.isfinite(g)), f"{what}: non-finite output"
    err = np.abs(g - r)
    bound = ELEM_TOL_F32 * (1 + np.abs(r)) + 2.0 ** -23 * nterms * term_rms
    worst = int(np.argmax(err - bound))
    rn = np.linalg.norm(r)
    fro = np.linalg.norm(g - r) / (rn if rn > 0 else 1.0)
    say(f"    {what}: max err/bound {float(np.max(err / bound)):.3f}, max err / (2^-23 n t) "
        f"{float(err.max() / (2.0 ** -23 * nterms * term_rms)):.3f}, Frobenius {fro:.2e} (bar {FRO_TOL_F32:.0e})")
    assert err[worst] <= bound[worst], f"{what}: element {worst} gpu={g[worst]!r} ref={r[worst]!r}"
    assert fro <= FRO_TOL_F32, f"{what}: Frobenius"


def _check(d, x, w, g, tag, sample=None, seed=0, layer=None):
    od = oracle_desc(d)
    ho, wo = sd.conv2d_out_shape(d)
    st = torch.cuda.current_stream().cuda_stream
    xd, wd, gd = to_dev(x), to_dev(w), to_dev(g)
    jobs = [(sd.FWD, sd.conv2d_fwd_f32, xd, wd, (d.N, ho, wo, d.K), oracle.conv2d_fwd_f32, x, w, d.R * d.S * d.C),
            (sd.DGRAD, sd.conv2d_dgrad_f32, gd, wd, (d.N, d.H, d.W, d.C), oracle.conv2d_dgrad_f32, g, w, d.R * d.S * d.K),
            (sd.WGRAD, sd.conv2d_wgrad_f32, xd, gd, (d.K, d.R, d.S, d.C), oracle.conv2d_wgrad_f32, x, g, d.N * ho * wo)]
    for pid, fn, a, b, shape, ofn, an, bn, nterms in jobs:
        term_rms = float(np.sqrt(np.mean(an.astype(np.float64) ** 2)) * np.sqrt(np.mean(bn.astype(np.float64) ** 2)))
        what = f"{tag} f32 pass {pid}"
        say(f"  run {what}")
        need = sd.conv2d_workspace_bytes_f32(d, pid)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
        out = GuardedOut(shape, torch.float32)
        fn(d, a, b, out.view, ws, st)
        torch.cuda.synchronize()
        out.check_guards()
        assert out.all_written(), f"{what}: some output elements were never written"
        got = out.numpy()
        if sample is None:
            _compare(got, ofn(od, an, bn), what, nterms, term_rms)
        else:
            idx = (workloads.stratified_indices(layer, pid, seed) if layer is not None
                   else workloads.sample_indices(got.size, sample, seed + pid))
            _compare(got.ravel()[idx], ofn(od, an, bn, idx=idx), what + f" ({idx.size} samples)", nterms, term_rms)


def _rand32(N, H, W, C, K, R, S, stride, pad, dil, seed):
    d = sd.make_desc(N, H, W, C, K, R, S, stride, pad, dil)
    ho, wo = sd.conv2d_out_shape(d)
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, H, W, C), dtype=np.float32)
    w = rng.standard_normal((K, R, S, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / (R * S * C)))
    g = rng.standard_normal((N, ho, wo, K), dtype=np.float32)
    return d, x, w, g


SMALL = [
    (1, 9, 11, 4, 4, 3, 3, (1, 1), (1, 1), (1, 1)),          # smallest channel counts
    (2, 10, 12, 8, 8, 1, 1, (1, 1), (0, 0), (1, 1)),
    (1, 12, 10, 24, 40, 3, 3, (2, 2), (1, 1), (1, 1)),       # strided: parity classes, ragged tiles
    (1, 15, 14, 40, 20, 3, 3, (3, 3), (2, 2), (2, 2)),       # stride 3, dilation 2, K = 20
    (1, 20, 17, 12, 16, 5, 3, (1, 2), (2, 1), (1, 2)),       # R != S
    (2, 23, 29, 64, 72, 3, 3, (1, 1), (1, 1), (1, 1)),       # several tiles, filter tail
    (1, 31, 37, 132, 200, 3, 3, (1, 1), (1, 1), (1, 1)),     # channel tail inside a 32-float step
    (1, 40, 50, 128, 260, 1, 1, (2, 2), (0, 0), (1, 1)),     # 1x1 stride 2: all-zero classes
    (1, 1, 1, 4, 4, 1, 1, (1, 1), (0, 0), (1, 1)),           # everything is 1
]


@pytest.mark.parametrize("case", SMALL, ids=lambda c: "x".join(str(v) for v in c[:7]))
def test_f32_small_shapes_full_tensor(case):
    say(f"f32 case {case}")
    d, x, w, g = _rand32(*case, seed=sum(case[:7]))
    _check(d, x, w, g, f"f32{case}")


def _distinct_backbone_and_head_shapes():
    """First instance of every layer shape of the detector workload after the RGB stem (the
    single-precision path takes channel counts in multiples of 4)."""
    seen, out = set(), []
    for li, l in enumerate(workloads.CONFIGS[5]):
        key = (l.N, l.H, l.W, l.C, l.K, l.R, l.stride, l.pad)
        if l.C % 4 or key in seen:
            continue
        seen.add(key)
        out.append(li)
    return out


@pytest.mark.parametrize("li", _distinct_backbone_and_head_shapes(), ids=lambda v: workloads.CONFIGS[5][v].name)
def test_f32_every_distinct_layer_shape_stratified_samples(li):
    """Every distinct res2-res5 shape at full size, the launch bench.py times, on at least 1e5
    stratified output elements per pass (workloads.stratified_indices)."""
    l = workloads.CONFIGS[5][li]
    say(f"f32 config layer {l.name} {l.x_shape} -> {l.y_shape}")
    d, x, w, g = _rand32(l.N, l.H, l.W, l.C, l.K, l.R, l.S, (l.stride, l.stride), (l.pad, l.pad), (l.dil, l.dil),
                         seed=1100 + li)
    _check(d, x, w, g, f"f32.{l.name}", sample=True, seed=3, layer=l)
    torch.cuda.empty_cache()


ODD = [
    (1, 9, 11, 3, 5, 3, 3, (1, 1), (1, 1), (1, 1)),          # channel / filter counts the matrix kernels do not take
    (2, 7, 8, 6, 4, 3, 3, (2, 2), (1, 1), (1, 1)),           # C = 6, strided
    (1, 12, 12, 4, 4, 9, 9, (1, 1), (4, 4), (1, 1)),         # 81 taps
    (1, 21, 23, 4, 4, 3, 3, (5, 5), (1, 1), (1, 1)),         # 25 stride classes
]


@pytest.mark.parametrize("case", ODD, ids=lambda c: "x".join(str(v) for v in c[:7]))
def test_f32_descriptors_outside_the_matrix_kernels(case):
    """Every valid descriptor is served: these take the one-thread-per-output kernels."""
    say(f"f32 direct case {case}")
    d, x, w, g = _rand32(*case, seed=sum(case[:7]) + 7)
    assert all(sd.conv2d_workspace_bytes_f32(d, p) == 0 for p in (sd.FWD, sd.DGRAD, sd.WGRAD))
    _check(d, x, w, g, f"f32direct{case}")


def test_f32_argument_checks():
    t = torch.zeros(4096, dtype=torch.float32, device="cuda")
    d = sd.make_desc(1, 8, 8, 8, 8, 3, 3, (1, 1), (1, 1), (1, 1))
    assert sd.conv2d_workspace_bytes_f32(d, sd.DGRAD) > 0
    with pytest.raises(sd.SdconvError) as e:
        sd.conv2d_dgrad_f32(d, t, t, t, None, 0)                            # workspace missing
    assert e.value.status == -3
