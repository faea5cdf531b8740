"""GPU parity of the single-precision companion path (conv2d_*_f32) against the fp64 oracle on
the same binary32 inputs.

Tolerance: binary32 products and accumulation over n terms give a typical error of about
sqrt(n) * 2^-24 * |ref| (n up to 4608 in the forward pass, 134400 in the weight gradient: below
3e-5 relative); the bar is 2e-4 * (1 + |ref|) per element and 2e-5 in the Frobenius norm."""
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
    assert err[worst] <= bound[worst], f"{what}: element {worst} gpu={g[worst]!r} ref={r[worst]!r}"
    rn = np.linalg.norm(r)
    assert np.linalg.norm(g - r) <= FRO_TOL_F32 * (rn if rn > 0 else 1.0), f"{what}: Frobenius"


def _check(d, x, w, g, tag, sample=None, seed=0):
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
            idx = workloads.sample_indices(got.size, sample, seed + pid)
            _compare(got.ravel()[idx], ofn(od, an, bn, idx=idx), what, nterms, term_rms)


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


@pytest.mark.parametrize("cfg,name", [(5, "res2.0a"), (5, "res3.0b"), (5, "res4.1b"), (5, "res5.1a"), (5, "res4.0p")])
def test_f32_config_layers_sampled(cfg, name):
    l = next(l for l in workloads.CONFIGS[cfg] if l.name == name)
    say(f"f32 config layer {name} {l.x_shape}")
    d, x, w, g = _rand32(l.N, l.H, l.W, l.C, l.K, l.R, l.S, (l.stride, l.stride), (l.pad, l.pad), (l.dil, l.dil), seed=11)
    _check(d, x, w, g, f"f32.{name}", sample=2000, seed=3)


def test_f32_unsupported_and_argument_checks():
    d = sd.make_desc(1, 8, 8, 3, 8, 3, 3, (1, 1), (1, 1), (1, 1))          # C = 3
    t = torch.zeros(4096, dtype=torch.float32, device="cuda")
    with pytest.raises(sd.SdconvError) as e:
        sd.conv2d_fwd_f32(d, t, t, t, None, 0)
    assert e.value.status == -2
    d = sd.make_desc(1, 8, 8, 8, 8, 3, 3, (1, 1), (1, 1), (1, 1))
    assert sd.conv2d_workspace_bytes_f32(d, sd.DGRAD) > 0
    with pytest.raises(sd.SdconvError) as e:
        sd.conv2d_dgrad_f32(d, t, t, t, None, 0)                            # workspace missing
    assert e.value.status == -3
