"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on
the same seeded binary16 inputs.  Bar: |err| <= 2e-2*(1+|ref|) per element and relative
Frobenius error <= 1e-3; overflow flag and unscaled values bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_1903_05831_amd as sd
from paper_1903_05831_amd import workloads

from gpu_harness import check_all_passes, say, to_dev

pytestmark = pytest.mark.gpu


def _rand_case(N, H, W, C, K, R, S, stride, pad, dil, seed):
    d = sd.make_desc(N, H, W, C, K, R, S, stride, pad, dil)
    ho, wo = sd.conv2d_out_shape(d)
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, H, W, C), dtype=np.float32).astype(np.float16)
    w = (rng.standard_normal((K, R, S, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / (R * S * C)))).astype(np.float16)
    g = rng.standard_normal((N, ho, wo, K), dtype=np.float32).astype(np.float16)
    return d, x, w, g


# Small shapes that span several tiles with ragged tails, odd channel counts (direct
# route), strides, pads, dilations, R != S, H != W.
SMALL = [
    # N  H   W   C   K  R  S  stride  pad     dil
    (1, 9, 11, 3, 5, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 13, 7, 1, 1, 3, 2, (2, 1), (1, 0), (1, 1)),
    (1, 12, 10, 24, 40, 3, 3, (2, 2), (1, 1), (1, 1)),
    (2, 10, 12, 8, 8, 1, 1, (1, 1), (0, 0), (1, 1)),
    (1, 15, 14, 40, 24, 3, 3, (3, 3), (2, 2), (2, 2)),
    (1, 20, 17, 8, 16, 5, 3, (1, 2), (2, 1), (1, 2)),
    (3, 11, 11, 16, 8, 1, 1, (2, 2), (0, 0), (1, 1)),
    (1, 9, 9, 8, 8, 1, 1, (3, 3), (0, 0), (1, 1)),
    (2, 23, 29, 64, 64, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 23, 29, 64, 72, 3, 3, (2, 2), (1, 1), (1, 1)),
    (1, 31, 37, 136, 200, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 31, 37, 128, 256, 1, 1, (1, 1), (0, 0), (1, 1)),
    (1, 30, 38, 256, 64, 1, 1, (2, 2), (0, 0), (1, 1)),
    (1, 17, 19, 64, 128, 3, 3, (1, 1), (2, 2), (2, 2)),
    (1, 40, 44, 3, 64, 7, 7, (2, 2), (3, 3), (1, 1)),
    (4, 14, 14, 128, 64, 3, 3, (2, 2), (1, 1), (1, 1)),
    (2, 19, 37, 4, 72, 3, 3, (1, 1), (1, 1), (1, 1)),    # thin-input route, K over one filter tile
    (1, 33, 70, 1, 8, 5, 8, (2, 1), (2, 3), (1, 1)),     # thin-input route, one channel, S = 8
    (1, 20, 50, 2, 16, 7, 7, (3, 2), (3, 3), (1, 1)),    # thin-input route, stride 3x2
    (1, 70, 9, 3, 64, 8, 1, (1, 1), (0, 0), (1, 1)),     # thin-input route, R = 8, S = 1
    (2, 37, 45, 3, 64, 3, 3, (1, 1), (1, 1), (1, 1)),    # thin dgrad on MFMA, stride 1
    (1, 41, 70, 4, 32, 5, 5, (2, 2), (2, 2), (1, 1)),    # thin dgrad on MFMA, K = 32, C = 4
    (1, 35, 67, 2, 64, 3, 4, (2, 1), (1, 2), (1, 1)),    # thin dgrad on MFMA, stride 2x1, C = 2
    (1, 30, 50, 3, 64, 3, 3, (2, 2), (2, 2), (2, 2)),    # thin dgrad on MFMA, dilation 2
    (1, 3, 3, 8, 8, 3, 3, (1, 1), (0, 0), (1, 1)),       # single output pixel
    (1, 1, 1, 8, 8, 1, 1, (1, 1), (0, 0), (1, 1)),       # everything is 1
    (1, 6, 6, 64, 64, 3, 3, (1, 1), (3, 3), (1, 1)),     # pad larger than needed
    (2, 25, 42, 256, 3, 1, 1, (1, 1), (0, 0), (1, 1)),   # padded-filter-count route: RPN objectness head
    (2, 25, 42, 256, 12, 1, 1, (1, 1), (0, 0), (1, 1)),  # ... RPN box head
    (1, 17, 23, 512, 60, 1, 1, (1, 1), (0, 0), (1, 1)),  # ... 15-anchor box head
    (2, 19, 21, 16, 20, 3, 3, (2, 2), (1, 1), (1, 1)),   # ... strided 3x3, K = 20
    (1, 9, 9, 8, 1, 3, 3, (1, 1), (1, 1), (2, 2)),       # ... a single filter, dilation 2
]


@pytest.mark.parametrize("case", SMALL, ids=lambda c: "x".join(str(v) for v in c[:7]) + f"_s{c[7][0]}{c[7][1]}p{c[8][0]}{c[8][1]}d{c[9][0]}{c[9][1]}")
def test_small_shapes_full_tensor(case):
    say(f"case {case}")
    d, x, w, g = _rand_case(*case, seed=hash(case) % 10000)
    check_all_passes(d, x, w, g, f"small{case}")


def test_config1_full_tensor_and_unscale():
    """Single 3x3 64->64 conv at 56x56: all three passes element by element, then the
    loss-scale removal (scale 1024) on the weight gradient, bit-exact."""
    l = workloads.CONFIGS[1][0]
    d = sd.desc_of(l)
    x, w, g = workloads.make_x(l, 1, 0), workloads.make_w(l, 1, 0), workloads.make_g(l, 1, 0)
    check_all_passes(d, x, w, g, "config1")
    dw = torch.empty(l.w_shape, dtype=torch.float32, device="cuda")
    ws_bytes = sd.conv2d_workspace_bytes(d, sd.WGRAD)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    sd.conv2d_wgrad(d, to_dev(x), to_dev(g), dw, ws, st)
    torch.cuda.synchronize()
    before = dw.cpu().numpy().copy()
    flag = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    sd.grad_unscale_check(dw, dw.numel(), 1.0 / 1024.0, flag, st)
    torch.cuda.synchronize()
    want, want_flag = oracle.unscale_check(before.ravel(), 1.0 / 1024.0)
    assert int(flag.item()) == want_flag == 0
    assert np.array_equal(dw.cpu().numpy().ravel().view(np.uint32), want.view(np.uint32))
    # run-to-run determinism of the split reduction
    dw2 = torch.empty_like(dw)
    sd.conv2d_wgrad(d, to_dev(x), to_dev(g), dw2, ws, st)
    torch.cuda.synchronize()
    assert np.array_equal(dw2.cpu().numpy().view(np.uint32), before.view(np.uint32))


def _unscale_case(g: np.ndarray, inv_scale: float, offset: int = 0):
    buf = torch.zeros(g.size + offset + 64, dtype=torch.float32, device="cuda")
    buf[offset:offset + g.size] = torch.from_numpy(g).cuda()
    sentinel = buf.cpu().numpy().copy()
    flag = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    view = buf[offset:offset + g.size] if g.size else None
    sd.grad_unscale_check(view if g.size else 0, g.size, inv_scale, flag, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = buf.cpu().numpy()
    want, want_flag = oracle.unscale_check(g, inv_scale)
    assert int(flag.item()) == want_flag
    a, b = got[offset:offset + g.size].view(np.uint32), want.view(np.uint32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got[offset:offset + g.size]), nan)
    assert np.array_equal(a[~nan], b[~nan])
    assert np.array_equal(got[:offset], sentinel[:offset]) and np.array_equal(got[offset + g.size:], sentinel[offset + g.size:])
    return want_flag


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 63, 64, 65, 255, 1023, 1024, 1025, 4096, 4097, 100003])
@pytest.mark.parametrize("offset", [0, 1, 3])
def test_unscale_sizes_and_alignment(n, offset):
    rng = np.random.default_rng(n * 4 + offset)
    g = (rng.standard_normal(n) * 10.0 ** rng.uniform(-40, 38, n)).astype(np.float32)
    assert _unscale_case(g, 2.0 ** -10, offset) == 0
    assert _unscale_case(g, float(np.float32(1.0 / 3.0)), offset) == 0
    if n:
        for pos in {0, n - 1, n // 2}:
            for bad in (np.inf, -np.inf, np.nan):
                h = g.copy(); h[pos] = bad
                assert _unscale_case(h, 2.0 ** -10, offset) == 1


def test_unscale_extremes_do_not_trip_flag():
    g = np.array([np.finfo(np.float32).max, -np.finfo(np.float32).max, 1e-45, -1e-45, 0.0, -0.0,
                  np.finfo(np.float32).tiny], dtype=np.float32)
    assert _unscale_case(g, 2.0 ** -10) == 0
    assert _unscale_case(g, 4.0) == 0          # finite in, inf out: flag looks at inputs


def test_unscale_full_size_with_seeded_infs():
    """All 23 454 912 weight-gradient elements of the detector workload, 1e-4 of them +inf."""
    n = sum(l.dw_numel for l in workloads.CONFIGS[5])
    rng = np.random.default_rng(5)
    g = (rng.standard_normal(n, dtype=np.float32) * np.float32(300.0))
    assert _unscale_case(g, 2.0 ** -10) == 0
    pos = workloads.inf_positions(n, 5)
    assert pos.size == int(np.ceil(1e-4 * n))
    g[pos] = np.inf
    assert _unscale_case(g, 2.0 ** -10) == 1
