"""Largest sizes the interface accepts: an activation tensor just below 2^31 elements (its last
byte offsets need all 32 bits of the kernels' offsets) through all three passes, and a gradient
buffer of more than 2^31 elements through grad_unscale_check (64-bit indexing).  Outputs are
checked on seeded samples that the oracle computes one by one, the same bar as everywhere."""
import numpy as np
import pytest
import torch

import oracle
import paper_1903_05831_amd as sd
from paper_1903_05831_amd import workloads

from gpu_harness import check_all_passes, say

pytestmark = pytest.mark.gpu


def test_activation_tensor_just_below_2_31_elements():
    """1x1 convolution 128 -> 8 channels on one 4096 x 4080 image: x and dx hold 2 139 095 040
    elements (99.6 % of 2^31); y, dy and dw are small, so the oracle's sampled sums stay cheap."""
    l = workloads.ConvLayer("limit", 1, 4096, 4080, 128, 8, 1, 1, 1, 0, 4096, 4080)
    assert l.N * l.H * l.W * l.C < 2 ** 31 <= l.N * l.H * (l.W + 16) * l.C
    d = sd.desc_of(l)
    say(f"limit layer {l.x_shape} -> {l.y_shape}")
    x, w, g = workloads.make_x(l, 9, 0), workloads.make_w(l, 9, 0), workloads.make_g(l, 9, 0)
    check_all_passes(d, x, w, g, "limit", sample=3000, seed=900)
    del x, w, g
    torch.cuda.empty_cache()


def test_padded_3x3_on_a_tensor_of_more_than_2_30_elements():
    """3x3, pad 1, 2048 -> 8 channels on one 724 x 725 image: x and dx hold 1 075 001 600 elements,
    so their byte offsets pass 2^31 -- the value the LDS-DMA kernels use to mark a load as masked
    (padding taps, ragged rows).  Such layers must take the kernels that index elements instead.
    The samples include the image corners and pixels on both sides of the 2 GiB byte offset.
    (Many channels rather than many pixels: the weight gradient then sums 524 900 pixels, as in the
    detector workload, and binary32 accumulation stays inside the parity bar.)"""
    l = workloads.ConvLayer("limit3x3", 1, 724, 725, 2048, 8, 3, 3, 1, 1, 724, 725)
    assert 2 ** 30 < l.N * l.H * l.W * l.C < 2 ** 31
    d = sd.desc_of(l)
    for p in (sd.FWD, sd.DGRAD, sd.WGRAD):
        name = sd.kernel_name(d, p)
        assert "dma" not in name and "_ws_" not in name and "patch" not in name, name
    say(f"limit layer {l.x_shape} -> {l.y_shape} 3x3 pad 1")
    x, w, g = workloads.make_x(l, 9, 1), workloads.make_w(l, 9, 1), workloads.make_g(l, 9, 1)
    # flat indices worth looking at: corners, last elements, both sides of byte offset 2^31
    pix_2g = (2 ** 31 // 2) // l.C
    extra_x = [0, l.C * (l.W - 1), l.C * l.W * (l.H - 1), l.C * (l.W * l.H - 1), l.C * l.W * l.H - 1] + \
              [l.C * (pix_2g + o) + c for o in (-l.W - 1, -1, 0, 1, 300) for c in (0, l.C - 1)]
    assert max(extra_x) < l.N * l.H * l.W * l.C
    # y is small; its pixels next to the x pixels at the 2 GiB offset read across that offset
    extra_y = [0, l.K * (l.Wo - 1), l.K * l.Wo * (l.Ho - 1), l.K * l.Wo * l.Ho - 1] + \
              [l.K * (pix_2g + o) + k for o in (-l.Wo - 1, -1, 0, 1, 300) for k in (0, l.K - 1)]
    check_all_passes(d, x, w, g, "limit3x3", sample=3000, seed=910,
                     extra={sd.FWD: extra_y, sd.DGRAD: extra_x})
    del x, w, g
    torch.cuda.empty_cache()


def test_unscale_more_than_2_31_elements():
    """n = 2^31 + 12345 fp32 gradients (8.6 GB), values from a seeded generator on the device
    (the host copy of each checked window is taken before the call and handed to the oracle):
    bit-exact results in windows at the start, around the 4 GiB and 8 GiB byte offsets and at
    the end; the flag is 0 without and 1 with a single +inf in the very last element."""
    n = 2 ** 31 + 12345
    dev = torch.device("cuda")
    gen = torch.Generator(device=dev)
    gen.manual_seed(workloads.BASE_SEED + 31)
    g = torch.empty(n, dtype=torch.float32, device=dev)
    step = 1 << 28
    for s in range(0, n, step):
        e = min(n, s + step)
        g[s:e] = torch.randn(e - s, generator=gen, device=dev, dtype=torch.float32) * 1000.0
    windows = [(0, 1 << 16), (2 ** 30 - 4096, 2 ** 30 + 4096), (2 ** 31 - 4096, 2 ** 31 + 4096), (n - 12345 - 64, n)]
    before = [g[a:b].cpu().numpy().copy() for a, b in windows]
    flag = torch.full((1,), -1, dtype=torch.int32, device=dev)
    st = torch.cuda.current_stream().cuda_stream
    inv = float(np.float32(1.0 / 1024.0))
    say(f"unscale n={n}")
    sd.grad_unscale_check(g, n, inv, flag, st)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    for (a, b), src in zip(windows, before):
        want, want_flag = oracle.unscale_check(src, inv)
        assert want_flag == 0
        got = g[a:b].cpu().numpy()
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"window {a}:{b}"
    g[n - 1] = float("inf")
    sd.grad_unscale_check(g, n, inv, flag, st)
    torch.cuda.synchronize()
    assert int(flag.item()) == 1
    assert bool(torch.isinf(g[n - 1]))
    del g
    torch.cuda.empty_cache()
