"""GPU parity of the fused epilogues (conv2d_fwd_fused, conv2d_dgrad_fused) against the fp64
oracle of oracle/epilogue.py, through every route of the dispatcher and every tile variant of
the pipelined kernels (their shared LDS-strip epilogue has one instantiation per wave-tile
shape and MFMA block size)."""
import numpy as np
import pytest
import torch

import paper_1903_05831_amd as sd

from gpu_harness import GuardedOut, check_fused, say, to_dev, workspace_for
from test_gpu_variants import ONE_SLAB, PATCH_VARIANTS, THREE_TAP_STEP, WS_VARIANTS, _rand_case, forced

pytestmark = pytest.mark.gpu

ROUTE_SHAPES = [
    # N  H   W   C    K   R  S  stride  pad     dil           route it takes by default
    (2, 37, 41, 3, 64, 7, 7, (2, 2), (3, 3), (1, 1)),       # thin (stem): C = 3
    (1, 19, 23, 5, 7, 3, 3, (1, 1), (1, 1), (1, 1)),        # direct: channel counts no MFMA tile takes
    (2, 21, 37, 64, 64, 3, 3, (1, 1), (1, 1), (1, 1)),      # patch kernel
    (1, 31, 37, 128, 264, 1, 1, (1, 1), (0, 0), (1, 1)),    # 1x1, filter tail
    (2, 23, 29, 64, 72, 3, 3, (2, 2), (1, 1), (1, 1)),      # strided 3x3: four classes in the data gradient
    (1, 40, 50, 128, 264, 1, 1, (2, 2), (0, 0), (1, 1)),    # 1x1 stride 2: three all-zero classes
    (1, 17, 19, 136, 200, 3, 3, (1, 1), (2, 2), (2, 2)),    # dilation 2, short last channel slab
    (2, 25, 42, 256, 12, 1, 1, (1, 1), (0, 0), (1, 1)),     # padded-filter-count route (K = 12)
    (2, 19, 21, 16, 20, 3, 3, (2, 2), (1, 1), (1, 1)),      # ... strided 3x3, K = 20
]


@pytest.mark.parametrize("case", ROUTE_SHAPES, ids=lambda c: "x".join(str(v) for v in c[:7]))
def test_fused_default_routes(case):
    say(f"fused default route case {case}")
    d, x, w, g = _rand_case(*case, seed=101)
    with forced(SDCONV_NO_TUNED_TABLE=1):
        check_fused(d, x, w, g, f"fused{case}", seed=1)


@pytest.mark.parametrize("fwd_opts,dgrad_opts", [
    (("scale",), ("scale",)), (("bias",), ("relu_mask",)), (("residual",), ()), (("relu",), ()),
    (("scale", "bias", "relu"), ("scale", "relu_mask")), (("residual", "relu"), ("relu_mask",))])
def test_fused_each_part_alone(fwd_opts, dgrad_opts):
    for case in (ROUTE_SHAPES[0], ROUTE_SHAPES[2], ROUTE_SHAPES[4]):
        say(f"fused parts {fwd_opts} {dgrad_opts} case {case}")
        d, x, w, g = _rand_case(*case, seed=202)
        with forced(SDCONV_NO_TUNED_TABLE=1):
            check_fused(d, x, w, g, f"parts{case}", seed=2, fwd_opts=fwd_opts, dgrad_opts=dgrad_opts)


def test_empty_tail_is_the_plain_pass_bit_for_bit():
    for case in ROUTE_SHAPES:
        say(f"fused empty tail case {case}")
        d, x, w, g = _rand_case(*case, seed=303)
        ho, wo = sd.conv2d_out_shape(d)
        st = torch.cuda.current_stream().cuda_stream
        xd, wd, gd = to_dev(x), to_dev(w), to_dev(g)
        a, b = GuardedOut((d.N, ho, wo, d.K), torch.float16), GuardedOut((d.N, ho, wo, d.K), torch.float16)
        sd.conv2d_fwd(d, xd, wd, a.view, workspace_for(d, sd.FWD), st)
        sd.conv2d_fwd_fused(d, xd, wd, b.view, workspace_for(d, sd.FWD), st)
        torch.cuda.synchronize()
        assert np.array_equal(a.numpy().view(np.uint16), b.numpy().view(np.uint16))
        a, b = GuardedOut((d.N, d.H, d.W, d.C), torch.float16), GuardedOut((d.N, d.H, d.W, d.C), torch.float16)
        sd.conv2d_dgrad(d, gd, wd, a.view, workspace_for(d, sd.DGRAD), st)
        sd.conv2d_dgrad_fused(d, gd, wd, b.view, workspace_for(d, sd.DGRAD), st)
        torch.cuda.synchronize()
        assert np.array_equal(a.numpy().view(np.uint16), b.numpy().view(np.uint16))


FUSED_WS_SHAPES = [
    (2, 23, 29, 64, 72, 3, 3, (2, 2), (1, 1), (1, 1)),
    (1, 31, 37, 136, 264, 1, 1, (1, 1), (0, 0), (1, 1)),
]
OLD_VARIANTS = [0, 1, 2, 3] + list(range(100, 112))


@pytest.mark.parametrize("variant", OLD_VARIANTS + WS_VARIANTS)
def test_fused_igemm_variants(variant):
    for case in FUSED_WS_SHAPES:
        say(f"fused variant {variant} case {case}")
        d, x, w, g = _rand_case(*case, seed=variant * 5 + 1)
        with forced(SDCONV_IGEMM_VARIANT=variant, SDCONV_NO_TUNED_TABLE=1):
            check_fused(d, x, w, g, f"fused_v{variant}{case}", seed=variant)


FUSED_PATCH_SHAPES = [
    (2, 21, 37, 64, 64, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 19, 18, 128, 192, 3, 3, (1, 1), (1, 1), (1, 1)),
]


@pytest.mark.parametrize("variant", PATCH_VARIANTS)
def test_fused_patch_variants(variant):
    for case in FUSED_PATCH_SHAPES:
        if variant in ONE_SLAB and (case[3] != 64 or case[4] != 64):
            continue
        say(f"fused patch variant {variant} case {case}")
        d, x, w, g = _rand_case(*case, seed=variant * 3 + 2)
        with forced(SDCONV_IGEMM_VARIANT=variant, SDCONV_NO_TUNED_TABLE=1):
            assert "patch" in sd.kernel_name(d, sd.FWD)
            check_fused(d, x, w, g, f"fused_p{variant}{case}", seed=variant)


def test_fused_argument_checks():
    d, x, w, g = _rand_case(1, 8, 8, 8, 8, 1, 1, (1, 1), (0, 0), (1, 1), seed=1)
    xd, wd = to_dev(x), to_dev(w)
    y = torch.empty((1, 8, 8, 8), dtype=torch.float16, device="cuda")
    sc = torch.ones(16, dtype=torch.float32, device="cuda")
    with pytest.raises(sd.SdconvError):
        sd.conv2d_fwd_fused(d, xd, wd, y, None, 0, scale=sc[1:9])          # 4-byte aligned only
    with pytest.raises(sd.SdconvError):
        sd.conv2d_dgrad_fused(d, y, wd, xd.clone(), None, 0, relu_mask=xd.view(-1)[1:])  # 2-byte aligned


def test_tail_pass_matches_the_elementwise_definition():
    """The separate pass used as the unfused baseline in the benchmark computes the same tail
    (on an already rounded binary16 tensor)."""
    rng = np.random.default_rng(7)
    pixels, C = 1237, 72
    t = rng.standard_normal((pixels, C)).astype(np.float16)
    scale = (rng.standard_normal(C) * 0.5 + 1).astype(np.float32)
    bias = rng.standard_normal(C).astype(np.float32)
    res = rng.standard_normal((pixels, C)).astype(np.float16)
    mask = np.maximum(rng.standard_normal((pixels, C)), 0).astype(np.float16)
    td = to_dev(t.copy())
    sd.sdconv_tail_pass(td, pixels, C, 0, scale=to_dev(scale), bias=to_dev(bias), residual=to_dev(res),
                        relu_mask=to_dev(mask), relu=True)
    torch.cuda.synchronize()
    v = t.astype(np.float64) * scale + bias + res.astype(np.float64)
    v = np.where(v > 0, v, 0.0)
    v = np.where(mask > 0, v, 0.0)
    got = td.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - v) <= 2e-3 * (1 + np.abs(v)))
    assert not got[mask <= 0].any()
    with pytest.raises(sd.SdconvError):
        sd.sdconv_tail_pass(td, pixels, 12, 0)          # channels not a multiple of 8
