"""GPU parity of every tile variant of the pipelined kernels, forced one by one through the
dispatcher's environment hooks (read per call), against the fp64 CPU oracle on full tensors.
The shapes give ragged row / spatial tiles, several images, filter-count tails and more than
one 64-channel slab, so every variant sees partial tiles on each axis."""
import os

import numpy as np
import pytest

import paper_1903_05831_amd as sd

from gpu_harness import check_all_passes, say

pytestmark = pytest.mark.gpu


def _rand_case(N, H, W, C, K, R, S, stride, pad, dil, seed):
    d = sd.make_desc(N, H, W, C, K, R, S, stride, pad, dil)
    ho, wo = sd.conv2d_out_shape(d)
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, H, W, C), dtype=np.float32).astype(np.float16)
    w = (rng.standard_normal((K, R, S, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / (R * S * C)))).astype(np.float16)
    g = rng.standard_normal((N, ho, wo, K), dtype=np.float32).astype(np.float16)
    return d, x, w, g


class forced:
    def __init__(self, **env):
        self.env = {k: str(v) for k, v in env.items()}

    def __enter__(self):
        self.old = {k: os.environ.get(k) for k in self.env}
        os.environ.update(self.env)

    def __exit__(self, *exc):
        for k, v in self.old.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v


# stride-1 layers the patch kernels accept (taps span two extra rows and columns, contraction
# channels in whole 64-channel slabs on both the forward and the data-gradient side)
PATCH_SHAPES = [
    # N  H   W   C    K   R  S  stride  pad     dil
    (2, 21, 37, 64, 64, 3, 3, (1, 1), (1, 1), (1, 1)),      # ragged tiles both ways, two images
    (1, 19, 18, 128, 192, 3, 3, (1, 1), (1, 1), (1, 1)),    # two slabs, filter tail (192 = 128 + 64)
    (1, 17, 33, 64, 128, 3, 3, (1, 1), (0, 0), (1, 1)),     # no padding: output smaller than input
    (1, 12, 20, 64, 64, 3, 3, (1, 1), (2, 2), (1, 1)),      # padding 2: output larger than input
    (1, 16, 16, 64, 64, 2, 2, (1, 1), (1, 1), (2, 2)),      # 2x2 taps, dilation 2
    (1, 9, 40, 64, 64, 3, 2, (1, 1), (1, 1), (1, 2)),       # 3x2 taps, dilation 1x2
]
PATCH_VARIANTS = list(range(400, 436))
# these take three taps per pipeline step: R*S must be a multiple of 3 and give at least
# (ring stages - 1) steps per channel slab; variant -> ring stages
THREE_TAP_STEP = {414: 3, 415: 2, 416: 2, 417: 2, 418: 3, 419: 4, 420: 3, 421: 2, 423: 2, 425: 2, 427: 2,
                  428: 4, 429: 3, 430: 2, 431: 2, 432: 2, 433: 2, 435: 4}
# these have a single patch buffer: one 64-channel slab on the contraction side of both passes
ONE_SLAB = set(range(422, 428)) | {433, 434}


@pytest.mark.parametrize("variant", PATCH_VARIANTS)
def test_patch_kernel_variants(variant):
    for case in PATCH_SHAPES:
        taps = case[5] * case[6]
        if variant in THREE_TAP_STEP and (taps % 3 or taps // 3 < THREE_TAP_STEP[variant] - 1):
            continue        # the dispatcher (rightly) does not hand such a layer to this variant
        if variant in ONE_SLAB and (case[3] != 64 or case[4] != 64):
            continue
        say(f"patch variant {variant} case {case}")
        d, x, w, g = _rand_case(*case, seed=variant * 31 + len(case))
        with forced(SDCONV_IGEMM_VARIANT=variant, SDCONV_NO_TUNED_TABLE=1):
            assert "patch" in sd.kernel_name(d, sd.FWD), "shape must reach the patch kernel"
            assert "patch" in sd.kernel_name(d, sd.DGRAD)
            check_all_passes(d, x, w, g, f"patch{variant}{case}")


WS_SHAPES = [
    (2, 23, 29, 64, 72, 3, 3, (2, 2), (1, 1), (1, 1)),      # strided: parity classes in the data gradient
    (1, 31, 37, 136, 200, 3, 3, (1, 1), (1, 1), (1, 1)),    # short last channel slab, filter tail
    (1, 31, 37, 128, 264, 1, 1, (1, 1), (0, 0), (1, 1)),    # 1x1, more than one 256-wide column tile
    (2, 23, 29, 72, 64, 1, 1, (2, 2), (0, 0), (1, 1)),      # 1x1 stride 2, odd image: three parity classes of the data gradient are all zeros
    (1, 21, 27, 64, 64, 1, 3, (2, 2), (0, 1), (1, 1)),      # 1x3 stride 2: the odd-row classes have no taps, both even-row classes do
]
WS_VARIANTS = list(range(300, 325))


@pytest.mark.parametrize("variant", WS_VARIANTS)
def test_split_role_kernel_variants(variant):
    for case in WS_SHAPES:
        say(f"ws variant {variant} case {case}")
        d, x, w, g = _rand_case(*case, seed=variant * 17 + 3)
        with forced(SDCONV_IGEMM_VARIANT=variant, SDCONV_NO_TUNED_TABLE=1):
            assert "_ws_" in sd.kernel_name(d, sd.FWD)
            check_all_passes(d, x, w, g, f"ws{variant}{case}")


def test_two_tile_widths_in_one_launch():
    """Variant 324 on a layer with 71 x 4 tiles of 224 x 256 (15 700 = 70 x 224 + 20 rows, so the
    last row tile is ragged): 256 of them stay that wide, the last seven row tiles are cut into 56
    tiles of 224 x 128; the data gradient of the same layer has 71 x 1 tiles and runs them all half
    as wide."""
    case = (1, 100, 157, 64, 1024, 1, 1, (1, 1), (0, 0), (1, 1))
    d, x, w, g = _rand_case(*case, seed=324)
    with forced(SDCONV_IGEMM_VARIANT=324, SDCONV_NO_TUNED_TABLE=1):
        assert "tail128" in sd.kernel_name(d, sd.FWD)
        check_all_passes(d, x, w, g, f"mixed{case}")


# the kernels in which every wave fetches its own share (igemm_dma.hip, 100-113) and the
# register-staged ones (igemm.hip, 0-3); their data gradient takes a transposed filter copy
DMA_VARIANTS = [0, 1, 2, 3] + list(range(100, 114))


@pytest.mark.parametrize("variant", DMA_VARIANTS)
def test_all_wave_fetch_kernel_variants(variant):
    for case in WS_SHAPES:
        say(f"dma variant {variant} case {case}")
        d, x, w, g = _rand_case(*case, seed=variant * 19 + 5)
        with forced(SDCONV_IGEMM_VARIANT=variant, SDCONV_NO_TUNED_TABLE=1):
            assert "_ws_" not in sd.kernel_name(d, sd.FWD) and "patch" not in sd.kernel_name(d, sd.FWD)
            check_all_passes(d, x, w, g, f"dma{variant}{case}")


WGRAD_SHAPES = [
    (2, 23, 29, 64, 72, 3, 3, (2, 2), (1, 1), (1, 1)),      # strided, gathered x rows, filter tail
    (1, 31, 37, 136, 200, 3, 3, (1, 1), (1, 1), (1, 1)),    # channel and filter tails
    (1, 31, 37, 128, 264, 1, 1, (1, 1), (0, 0), (1, 1)),    # 1x1 unpadded: linear x addressing
]
WGRAD_VARIANTS = [0, 1] + list(range(100, 121))      # 0, 1: the register-staged kernels of wgrad.hip


@pytest.mark.parametrize("variant", WGRAD_VARIANTS)
def test_wgrad_kernel_variants(variant):
    for splits in (1, 3):
        for case in WGRAD_SHAPES:
            say(f"wgrad variant {variant} splits {splits} case {case}")
            d, x, w, g = _rand_case(*case, seed=variant * 13 + splits)
            with forced(SDCONV_WGRAD_VARIANT=variant, SDCONV_WGRAD_SPLITS=splits, SDCONV_NO_TUNED_TABLE=1):
                check_all_passes(d, x, w, g, f"wgrad{variant}s{splits}{case}")
