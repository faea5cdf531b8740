"""Synthetic workloads: layer shapes of the five benchmark configurations and the
seeded input generators that both the HIP path and the CPU checker are fed from.

This module holds no convolution arithmetic.  Output extents are written out as
literals in the tables (they are the shapes of a ResNet-50-C4 Faster R-CNN at
800x1344 input, the detector the paper's Figure 1 is measured on); tests check that
the library and the checker both derive the same extents from the descriptors.

Value distributions: activations and upstream gradients ~ N(0,1); weights He-normal
with variance 2/(R*S*C); all drawn in fp32 and rounded once to binary16 (RNE).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List

import numpy as np

BASE_SEED = 190305831
ROLE_X, ROLE_W, ROLE_G, ROLE_INF = 0, 1, 2, 3


@dataclass(frozen=True)
class ConvLayer:
    name: str
    N: int
    H: int
    W: int
    C: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    Ho: int
    Wo: int
    dil: int = 1

    @property
    def x_shape(self):
        return (self.N, self.H, self.W, self.C)

    @property
    def w_shape(self):
        return (self.K, self.R, self.S, self.C)

    @property
    def y_shape(self):
        return (self.N, self.Ho, self.Wo, self.K)

    @property
    def flops(self) -> int:
        """Algorithmic FLOPs of ONE pass (2 per multiply-add, padding taps counted)."""
        return 2 * self.N * self.Ho * self.Wo * self.K * self.R * self.S * self.C

    @property
    def dw_numel(self) -> int:
        return self.K * self.R * self.S * self.C

    def compulsory_bytes(self, pass_name: str) -> int:
        """Bytes each tensor moves once: fp16 activations and weights, fp32 dw."""
        xb = 2 * self.N * self.H * self.W * self.C
        yb = 2 * self.N * self.Ho * self.Wo * self.K
        wb = self.dw_numel
        if pass_name == "wgrad":
            return xb + yb + 4 * wb
        return xb + yb + 2 * wb


def _L(name, N, H, W, C, K, R, stride, pad, Ho, Wo):
    return ConvLayer(name, N, H, W, C, K, R, R, stride, pad, Ho, Wo)


def _res2_block(prefix, first: bool) -> List[ConvLayer]:
    cin = 64 if first else 256
    out = [_L(prefix + "a", 2, 200, 336, cin, 64, 1, 1, 0, 200, 336),
           _L(prefix + "b", 2, 200, 336, 64, 64, 3, 1, 1, 200, 336),
           _L(prefix + "c", 2, 200, 336, 64, 256, 1, 1, 0, 200, 336)]
    if first:
        out.append(_L(prefix + "p", 2, 200, 336, 64, 256, 1, 1, 0, 200, 336))
    return out


def _res3_block0() -> List[ConvLayer]:
    return [_L("res3.0a", 2, 200, 336, 256, 128, 1, 1, 0, 200, 336),
            _L("res3.0b", 2, 200, 336, 128, 128, 3, 2, 1, 100, 168),
            _L("res3.0c", 2, 100, 168, 128, 512, 1, 1, 0, 100, 168),
            _L("res3.0p", 2, 200, 336, 256, 512, 1, 2, 0, 100, 168)]


def _res3_block(i) -> List[ConvLayer]:
    p = f"res3.{i}"
    return [_L(p + "a", 2, 100, 168, 512, 128, 1, 1, 0, 100, 168),
            _L(p + "b", 2, 100, 168, 128, 128, 3, 1, 1, 100, 168),
            _L(p + "c", 2, 100, 168, 128, 512, 1, 1, 0, 100, 168)]


def _res4() -> List[ConvLayer]:
    out = [_L("res4.0a", 2, 100, 168, 512, 256, 1, 1, 0, 100, 168),
           _L("res4.0b", 2, 100, 168, 256, 256, 3, 2, 1, 50, 84),
           _L("res4.0c", 2, 50, 84, 256, 1024, 1, 1, 0, 50, 84),
           _L("res4.0p", 2, 100, 168, 512, 1024, 1, 2, 0, 50, 84)]
    for i in range(1, 6):
        p = f"res4.{i}"
        out += [_L(p + "a", 2, 50, 84, 1024, 256, 1, 1, 0, 50, 84),
                _L(p + "b", 2, 50, 84, 256, 256, 3, 1, 1, 50, 84),
                _L(p + "c", 2, 50, 84, 256, 1024, 1, 1, 0, 50, 84)]
    return out


def _res5() -> List[ConvLayer]:
    out = [_L("res5.0a", 512, 14, 14, 1024, 512, 1, 1, 0, 14, 14),
           _L("res5.0b", 512, 14, 14, 512, 512, 3, 2, 1, 7, 7),
           _L("res5.0c", 512, 7, 7, 512, 2048, 1, 1, 0, 7, 7),
           _L("res5.0p", 512, 14, 14, 1024, 2048, 1, 2, 0, 7, 7)]
    for i in range(1, 3):
        p = f"res5.{i}"
        out += [_L(p + "a", 512, 7, 7, 2048, 512, 1, 1, 0, 7, 7),
                _L(p + "b", 512, 7, 7, 512, 512, 3, 1, 1, 7, 7),
                _L(p + "c", 512, 7, 7, 512, 2048, 1, 1, 0, 7, 7)]
    return out


def _config5() -> List[ConvLayer]:
    out = [_L("stem", 2, 800, 1344, 3, 64, 7, 2, 3, 400, 672)]
    out += _res2_block("res2.0", True) + _res2_block("res2.1", False) + _res2_block("res2.2", False)
    out += _res3_block0() + _res3_block(1) + _res3_block(2) + _res3_block(3)
    out += _res4()
    out += _res5()
    return out


def _fpn_rpn() -> List[ConvLayer]:
    """Convolutions a ResNet-50-FPN Faster R-CNN adds to (or runs differently from) the C4 model,
    N = 2 images of 800x1344 (Table 1 of the paper quotes its training speed on this model):
    res5 on the whole image instead of on RoIs, the FPN lateral 1x1 and output 3x3 convs at strides
    4-32, the RPN head shared by the pyramid levels P2-P6 (3 anchors per position), the two
    fully connected layers of the box head on 512 RoIs of 7x7x256 written as 1x1 convs on 1x1
    images, and the RPN of the C4 model (3x3 1024->512, 15 anchors)."""
    out = [_L("res5i.0a", 2, 50, 84, 1024, 512, 1, 1, 0, 50, 84),
           _L("res5i.0b", 2, 50, 84, 512, 512, 3, 2, 1, 25, 42),
           _L("res5i.0c", 2, 25, 42, 512, 2048, 1, 1, 0, 25, 42),
           _L("res5i.0p", 2, 50, 84, 1024, 2048, 1, 2, 0, 25, 42)]
    for i in range(1, 3):
        q = f"res5i.{i}"
        out += [_L(q + "a", 2, 25, 42, 2048, 512, 1, 1, 0, 25, 42),
                _L(q + "b", 2, 25, 42, 512, 512, 3, 1, 1, 25, 42),
                _L(q + "c", 2, 25, 42, 512, 2048, 1, 1, 0, 25, 42)]
    levels = [(2, 200, 336, 256), (3, 100, 168, 512), (4, 50, 84, 1024), (5, 25, 42, 2048)]
    for lv, h, w, c in levels:
        out.append(_L(f"fpn.lat{lv}", 2, h, w, c, 256, 1, 1, 0, h, w))
    for lv, h, w, c in levels:
        out.append(_L(f"fpn.out{lv}", 2, h, w, 256, 256, 3, 1, 1, h, w))
    for lv, h, w in [(2, 200, 336), (3, 100, 168), (4, 50, 84), (5, 25, 42), (6, 13, 21)]:
        out += [_L(f"rpn.conv{lv}", 2, h, w, 256, 256, 3, 1, 1, h, w),
                _L(f"rpn.cls{lv}", 2, h, w, 256, 3, 1, 1, 0, h, w),
                _L(f"rpn.box{lv}", 2, h, w, 256, 12, 1, 1, 0, h, w)]
    out += [_L("head.fc6", 512, 1, 1, 7 * 7 * 256, 1024, 1, 1, 0, 1, 1),
            _L("head.fc7", 512, 1, 1, 1024, 1024, 1, 1, 0, 1, 1)]
    out += [_L("c4rpn.conv", 2, 50, 84, 1024, 512, 3, 1, 1, 50, 84),
            _L("c4rpn.cls", 2, 50, 84, 512, 15, 1, 1, 0, 50, 84),
            _L("c4rpn.box", 2, 50, 84, 512, 60, 1, 1, 0, 50, 84)]
    return out


CONFIGS: Dict[int, List[ConvLayer]] = {
    1: [_L("conv3x3_64", 1, 56, 56, 64, 64, 3, 1, 1, 56, 56)],
    2: _res2_block("res2.", False),
    3: _res3_block0(),
    4: _res4(),
    5: _config5(),
    6: _fpn_rpn(),
}

CONFIG_NAMES = {
    1: "single 3x3 64->64 conv at 56x56, N=1",
    2: "ResNet-50 res2 bottleneck convs at 200x336, N=2",
    3: "ResNet-50 res3 first block from 200x336x256, N=2",
    4: "ResNet-50-C4 res4 trunk (6 bottlenecks) at 50x84, N=2",
    5: "ResNet-50-C4 Faster R-CNN, all 53 convs, N=2 x 800x1344 + 512 RoIs",
    6: "ResNet-50-FPN Faster R-CNN additions: res5 on the image, FPN, RPN heads on P2-P6, box-head FCs, C4 RPN",
}


def _rng(config_id: int, layer_index: int, role: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([BASE_SEED, config_id, layer_index, role]))


def _normal_half(rng: np.random.Generator, shape, sigma: float) -> np.ndarray:
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if sigma != 1.0:
        a *= np.float32(sigma)
    return a.astype(np.float16)


def make_x(layer: ConvLayer, config_id: int, layer_index: int) -> np.ndarray:
    return _normal_half(_rng(config_id, layer_index, ROLE_X), layer.x_shape, 1.0)


def make_w(layer: ConvLayer, config_id: int, layer_index: int) -> np.ndarray:
    sigma = float(np.sqrt(2.0 / (layer.R * layer.S * layer.C)))
    return _normal_half(_rng(config_id, layer_index, ROLE_W), layer.w_shape, sigma)


def make_g(layer: ConvLayer, config_id: int, layer_index: int) -> np.ndarray:
    return _normal_half(_rng(config_id, layer_index, ROLE_G), layer.y_shape, 1.0)


def inf_positions(n: int, config_id: int, fraction: float = 1e-4) -> np.ndarray:
    """ceil(fraction*n) distinct flat indices at which a gradient buffer is set to +inf."""
    count = int(np.ceil(fraction * n))
    return np.sort(_rng(config_id, 0, ROLE_INF).choice(n, size=count, replace=False))


def sample_indices(total: int, count: int, seed: int) -> np.ndarray:
    """Seeded flat output indices for sampled parity checks (always holds first and last)."""
    rng = np.random.default_rng(np.random.SeedSequence([BASE_SEED, 77, seed]))
    count = min(count, total)
    idx = rng.choice(total, size=count, replace=False) if count < total else np.arange(total)
    idx[0] = 0
    idx[-1] = total - 1
    return np.unique(idx).astype(np.int64)


def stratified_indices(layer: ConvLayer, pass_id: int, seed: int, min_count: int = 100_000,
                       row_window: int = 8) -> np.ndarray:
    """Seeded flat output indices of one pass (0 forward: y, 1 data gradient: dx, 2 weight
    gradient: dw) spread so that no tile of a kernel can be missed, whatever its shape:

    y / dx: the pixels are listed per stride-parity class of the data gradient (one class for the
    forward pass), in image order; of every `row_window` consecutive pixels of a list one is
    drawn, plus the first and last pixel of the list; of every drawn pixel the first and last
    channel and one channel out of each of `cpr` equal channel ranges are taken (cpr >= 4, raised
    until min_count elements are reached); the first and last pixel of a list are taken whole.
    dw: one element out of every (8 filters x tap x 8 channels) cell, plus uniform draws up to
    min_count; tensors of up to 1.5 * min_count elements are taken whole."""
    rng = np.random.default_rng(np.random.SeedSequence([BASE_SEED, 78, seed, pass_id]))
    if pass_id == 2:
        total = layer.K * layer.R * layer.S * layer.C
        if total <= min_count * 3 // 2:
            return np.arange(total, dtype=np.int64)
        taps = layer.R * layer.S
        kw, cw = (layer.K + 7) // 8, (layer.C + 7) // 8
        k = np.minimum(np.arange(kw)[:, None, None] * 8 + rng.integers(0, 8, (kw, taps, cw)), layer.K - 1)
        c = np.minimum(np.arange(cw)[None, None, :] * 8 + rng.integers(0, 8, (kw, taps, cw)), layer.C - 1)
        t = np.arange(taps)[None, :, None]
        idx = ((k * taps + t) * layer.C + c).ravel()
        idx = np.unique(np.concatenate([idx, [0, total - 1]]))
        while idx.size < min_count:
            idx = np.unique(np.concatenate([idx, rng.integers(0, total, 2 * (min_count - idx.size))]))
        return idx.astype(np.int64)
    if pass_id == 0:
        H, W, ncols, sh, sw = layer.Ho, layer.Wo, layer.K, 1, 1
    else:
        H, W, ncols, sh, sw = layer.H, layer.W, layer.C, layer.stride, layer.stride
    if layer.N * H * W * ncols <= min_count * 3 // 2:
        return np.arange(layer.N * H * W * ncols, dtype=np.int64)
    lists = []
    for a in range(sh):
        for b in range(sw):
            hh, ww = np.arange(a, H, sh), np.arange(b, W, sw)
            if hh.size == 0 or ww.size == 0:
                continue
            pix = (np.arange(layer.N)[:, None, None] * H + hh[None, :, None]) * W + ww[None, None, :]
            lists.append(pix.ravel())
    nrows = sum((len(p) + row_window - 1) // row_window + 2 for p in lists)
    cpr = int(min(ncols, max(4, -(-min_count // max(nrows, 1)))))
    edges = np.linspace(0, ncols, cpr + 1).astype(np.int64)
    out = []
    for pix in lists:
        m = len(pix)
        nwin = (m + row_window - 1) // row_window
        pos = np.minimum(np.arange(nwin) * row_window + rng.integers(0, row_window, nwin), m - 1)
        pos = np.unique(np.concatenate([pos, [0, m - 1]]))
        rows = pix[pos].astype(np.int64)
        lo, hi = edges[:-1][None, :], edges[1:][None, :]
        cols = lo + (rng.random((rows.size, cpr)) * (hi - lo)).astype(np.int64)
        cols = np.concatenate([cols, np.zeros((rows.size, 1), np.int64),
                               np.full((rows.size, 1), ncols - 1, np.int64)], axis=1)
        out.append((rows[:, None] * ncols + cols).ravel())
        for p in (pix[0], pix[-1]):
            out.append(int(p) * ncols + np.arange(ncols, dtype=np.int64))
    return np.unique(np.concatenate(out)).astype(np.int64)
