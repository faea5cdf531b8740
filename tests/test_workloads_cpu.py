"""The stratified sample of output elements used by the full-size GPU parity tests: its coverage
properties, checked on the CPU.  The tests' claim that no tile of a kernel can go unchecked rests on
them: whatever the tile shape, a block of 16 GEMM rows contains two 8-pixel windows of one
stride-parity class, each with a sampled pixel, and every sampled pixel has samples in at least four
channel ranges plus the first and last channel."""
import numpy as np
import pytest

from paper_1903_05831_amd import workloads


def _layer(cfg, name):
    return next(l for l in workloads.CONFIGS[cfg] if l.name == name)


CASES = [(5, "res5.1b", 0), (5, "res3.0b", 1), (5, "res4.0p", 1), (5, "res2.0c", 0), (6, "rpn.conv2", 1), (6, "res5i.0b", 1)]


@pytest.mark.parametrize("cfg,name,pass_id", CASES)
def test_every_window_of_eight_class_pixels_and_every_channel_range_is_sampled(cfg, name, pass_id):
    l = _layer(cfg, name)
    idx = workloads.stratified_indices(l, pass_id, 7)
    if pass_id == 0:
        H, W, ncols, s = l.Ho, l.Wo, l.K, 1
    else:
        H, W, ncols, s = l.H, l.W, l.C, l.stride
    total = l.N * H * W * ncols
    assert idx.dtype == np.int64 and idx.ndim == 1
    assert np.all(np.diff(idx) > 0) and idx[0] == 0 and idx[-1] == total - 1
    assert idx.size >= min(total, 100_000)
    pix, col = idx // ncols, idx % ncols
    sampled = np.zeros(l.N * H * W, bool)
    sampled[pix] = True
    for a in range(s):
        for b in range(s):
            hh, ww = np.arange(a, H, s), np.arange(b, W, s)
            order = ((np.arange(l.N)[:, None, None] * H + hh[None, :, None]) * W + ww[None, None, :]).ravel()
            hit = sampled[order]
            pad = (-hit.size) % 8
            windows = np.concatenate([hit, np.zeros(pad, bool)]).reshape(-1, 8)
            assert windows.any(axis=1).all(), f"class ({a},{b}): a window of 8 consecutive pixels has no sample"
            assert hit[0] and hit[-1]
    # per sampled pixel: first and last channel, and at least four distinct quarters of the channel axis
    first = np.zeros(l.N * H * W, bool); last = np.zeros_like(first)
    first[pix[col == 0]] = True
    last[pix[col == ncols - 1]] = True
    assert first[sampled].all() and last[sampled].all()
    quarter = np.minimum(col * 4 // ncols, 3)
    seen = np.zeros((l.N * H * W, 4), bool)
    seen[pix, quarter] = True
    assert seen[sampled].all()


@pytest.mark.parametrize("cfg,name", [(5, "res5.1b"), (5, "res4.1a"), (5, "res3.0b")])
def test_every_cell_of_the_weight_gradient_is_sampled(cfg, name):
    l = _layer(cfg, name)
    idx = workloads.stratified_indices(l, 2, 11)
    total = l.K * l.R * l.S * l.C
    assert np.all(np.diff(idx) > 0) and idx[0] >= 0 and idx[-1] == total - 1
    if total <= 150_000:
        assert idx.size == total
        return
    assert idx.size >= 100_000
    taps = l.R * l.S
    k, t, c = idx // (taps * l.C), (idx // l.C) % taps, idx % l.C
    cells = np.zeros(((l.K + 7) // 8, taps, (l.C + 7) // 8), bool)
    cells[k // 8, t, c // 8] = True
    assert cells.all(), "an (8 filters x tap x 8 channels) cell has no sample"


def test_small_tensors_are_taken_whole_and_draws_are_seeded():
    l = workloads.CONFIGS[1][0]
    for p in (0, 1, 2):
        n = {0: l.N * l.Ho * l.Wo * l.K, 1: l.N * l.H * l.W * l.C, 2: l.K * l.R * l.S * l.C}[p]
        idx = workloads.stratified_indices(l, p, 3, min_count=10 ** 9)
        assert np.array_equal(idx, np.arange(n))
    big = _layer(5, "res5.1b")
    a = workloads.stratified_indices(big, 0, 1)
    assert np.array_equal(a, workloads.stratified_indices(big, 0, 1))
    assert not np.array_equal(a, workloads.stratified_indices(big, 0, 2))
