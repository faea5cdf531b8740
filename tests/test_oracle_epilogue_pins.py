"""Pins of the fused-epilogue oracle against things other than itself: a hand-worked example,
the folding of the affine map into the filter (checked through the separately pinned plain
convolution), the batch-normalisation inference formula, an identity convolution that leaves
only the elementwise part, and finite differences of a brute-force loss for the data gradient."""
import os

import numpy as np
import pytest

import oracle
from oracle import epilogue as ep

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fused_epilogue_example.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        out[k] = np.array([float(t) for t in v])
    return out


def test_hand_worked_example():
    g = _golden()
    d = oracle.make_desc(1, 1, 2, 2, 2, 1, 1)
    x = g["x"].reshape(1, 1, 2, 2).astype(np.float16)
    w = g["w"].reshape(2, 1, 1, 2).astype(np.float16)
    sc, bi = g["scale"].astype(np.float32), g["bias"].astype(np.float32)
    res = g["residual"].reshape(1, 1, 2, 2).astype(np.float16)
    assert np.array_equal(ep.conv2d_fwd_fused(d, x, w).ravel(), g["conv"])
    assert np.array_equal(ep.conv2d_fwd_fused(d, x, w, sc, bi).ravel(), g["affine"])
    assert np.array_equal(ep.conv2d_fwd_fused(d, x, w, sc, bi, res).ravel(), g["sum"])
    assert np.array_equal(ep.conv2d_fwd_fused(d, x, w, sc, bi, res, relu=True).ravel(), g["relu_sum"])
    assert np.array_equal(ep.conv2d_fwd_fused(d, x, w, sc, bi, None, relu=True).ravel(), g["relu_affine"])


def _case(seed, N=2, H=7, W=6, C=8, K=5, R=3, S=3, stride=(1, 1), pad=(1, 1), dil=(1, 1)):
    rng = np.random.default_rng(seed)
    d = oracle.make_desc(N, H, W, C, K, R, S, stride, pad, dil)
    ho, wo = oracle.out_shape(d)
    x = rng.standard_normal((N, H, W, C)).astype(np.float16)
    w = (rng.standard_normal((K, R, S, C)) * 0.25).astype(np.float16)
    dy = rng.standard_normal((N, ho, wo, K)).astype(np.float16)
    return d, x, w, dy, rng


def test_scale_folds_into_the_filter_per_output_channel():
    """Power-of-two factors keep scale[k]*w[k] exact in binary16, so the affine map must equal
    the plain (separately pinned) convolution with the folded filter, plus the bias."""
    d, x, w, _, rng = _case(1, stride=(2, 1))
    scale = np.array([0.5, -2.0, 4.0, 1.0, -0.25], dtype=np.float32)
    bias = rng.standard_normal(d.K).astype(np.float32)
    folded = (w.astype(np.float64) * scale.astype(np.float64)[:, None, None, None]).astype(np.float16)
    assert np.array_equal(folded.astype(np.float64), w.astype(np.float64) * scale[:, None, None, None])
    want = oracle.conv2d_fwd(d, x, folded) + bias.astype(np.float64)[None, None, None, :]
    got = ep.conv2d_fwd_fused(d, x, w, scale, bias)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)


def test_frozen_batch_norm_formula():
    d, x, w, _, rng = _case(2)
    gamma, beta = rng.standard_normal(d.K), rng.standard_normal(d.K)
    mean, var = rng.standard_normal(d.K), rng.uniform(0.5, 2.0, d.K)
    eps = 1e-5
    scale, bias = ep.frozen_bn_affine(gamma, beta, mean, var, eps)
    s32, b32 = scale.astype(np.float32), bias.astype(np.float32)
    z = oracle.conv2d_fwd(d, x, w)
    # inference formula with the binary32 factors the fused call is given
    want = s32.astype(np.float64) * z + b32.astype(np.float64)
    np.testing.assert_allclose(ep.conv2d_fwd_fused(d, x, w, s32, b32), want, rtol=1e-13, atol=1e-13)
    # and the folding itself against the textbook normalisation
    bn = gamma * (z - mean) / np.sqrt(var + eps) + beta
    np.testing.assert_allclose(scale * z + bias, bn, rtol=1e-12, atol=1e-12)


def test_identity_convolution_leaves_the_elementwise_part():
    rng = np.random.default_rng(3)
    C = 6
    d = oracle.make_desc(2, 5, 4, C, C, 1, 1)
    x = rng.standard_normal((2, 5, 4, C)).astype(np.float16)
    w = np.eye(C, dtype=np.float16).reshape(C, 1, 1, C)
    scale, bias = rng.standard_normal(C).astype(np.float32), rng.standard_normal(C).astype(np.float32)
    res = rng.standard_normal((2, 5, 4, C)).astype(np.float16)
    v = x.astype(np.float64) * scale.astype(np.float64) + bias.astype(np.float64) + res.astype(np.float64)
    assert np.array_equal(ep.conv2d_fwd_fused(d, x, w, scale, bias, res, relu=True), np.maximum(v, 0.0))
    assert np.array_equal(ep.conv2d_fwd_fused(d, x, w, scale, bias, res, relu=False), v)
    # order matters: the shortcut is added before the ReLU, not after it
    after = np.maximum(x.astype(np.float64) * scale + bias, 0.0) + res.astype(np.float64)
    assert not np.array_equal(ep.conv2d_fwd_fused(d, x, w, scale, bias, res, relu=True), after)


def _brute_conv(a, w, stride, pad, dil):
    """Direct convolution of an fp64 NHWC tensor (tiny sizes only)."""
    N, H, W, C = a.shape
    K, R, S, _ = w.shape
    ho = (H + 2 * pad[0] - dil[0] * (R - 1) - 1) // stride[0] + 1
    wo = (W + 2 * pad[1] - dil[1] * (S - 1) - 1) // stride[1] + 1
    y = np.zeros((N, ho, wo, K))
    for n in range(N):
        for i in range(ho):
            for j in range(wo):
                for r in range(R):
                    for s in range(S):
                        h, q = i * stride[0] - pad[0] + r * dil[0], j * stride[1] - pad[1] + s * dil[1]
                        if 0 <= h < H and 0 <= q < W:
                            y[n, i, j, :] += w[:, r, s, :] @ a[n, h, q, :]
    return y


@pytest.mark.parametrize("stride,pad,dil", [((1, 1), (1, 1), (1, 1)), ((2, 2), (1, 1), (1, 1)), ((1, 2), (2, 2), (2, 2))])
def test_data_gradient_matches_finite_differences(stride, pad, dil):
    """L(z) = <conv(relu(s*z + b), w), dy>; dL/dz by central differences of a brute-force
    forward, at points away from the ReLU kink."""
    rng = np.random.default_rng(4)
    N, H, W, C, K, R, S = 1, 5, 4, 3, 2, 3, 3
    d = oracle.make_desc(N, H, W, C, K, R, S, stride, pad, dil)
    ho, wo = oracle.out_shape(d)
    s = np.array([0.5, -2.0, 1.0], dtype=np.float32)       # powers of two: a = s*z + b stays exact
    b = np.array([0.25, -0.5, 0.0], dtype=np.float32)
    z = (rng.integers(-8, 9, (N, H, W, C)) / 4.0 + 0.125)   # multiples of 1/8, never on the kink
    a = np.maximum(z * s + b, 0.0)
    a16 = a.astype(np.float16)
    assert np.array_equal(a16.astype(np.float64), a)
    w = (rng.integers(-4, 5, (K, R, S, C)) / 4.0).astype(np.float16)
    dy = (rng.integers(-4, 5, (N, ho, wo, K)) / 2.0).astype(np.float16)

    def loss(zz):
        return float(np.sum(_brute_conv(np.maximum(zz * s + b, 0.0), w.astype(np.float64), stride, pad, dil)
                            * dy.astype(np.float64)))

    got = ep.conv2d_dgrad_fused(d, dy, w, scale=s, relu_mask=a16)
    h = 1.0 / 64
    for idx in np.ndindex(z.shape):
        zp, zm = z.copy(), z.copy()
        zp[idx] += h
        zm[idx] -= h
        fd = (loss(zp) - loss(zm)) / (2 * h)                # L is piecewise linear: exact up to rounding
        assert abs(got[idx] - fd) < 1e-9, (idx, got[idx], fd)


def test_data_gradient_mask_is_strict_and_optional():
    d, x, w, dy, rng = _case(5)
    plain = oracle.conv2d_dgrad(d, dy, w)
    assert np.array_equal(ep.conv2d_dgrad_fused(d, dy, w), plain)
    ones = np.ones((d.N, d.H, d.W, d.C), dtype=np.float16)
    assert np.array_equal(ep.conv2d_dgrad_fused(d, dy, w, relu_mask=ones), plain)
    assert not ep.conv2d_dgrad_fused(d, dy, w, relu_mask=ones * 0).any()        # gradient 0 at 0
    assert not ep.conv2d_dgrad_fused(d, dy, w, relu_mask=-ones).any()
    scale = rng.standard_normal(d.C).astype(np.float32)
    assert np.array_equal(ep.conv2d_dgrad_fused(d, dy, w, scale=scale, relu_mask=ones),
                          plain * scale.astype(np.float64)[None, None, None, :])


def test_argument_checks():
    d, x, w, dy, _ = _case(6)
    with pytest.raises(TypeError):
        ep.conv2d_fwd_fused(d, x, w, scale=np.ones(d.K))                 # fp64 vector
    with pytest.raises(TypeError):
        ep.conv2d_fwd_fused(d, x, w, scale=np.ones(d.C + 1, np.float32))  # wrong length
    with pytest.raises(TypeError):
        ep.conv2d_dgrad_fused(d, dy, w, relu_mask=np.ones((d.N, d.H, d.W, d.C), np.float32))


def test_sampled_mode_picks_the_same_elements_and_channels():
    """fwd_tail / dgrad_tail on flat elements idx must give what indexing the whole result gives:
    the channel of a flat NHWC index is its remainder modulo the channel count (checked with
    per-channel vectors that hold the channel number, whose effect can be read off the result)."""
    d, x, w, dy, rng = _case(9, stride=(2, 2))
    ho, wo = oracle.out_shape(d)
    idx = np.array([0, 1, d.K - 1, d.K, 3 * d.K + 2, d.N * ho * wo * d.K - 1])
    sc = rng.standard_normal(d.K).astype(np.float32)
    bi = rng.standard_normal(d.K).astype(np.float32)
    res = rng.standard_normal((d.N, ho, wo, d.K)).astype(np.float16)
    full = ep.conv2d_fwd_fused(d, x, w, sc, bi, res, relu=True)
    assert np.array_equal(ep.conv2d_fwd_fused(d, x, w, sc, bi, res, relu=True, idx=idx), full.ravel()[idx])
    # bias = channel number on a zero convolution: the sampled result is the channel of each index
    chan = np.arange(d.K, dtype=np.float32)
    got = ep.fwd_tail(np.zeros(idx.size), d, bias=chan, idx=idx)
    assert np.array_equal(got, [0, 1, d.K - 1, 0, 2, d.K - 1])
    jdx = np.array([0, d.C - 1, d.C, 5 * d.C + 3, d.N * d.H * d.W * d.C - 1])
    dsc = rng.standard_normal(d.C).astype(np.float32)
    mask = np.maximum(rng.standard_normal((d.N, d.H, d.W, d.C)), 0).astype(np.float16)
    fulld = ep.conv2d_dgrad_fused(d, dy, w, dsc, mask)
    assert np.array_equal(ep.conv2d_dgrad_fused(d, dy, w, dsc, mask, idx=jdx), fulld.ravel()[jdx])
    got = ep.dgrad_tail(np.ones(jdx.size), d, scale=np.arange(d.C, dtype=np.float32), idx=jdx)
    assert np.array_equal(got, [0, d.C - 1, 0, 3, d.C - 1])
    # the tails applied to a precomputed convolution are the fused calls
    assert np.array_equal(ep.fwd_tail(oracle.conv2d_fwd(d, x, w), d, sc, bi, res, True), full)
    assert np.array_equal(ep.dgrad_tail(oracle.conv2d_dgrad(d, dy, w), d, dsc, mask), fulld)
