"""Pins of the single-precision entry points of the convolution oracle: they must give what
the (separately pinned) half-precision entry points give on values that both formats hold
exactly, and on values only binary32 holds they must match a brute-force float64 contraction
written with a library einsum over an explicitly gathered patch tensor, and the adjoint
identities."""
import numpy as np
import pytest

import oracle

CASES = [
    # N  H  W  C  K  R  S  stride  pad     dil
    (2, 7, 6, 4, 5, 3, 3, (1, 1), (1, 1), (1, 1)),
    (1, 9, 8, 3, 4, 3, 2, (2, 1), (1, 0), (1, 2)),
    (1, 6, 6, 8, 8, 1, 1, (2, 2), (0, 0), (1, 1)),
]


def _mk(case, seed, dtype):
    N, H, W, C, K, R, S, st, pd, dl = case
    d = oracle.make_desc(N, H, W, C, K, R, S, st, pd, dl)
    ho, wo = oracle.out_shape(d)
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, H, W, C)).astype(dtype)
    w = rng.standard_normal((K, R, S, C)).astype(dtype)
    g = rng.standard_normal((N, ho, wo, K)).astype(dtype)
    return d, x, w, g


@pytest.mark.parametrize("case", CASES)
def test_same_as_half_entry_points_on_half_values(case):
    d, x, w, g = _mk(case, 1, np.float16)
    x32, w32, g32 = x.astype(np.float32), w.astype(np.float32), g.astype(np.float32)
    assert np.array_equal(oracle.conv2d_fwd_f32(d, x32, w32), oracle.conv2d_fwd(d, x, w))
    assert np.array_equal(oracle.conv2d_dgrad_f32(d, g32, w32), oracle.conv2d_dgrad(d, g, w))
    assert np.array_equal(oracle.conv2d_wgrad_f32(d, x32, g32), oracle.conv2d_wgrad(d, x, g))


def _patches(x, case, ho, wo):
    """[N][ho][wo][R][S][C] gather of x with zero padding, float64."""
    N, H, W, C, K, R, S, st, pd, dl = case
    p = np.zeros((N, ho, wo, R, S, C))
    for i in range(ho):
        for j in range(wo):
            for r in range(R):
                for s in range(S):
                    h, q = i * st[0] - pd[0] + r * dl[0], j * st[1] - pd[1] + s * dl[1]
                    if 0 <= h < H and 0 <= q < W:
                        p[:, i, j, r, s, :] = x[:, h, q, :]
    return p


@pytest.mark.parametrize("case", CASES)
def test_against_einsum_on_binary32_only_values(case):
    d, x, w, g = _mk(case, 2, np.float32)
    assert not np.array_equal(x.astype(np.float16).astype(np.float32), x)     # really beyond binary16
    ho, wo = oracle.out_shape(d)
    x64, w64, g64 = x.astype(np.float64), w.astype(np.float64), g.astype(np.float64)
    pt = _patches(x64, case, ho, wo)
    np.testing.assert_allclose(oracle.conv2d_fwd_f32(d, x, w), np.einsum("nijrsc,krsc->nijk", pt, w64),
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_wgrad_f32(d, x, g), np.einsum("nijk,nijrsc->krsc", g64, pt),
                               rtol=1e-12, atol=1e-12)
    # adjoint identity <fwd(x, w), g> == <x, dgrad(g, w)>
    lhs = float(np.sum(oracle.conv2d_fwd_f32(d, x, w) * g64))
    rhs = float(np.sum(x64 * oracle.conv2d_dgrad_f32(d, g, w)))
    assert abs(lhs - rhs) <= 1e-10 * (1 + abs(lhs))
    # and dgrad element by element through one-hot probes of the forward map
    dx = oracle.conv2d_dgrad_f32(d, g, w)
    rng = np.random.default_rng(3)
    for _ in range(8):
        idx = tuple(rng.integers(0, n) for n in x.shape)
        e = np.zeros_like(x)
        e[idx] = 1.0
        want = float(np.sum(oracle.conv2d_fwd_f32(d, e, w) * g64))
        assert abs(dx[idx] - want) <= 1e-12 * (1 + abs(want))


def test_dtype_is_checked():
    d, x, w, g = _mk(CASES[0], 4, np.float32)
    with pytest.raises(TypeError):
        oracle.conv2d_fwd_f32(d, x.astype(np.float64), w)
    with pytest.raises(TypeError):
        oracle.conv2d_fwd(d, x, w)
