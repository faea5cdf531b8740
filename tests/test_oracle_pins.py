"""Pins for the CPU oracle: each test checks it against something other than itself --
a brute-force im2col + library matmul, plain matmul for 1x1, adjoint identities probed
with one-hot tensors, hand-written closed forms, invariants, and an independent library
convolution in float64.  No GPU needed."""
import itertools
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

# (N,H,W,C,K,R,S,stride,pad,dil): odd sizes, R != S, H != W, stride/pad/dil mixes
CASES = [
    (1, 5, 6, 3, 4, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 7, 5, 4, 3, 3, 2, (2, 1), (1, 0), (1, 1)),
    (1, 9, 8, 2, 5, 3, 3, (2, 2), (1, 1), (1, 1)),
    (2, 8, 9, 3, 2, 2, 3, (1, 2), (0, 2), (2, 1)),
    (1, 11, 10, 1, 1, 3, 3, (3, 2), (2, 3), (2, 2)),
    (1, 6, 6, 5, 7, 1, 1, (2, 2), (0, 0), (1, 1)),
    (1, 4, 4, 2, 3, 1, 1, (3, 3), (0, 0), (1, 1)),
    (2, 10, 7, 3, 4, 7, 7, (2, 2), (3, 3), (1, 1)),
    (1, 6, 7, 2, 2, 3, 3, (1, 1), (0, 0), (1, 1)),
]


def _rand_half(rng, shape, sigma=1.0):
    return (rng.standard_normal(shape) * sigma).astype(np.float16)


def _tensors(case, seed=0):
    N, H, W, C, K, R, S, st, pd, dl = case
    d = oracle.make_desc(N, H, W, C, K, R, S, st, pd, dl)
    Ho, Wo = oracle.out_shape(d)
    rng = np.random.default_rng(seed)
    x = _rand_half(rng, (N, H, W, C))
    w = _rand_half(rng, (K, R, S, C), 0.5)
    g = _rand_half(rng, (N, Ho, Wo, K))
    return d, x, w, g, Ho, Wo


def _im2col(x, R, S, st, pd, dl, Ho, Wo):
    """Explicit [N*Ho*Wo, R*S*C] patch matrix by indexing, zeros outside the image."""
    N, H, W, C = x.shape
    cols = np.zeros((N, Ho, Wo, R, S, C), dtype=np.float64)
    for n, ho, wo, r, s in itertools.product(range(N), range(Ho), range(Wo), range(R), range(S)):
        h = ho * st[0] - pd[0] + r * dl[0]
        wi = wo * st[1] - pd[1] + s * dl[1]
        if 0 <= h < H and 0 <= wi < W:
            cols[n, ho, wo, r, s, :] = x[n, h, wi, :]
    return cols.reshape(N * Ho * Wo, R * S * C)


@pytest.mark.parametrize("case", CASES)
def test_out_shape_matches_counting(case):
    """Output extent = number of window positions that fit, counted one by one."""
    N, H, W, C, K, R, S, st, pd, dl = case
    d = oracle.make_desc(N, H, W, C, K, R, S, st, pd, dl)
    Ho, Wo = oracle.out_shape(d)
    cnt_h = sum(1 for o in range(0, H + 2 * pd[0], st[0]) if o + dl[0] * (R - 1) < H + 2 * pd[0])
    cnt_w = sum(1 for o in range(0, W + 2 * pd[1], st[1]) if o + dl[1] * (S - 1) < W + 2 * pd[1])
    assert (Ho, Wo) == (cnt_h, cnt_w)


@pytest.mark.parametrize("case", CASES)
def test_fwd_equals_im2col_matmul(case):
    d, x, w, g, Ho, Wo = _tensors(case)
    N, H, W, C, K, R, S, st, pd, dl = case
    cols = _im2col(x.astype(np.float64), R, S, st, pd, dl, Ho, Wo)
    ref = (cols @ w.astype(np.float64).reshape(K, R * S * C).T).reshape(N, Ho, Wo, K)
    got = oracle.conv2d_fwd(d, x, w)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("case", CASES)
def test_wgrad_and_dgrad_equal_im2col_transposes(case):
    """With A = im2col(x): dw = g^T A, and dx = col2im(g W) (scatter-add of patches)."""
    d, x, w, g, Ho, Wo = _tensors(case, seed=1)
    N, H, W, C, K, R, S, st, pd, dl = case
    A = _im2col(x.astype(np.float64), R, S, st, pd, dl, Ho, Wo)
    G = g.astype(np.float64).reshape(-1, K)
    dw_ref = (G.T @ A).reshape(K, R, S, C)
    np.testing.assert_allclose(oracle.conv2d_wgrad(d, x, g), dw_ref, rtol=1e-12, atol=1e-12)
    P = (G @ w.astype(np.float64).reshape(K, R * S * C)).reshape(N, Ho, Wo, R, S, C)
    dx_ref = np.zeros((N, H, W, C))
    for n, ho, wo, r, s in itertools.product(range(N), range(Ho), range(Wo), range(R), range(S)):
        h = ho * st[0] - pd[0] + r * dl[0]
        wi = wo * st[1] - pd[1] + s * dl[1]
        if 0 <= h < H and 0 <= wi < W:
            dx_ref[n, h, wi, :] += P[n, ho, wo, r, s, :]
    np.testing.assert_allclose(oracle.conv2d_dgrad(d, g, w), dx_ref, rtol=1e-12, atol=1e-12)


def test_1x1_is_matmul_all_passes():
    N, H, W, C, K = 2, 5, 7, 6, 9
    d = oracle.make_desc(N, H, W, C, K, 1, 1)
    rng = np.random.default_rng(3)
    x, w, g = _rand_half(rng, (N, H, W, C)), _rand_half(rng, (K, 1, 1, C)), _rand_half(rng, (N, H, W, K))
    X, Wm, G = x.astype(np.float64).reshape(-1, C), w.astype(np.float64).reshape(K, C), g.astype(np.float64).reshape(-1, K)
    np.testing.assert_allclose(oracle.conv2d_fwd(d, x, w).reshape(-1, K), X @ Wm.T, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.conv2d_dgrad(d, g, w).reshape(-1, C), G @ Wm, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.conv2d_wgrad(d, x, g).reshape(K, C), G.T @ X, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("case", CASES)
def test_adjoint_identities(case):
    d, x, w, g, Ho, Wo = _tensors(case, seed=2)
    y = oracle.conv2d_fwd(d, x, w)
    dx = oracle.conv2d_dgrad(d, g, w)
    dw = oracle.conv2d_wgrad(d, x, g)
    a = np.sum(y * g.astype(np.float64))
    b = np.sum(x.astype(np.float64) * dx)
    c = np.sum(w.astype(np.float64) * dw)
    scale = max(1.0, abs(a))
    assert abs(a - b) <= 1e-11 * scale
    assert abs(a - c) <= 1e-11 * scale


@pytest.mark.parametrize("case", CASES[:6])
def test_adjoints_entrywise_with_one_hot_probes(case):
    """dx[i] = <fwd(e_i, w), g> and dw[j] = <fwd(x, e_j), g>: pins every entry, not only
    the inner product."""
    d, x, w, g, Ho, Wo = _tensors(case, seed=4)
    g64 = g.astype(np.float64)
    dx = oracle.conv2d_dgrad(d, g, w).ravel()
    dw = oracle.conv2d_wgrad(d, x, g).ravel()
    rng = np.random.default_rng(5)
    for i in rng.choice(x.size, size=min(x.size, 25), replace=False):
        e = np.zeros(x.size, np.float16); e[i] = 1
        assert abs(np.sum(oracle.conv2d_fwd(d, e.reshape(x.shape), w) * g64) - dx[i]) <= 1e-11 * (1 + abs(dx[i]))
    for j in rng.choice(w.size, size=min(w.size, 25), replace=False):
        e = np.zeros(w.size, np.float16); e[j] = 1
        assert abs(np.sum(oracle.conv2d_fwd(d, x, e.reshape(w.shape)) * g64) - dw[j]) <= 1e-11 * (1 + abs(dw[j]))


@pytest.mark.parametrize("r0,s0,stride,pad,dil", [(0, 0, 1, 1, 1), (2, 1, 1, 1, 1), (1, 2, 2, 1, 1), (0, 2, 1, 2, 2)])
def test_delta_kernel_is_shifted_copy(r0, s0, stride, pad, dil):
    """A one-tap identity kernel copies x at offset (r0*dil - pad, s0*dil - pad): pins
    orientation (no flip) and the padding offset."""
    N, H, W, C = 1, 7, 8, 3
    d = oracle.make_desc(N, H, W, C, C, 3, 3, (stride, stride), (pad, pad), (dil, dil))
    Ho, Wo = oracle.out_shape(d)
    x = _rand_half(np.random.default_rng(6), (N, H, W, C))
    w = np.zeros((C, 3, 3, C), np.float16)
    for c in range(C):
        w[c, r0, s0, c] = 1
    y = oracle.conv2d_fwd(d, x, w)
    for ho, wo in itertools.product(range(Ho), range(Wo)):
        h, wi = ho * stride - pad + r0 * dil, wo * stride - pad + s0 * dil
        ref = x[0, h, wi].astype(np.float64) if (0 <= h < H and 0 <= wi < W) else np.zeros(C)
        assert np.array_equal(y[0, ho, wo], ref)


def _load_grid(name):
    rows = [l.split() for l in open(os.path.join(GOLDEN, name)) if l.strip() and not l.startswith("#")]
    return np.array(rows, dtype=np.float64)


def test_all_ones_border_counts_golden():
    counts = _load_grid("ones_border_counts.txt")
    C, K = 5, 2
    d = oracle.make_desc(1, 4, 5, C, K, 3, 3, pad=(1, 1))
    y = oracle.conv2d_fwd(d, np.ones((1, 4, 5, C), np.float16), np.ones((K, 3, 3, C), np.float16))
    for k in range(K):
        assert np.array_equal(y[0, :, :, k], C * counts)
    # adjoint views of the same picture: dx with dy == 1 counts the windows covering a pixel
    # (same table for 3x3 p1 s1 times K); dw sums the number of outputs whose tap is in range.
    dx = oracle.conv2d_dgrad(d, np.ones((1, 4, 5, K), np.float16), np.ones((K, 3, 3, C), np.float16))
    assert np.array_equal(dx[0, :, :, 0], K * counts)
    dw = oracle.conv2d_wgrad(d, np.ones((1, 4, 5, C), np.float16), np.ones((1, 4, 5, K), np.float16))
    rows = np.array([3, 4, 3]); cols = np.array([4, 5, 4])   # valid output rows/cols per tap
    assert np.array_equal(dw[0, :, :, 0], np.outer(rows, cols))


def test_all_ones_counts_stride2_dilation2_golden():
    counts = _load_grid("ones_border_counts_s2_d2.txt")
    C = 3
    d = oracle.make_desc(1, 5, 6, C, 1, 3, 3, (2, 2), (2, 2), (2, 2))
    assert oracle.out_shape(d) == (3, 3)
    y = oracle.conv2d_fwd(d, np.ones((1, 5, 6, C), np.float16), np.ones((1, 3, 3, C), np.float16))
    assert np.array_equal(y[0, :, :, 0], C * counts)


def test_stride_is_subsampling_of_stride1():
    N, H, W, C, K = 1, 9, 10, 3, 2
    rng = np.random.default_rng(7)
    x, w = _rand_half(rng, (N, H, W, C)), _rand_half(rng, (K, 3, 3, C))
    y1 = oracle.conv2d_fwd(oracle.make_desc(N, H, W, C, K, 3, 3, (1, 1), (1, 1)), x, w)
    for sh, sw in [(2, 2), (3, 2), (2, 3)]:
        ys = oracle.conv2d_fwd(oracle.make_desc(N, H, W, C, K, 3, 3, (sh, sw), (1, 1)), x, w)
        assert np.array_equal(ys, y1[:, ::sh, ::sw, :][:, :ys.shape[1], :ys.shape[2], :])


def test_dilation_equals_zero_stuffed_kernel():
    N, H, W, C, K = 1, 10, 9, 2, 3
    rng = np.random.default_rng(8)
    x, w = _rand_half(rng, (N, H, W, C)), _rand_half(rng, (K, 3, 3, C))
    g_shape = None
    for dh, dw_ in [(2, 2), (2, 1), (1, 3)]:
        big = np.zeros((K, 2 * dh + 1, 2 * dw_ + 1, C), np.float16)
        big[:, ::dh, ::dw_, :] = w
        dd = oracle.make_desc(N, H, W, C, K, 3, 3, (1, 1), (2, 2), (dh, dw_))
        ds = oracle.make_desc(N, H, W, C, K, 2 * dh + 1, 2 * dw_ + 1, (1, 1), (2, 2), (1, 1))
        yd, ys = oracle.conv2d_fwd(dd, x, w), oracle.conv2d_fwd(ds, x, big)
        np.testing.assert_allclose(yd, ys, rtol=1e-13, atol=1e-13)
        g = _rand_half(rng, yd.shape)
        np.testing.assert_allclose(oracle.conv2d_dgrad(dd, g, w), oracle.conv2d_dgrad(ds, g, big), rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(oracle.conv2d_wgrad(dd, x, g), oracle.conv2d_wgrad(ds, x, g)[:, ::dh, ::dw_, :], rtol=1e-13, atol=1e-13)


def test_linearity_in_each_argument():
    case = CASES[2]
    d, x1, w, g, Ho, Wo = _tensors(case, seed=9)
    _, x2, w2, g2, _, _ = _tensors(case, seed=10)
    # sums of binary16 values are not binary16: check on values with few mantissa bits
    q = lambda a: (np.round(a.astype(np.float64) * 8) / 8).astype(np.float16)
    x1, x2, w, w2 = q(x1), q(x2), q(w), q(w2)
    y = oracle.conv2d_fwd(d, (x1.astype(np.float32) + 2 * x2.astype(np.float32)).astype(np.float16), w)
    np.testing.assert_allclose(y, oracle.conv2d_fwd(d, x1, w) + 2 * oracle.conv2d_fwd(d, x2, w), rtol=1e-13, atol=1e-12)
    y = oracle.conv2d_fwd(d, x1, (w.astype(np.float32) - w2.astype(np.float32)).astype(np.float16))
    np.testing.assert_allclose(y, oracle.conv2d_fwd(d, x1, w) - oracle.conv2d_fwd(d, x1, w2), rtol=1e-13, atol=1e-12)


@pytest.mark.parametrize("case", CASES)
def test_against_library_conv_float64(case):
    """Third opinion: torch's CPU float64 convolution and its autograd."""
    d, x, w, g, Ho, Wo = _tensors(case, seed=11)
    N, H, W, C, K, R, S, st, pd, dl = case
    xt = torch.tensor(x.astype(np.float64)).permute(0, 3, 1, 2).requires_grad_(True)
    wt = torch.tensor(w.astype(np.float64)).permute(0, 3, 1, 2).requires_grad_(True)
    yt = torch.nn.functional.conv2d(xt, wt, stride=st, padding=pd, dilation=dl)
    gt = torch.tensor(g.astype(np.float64)).permute(0, 3, 1, 2)
    dxt, dwt = torch.autograd.grad(yt, (xt, wt), gt)
    np.testing.assert_allclose(oracle.conv2d_fwd(d, x, w), yt.detach().permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_dgrad(d, g, w), dxt.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oracle.conv2d_wgrad(d, x, g), dwt.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)


def test_dgrad_untouched_positions_are_zero():
    """1x1 stride 2: only even pixels receive gradient; the rest is the empty sum."""
    d = oracle.make_desc(1, 6, 6, 2, 3, 1, 1, (2, 2))
    rng = np.random.default_rng(12)
    g, w = _rand_half(rng, (1, 3, 3, 3)), _rand_half(rng, (3, 1, 1, 2))
    dx = oracle.conv2d_dgrad(d, g, w)
    mask = np.zeros((6, 6), bool); mask[::2, ::2] = True
    assert np.all(dx[0][~mask] == 0.0)
    np.testing.assert_allclose(dx[0][::2, ::2].reshape(-1, 2), g.astype(np.float64).reshape(-1, 3) @ w.astype(np.float64).reshape(3, 2), rtol=1e-13)


def test_sampled_elements_equal_full_tensor():
    d, x, w, g, Ho, Wo = _tensors(CASES[1], seed=13)
    for fn, a, b in [(oracle.conv2d_fwd, x, w), (oracle.conv2d_dgrad, g, w), (oracle.conv2d_wgrad, x, g)]:
        full = fn(d, a, b).ravel()
        idx = np.random.default_rng(14).choice(full.size, size=17, replace=False)
        assert np.array_equal(fn(d, a, b, idx=idx), full[idx])


def test_half_decoding_is_exact_for_all_bit_patterns():
    """All 65536 binary16 patterns through a 1x1 conv with weight 1 reproduce numpy's
    widening (subnormals kept, inf/NaN propagate)."""
    bits = np.arange(65536, dtype=np.uint16).view(np.float16)
    d = oracle.make_desc(1, 256, 256, 1, 1, 1, 1)
    with np.errstate(invalid="ignore"):
        y = oracle.conv2d_fwd(d, bits.reshape(1, 256, 256, 1), np.ones((1, 1, 1, 1), np.float16)).ravel()
    ref = bits.astype(np.float64)
    assert np.array_equal(np.isnan(y), np.isnan(ref))
    ok = ~np.isnan(ref)
    assert np.array_equal(y[ok], ref[ok])


# ---- unscale + overflow flag -------------------------------------------------------

def test_unscale_bits_golden():
    rows = [l.split()[:2] for l in open(os.path.join(GOLDEN, "unscale_bits.txt")) if l.strip() and not l.startswith("#")]
    g = np.array([int(a, 16) for a, _ in rows], dtype=np.uint32).view(np.float32)
    want = np.array([int(b, 16) for _, b in rows], dtype=np.uint32)
    out, flag = oracle.unscale_check(g, 2.0 ** -10)
    assert np.array_equal(out.view(np.uint32), want)
    assert flag == 1   # the fixture holds +inf and -inf


def test_unscale_general_factor_is_correctly_rounded():
    rng = np.random.default_rng(15)
    g = (rng.standard_normal(4099) * 10.0 ** rng.uniform(-30, 30, 4099)).astype(np.float32)
    inv = np.float32(1.0 / 3.0)
    out, flag = oracle.unscale_check(g, float(inv))
    assert flag == 0
    assert np.array_equal(out, g * inv)          # numpy's fp32 multiply is correctly rounded
    # exact check through integers: |out - g*inv| <= half an ulp of out
    exact = g.astype(np.float64) * np.float64(inv)
    ulp = np.spacing(np.abs(out)).astype(np.float64)
    assert np.all(np.abs(out.astype(np.float64) - exact) <= 0.5 * ulp)


@pytest.mark.parametrize("n", [0, 1, 63, 64, 65, 1000])
def test_flag_cases(n):
    base = np.linspace(-3, 3, n).astype(np.float32)
    out, flag = oracle.unscale_check(base, 0.5)
    assert flag == 0 and np.array_equal(out, base * np.float32(0.5))
    if n == 0:
        return
    for pos in {0, n - 1, n // 2}:
        for bad in (np.inf, -np.inf, np.nan):
            g = base.copy(); g[pos] = bad
            out, flag = oracle.unscale_check(g, 0.5)
            assert flag == 1
            assert (np.isnan(out[pos]) if np.isnan(bad) else out[pos] == bad)
    g = base.copy(); g[0] = np.finfo(np.float32).max; g[-1] = np.float32(1e-45)
    assert oracle.unscale_check(g, 0.5)[1] == 0


def test_flag_looks_at_inputs_not_outputs():
    g = np.array([np.finfo(np.float32).max, 1.0], np.float32)
    out, flag = oracle.unscale_check(g, 4.0)      # finite in, inf out
    assert flag == 0 and np.isinf(out[0])
