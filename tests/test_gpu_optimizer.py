"""GPU parity of the optimizer tail against oracle/optimizer.py, through the C ABI.
Everything here is a chain of single binary32 operations plus one binary16 cast, so the bar
is bit-exact: master weights, momentum, half weights, unscaled gradients, flag and state."""
import numpy as np
import pytest
import torch

import paper_1903_05831_amd as sd
from oracle import optimizer as opt

from gpu_harness import say

pytestmark = pytest.mark.gpu
F = np.float32


def _state(scale, good):
    a = np.zeros(2, dtype=np.int32)
    a[0] = np.array([scale], dtype=F).view(np.int32)[0]
    a[1] = good
    return torch.from_numpy(a).cuda()


def _read_state(t):
    a = t.cpu().numpy()
    return float(a[:1].view(F)[0]), int(a[1])


def _bits(a):
    return np.ascontiguousarray(a).view(np.uint32 if a.dtype == F else np.uint16)


@pytest.mark.parametrize("n", [0, 1, 3, 4, 5, 2047, 2048, 2049, 100003, 1 << 20])
@pytest.mark.parametrize("overflow", [False, True])
def test_sgd_momentum_update_bit_exact(n, overflow):
    say(f"sgd n={n} overflow={overflow}")
    rng = np.random.default_rng(n * 2 + int(overflow))
    w = (rng.standard_normal(n) * 0.05).astype(F)
    m = (rng.standard_normal(n) * 0.01).astype(F)
    g = rng.standard_normal(n).astype(F)
    if n > 8:
        w[:4] = [65520.0, 2.0 ** -24, 2.0 ** -25, 1.0 + 2.0 ** -11]      # cast: overflow, subnormals, tie
        w[4] = -0.0
        g[5] = 1e-40                                                      # fp32 subnormal gradient
    lr, mu, wd = 0.02, 0.9, 1e-4
    st = torch.cuda.current_stream().cuda_stream
    dw, dm, dg = (torch.from_numpy(a.copy()).cuda() for a in (w, m, g))
    dh = torch.full((max(n, 1),), 7.0, dtype=torch.float16, device="cuda")
    flag = torch.tensor([1 if overflow else 0], dtype=torch.int32, device="cuda")
    state = _state(1024.0, 1)
    sd.sgd_momentum_update(dw, dm, dg, dh, n, lr, mu, wd, flag, state, 2.0, 0.5, 2, st)
    torch.cuda.synchronize()
    rw, rm, rh = opt.sgd_momentum_update(w, m, g, lr, mu, wd, overflow)
    assert np.array_equal(_bits(dw.cpu().numpy()), _bits(rw))
    assert np.array_equal(_bits(dm.cpu().numpy()), _bits(rm))
    assert np.array_equal(_bits(dh.cpu().numpy()[:n]), _bits(rh))
    assert np.array_equal(dg.cpu().numpy().view(np.uint32), g.view(np.uint32)), "grad is read only"
    assert int(flag.item()) == int(overflow), "flag is read only"
    rs, rgood = opt.loss_scale_next(1024.0, 1, overflow, 2.0, 0.5, 2)
    assert _read_state(state) == (float(rs), rgood)


def test_loss_scale_state_machine_on_device():
    """A sequence of flags drives the device-side state like the oracle's (growth 2, backoff 1/2, interval 3)."""
    st = torch.cuda.current_stream().cuda_stream
    state = _state(65536.0, 0)
    z = torch.zeros(4, dtype=torch.float32, device="cuda")
    h = torch.zeros(4, dtype=torch.float16, device="cuda")
    s, gd = F(65536.0), 0
    for ov in (0, 0, 0, 1, 1, 0, 0, 1, 0, 0, 0, 0, 0, 0):
        flag = torch.tensor([ov], dtype=torch.int32, device="cuda")
        sd.sgd_momentum_update(z, z.clone(), z.clone(), h, 0, 0.1, 0.9, 0.0, flag, state, 2.0, 0.5, 3, st)
        torch.cuda.synchronize()
        s, gd = opt.loss_scale_next(s, gd, bool(ov), 2.0, 0.5, 3)
        assert _read_state(state) == (float(s), gd)


@pytest.mark.parametrize("scale", [1024.0, 3.0, 65536.0, 0.5, 1e-3])
@pytest.mark.parametrize("n", [0, 5, 4099, 1 << 18])
def test_dynamic_unscale_bit_exact(scale, n):
    say(f"dynamic unscale scale={scale} n={n}")
    rng = np.random.default_rng(int(scale * 10) + n)
    g = (rng.standard_normal(n) * 100.0).astype(F)
    bad = n > 100 and scale == 3.0
    if bad:
        g[n // 2] = -np.inf
        g[7] = np.nan
    st = torch.cuda.current_stream().cuda_stream
    dg = torch.from_numpy(g.copy()).cuda() if n else torch.zeros(1, device="cuda")
    flag = torch.tensor([5], dtype=torch.int32, device="cuda")
    state = _state(scale, 4)
    sd.grad_unscale_check_dynamic(dg, n, state, flag, st)
    torch.cuda.synchronize()
    ref, rflag = opt.unscale_check_dynamic(g, scale)
    got = dg.cpu().numpy()[:n]
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))
    assert int(flag.item()) == rflag == int(bad)
    assert _read_state(state) == (float(F(scale)), 4), "state is read only"


def test_full_tail_two_steps():
    """unscale (dynamic) -> update -> unscale -> update on the workload's gradient size, second
    step with an overflow: chained device results equal the chained oracle bit for bit."""
    n = 23454912 // 16
    rng = np.random.default_rng(99)
    w = (rng.standard_normal(n) * 0.05).astype(F)
    m = np.zeros(n, dtype=F)
    st = torch.cuda.current_stream().cuda_stream
    dw, dm = torch.from_numpy(w.copy()).cuda(), torch.from_numpy(m.copy()).cuda()
    dh = torch.empty(n, dtype=torch.float16, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    state = _state(1024.0, 0)
    s, gd = F(1024.0), 0
    for step in range(2):
        g = (rng.standard_normal(n) * 1024.0).astype(F)
        if step == 1:
            g[12345] = np.inf
        dg = torch.from_numpy(g.copy()).cuda()
        sd.grad_unscale_check_dynamic(dg, n, state, flag, st)
        sd.sgd_momentum_update(dw, dm, dg, dh, n, 0.01, 0.9, 1e-4, flag, state, 2.0, 0.5, 1, st)
        torch.cuda.synchronize()
        ug, ov = opt.unscale_check_dynamic(g, s)
        w, m, h = opt.sgd_momentum_update(w, m, ug, 0.01, 0.9, 1e-4, bool(ov))
        s, gd = opt.loss_scale_next(s, gd, bool(ov), 2.0, 0.5, 1)
        assert int(flag.item()) == ov == step
        assert np.array_equal(_bits(dw.cpu().numpy()), _bits(w))
        assert np.array_equal(_bits(dm.cpu().numpy()), _bits(m))
        assert np.array_equal(_bits(dh.cpu().numpy()), _bits(h))
        assert _read_state(state) == (float(s), gd)
