"""Pins for oracle/optimizer.py: closed forms, hand-derived bit patterns and a written-out
transition table, so that a wrong sign, a dropped term, a fused multiply-add or a different
rounding anywhere in it fails one of them.  CPU only."""
import os

import numpy as np
import pytest

from oracle import optimizer as opt

F = np.float32
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits32(x):
    return np.asarray(x, dtype=F).view(np.uint32)


def test_plain_sgd_closed_form():
    # mu = 0, wd = 0: w' = w - lr*g, mom' = -lr*g; powers of two keep everything exact
    w = np.array([1.0, -2.0, 0.5, 0.0], dtype=F)
    g = np.array([4.0, 0.25, -8.0, 1.0], dtype=F)
    w2, m2, h = opt.sgd_momentum_update(w, np.zeros(4, F), g, lr=0.125, mu=0.0, wd=0.0, overflow=False)
    assert np.array_equal(w2, np.array([0.5, -2.03125, 1.5, -0.125], dtype=F))
    assert np.array_equal(m2, np.array([-0.5, -0.03125, 1.0, -0.125], dtype=F))
    assert np.array_equal(h, w2.astype(np.float16))


def test_momentum_geometric_series():
    # constant gradient 1, lr = 1, mu = 1/2: mom_t = -(2 - 2^(1-t)), w_t = -sum_{i<=t} (2 - 2^(1-i))
    w, m = np.zeros(1, F), np.zeros(1, F)
    g = np.ones(1, F)
    acc = 0.0
    for t in range(1, 12):
        w, m, _ = opt.sgd_momentum_update(w, m, g, lr=1.0, mu=0.5, wd=0.0, overflow=False)
        mom_t = -(2.0 - 2.0 ** (1 - t))
        acc += mom_t
        assert m[0] == F(mom_t) and w[0] == F(acc)


def test_weight_decay_only():
    # g = 0, mu = 0: w' = w - lr*wd*w; lr*wd = 1/4 -> w_t = (3/4)^t exactly while 3^t fits 24 bits
    w, m = np.ones(1, F), np.zeros(1, F)
    for t in range(1, 12):
        w, m, _ = opt.sgd_momentum_update(w, m, np.zeros(1, F), lr=0.5, mu=0.0, wd=0.5, overflow=False)
        assert w[0] == F(0.75 ** t)


def test_sign_of_the_gradient_term():
    # a positive gradient must lower the weight, weight decay must pull towards zero
    w2, _, _ = opt.sgd_momentum_update(np.array([1.0], F), np.zeros(1, F), np.array([1.0], F), 0.1, 0.9, 0.0, False)
    assert w2[0] < 1.0
    w3, _, _ = opt.sgd_momentum_update(np.array([-1.0], F), np.zeros(1, F), np.zeros(1, F), 0.1, 0.0, 0.5, False)
    assert -1.0 < w3[0] < 0.0


def test_each_operation_rounds_on_its_own():
    # values for which a fused multiply-add (one rounding) differs from multiply, round, add:
    # mu*mom = (1 + 2^-12)^2 = 1 + 2^-11 + 2^-24 rounds to 1 + 2^-11 (tie to even); minus
    # lr*g = 1 + 2^-11 gives exactly 0 unfused, but -2^-24 ... fused would keep the 2^-24
    mu = F(1.0 + 2.0 ** -12)
    mom = np.array([1.0 + 2.0 ** -12], dtype=F)
    g = np.array([1.0 + 2.0 ** -11], dtype=F)
    _, m2, _ = opt.sgd_momentum_update(np.zeros(1, F), mom, g, lr=1.0, mu=mu, wd=0.0, overflow=False)
    assert m2[0] == F(0.0)
    fused = float(mu) * float(mom[0]) - float(g[0])
    assert fused != 0.0                                # the fused result is the one that must NOT come out


def test_half_cast_bit_patterns():
    # hand-derived binary16 patterns: exact, ties to even both ways, overflow, smallest subnormal
    w = np.array([1.0, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 65504.0, 65520.0, 2.0 ** -24,
                  2.0 ** -25, -0.0, 3 * 2.0 ** -25], dtype=F)
    _, _, h = opt.sgd_momentum_update(w, np.zeros_like(w), np.zeros_like(w), 0.0, 0.0, 0.0, overflow=True)
    want = np.array([0x3C00, 0x3C00, 0x3C02, 0x7BFF, 0x7C00, 0x0001, 0x0000, 0x8000, 0x0002], dtype=np.uint16)
    assert np.array_equal(h.view(np.uint16), want)


def test_overflow_skips_the_update():
    w = np.array([1.5, -2.5], dtype=F)
    m = np.array([0.25, 0.5], dtype=F)
    g = np.array([np.inf, 1.0], dtype=F)
    w2, m2, h = opt.sgd_momentum_update(w, m, g, 0.1, 0.9, 1e-4, overflow=True)
    assert np.array_equal(bits32(w2), bits32(w)) and np.array_equal(bits32(m2), bits32(m))
    assert np.array_equal(h, w.astype(np.float16))


def test_loss_scale_transition_table():
    # tests/golden/loss_scale_transitions.txt: scale good overflow -> scale' good'  (growth 2, backoff 1/2, interval 3)
    rows = [l.split() for l in open(os.path.join(GOLDEN, "loss_scale_transitions.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) >= 8
    for s, gd, ov, s2, gd2 in rows:
        got = opt.loss_scale_next(float(s), int(gd), bool(int(ov)), 2.0, 0.5, 3)
        assert (float(got[0]), got[1]) == (float(s2), int(gd2)), (s, gd, ov)


def test_loss_scale_sequence():
    # 1024, interval 2: clean, clean -> 2048; overflow -> 1024; clean, overflow -> 512 (count restarted)
    s, gd = F(1024.0), 0
    seen = []
    for ov in (0, 0, 1, 0, 1, 0, 0):
        s, gd = opt.loss_scale_next(s, gd, bool(ov), 2.0, 0.5, 2)
        seen.append((float(s), gd))
    assert seen == [(1024.0, 1), (2048.0, 0), (1024.0, 0), (1024.0, 1), (512.0, 0), (512.0, 1), (1024.0, 0)]


def test_dynamic_unscale_matches_the_static_one_for_powers_of_two():
    import oracle
    rng = np.random.default_rng(5)
    g = rng.standard_normal(1000).astype(F) * F(1000.0)
    g[17] = np.inf
    out_dyn, flag_dyn = opt.unscale_check_dynamic(g, 1024.0)
    out_st, flag_st = oracle.unscale_check(g, 1.0 / 1024.0)
    assert flag_dyn == flag_st == 1
    assert np.array_equal(bits32(out_dyn), bits32(out_st))


def test_dynamic_unscale_reciprocal_is_rounded_once():
    # scale 3: 1/3 in binary32 is 0x3EAAAAAB; g = 3 gives 3 * fl(1/3) = 1.0000000298 -> rounds to 1
    out, flag = opt.unscale_check_dynamic(np.array([3.0, 1.0], dtype=F), 3.0)
    assert flag == 0
    assert bits32(out)[1] == 0x3EAAAAAB and out[0] == F(1.0)
