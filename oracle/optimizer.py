"""CPU oracle for the optimizer tail of a mixed-precision step -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module.  It
shares nothing with the HIP library.

Section 2.2 of the paper adopts the loss scaling of its cited mixed-precision recipe: weight
gradients carry a factor S, are unscaled and checked for overflow, and the update is skipped
when the check fires.  The paper names neither the scale schedule nor the optimizer; the
readings taken here (and listed in the design notes) are

  * dynamic schedule of the cited recipe: on overflow the scale is multiplied by `backoff`
    and the count of clean steps restarts; after `interval` clean steps in a row it is
    multiplied by `growth` and the count restarts;
  * SGD with momentum and weight decay on fp32 master weights in the formulation of the
    framework the paper builds on:  mom <- mu*mom - lr*(g + wd*w);  w <- w + mom;
    followed by the fp32 -> binary16 cast (round to nearest even) of the updated weight.

Every operation below is a single IEEE binary32 operation with its own rounding, in the order
written (numpy float32 scalars and arrays do exactly that; nothing is fused).

Pins: tests/test_oracle_optimizer_pins.py (nothing here is "parity unpinned").
"""
from __future__ import annotations

import numpy as np

F = np.float32


def loss_scale_next(scale, good_steps: int, overflow: bool, growth, backoff, interval: int):
    """One transition of the loss-scale state machine -> (scale', good_steps')."""
    scale = F(scale)
    if overflow:
        return F(scale * F(backoff)), 0
    good_steps += 1
    if good_steps >= interval:
        return F(scale * F(growth)), 0
    return scale, good_steps


def unscale_check_dynamic(g: np.ndarray, scale):
    """g * (1/scale) with the reciprocal rounded once to binary32, and the overflow flag of the
    *inputs* (any +-inf or NaN) -> (out fp32, flag)."""
    g = np.asarray(g, dtype=F)
    with np.errstate(all="ignore"):
        inv = F(F(1.0) / F(scale))
        out = (g * inv).astype(F)
    return out, int(not np.isfinite(g).all())


def sgd_momentum_update(w: np.ndarray, mom: np.ndarray, g: np.ndarray, lr, mu, wd, overflow: bool):
    """-> (w', mom', w16).  With overflow the step is skipped: w and mom come back unchanged and
    w16 is the cast of the unchanged w."""
    w = np.asarray(w, dtype=F).copy()
    mom = np.asarray(mom, dtype=F).copy()
    g = np.asarray(g, dtype=F)
    lr, mu, wd = F(lr), F(mu), F(wd)
    with np.errstate(all="ignore"):
        if not overflow:
            t = (wd * w).astype(F)
            gg = (g + t).astype(F)
            a = (mu * mom).astype(F)
            b = (lr * gg).astype(F)
            mom = (a - b).astype(F)
            w = (w + mom).astype(F)
        w16 = w.astype(np.float16)
    return w, mom, w16
