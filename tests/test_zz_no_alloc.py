"""conv2d_wgrad_static_scratch (the weight gradient on the library's own fixed device scratch,
for callers that cannot allocate) against conv2d_wgrad with a caller workspace: same kernels, so
the results must agree bit for bit, on two calls in a row, the second on a smaller layer that
finds the first call's partial sums in the scratch.  Runs last (file name) so that a failure
here hides no other test."""
import numpy as np
import pytest
import torch

import paper_1903_05831_amd as sd
from paper_1903_05831_amd import workloads

from gpu_harness import GuardedOut, say, to_dev, workspace_for

pytestmark = pytest.mark.gpu


def _both(cfg, li):
    l = workloads.CONFIGS[cfg][li]
    d = sd.desc_of(l)
    need = sd.conv2d_workspace_bytes(d, sd.WGRAD)
    say(f"static scratch: cfg{cfg}.{l.name} {l.x_shape} -> {l.w_shape} workspace {need} B "
        f"[{sd.kernel_name(d, sd.WGRAD)}]")
    assert 0 < need <= sd.STATIC_SCRATCH_BYTES
    x, g = to_dev(workloads.make_x(l, cfg, li)), to_dev(workloads.make_g(l, cfg, li))
    st = torch.cuda.current_stream().cuda_stream
    ref = GuardedOut(l.w_shape, torch.float32)
    sd.conv2d_wgrad(d, x, g, ref.view, workspace_for(d, sd.WGRAD), st)
    out = GuardedOut(l.w_shape, torch.float32)
    sd.conv2d_wgrad_static_scratch(d, x, g, out.view, st)
    torch.cuda.synchronize()
    out.check_guards()
    assert out.all_written()
    a, b = out.numpy().view(np.uint32), ref.numpy().view(np.uint32)
    assert np.array_equal(a, b), f"cfg{cfg}.{l.name}: {int((a != b).sum())} of {a.size} elements differ"


def test_two_calls_in_a_row_second_smaller():
    # res4 3x3 256 -> 256 (split-K partials of 589 824 weights), then res2 1x1 64 -> 256 (16 384)
    _both(4, 5)
    _both(2, 2)
    # and the RGB stem (its own partial layout) after them
    _both(5, 0)


def test_oversize_is_rejected_before_any_launch():
    d = sd.make_desc(8, 56, 56, 1024, 1024, 3, 3, (1, 1), (1, 1))
    assert sd.conv2d_workspace_bytes(d, sd.WGRAD) > sd.STATIC_SCRATCH_BYTES
    with pytest.raises(sd.SdconvError) as e:
        sd.conv2d_wgrad_static_scratch(d, 0x1000, 0x1000, 0x1000, 0)
    assert e.value.status == sd.EWORKSPACE
