"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, derives output shapes, and rejects bad arguments before
anything is launched."""
import ctypes
import os
import re

import pytest

import paper_1903_05831_amd as sd
from paper_1903_05831_amd import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("sdconv.h", "sdconv_bench.h"))
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(\w+)\s*\(", header)) - {"defined"}
    assert declared == set(sd.EXPORTS)
    L = sd.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_out_shape_matches_workload_tables_and_oracle():
    import oracle
    for cfg, layers in workloads.CONFIGS.items():
        for l in layers:
            d = sd.desc_of(l)
            assert sd.conv2d_out_shape(d) == (l.Ho, l.Wo), (cfg, l.name)
            od = oracle.make_desc(l.N, l.H, l.W, l.C, l.K, l.R, l.S, (l.stride,) * 2, (l.pad,) * 2, (l.dil,) * 2)
            assert oracle.out_shape(od) == (l.Ho, l.Wo)


def test_workload_totals():
    """53 conv layers, 1109.62 GFLOP per pass and 23 454 912 weight-gradient elements for the
    full detector workload (hand-checked sums of the layer table)."""
    l5 = workloads.CONFIGS[5]
    assert len(l5) == 53
    assert sum(l.dw_numel for l in l5) == 23454912
    assert abs(sum(l.flops for l in l5) / 1e9 - 1109.62) < 0.01
    assert [len(workloads.CONFIGS[c]) for c in (1, 2, 3, 4)] == [1, 3, 4, 19]


BAD_DESCS = [
    dict(N=0), dict(H=0), dict(W=-1), dict(C=0), dict(K=0), dict(R=0), dict(S=0),
    dict(stride_h=0), dict(stride_w=0), dict(pad_h=-1), dict(pad_w=-1), dict(dil_h=0), dict(dil_w=0),
    dict(H=2, R=3, pad_h=0),                 # empty output
    dict(N=70000, H=256, W=256, C=64),       # >= 2^31 elements
]


def _desc(**over):
    base = dict(N=1, H=8, W=8, C=8, K=8, R=3, S=3, stride_h=1, stride_w=1, pad_h=1, pad_w=1, dil_h=1, dil_w=1)
    base.update(over)
    return sd.conv2d_desc(**base)


@pytest.mark.parametrize("over", BAD_DESCS)
def test_invalid_descriptors_are_rejected(over):
    d = _desc(**over)
    ho, wo = ctypes.c_int32(), ctypes.c_int32()
    L = sd.lib()
    assert L.conv2d_out_shape(ctypes.byref(d), ctypes.byref(ho), ctypes.byref(wo)) == sd.EINVAL
    assert sd.conv2d_workspace_bytes(d, sd.FWD) == 0
    fake = 0x1000  # never dereferenced: validation fails first
    for name in ("conv2d_fwd", "conv2d_dgrad", "conv2d_wgrad"):
        assert getattr(L, name)(ctypes.byref(d), fake, fake, fake, None, 0, None) == sd.EINVAL
    assert sd.kernel_name(d, sd.FWD) == "invalid"


def test_null_and_misaligned_pointers_are_rejected():
    d = _desc()
    L = sd.lib()
    ok = 0x1000
    for name in ("conv2d_fwd", "conv2d_dgrad", "conv2d_wgrad"):
        fn = getattr(L, name)
        assert fn(None, ok, ok, ok, None, 0, None) == sd.EINVAL
        assert fn(ctypes.byref(d), None, ok, ok, None, 0, None) == sd.EINVAL
        assert fn(ctypes.byref(d), ok, None, ok, None, 0, None) == sd.EINVAL
        assert fn(ctypes.byref(d), ok, ok, None, None, 0, None) == sd.EINVAL
        assert fn(ctypes.byref(d), ok + 2, ok, ok, None, 0, None) == sd.EINVAL
    assert L.conv2d_out_shape(ctypes.byref(d), None, None) == sd.EINVAL


def test_workspace_is_checked_before_launch():
    l = workloads.CONFIGS[4][1]
    d = sd.desc_of(l)
    L = sd.lib()
    ok = 0x1000
    for pass_id, name in ((sd.DGRAD, "conv2d_dgrad"), (sd.WGRAD, "conv2d_wgrad")):
        need = sd.conv2d_workspace_bytes(d, pass_id)
        if need == 0:
            continue
        fn = getattr(L, name)
        assert fn(ctypes.byref(d), ok, ok, ok, None, 0, None) == sd.EWORKSPACE
        assert fn(ctypes.byref(d), ok, ok, ok, ok, need - 1, None) == sd.EWORKSPACE
    assert sd.conv2d_workspace_bytes(d, 7) == 0


def test_unscale_argument_checks():
    L = sd.lib()
    ok = 0x1000
    inf, nan = float("inf"), float("nan")
    assert L.grad_unscale_check(ok, 16, ctypes.c_float(1.0), None, None) == sd.EINVAL
    assert L.grad_unscale_check(None, 16, ctypes.c_float(1.0), ok, None) == sd.EINVAL
    assert L.grad_unscale_check(ok + 2, 16, ctypes.c_float(1.0), ok, None) == sd.EINVAL
    for bad in (0.0, -1.0, inf, nan):
        assert L.grad_unscale_check(ok, 16, ctypes.c_float(bad), ok, None) == sd.EINVAL


def test_optimizer_tail_argument_checks():
    """Nothing is launched for a bad argument (there is no GPU here: a launch would fail differently)."""
    L = sd.lib()
    ok = 0x1000
    f = ctypes.c_float
    inf, nan = float("inf"), float("nan")
    assert L.grad_unscale_check_dynamic(ok, 16, None, ok, None) == sd.EINVAL
    assert L.grad_unscale_check_dynamic(ok, 16, ok, None, None) == sd.EINVAL
    assert L.grad_unscale_check_dynamic(None, 16, ok, ok, None) == sd.EINVAL
    assert L.grad_unscale_check_dynamic(ok + 2, 16, ok, ok, None) == sd.EINVAL

    def upd(w=ok, m=ok, g=ok, h=ok, n=16, lr=0.1, mu=0.9, wd=0.0, flag=ok, st=ok, gr=2.0, bo=0.5, iv=2000):
        return L.sgd_momentum_update(w, m, g, h, n, f(lr), f(mu), f(wd), flag, st, f(gr), f(bo), iv, None)

    for kw in (dict(w=None), dict(m=None), dict(g=None), dict(h=None), dict(flag=None), dict(st=None),
               dict(w=ok + 4), dict(m=ok + 8), dict(g=ok + 4), dict(h=ok + 2), dict(flag=ok + 1), dict(st=ok + 2),
               dict(lr=nan), dict(mu=inf), dict(wd=nan), dict(gr=0.0), dict(gr=inf), dict(bo=-1.0), dict(bo=nan),
               dict(iv=0)):
        assert upd(**kw) == sd.EINVAL, kw


def test_status_strings():
    assert sd.status_string(sd.OK) == "ok"
    for code in (sd.EINVAL, sd.EUNSUPPORTED, sd.EWORKSPACE, sd.EHIP, 99):
        assert isinstance(sd.status_string(code), str) and sd.status_string(code)
    assert sd.last_hip_error() == 0


def test_tensors_of_2_30_elements_or_more_avoid_the_byte_offset_kernels():
    """The LDS-DMA kernels use 32-bit byte offsets whose bit 31 marks a masked load (padding tap,
    ragged row): 0x80000000 must not be the address of real data.  A binary16 tensor of 2^30
    elements or more has data at byte 2^31 and beyond (host-side arithmetic below), so such layers
    must be served by the kernels that index elements; smaller ones keep the LDS-DMA kernels."""
    big = _desc(N=1, H=724, W=725, C=2048, K=8)
    last_byte_offset = (big.N * big.H * big.W * big.C - 1) * 2
    assert last_byte_offset >= 0x80000000          # a valid pixel would look like a masked one
    for p in (sd.FWD, sd.DGRAD, sd.WGRAD):
        name = sd.kernel_name(big, p)
        assert "dma" not in name and "_ws_" not in name and "patch" not in name, name
    small = _desc(N=1, H=724, W=724, C=2048, K=8)
    assert (small.N * small.H * small.W * small.C - 1) * 2 < 0x80000000
    assert any(t in sd.kernel_name(small, sd.FWD) for t in ("dma", "_ws_", "patch"))
    # large y with a small x (many filters), and a large filter bank
    assert "dma" not in sd.kernel_name(_desc(N=1, H=2048, W=2048, C=8, K=256, R=1, S=1, pad_h=0, pad_w=0), sd.WGRAD)


def test_neighbouring_batch_sizes_take_the_tuned_entries():
    """The measured table holds the layers of the workloads at their batch sizes; the same geometry
    at half or twice the batch takes the same kernel variant, four times the batch does not."""
    import dataclasses
    hits = 0
    for l in workloads.CONFIGS[5][1:40]:
        base = [sd.kernel_name(sd.desc_of(l), p) for p in (sd.FWD, sd.DGRAD, sd.WGRAD)]
        for n in (1, 4):
            other = [sd.kernel_name(sd.desc_of(dataclasses.replace(l, N=n)), p) for p in (sd.FWD, sd.DGRAD, sd.WGRAD)]
            assert other == base, (l.name, n, base, other)
            hits += 1
    assert hits == 78
    # the pixel ranges of the weight gradient follow the batch
    l = next(l for l in workloads.CONFIGS[5] if l.name == "res4.1b")
    ws = [sd.conv2d_workspace_bytes(sd.desc_of(dataclasses.replace(l, N=n)), sd.WGRAD) for n in (1, 2, 4)]
    assert ws[0] < ws[1] < ws[2]
