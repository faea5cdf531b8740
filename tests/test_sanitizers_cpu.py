"""Host sanitizer legs (no GPU): the CPU oracle and the argument-validation layer of the C ABI,
each compiled with -fsanitize=address,undefined and driven through their edge cases by a small C
program.  A sanitizer report aborts the program, which fails the test; the oracle's results from
the sanitized build must also equal those of the ordinary build bit for bit."""
import ctypes
import os
import shutil
import subprocess

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
SAN_ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def _lcg_stream(seed):
    state = seed
    while True:
        state = (state * 6364136223846793005 + 1442695040888963407) & 0xFFFFFFFFFFFFFFFF
        yield state


def _inputs(case_index, nx, nw, ny):
    """The driver's inputs: per tensor element one draw for the binary16 and one for the binary32 value."""
    it = _lcg_stream(1000 + case_index)

    def tensor(n):
        h = np.empty(n, np.uint16)
        f = np.empty(n, np.float32)
        for i in range(n):
            b = (next(it) >> 40) & 0xFFFF
            if (b & 0x7C00) == 0x7C00:
                b ^= 0x4000
            h[i] = b
            f[i] = (((next(it) >> 40) & 1023) - 512) / 8.0
        return h.view(np.float16), f

    return tensor(nx), tensor(nw), tensor(ny)


CASES = [
    (1, 5, 6, 3, 4, 3, 3, (1, 1), (1, 1), (1, 1)),
    (2, 7, 5, 4, 2, 3, 2, (2, 2), (1, 0), (1, 1)),
    (1, 6, 6, 2, 3, 1, 1, (3, 3), (0, 0), (1, 1)),
    (1, 9, 8, 2, 2, 3, 3, (1, 2), (2, 2), (2, 2)),
    (2, 4, 4, 5, 1, 2, 2, (1, 1), (0, 1), (1, 1)),
    (1, 1, 1, 1, 1, 1, 1, (1, 1), (0, 0), (1, 1)),
]


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no gcc")
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe, res = str(tmp_path / "oracle_driver"), str(tmp_path / "results.bin")
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-o", exe,
                    os.path.join(HERE, "oracle_driver.c"), os.path.join(ROOT, "oracle", "oracle_conv.c"), "-lm"],
                   check=True)
    p = subprocess.run([exe, res], env=SAN_ENV, capture_output=True, text=True, timeout=300)
    assert p.returncode == 0, p.stdout + p.stderr
    assert "oracle_driver status 0" in p.stdout
    got = np.fromfile(res, dtype=np.float64)
    want = []
    for ci, (N, H, W, C, K, R, S, st, pd, dl) in enumerate(CASES):
        d = oracle.make_desc(N, H, W, C, K, R, S, st, pd, dl)
        ho, wo = oracle.out_shape(d)
        nx, nw, ny = N * H * W * C, K * R * S * C, N * ho * wo * K
        (x, xf), (w, wf), (g, gf) = _inputs(ci, nx, nw, ny)
        x, xf = x.reshape(N, H, W, C), xf.reshape(N, H, W, C)
        w, wf = w.reshape(K, R, S, C), wf.reshape(K, R, S, C)
        g, gf = g.reshape(N, ho, wo, K), gf.reshape(N, ho, wo, K)
        want += [oracle.conv2d_fwd(d, x, w).ravel(), oracle.conv2d_dgrad(d, g, w).ravel(),
                 oracle.conv2d_wgrad(d, x, g).ravel(), oracle.conv2d_fwd_f32(d, xf, wf).ravel(),
                 oracle.conv2d_dgrad_f32(d, gf, wf).ravel(), oracle.conv2d_wgrad_f32(d, xf, gf).ravel(),
                 oracle.conv2d_fwd(d, x, w, idx=np.array([ny - 1, 0, ny // 2])),
                 oracle.conv2d_dgrad(d, g, w, idx=np.array([nx - 1, 0, nx // 2])),
                 oracle.conv2d_wgrad(d, x, g, idx=np.array([nw - 1, 0, nw // 2]))]
    want = np.concatenate(want)
    assert got.shape == want.shape
    assert np.array_equal(got.view(np.uint64), want.view(np.uint64))


HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = "/opt/rocm/llvm/bin/clang"


@pytest.mark.skipif(not (os.path.exists(HIPCC) and os.path.exists(CLANG)), reason="no ROCm toolchain")
def test_abi_validation_layer_under_host_sanitizers(tmp_path):
    """api.hip, dispatch.hip and static_scratch.hip rebuilt with the host side under ASan + UBSan
    and linked with the kernels' objects of the ordinary build; the driver sweeps descriptors and
    bad arguments through every entry point (nothing it does reaches a GPU)."""
    from paper_1903_05831_amd import build as hip_build
    bdir = os.path.join(os.path.dirname(hip_build.LIB), "_build")
    if hip_build.stale() or not os.path.isdir(bdir):
        hip_build.build(force=True)
    host = ("api", "dispatch", "static_scratch")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    objs = []
    for name in host:
        obj = str(tmp_path / f"{name}.o")
        subprocess.run([HIPCC] + [f for f in hip_build.FLAGS if f not in ("-shared", "-O3")] + ["-O1", "-g"] + san +
                       ["-c", os.path.join(hip_build.CSRC, name + ".hip"), "-o", obj], check=True,
                       stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        objs.append(obj)
    others = [os.path.join(bdir, os.path.basename(s) + ".o") for s in hip_build.sources()
              if os.path.basename(s)[:-4] not in host]
    lib = str(tmp_path / "libsdconv_san.so")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Xarch_host", "-fsanitize=address",
                    "-Xarch_host", "-fsanitize=undefined", "-o", lib] + objs + others, check=True)
    exe = str(tmp_path / "abi_driver")
    subprocess.run([CLANG, "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-I", os.path.join(ROOT, "include"), os.path.join(HERE, "abi_driver.c"), "-o", exe,
                    "-L", str(tmp_path), "-lsdconv_san", f"-Wl,-rpath,{tmp_path}", "-lm"], check=True)
    env = dict(SAN_ENV, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=0")
    p = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=600)
    assert p.returncode == 0, p.stdout[-3000:] + p.stderr[-3000:]
    assert "0 failures" in p.stdout
