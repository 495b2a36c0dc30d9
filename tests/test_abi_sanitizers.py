"""Host hardening of the C ABI (CPU only): the ABI translation unit is rebuilt with AddressSanitizer and
UndefinedBehaviorSanitizer on its host code, linked into a small driver (tests/host/abi_host_driver.cpp) that
walks every entry point's argument-error and no-op paths and sweeps the size queries; and a hypothesis test
checks the size queries and the shape validator against a Python model on random shapes."""
import ctypes
import os
import shutil
import subprocess

import pytest
from hypothesis import given, settings, strategies as st

from paper_2605_16732_amd import binding as B
from paper_2605_16732_amd import build as BLD

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_abi_host_code_under_asan_and_ubsan():
    objdir = os.path.join(BLD.HERE, "_build")
    others = [os.path.join(objdir, s.replace(".hip", ".o")) for s in BLD.SOURCES if s != "dirotq_abi.hip"]
    if not all(os.path.exists(o) for o in others):
        BLD.build(verbose=False)
    cc = BLD.hipcc()
    clangxx = os.path.join(os.path.dirname(os.path.realpath(cc)), "..", "lib", "llvm", "bin", "clang++")
    if not os.path.exists(clangxx):
        clangxx = shutil.which("clang++") or "/opt/rocm/lib/llvm/bin/clang++"
    san_obj = os.path.join(objdir, "dirotq_abi_san.o")
    drv_obj = os.path.join(objdir, "abi_host_driver.o")
    exe = os.path.join(objdir, "abi_host_driver_san")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", BLD.CSRC]
    # the sanitizers go on the host pass only (-Xarch_host); the device code of the unit is compiled as usual
    subprocess.run([cc, *BLD.HIPCC_FLAGS, "-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host",
                    "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined", *inc, "-c",
                    os.path.join(BLD.CSRC, "dirotq_abi.hip"), "-o", san_obj], check=True, capture_output=True)
    subprocess.run([clangxx, "-O1", "-g", "-std=c++17", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", *inc, "-c", os.path.join(ROOT, "tests", "host", "abi_host_driver.cpp"),
                    "-o", drv_obj], check=True, capture_output=True)
    subprocess.run([cc, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", drv_obj, san_obj,
                    *others, "-o", exe], check=True, capture_output=True)
    syms = subprocess.run(["nm", san_obj], check=True, capture_output=True, text=True).stdout
    assert "__asan" in syms and "__ubsan" in syms              # the host code really is instrumented
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "0 failure(s)" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr


def _pad(v, a=256):
    return (v + a - 1) // a * a


def _shape_ok(M, N, K, r, g):
    return (M >= 0 and N >= 1 and 32 <= K <= (1 << 20) and K % 32 == 0 and 0 <= r <= K and r % 32 == 0 and
            g in (32, 64, 128) and (K - r) % g == 0 and M <= (1 << 24) and N <= (1 << 24) and
            ((M + 127) // 128) * ((N + 127) // 128) <= (1 << 30))


dims = st.one_of(st.integers(-64, 4096), st.sampled_from([0, 1, 31, 32, 33, 1152, 3072, 12288, 1 << 20, (1 << 20) + 32,
                                                         1 << 24, (1 << 24) + 1]))


@settings(max_examples=400, deadline=None)
@given(M=dims, N=dims, K=st.one_of(dims, st.integers(1, 512).map(lambda v: 32 * v)),
       r=st.one_of(dims, st.integers(0, 64).map(lambda v: 32 * v)), g=st.sampled_from([0, 16, 32, 48, 64, 96, 128, 256]))
def test_size_queries_against_a_model(M, N, K, r, g):
    L = B.lib()
    out = ctypes.c_size_t(7)
    st_w = L.dirotq_weights_bytes(N, K, r, g, ctypes.byref(out))
    if _shape_ok(0, N, K, r, g):
        G = (K - r) // g
        assert st_w == B.OK
        assert out.value == max(_pad(N * r * 2) + _pad(N * (K - r) // 2) + 2 * _pad(G * N * 2), 256)
    else:
        assert st_w == B.ERR_SHAPE and out.value == 7
    out = ctypes.c_size_t(7)
    st_ws = L.dirotq_workspace_bytes(M, K, r, g, ctypes.byref(out))
    if _shape_ok(M, 1, K, r, g):
        G = (K - r) // g
        assert st_ws == B.OK
        assert out.value == max(_pad(M * r * 2) + _pad(M * (K - r) // 2) + 2 * _pad(G * M * 2), 256)
    else:
        assert st_ws == B.ERR_SHAPE and out.value == 7
    # the validator of an online call agrees with the model (fake aligned pointers: rejected or a no-op first)
    # (a valid shape with M > 0 is never called with these pointers: it would be launched)
    a = 0x1000
    if not _shape_ok(M, N, K, r, g):
        assert L.dirotq_w4a4_gemm(a, a, a, a, None, M, N, K, r, g, a, 0, None) == B.ERR_SHAPE
    elif M == 0:
        assert L.dirotq_w4a4_gemm(a, a, a, a, None, M, N, K, r, g, a, 0, None) == B.OK
