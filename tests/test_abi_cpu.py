"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_2605_16732_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "dirotq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dirotq_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    names = _declared()
    assert len(names) >= 12
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
        assert n in B.SIGNATURES, n
    assert sorted(B.SIGNATURES) == names


def test_strerror():
    L = B.lib()
    assert L.dirotq_strerror(0) == b"ok"
    seen = {L.dirotq_strerror(s) for s in range(-7, 1)}
    assert len(seen) == 8
    assert L.dirotq_last_hip_error() == 0


def test_size_queries():
    # blob: Wh bf16 [N,r] | packed codes [N,(K-r)/2] | fp16 scales [G,N] | i16 code sums [G,N];
    # workspace: xh | xl | sx | zx; each section padded to 256 B
    N, K, r, g = 1152, 1152, 64, 64
    G = (K - r) // g
    pad = lambda v: (v + 255) // 256 * 256
    assert B.weights_bytes(N, K, r, g) == pad(N * r * 2) + pad(N * (K - r) // 2) + 2 * pad(G * N * 2)
    assert B.workspace_bytes(256, K, r, g) == pad(256 * r * 2) + pad(256 * (K - r) // 2) + 2 * pad(G * 256 * 2)
    assert B.prepare_scratch_bytes(N, K) == N * K * 4
    assert B.workspace_bytes(0, K, r, g) >= 0
    # 8-bit activations: xh | x8 u8 [M,K-r] | sx fp16 [M] | scratch = fp32 [M,K-r] | fp32 [ceil((K-r)/128),M]
    M, KL = 256, K - r
    scratch = pad(M * KL * 4) + pad((KL + 127) // 128 * M * 4)
    assert B.a8_scratch_bytes(M, K, r) == scratch
    assert B.a8_workspace_bytes(M, K, r) == pad(M * r * 2) + pad(M * KL) + pad(M * 2) + scratch


@pytest.mark.parametrize("N,K,r,g", [
    (0, 64, 0, 32),      # N < 1
    (8, 48, 0, 32),      # K % 32
    (8, 64, -32, 32),    # r < 0
    (8, 64, 96, 32),     # r > K
    (8, 64, 16, 32),     # r % 32
    (8, 128, 0, 48),     # g not in {32,64,128}
    (8, 128, 32, 64),    # (K - r) % g
    (8, 0, 0, 32),       # K < 32
    ((1 << 24) + 1, 64, 0, 32),   # N beyond the limit
    (8, (1 << 20) + 32, 0, 32),   # K beyond the limit
])
def test_bad_shapes_are_rejected(N, K, r, g):
    out = ctypes.c_size_t(7)
    assert B.lib().dirotq_weights_bytes(N, K, r, g, ctypes.byref(out)) == B.ERR_SHAPE
    assert out.value == 7          # nothing written on error


def test_argument_errors_before_any_launch():
    L = B.lib()
    a = 0x1000                      # fake, aligned, never dereferenced: validation fails first
    assert L.dirotq_weights_bytes(8, 64, 0, 32, None) == B.ERR_NULL
    assert L.dirotq_rotate_quantize(None, a, 4, 64, 0, 32, None, a, a, None) == B.ERR_NULL
    assert L.dirotq_rotate_quantize(a, a, 4, 64, 32, 32, None, a, a, None) == B.ERR_NULL     # xh needed
    assert L.dirotq_rotate_quantize(a, a, 4, 64, 0, 32, None, None, a, None) == B.ERR_NULL   # xl needed
    assert L.dirotq_rotate_quantize(a, a, -1, 64, 0, 32, None, a, a, None) == B.ERR_SHAPE
    assert L.dirotq_rotate_quantize(a + 2, a, 4, 64, 0, 32, None, a, a, None) == B.ERR_ALIGN
    assert L.dirotq_w4a4_gemm(None, a, a, None, None, 4, 8, 64, 0, 32, a, 0, None) == B.ERR_NULL
    assert L.dirotq_w4a4_gemm(None, a, a, a, None, 4, 8, 64, 0, 32, a, 2, None) == B.ERR_UNSUPPORTED
    assert L.dirotq_w4a4_gemm(None, a, a, a, None, 4, 8, 64, 0, 48, a, 0, None) == B.ERR_SHAPE
    assert L.dirotq_linear(a, a, a, None, 4, 8, 64, 0, 32, a, a, 16, None) == B.ERR_WORKSPACE
    assert L.dirotq_linear(a, a, a, None, 4, 8, 64, 0, 32, a, a + 16, 1 << 20, None) == B.ERR_ALIGN
    assert L.dirotq_prepare_weights(a, a, 8, 64, 0, 32, a, a, 8, None) == B.ERR_WORKSPACE
    assert L.dirotq_prepare_rotation(a, 48, a, None) == B.ERR_SHAPE
    assert L.dirotq_import_weights(None, None, None, 8, 64, 0, 32, a, None) == B.ERR_NULL
    assert L.dirotq_export_weights(None, 8, 64, 0, 32, a, a, a, None) == B.ERR_NULL
    # asymmetric-activation entry points: same rules, plus the zero-point array
    assert L.dirotq_rotate_quantize_asym(a, a, 4, 64, 0, 32, None, a, a, None, None) == B.ERR_NULL       # zx needed
    assert L.dirotq_rotate_quantize_asym(a, a, 4, 64, 0, 32, None, a, a, a + 2, None) == B.ERR_ALIGN
    assert L.dirotq_rotate_quantize_asym(a, a, 4, 64, 0, 96, None, a, a, a, None) == B.ERR_SHAPE
    assert L.dirotq_w4a4_gemm_asym(None, a, a, None, a, None, 4, 8, 64, 0, 32, a, 0, None) == B.ERR_NULL   # zx needed
    assert L.dirotq_w4a4_gemm_asym(None, a, a, a, a, None, 4, 8, 64, 0, 32, a, 3, None) == B.ERR_UNSUPPORTED
    assert L.dirotq_linear_asym(a, a, a, None, 4, 8, 64, 0, 32, a, a, 16, None) == B.ERR_WORKSPACE
    assert L.dirotq_rotate_quantize_asym(a, a, 0, 64, 0, 32, None, a, a, a, None) == B.OK
    assert L.dirotq_w4a4_gemm_asym(None, a, a, a, a, None, 0, 8, 64, 0, 32, a, 0, None) == B.OK
    assert L.dirotq_linear_asym(a, a, a, None, 0, 8, 64, 0, 32, a, a, 0, None) == B.OK
    # entry point that keeps its intermediates in the library's fixed device array
    assert L.dirotq_linear_static(a, a, a, None, 4, 8, 48, 0, 32, a, None) == B.ERR_SHAPE
    assert L.dirotq_linear_static(a, a, None, None, 4, 8, 64, 0, 32, a, None) == B.ERR_NULL
    assert L.dirotq_linear_static(a, a + 8, a, None, 4, 8, 64, 0, 32, a, None) == B.ERR_ALIGN
    assert L.dirotq_linear_static(a, a, a, None, 0, 8, 64, 0, 32, a, None) == B.OK
    # beyond the fixed size: refused before any device is touched
    assert B.workspace_bytes(16384, 12288, 128, 64) > B.STATIC_SCRATCH_BYTES
    assert L.dirotq_linear_static(a, a, a, None, 16384, 8, 12288, 128, 64, a, None) == B.ERR_STATIC_LIMIT
    assert b"64 MiB" in L.dirotq_strerror(B.ERR_STATIC_LIMIT)
    # shared-input entry point: host arrays of device pointers
    vp2 = (ctypes.c_void_p * 2)(a, a)
    ns2 = (ctypes.c_int * 2)(8, 16)
    assert L.dirotq_linear_shared(a, a, 0, vp2, None, ns2, vp2, 4, 64, 0, 32, a, 1 << 20, None) == B.ERR_SHAPE   # n_out < 1
    assert L.dirotq_linear_shared(a, a, 17, vp2, None, ns2, vp2, 4, 64, 0, 32, a, 1 << 20, None) == B.ERR_SHAPE
    assert L.dirotq_linear_shared(a, a, 2, None, None, ns2, vp2, 4, 64, 0, 32, a, 1 << 20, None) == B.ERR_NULL
    assert L.dirotq_linear_shared(a, a, 2, vp2, None, (ctypes.c_int * 2)(8, 0), vp2, 4, 64, 0, 32, a, 1 << 20, None) == B.ERR_SHAPE
    assert L.dirotq_linear_shared(a, a, 2, (ctypes.c_void_p * 2)(a, None), None, ns2, vp2, 4, 64, 0, 32, a, 1 << 20, None) == B.ERR_NULL
    assert L.dirotq_linear_shared(a, a, 2, vp2, None, ns2, vp2, 4, 64, 0, 32, a, 16, None) == B.ERR_WORKSPACE
    assert L.dirotq_linear_shared(a, a, 2, vp2, None, ns2, vp2, 0, 64, 0, 32, a, 0, None) == B.OK
    # 8-bit-activation entry points
    assert L.dirotq_a8_scratch_bytes(4, 64, 0, None) == B.ERR_NULL
    assert L.dirotq_a8_workspace_bytes(4, 48, 0, ctypes.byref(ctypes.c_size_t())) == B.ERR_SHAPE
    A = 0x1000                      # 256-byte aligned
    assert L.dirotq_rotate_quantize_a8(a, a, 4, 64, 0, None, None, a, A, 1 << 20, None) == B.ERR_NULL     # x8 needed
    assert L.dirotq_rotate_quantize_a8(a, a, 4, 64, 0, None, a, a, None, 1 << 20, None) == B.ERR_NULL     # scratch needed
    assert L.dirotq_rotate_quantize_a8(a, a, 4, 64, 0, None, a, a, A + 16, 1 << 20, None) == B.ERR_ALIGN
    assert L.dirotq_rotate_quantize_a8(a, a, 4, 64, 0, None, a, a, A, 16, None) == B.ERR_WORKSPACE
    assert L.dirotq_rotate_quantize_a8(a, a, 4, 64, 16, a, a, a, A, 1 << 20, None) == B.ERR_SHAPE
    assert L.dirotq_rotate_quantize_a8(a, a, 0, 64, 0, None, a, a, A, 0, None) == B.OK
    assert L.dirotq_w4a8_gemm(None, a, None, a, None, 4, 8, 64, 0, 32, a, 0, None) == B.ERR_NULL           # sx needed
    assert L.dirotq_w4a8_gemm(None, a, a, a, None, 4, 8, 64, 0, 32, a, 2, None) == B.ERR_UNSUPPORTED
    assert L.dirotq_w4a8_gemm(None, a, a, a, None, 4, 8, 64, 0, 48, a, 0, None) == B.ERR_SHAPE
    assert L.dirotq_w4a8_gemm(None, a, a, a, None, 0, 8, 64, 0, 32, a, 0, None) == B.OK
    assert L.dirotq_linear_a8(a, a, a, None, 4, 8, 64, 0, 32, a, A, 16, None) == B.ERR_WORKSPACE
    assert L.dirotq_linear_a8(a, a, a, None, 4, 8, 64, 0, 32, a, None, 1 << 20, None) == B.ERR_NULL
    assert L.dirotq_linear_a8(a, a, a, None, 0, 8, 64, 0, 32, a, A, 0, None) == B.OK
    # W4A16
    assert L.dirotq_w4a16_gemm(None, a, None, 4, 8, 64, 32, a, 0, None) == B.ERR_NULL
    assert L.dirotq_w4a16_gemm(a, a, None, 4, 8, 64, 32, a, 5, None) == B.ERR_UNSUPPORTED
    assert L.dirotq_w4a16_gemm(a, a, None, 4, 8, 96, 64, a, 0, None) == B.ERR_SHAPE
    assert L.dirotq_w4a16_gemm(a + 4, a, None, 4, 8, 64, 32, a, 0, None) == B.ERR_ALIGN
    assert L.dirotq_w4a16_gemm(a, a, None, 0, 8, 64, 32, a, 0, None) == B.OK
    # M == 0 is a valid no-op and launches nothing
    assert L.dirotq_rotate_quantize(a, a, 0, 64, 0, 32, None, a, a, None) == B.OK
    assert L.dirotq_w4a4_gemm(None, a, a, a, None, 0, 8, 64, 0, 32, a, 0, None) == B.OK


def test_output_tilings_beyond_32_bit_grids_are_rejected():
    L = B.lib()
    a = 0x1000
    big = 1 << 24                  # 131072 x 131072 tiles of 128 x 128 would overflow the grid index
    assert L.dirotq_w4a4_gemm(None, a, a, a, None, big, big, 64, 0, 32, a, 0, None) == B.ERR_SHAPE
    assert L.dirotq_linear(a, a, a, None, big, big, 64, 0, 32, a, a, 1 << 62, None) == B.ERR_SHAPE
    assert L.dirotq_w4a16_gemm(a, a, None, big, big, 64, 32, a, 0, None) == B.ERR_SHAPE
    out = ctypes.c_size_t(0)
    assert L.dirotq_workspace_bytes(big, 1 << 20, 0, 32, ctypes.byref(out)) == B.OK     # sizes are 64-bit
    assert out.value > (1 << 42)


def test_error_type_carries_message():
    with pytest.raises(B.DirotqError) as e:
        B.weights_bytes(8, 48, 0, 32)
    assert e.value.status == B.ERR_SHAPE and "K%32" in str(e.value)
