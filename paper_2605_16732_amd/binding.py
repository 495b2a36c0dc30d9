"""ctypes binding of libdirotq.so: argument marshalling only.

Every function mirrors the C entry point of the same name in include/dirotq.h and
takes torch tensors that already live on the GPU (PyTorch only supplies device memory
and the stream).  Nothing here computes; if the library is missing the import of the
entry points fails loudly -- there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdirotq.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_HIP = -1, -2, -3, -4, -5, -6
ERR_STATIC_LIMIT = -7
STATIC_SCRATCH_BYTES = 64 << 20

_c_int, _c_size_t, _c_void_p = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p
_size_p = ctypes.POINTER(ctypes.c_size_t)

# name -> (restype, argtypes); one entry per declaration in include/dirotq.h
SIGNATURES = {
    "dirotq_strerror": (ctypes.c_char_p, [_c_int]),
    "dirotq_last_hip_error": (_c_int, []),
    "dirotq_weights_bytes": (_c_int, [_c_int] * 4 + [_size_p]),
    "dirotq_prepare_scratch_bytes": (_c_int, [_c_int] * 2 + [_size_p]),
    "dirotq_workspace_bytes": (_c_int, [_c_int] * 4 + [_size_p]),
    "dirotq_prepare_rotation": (_c_int, [_c_void_p, _c_int, _c_void_p, _c_void_p]),
    "dirotq_prepare_weights": (_c_int, [_c_void_p, _c_void_p] + [_c_int] * 4 + [_c_void_p, _c_void_p, _c_size_t, _c_void_p]),
    "dirotq_import_weights": (_c_int, [_c_void_p] * 3 + [_c_int] * 4 + [_c_void_p, _c_void_p]),
    "dirotq_export_weights": (_c_int, [_c_void_p] + [_c_int] * 4 + [_c_void_p] * 4),
    "dirotq_rotate_quantize": (_c_int, [_c_void_p, _c_void_p] + [_c_int] * 4 + [_c_void_p] * 4),
    "dirotq_w4a4_gemm": (_c_int, [_c_void_p] * 5 + [_c_int] * 5 + [_c_void_p, _c_int, _c_void_p]),
    "dirotq_linear": (_c_int, [_c_void_p] * 4 + [_c_int] * 5 + [_c_void_p, _c_void_p, _c_size_t, _c_void_p]),
    "dirotq_linear_static": (_c_int, [_c_void_p] * 4 + [_c_int] * 5 + [_c_void_p, _c_void_p]),
    "dirotq_linear_shared": (_c_int, [_c_void_p, _c_void_p, _c_int] + [_c_void_p] * 4 + [_c_int] * 4 + [_c_void_p, _c_size_t, _c_void_p]),
    "dirotq_rotate_quantize_asym": (_c_int, [_c_void_p, _c_void_p] + [_c_int] * 4 + [_c_void_p] * 5),
    "dirotq_w4a4_gemm_asym": (_c_int, [_c_void_p] * 6 + [_c_int] * 5 + [_c_void_p, _c_int, _c_void_p]),
    "dirotq_linear_asym": (_c_int, [_c_void_p] * 4 + [_c_int] * 5 + [_c_void_p, _c_void_p, _c_size_t, _c_void_p]),
    "dirotq_a8_scratch_bytes": (_c_int, [_c_int] * 3 + [_size_p]),
    "dirotq_a8_workspace_bytes": (_c_int, [_c_int] * 3 + [_size_p]),
    "dirotq_rotate_quantize_a8": (_c_int, [_c_void_p, _c_void_p] + [_c_int] * 3 + [_c_void_p] * 4 + [_c_size_t, _c_void_p]),
    "dirotq_w4a8_gemm": (_c_int, [_c_void_p] * 5 + [_c_int] * 5 + [_c_void_p, _c_int, _c_void_p]),
    "dirotq_linear_a8": (_c_int, [_c_void_p] * 4 + [_c_int] * 5 + [_c_void_p, _c_void_p, _c_size_t, _c_void_p]),
    "dirotq_w4a16_gemm": (_c_int, [_c_void_p] * 3 + [_c_int] * 4 + [_c_void_p, _c_int, _c_void_p]),
}


class DirotqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().dirotq_strerror(status).decode()
        if status == ERR_HIP:
            msg += f" [hipError {lib().dirotq_last_hip_error()}]"
        super().__init__(f"{where}: {msg} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2605_16732_amd.build` "
                               "(there is no fallback implementation)")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != OK:
        raise DirotqError(status, where)


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "tensors must be contiguous GPU tensors"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _size(fn_name: str, *ints) -> int:
    out = ctypes.c_size_t(0)
    _check(getattr(lib(), fn_name)(*ints, ctypes.byref(out)), fn_name)
    return out.value


def weights_bytes(N, K, r, g) -> int:
    return _size("dirotq_weights_bytes", N, K, r, g)


def prepare_scratch_bytes(N, K) -> int:
    return _size("dirotq_prepare_scratch_bytes", N, K)


def workspace_bytes(M, K, r, g) -> int:
    return _size("dirotq_workspace_bytes", M, K, r, g)


def a8_scratch_bytes(M, K, r) -> int:
    return _size("dirotq_a8_scratch_bytes", M, K, r)


def a8_workspace_bytes(M, K, r) -> int:
    return _size("dirotq_a8_workspace_bytes", M, K, r)


def _new(shape, dtype, like):
    return torch.empty(shape, dtype=dtype, device=like.device)


def prepare_rotation(Q32: torch.Tensor) -> torch.Tensor:
    """fp32 [K,K] basis (column = direction) -> bf16 [K,K] operand, one direction per row."""
    K = Q32.shape[0]
    Qt = _new((K, K), torch.bfloat16, Q32)
    _check(lib().dirotq_prepare_rotation(_ptr(Q32), K, _ptr(Qt), _stream()), "dirotq_prepare_rotation")
    return Qt


def prepare_weights(W: torch.Tensor, Q32: torch.Tensor, r: int, g: int) -> torch.Tensor:
    N, K = W.shape
    blob = _new((weights_bytes(N, K, r, g),), torch.uint8, W)
    nscr = prepare_scratch_bytes(N, K)
    scratch = _new((nscr,), torch.uint8, W)
    _check(lib().dirotq_prepare_weights(_ptr(W), _ptr(Q32), N, K, r, g, _ptr(blob), _ptr(scratch), nscr,
                                        _stream()), "dirotq_prepare_weights")
    return blob


def import_weights(Wh, codes, sw, N, K, r, g, device="cuda") -> torch.Tensor:
    blob = torch.zeros((weights_bytes(N, K, r, g),), dtype=torch.uint8, device=device)
    _check(lib().dirotq_import_weights(_ptr(Wh), _ptr(codes), _ptr(sw), N, K, r, g, _ptr(blob), _stream()),
           "dirotq_import_weights")
    return blob


def export_weights(blob, N, K, r, g):
    G = (K - r) // g
    Wh = _new((N, r), torch.bfloat16, blob)
    codes = _new((N, K - r), torch.int8, blob)
    sw = _new((N, G), torch.float16, blob)
    _check(lib().dirotq_export_weights(_ptr(blob), N, K, r, g, _ptr(Wh) if r else None,
                                       _ptr(codes) if r < K else None, _ptr(sw) if r < K else None,
                                       _stream()), "dirotq_export_weights")
    return Wh, codes, sw


def rotate_quantize(x, Qt, r, g, out=None):
    """x bf16 [M,K], Qt bf16 [K,K] -> (xh bf16 [M,r], xl uint8 [M,(K-r)/2], sx fp16 [G,M])."""
    M, K = x.shape
    G = (K - r) // g
    if out is None:
        out = (_new((M, r), torch.bfloat16, x), _new((M, (K - r) // 2), torch.uint8, x),
               _new((G, M), torch.float16, x))
    xh, xl, sx = out
    _check(lib().dirotq_rotate_quantize(_ptr(x), _ptr(Qt), M, K, r, g, _ptr(xh) if r else None,
                                        _ptr(xl) if r < K else None, _ptr(sx) if r < K else None,
                                        _stream()), "dirotq_rotate_quantize")
    return xh, xl, sx


def w4a4_gemm(xh, xl, sx, blob, M, N, K, r, g, bias=None, out_dtype=torch.bfloat16, out=None):
    y = out if out is not None else torch.empty((M, N), dtype=out_dtype, device=blob.device)
    code = {torch.bfloat16: 0, torch.float32: 1}[y.dtype]
    _check(lib().dirotq_w4a4_gemm(_ptr(xh) if r else None, _ptr(xl) if r < K else None,
                                  _ptr(sx) if r < K else None, _ptr(blob), _ptr(bias), M, N, K, r, g,
                                  _ptr(y), code, _stream()), "dirotq_w4a4_gemm")
    return y


def linear(x, Qt, blob, N, r, g, bias=None, workspace=None, out=None):
    M, K = x.shape
    nws = workspace_bytes(M, K, r, g)
    if workspace is None:
        workspace = _new((nws,), torch.uint8, x)
    y = out if out is not None else _new((M, N), torch.bfloat16, x)
    _check(lib().dirotq_linear(_ptr(x), _ptr(Qt), _ptr(blob), _ptr(bias), M, N, K, r, g, _ptr(y),
                               _ptr(workspace), workspace.numel(), _stream()), "dirotq_linear")
    return y


def linear_static(x, Qt, blob, N, r, g, out, bias=None):
    """dirotq_linear_static: intermediates live in the library's fixed device array; `out` is
    required so that this wrapper allocates nothing either."""
    M, K = x.shape
    _check(lib().dirotq_linear_static(_ptr(x), _ptr(Qt), _ptr(blob), _ptr(bias), M, N, K, r, g, _ptr(out),
                                      _stream()), "dirotq_linear_static")
    return out


def rotate_quantize_asym(x, Qt, r, g, out=None):
    """x bf16 [M,K], Qt bf16 [K,K] -> (xh bf16 [M,r], xl uint8 [M,(K-r)/2] unsigned nibbles,
    sx fp16 [G,M], zx fp16 [G,M])."""
    M, K = x.shape
    G = (K - r) // g
    if out is None:
        out = (_new((M, r), torch.bfloat16, x), _new((M, (K - r) // 2), torch.uint8, x),
               _new((G, M), torch.float16, x), _new((G, M), torch.float16, x))
    xh, xl, sx, zx = out
    low = r < K
    _check(lib().dirotq_rotate_quantize_asym(_ptr(x), _ptr(Qt), M, K, r, g, _ptr(xh) if r else None,
                                             _ptr(xl) if low else None, _ptr(sx) if low else None,
                                             _ptr(zx) if low else None, _stream()), "dirotq_rotate_quantize_asym")
    return xh, xl, sx, zx


def w4a4_gemm_asym(xh, xl, sx, zx, blob, M, N, K, r, g, bias=None, out_dtype=torch.bfloat16, out=None):
    y = out if out is not None else torch.empty((M, N), dtype=out_dtype, device=blob.device)
    code = {torch.bfloat16: 0, torch.float32: 1}[y.dtype]
    low = r < K
    _check(lib().dirotq_w4a4_gemm_asym(_ptr(xh) if r else None, _ptr(xl) if low else None,
                                       _ptr(sx) if low else None, _ptr(zx) if low else None, _ptr(blob),
                                       _ptr(bias), M, N, K, r, g, _ptr(y), code, _stream()),
           "dirotq_w4a4_gemm_asym")
    return y


def linear_asym(x, Qt, blob, N, r, g, bias=None, workspace=None, out=None):
    M, K = x.shape
    nws = workspace_bytes(M, K, r, g)
    if workspace is None:
        workspace = _new((nws,), torch.uint8, x)
    y = out if out is not None else _new((M, N), torch.bfloat16, x)
    _check(lib().dirotq_linear_asym(_ptr(x), _ptr(Qt), _ptr(blob), _ptr(bias), M, N, K, r, g, _ptr(y),
                                    _ptr(workspace), workspace.numel(), _stream()), "dirotq_linear_asym")
    return y


def linear_shared(x, Qt, blobs, Ns, r, g, biases=None, workspace=None, outs=None):
    """One rotation + quantization of x, then one GEMM per (blob, N).  Returns the list of outputs."""
    M, K = x.shape
    n = len(blobs)
    if workspace is None:
        workspace = _new((workspace_bytes(M, K, r, g),), torch.uint8, x)
    if outs is None:
        outs = [_new((M, N), torch.bfloat16, x) for N in Ns]
    vp = ctypes.c_void_p * n
    c_blobs = vp(*[_ptr(b) for b in blobs])
    c_bias = vp(*[_ptr(b) for b in biases]) if biases is not None else None
    c_ys = vp(*[_ptr(y) for y in outs])
    c_Ns = (ctypes.c_int * n)(*Ns)
    _check(lib().dirotq_linear_shared(_ptr(x), _ptr(Qt), n, c_blobs, c_bias, c_Ns, c_ys, M, K, r, g, _ptr(workspace),
                                      workspace.numel(), _stream()), "dirotq_linear_shared")
    return outs


def rotate_quantize_a8(x, Qt, r, out=None, scratch=None):
    """x bf16 [M,K], Qt bf16 [K,K] -> (xh bf16 [M,r], x8 uint8 [M,K-r] sign-magnitude bytes in the
    even|odd order of each 32-channel block, sx fp16 [M])."""
    M, K = x.shape
    if out is None:
        out = (_new((M, r), torch.bfloat16, x), _new((M, K - r), torch.uint8, x), _new((M,), torch.float16, x))
    xh, x8, sx = out
    if scratch is None:
        scratch = _new((a8_scratch_bytes(M, K, r),), torch.uint8, x)
    low = r < K
    _check(lib().dirotq_rotate_quantize_a8(_ptr(x), _ptr(Qt), M, K, r, _ptr(xh) if r else None,
                                           _ptr(x8) if low else None, _ptr(sx) if low else None,
                                           _ptr(scratch) if low else None, scratch.numel(), _stream()),
           "dirotq_rotate_quantize_a8")
    return xh, x8, sx


def w4a8_gemm(xh, x8, sx, blob, M, N, K, r, g, bias=None, out_dtype=torch.bfloat16, out=None):
    y = out if out is not None else torch.empty((M, N), dtype=out_dtype, device=blob.device)
    code = {torch.bfloat16: 0, torch.float32: 1}[y.dtype]
    low = r < K
    _check(lib().dirotq_w4a8_gemm(_ptr(xh) if r else None, _ptr(x8) if low else None, _ptr(sx) if low else None,
                                  _ptr(blob), _ptr(bias), M, N, K, r, g, _ptr(y), code, _stream()),
           "dirotq_w4a8_gemm")
    return y


def linear_a8(x, Qt, blob, N, r, g, bias=None, workspace=None, out=None):
    M, K = x.shape
    if workspace is None:
        workspace = _new((a8_workspace_bytes(M, K, r),), torch.uint8, x)
    y = out if out is not None else _new((M, N), torch.bfloat16, x)
    _check(lib().dirotq_linear_a8(_ptr(x), _ptr(Qt), _ptr(blob), _ptr(bias), M, N, K, r, g, _ptr(y),
                                  _ptr(workspace), workspace.numel(), _stream()), "dirotq_linear_a8")
    return y


def w4a16_gemm(x, blob, N, g, bias=None, out_dtype=torch.bfloat16, out=None):
    """x bf16 [M,K] against a prepared r = 0 blob -> y [M,N]."""
    M, K = x.shape
    y = out if out is not None else torch.empty((M, N), dtype=out_dtype, device=x.device)
    code = {torch.bfloat16: 0, torch.float32: 1}[y.dtype]
    _check(lib().dirotq_w4a16_gemm(_ptr(x), _ptr(blob), _ptr(bias), M, N, K, g, _ptr(y), code, _stream()),
           "dirotq_w4a16_gemm")
    return y
