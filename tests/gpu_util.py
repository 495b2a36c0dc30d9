"""Helpers shared by the GPU parity tests: host<->device marshalling and the
comparison rules.  The HIP path is always reached through the C-ABI binding."""
from __future__ import annotations

import numpy as np
import torch

from oracle import dirotq_oracle as O
from paper_2605_16732_amd import binding as B
from paper_2605_16732_amd import inputs as I

DEV = "cuda"


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV).view(torch.bfloat16)


def host_bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_f16(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.float16)


def dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.float16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV).view(torch.float16)
    if a.dtype == np.uint16:
        return dev_bf16(a)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def pack_codes(q: np.ndarray) -> np.ndarray:
    """int codes in [-7, 7], shape [rows, C] -> the library's packed form [rows, C/2]: two
    sign-magnitude nibbles per byte (bit 3 = sign, bits 0-2 = |q|), even channel low."""
    q = np.asarray(q).astype(np.int16)
    assert q.min() >= -7 and q.max() <= 7 and q.shape[-1] % 2 == 0
    nib = (np.abs(q) | np.where(q < 0, 8, 0)).astype(np.uint8)
    return np.ascontiguousarray(nib[..., 0::2] | (nib[..., 1::2] << 4))


def unpack_codes(b: np.ndarray) -> np.ndarray:
    """Inverse of pack_codes -> int8 codes [rows, C]; a stored "minus zero" (0x8) is rejected."""
    b = np.asarray(b, dtype=np.uint8)
    nib = np.stack([b & 15, b >> 4], axis=-1).reshape(*b.shape[:-1], b.shape[-1] * 2)
    assert not np.any(nib == 8), "sign bit set on a zero code"
    mag = (nib & 7).astype(np.int8)
    return np.where(nib & 8, -mag, mag).astype(np.int8)


def import_blob(Wh, qw, sw, N, K, r, g):
    """Oracle-side prepared weights -> device blob through dirotq_import_weights."""
    Wh_d = dev_bf16(O.bf16_bits(Wh)) if r else None
    qw_d = dev(qw) if r < K else None
    sw_d = dev(sw) if r < K else None
    return B.import_weights(Wh_d, qw_d, sw_d, N, K, r, g)


def gpu_rotate_quantize(x_bits, Qt_dev, r, g):
    xh, xl, sx = B.rotate_quantize(dev_bf16(x_bits), Qt_dev, r, g)
    torch.cuda.synchronize()
    K = x_bits.shape[1]
    xh_h = O.from_bf16_bits(host_bf16_bits(xh)) if r else np.zeros((x_bits.shape[0], 0), np.float32)
    if r < K:
        qx = unpack_codes(xl.cpu().numpy())
        sx_h = np.ascontiguousarray(host_f16(sx).T)           # -> [M, G] like the oracle
    else:
        qx = np.zeros((x_bits.shape[0], 0), np.int8)
        sx_h = np.zeros((x_bits.shape[0], 0), np.float16)
    return (xh, xl, sx), (xh_h, qx, sx_h)


def check_codes_statistical(xhat, qx_gpu, sx_gpu, qx_ref, sx_ref, g, min_agree=0.999, band=1e-3,
                            max_scale_flip_frac=5e-3):
    """The end-to-end code contract: at least 99.9% of the INT4 codes equal the
    oracle's; a differing code is accepted only if the oracle's fp32 rotated value sits
    within `band` scale units of a rounding boundary.  A group whose stored scale
    differs (the absmax landed on the other side of an fp16 rounding midpoint) must
    differ by one fp16 ulp, and its codes are judged against the oracle's rotated values
    re-quantized with the GPU's scale.  Returns a dict of counts."""
    M, C = qx_ref.shape
    G = C // g
    sxg = sx_gpu.astype(np.float32)
    sxr = sx_ref.astype(np.float32)
    scale_diff = sx_gpu.view(np.uint16) != sx_ref.view(np.uint16)
    n_scale_flip = int(scale_diff.sum())
    if n_scale_flip:
        ulps = np.abs(sx_gpu.view(np.uint16).astype(np.int32) - sx_ref.view(np.uint16).astype(np.int32))
        assert ulps[scale_diff].max() == 1, "a scale differs by more than one fp16 ulp"
        assert n_scale_flip <= max(2, max_scale_flip_frac * M * G), f"{n_scale_flip} scale flips of {M * G}"
    # judge every code against the GPU's scale (equal to the oracle's in almost all groups)
    with np.errstate(divide="ignore"):
        inv = np.where(sxg == 0, np.float32(0), (np.float32(1.0) / sxg).astype(np.float32))
    t = (xhat.reshape(M, G, g) * inv[..., None]).astype(np.float32)
    want = np.clip(np.rint(t), -7, 7).astype(np.int8).reshape(M, C)
    diff = qx_gpu != want
    n_diff = int(diff.sum())
    if n_diff:
        tt = t.reshape(M, C)[diff].astype(np.float64)
        frac = np.abs(tt - np.floor(tt) - 0.5)          # distance to the nearest n + 1/2
        assert np.all(frac <= band), f"code flip {frac.max():.3g} scale units away from a boundary"
        assert np.all(np.abs(qx_gpu[diff].astype(np.int32) - want[diff]) == 1)
    agree = float((qx_gpu == qx_ref).mean())
    assert agree >= min_agree, f"only {agree:.5f} of the codes agree with the oracle"
    return dict(agree=agree, code_flips=n_diff, scale_flips=n_scale_flip, groups=M * G)


def check_output(y_gpu: np.ndarray, y32: np.ndarray, tol=1e-2):
    """Final output contract: per-token relative L2 error and max-abs error relative to the
    largest output are both at most `tol` against the oracle's fp32 output."""
    d = y_gpu.astype(np.float64) - y32.astype(np.float64)
    row = np.linalg.norm(d, axis=1) / np.maximum(np.linalg.norm(y32.astype(np.float64), axis=1), 1e-30)
    mx = np.abs(d).max() / np.abs(y32).max()
    assert row.max() <= tol, f"per-token relative error {row.max():.3g}"
    assert mx <= tol, f"max-abs relative error {mx:.3g}"
    return float(row.max()), float(mx)


_layer_cache: dict = {}


def layer_with_oracle(shape: I.LayerShape, M: int | None = None, rows=None, residual_rotation: bool = False):
    """Inputs of a layer plus the oracle's full result (cached per shape).  `rows`
    selects a subset of tokens for the oracle (tokens are independent)."""
    key = (shape, M, None if rows is None else tuple(rows), residual_rotation)
    if key in _layer_cache:
        return _layer_cache[key]
    L = I.make_layer(shape, M=M, residual_rotation=residual_rotation)
    x = I.bf16_bits_to_f32(L.x_bits)
    Q = I.bf16_bits_to_f32(L.Q_bits)
    Wh, qw, sw = O.prepare_weights(L.W, L.Q32, shape.r, shape.g)
    xs = x if rows is None else x[np.asarray(rows)]
    ref = O.linear(xs, Q, Wh, qw, sw, shape.r, shape.g)
    out = (L, (Wh, qw, sw), ref)
    _layer_cache.clear()             # keep at most one big layer alive
    _layer_cache[key] = out
    return out
