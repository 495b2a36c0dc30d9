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


def accumulation_slack(x_rows: np.ndarray, Q: np.ndarray, cols: np.ndarray, K: int) -> np.ndarray:
    """How far the GPU's fp32 rotated value x_hat[m, c] = sum_k x[m,k] Q[k,c] may sit from the
    oracle's (float64 sum, rounded once): the GPU accumulates ~K rounded partial sums, each off by at
    most 2^-24 of its magnitude; modelled as a random walk over partial sums of typical size
    B2 = sqrt(sum_k (x_k Q_kc)^2), with a safety factor of 4:  4 sqrt(K) 2^-24 B2
    (observed flips sit within a fifth of that distance).
    x_rows [n, K] and cols [n] name the (token, channel) pairs; returns [n] float64."""
    xr = x_rows.astype(np.float64)
    qc = Q[:, cols].T.astype(np.float64)                  # [n, K]
    b2 = np.sqrt(np.sum((xr * qc) ** 2, axis=1))
    return 4.0 * np.sqrt(K) * 2.0 ** -24 * b2


def check_flips_near_midpoint(unrounded: np.ndarray, got16: np.ndarray, ref16: np.ndarray, slack: np.ndarray, what: str):
    """A stored fp16 value may differ from the oracle's only by one ulp and only if the oracle's unrounded
    fp32 value lies within `slack` of the rounding midpoint between the two candidates."""
    ulps = np.abs(got16.view(np.uint16).astype(np.int32) - ref16.view(np.uint16).astype(np.int32))
    assert ulps.max() == 1, f"{what}: differs by more than one fp16 ulp"
    mid = 0.5 * (got16.astype(np.float64) + ref16.astype(np.float64))
    dist = np.abs(unrounded.astype(np.float64) - mid)
    bad = dist > slack + 2.0 ** -22 * np.abs(mid)          # (+ the fp32 rounding of the division itself)
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {len(bad)} flips are not explained by fp32 accumulation noise "
                           f"(worst: {dist[bad].max():.3g} from the midpoint, allowed {slack[bad].min():.3g})")
    return float((dist / np.maximum(slack, 1e-300)).max())


def check_codes_statistical(xhat, qx_gpu, sx_gpu, qx_ref, sx_ref, g, min_agree=0.999, band=1e-3,
                            max_scale_flip_frac=5e-3, x=None, Q=None, col0=0):
    """The end-to-end code contract: at least 99.9% of the INT4 codes equal the
    oracle's; a differing code is accepted only if the oracle's fp32 rotated value sits
    within `band` scale units of a rounding boundary.  A group whose stored scale
    differs must differ by one fp16 ulp, and -- when the activations `x` [M,K] and the basis `Q`
    [K,K] are given (`col0` = first rotated channel of `xhat`) -- only because the oracle's
    unrounded amax / 7 lies next to the fp16 rounding midpoint, closer than the fp32 accumulation
    noise of the absmax channel allows (accumulation_slack / 7).  The codes of such a group are
    judged against the oracle's rotated values re-quantized with the GPU's scale.  Returns a
    dict of counts."""
    M, C = qx_ref.shape
    G = C // g
    sxg = sx_gpu.astype(np.float32)
    scale_diff = sx_gpu.view(np.uint16) != sx_ref.view(np.uint16)
    n_scale_flip = int(scale_diff.sum())
    worst = 0.0
    if n_scale_flip:
        ulps = np.abs(sx_gpu.view(np.uint16).astype(np.int32) - sx_ref.view(np.uint16).astype(np.int32))
        assert ulps[scale_diff].max() == 1, "a scale differs by more than one fp16 ulp"
        assert n_scale_flip <= max(2, max_scale_flip_frac * M * G), f"{n_scale_flip} scale flips of {M * G}"
        if x is not None:
            mi, ji = np.nonzero(scale_diff)
            grp = np.abs(xhat.reshape(M, G, g)[mi, ji])                      # [n, g]
            cpos = np.argmax(grp, axis=1)
            amax = grp[np.arange(len(mi)), cpos]
            s32 = (amax / np.float32(7.0)).astype(np.float32)
            slack = accumulation_slack(x[mi], Q, col0 + ji * g + cpos, x.shape[1]) / 7.0
            worst = check_flips_near_midpoint(s32, sx_gpu[mi, ji], sx_ref[mi, ji], slack, "activation scale")
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
    return dict(agree=agree, code_flips=n_diff, scale_flips=n_scale_flip, groups=M * G, worst_flip_slack=worst)


def check_xh(xh_gpu, xh_ref, x, K):
    """bf16 part against the oracle's.  Both sides round an fp32 rotated value to bf16; the GPU's fp32 value
    differs from the oracle's by accumulation noise (random-walk model: ~sqrt(K) 2^-24 times the size of the
    partial sums, bounded here by 1e-5 |x_m|), so an element may land on the neighbouring bf16 number when
    the value sits next to a rounding boundary: |err| <= one bf16 ulp (2^-7 relative) + that noise, and the
    share of such elements is about 2 * noise / ulp = sqrt(K) 2^-15 A with A = partial-sum size over value
    size (a few units for the high-variance channels): at most 4 sqrt(K) 2^-16 of the elements (observed:
    2e-4 to 5e-4)."""
    xn = np.linalg.norm(x.astype(np.float64), axis=1)[:, None]
    err = np.abs(xh_gpu.astype(np.float64) - xh_ref)
    assert np.all(err <= 2.0 ** -7 * np.abs(xh_ref) + 1e-5 * xn)
    frac = float((err != 0).mean())
    assert frac <= max(4.0 * np.sqrt(K) * 2.0 ** -16, 8.0 / err.size), f"{frac:.4f} of the bf16 coefficients differ"
    return frac


def check_output(y_gpu: np.ndarray, y32: np.ndarray, tol=1e-2):
    """Final output contract: per-token relative L2 error and max-abs error relative to the
    largest output are both at most `tol` against the oracle's fp32 output."""
    d = y_gpu.astype(np.float64) - y32.astype(np.float64)
    row = np.linalg.norm(d, axis=1) / np.maximum(np.linalg.norm(y32.astype(np.float64), axis=1), 1e-30)
    mx = np.abs(d).max() / np.abs(y32).max()
    assert row.max() <= tol, f"per-token relative error {row.max():.3g}"
    assert mx <= tol, f"max-abs relative error {mx:.3g}"
    return float(row.max()), float(mx)


_big: dict = {}          # one layer's draws and oracle intermediates at a time (they are large)


def _layer_key(shape: I.LayerShape, M, residual_rotation):
    return (shape.config_id, shape.layer_id, shape.K, shape.N, shape.M if M is None else M, shape.n_outliers,
            bool(residual_rotation))


def layer_inputs(shape: I.LayerShape, M: int | None = None, residual_rotation: bool = False):
    """The seeded draws of a layer (they do not depend on r and g), cached for the latest layer only."""
    key = _layer_key(shape, M, residual_rotation)
    if _big.get("key") != key:
        _big.clear()
        _big["key"] = key
        _big["L"] = I.make_layer(shape, M=M, residual_rotation=residual_rotation)
    return _big["L"]


def oracle_rotation(shape: I.LayerShape, M: int | None = None, residual_rotation: bool = False):
    """(L, x float32 [M,K], Q float32 [K,K] bf16-valued, xhat = oracle rotation of all tokens), cached."""
    L = layer_inputs(shape, M, residual_rotation)
    if "xhat" not in _big:
        _big["x"] = I.bf16_bits_to_f32(L.x_bits)
        _big["Q"] = I.bf16_bits_to_f32(L.Q_bits)
        _big["xhat"] = O.rotate(_big["x"], _big["Q"])
    return L, _big["x"], _big["Q"], _big["xhat"]


def oracle_fused_weights(shape: I.LayerShape, M: int | None = None, residual_rotation: bool = False):
    """W' = W Q of the layer (oracle, fp32), cached: every (r, g) split of the same layer starts from it."""
    L = layer_inputs(shape, M, residual_rotation)
    if "Wp" not in _big:
        _big["Wp"] = O.fuse_weights(L.W, L.Q32)
    return _big["Wp"]


def layer_with_oracle(shape: I.LayerShape, M: int | None = None, rows=None, residual_rotation: bool = False):
    """Inputs of a layer plus the oracle's result.  Rotation and quantization cover every token;
    `rows` restricts the mixed-precision product (y32, y) to a subset of tokens (tokens are independent
    rows of the layer).  Returns (L, (Wh, qw, sw), ref) with ref["rows"] = the tokens y32 covers."""
    L, x, Q, xhat = oracle_rotation(shape, M, residual_rotation)
    Wh, qw, sw = O.split_quantize_weights(oracle_fused_weights(shape, M, residual_rotation), shape.r, shape.g)
    xh, qx, sx = O.split_quantize(xhat, shape.r, shape.g)
    sel = slice(None) if rows is None else np.asarray(rows)
    y32, y = O.combine(xh[sel], qx[sel], sx[sel], Wh, qw, sw, shape.g)
    ref = dict(xhat=xhat, xh=xh, qx=qx, sx=sx, y32=y32, y=y, rows=sel, x=x, Q=Q)
    return L, (Wh, qw, sw), ref
