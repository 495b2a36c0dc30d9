"""CPU oracle for the rotation-aware W4A4 linear layer (DiRotQ).

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, obviously-correct NumPy
statement of what the layer computes, written from the paper; it shares no code
with the HIP library and must never be imported by the product path.  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may call it.

Notation.  The paper writes Y = X W with X in R^{b x m}, W in R^{m x n}, rotation
V = [U_h, U_l R] and rank k = r m ("Problem formulation" and "PCA-guided rotated
quantization").  Here the nn.Linear convention is used: M tokens, K input
channels, N output channels, W in R^{N x K}, y = W x, Q = V (column j = j-th
basis direction), `r` = the rank itself (the paper's k), `g` = group size,
G = (K - r) / g groups.  W' = W Q is the offline-fused weight (the paper's
V^T W, transposed).

The layer is an approximation of X W (the forward-computation equation has an
"approximately equal"), so the oracle is the algorithm step by step.  Storage
roundings (BF16 for the kept coefficients, INT4 + fp16 scale for the rest, fp32
for the rotated activations) are part of the definition; summation order is not,
so every sum is taken in float64.

Readings where the paper is silent (each is listed in the design notes too):
  * symmetric quantizer for activations and weights, codes clipped to [-7, 7]
    (the paper formulates everything in the symmetric form of its quantizer
    equation, q_max = 2^(4-1) - 1 = 7);
  * round-half-to-even in the round-and-clip operator;
  * groups are g consecutive rotated channels starting at channel r, per token for
    activations and per output channel for weights ("per-group ... group size 64"
    with "16-bit scaling factors");
  * scales are stored as IEEE fp16 and codes are computed against the *stored*
    scale, with the fixed fp32 operation sequence of `quantize_groups`;
  * the quantizer reads the fp32 rotated activation, not a BF16-rounded copy;
  * the W4A8 variant (`*_a8`) follows the paper's implementation details for 8-bit
    settings on the activation side: per-token dynamic quantization, here symmetric INT8
    over the K - r rotated channels that are not kept in BF16, one fp16 scale per token;
    weights stay 4-bit per group;
  * the W4A16 layers (`linear_w4a16`: the appendix on quantization details keeps the input
    activations of some layers in 16 bits) are read as weight-only quantization without
    rotation: BF16 activations against the same per-group 4-bit weights, dequantized
    exactly (code x fp16 scale);
  * the asymmetric activation variant (`*_asym`, the form the paper's experiments use
    for activations: z = min X, s = (max X - min X) / 15, codes in [0, 15]) stores the
    zero-point as fp16 next to the fp16 scale and quantizes against the stored pair.

Pins (see tests/test_oracle_*.py): hand-worked quantizer cases from the quantizer
equation, nibble packing bytes, a pure-Python-loop brute force of the whole layer on
tiny shapes, the identity X W = X V V^T W (exact mode, any r), reduction to a plain
BF16 GEMM at r = K, reduction to plain per-group RTN at Q = I, quantizer error
bounds; for the W4A16 layer a Python-loop brute force, exact integer and power-of-two cases
and agreement with `combine` on activations that are themselves code x scale; for the asymmetric variant hand-worked cases, shift equivariance, its error
bound, and a brute force that dequantizes every element (q s + z) and multiplies
out, which pins the zero-point term of `combine_asym`.  Unpinned: absolute QSNR / image-quality numbers of the paper (they need
its models and data) -- "parity unpinned" for those, none of which is computed here.
"""
from __future__ import annotations

import numpy as np

QMAX = 7                       # 2^(4-1) - 1, quantizer equation, symmetric case
UQMAX = 15                     # 2^4 - 1, quantizer equation, asymmetric case (q_min = 0)
QMAX8 = 127                    # 2^(8-1) - 1, quantizer equation, symmetric case, 8 bits
FP16_MAX = np.float32(65504.0)


# --------------------------------------------------------------------------
# storage formats
# --------------------------------------------------------------------------
def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns the
    rounded values as float32.  NaN/inf do not occur in this workload."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a_bf16_valued: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bfloat16-valued."""
    a = np.ascontiguousarray(a_bf16_valued, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16).reshape(a.shape)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b).astype(np.uint32) << np.uint32(16)).view(np.float32)


def pack_int4(codes: np.ndarray) -> np.ndarray:
    """[..., C] int8 codes in [-8, 7] -> [..., C/2] uint8.  Byte i holds channel 2i
    in bits 0-3 and channel 2i+1 in bits 4-7, two's-complement nibbles."""
    c = np.asarray(codes).astype(np.int16)
    assert c.shape[-1] % 2 == 0
    lo = c[..., 0::2] & 0xF
    hi = c[..., 1::2] & 0xF
    return (lo | (hi << 4)).astype(np.uint8)


def unpack_int4(packed: np.ndarray) -> np.ndarray:
    p = np.asarray(packed).astype(np.int16)
    lo = p & 0xF
    hi = (p >> 4) & 0xF
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty(p.shape[:-1] + (2 * p.shape[-1],), dtype=np.int8)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


# --------------------------------------------------------------------------
# the quantizer  (quantizer equation, symmetric: z = 0, s = max|X| / q_max)
# --------------------------------------------------------------------------
def quantize_groups(v: np.ndarray, g: int):
    """Symmetric INT4 quantization of the last axis in groups of g.

    v: float32 [..., C], C % g == 0.  Returns (codes int8 [..., C] in [-7,7],
    scales float16 [..., C/g]).  The dequantised value is codes * float32(scale).

    Fixed IEEE-fp32 sequence (so that another implementation can reproduce it
    bit for bit):  amax = max|v|;  s32 = amax / 7 (fp32 division);
    s16 = fp16(s32) (round to nearest even, saturating at 65504);
    sf = float32(s16);  sf == 0 -> all codes 0;  else inv = 1 / sf (fp32 division),
    t = v * inv (fp32), code = clip(rint(t), -7, 7) with rint = ties to even.
    """
    v = np.ascontiguousarray(v, dtype=np.float32)
    C = v.shape[-1]
    assert C % g == 0
    vg = v.reshape(v.shape[:-1] + (C // g, g))
    amax = np.max(np.abs(vg), axis=-1)                               # exact
    s32 = (amax / np.float32(QMAX)).astype(np.float32)
    s32 = np.minimum(s32, FP16_MAX)
    s16 = s32.astype(np.float16)                                     # RNE
    sf = s16.astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = (np.float32(1.0) / sf).astype(np.float32)
    inv = np.where(sf == 0, np.float32(0.0), inv).astype(np.float32)
    t = (vg * inv[..., None]).astype(np.float32)
    q = np.clip(np.rint(t), -QMAX, QMAX).astype(np.int8)
    return q.reshape(v.shape), s16


def dequantize_groups(codes: np.ndarray, scales: np.ndarray, g: int) -> np.ndarray:
    """codes * scale, in float64 (exact: 3-bit by 11-bit significands)."""
    c = np.asarray(codes).astype(np.float64)
    s = np.repeat(np.asarray(scales).astype(np.float64), g, axis=-1)
    return c * s


# --------------------------------------------------------------------------
# the quantizer, asymmetric case  (quantizer equation: z = min X,
# s = (max X - min X) / (q_max - q_min), q_min = 0, q_max = 2^4 - 1)
# --------------------------------------------------------------------------
def quantize_groups_asym(v: np.ndarray, g: int):
    """Asymmetric UINT4 quantization of the last axis in groups of g.

    v: float32 [..., C], C % g == 0.  Returns (codes uint8 [..., C] in [0,15],
    scales float16 [..., C/g], zeros float16 [..., C/g]).  The dequantised value is
    codes * float32(scale) + float32(zero).

    Fixed IEEE-fp32 sequence:  mn = min v, mx = max v;  z16 = fp16(mn) (round to
    nearest even, saturating at +-65504), zf = float32(z16);  s32 = (mx - mn) / 15
    (fp32 subtraction, then fp32 division);  s16 = fp16(min(s32, 65504));
    sf = float32(s16);  sf == 0 -> all codes 0;  else inv = 1 / sf (fp32 division),
    t = (v - zf) * inv (fp32 subtraction, then fp32 product),
    code = clip(rint(t), 0, 15) with rint = ties to even.
    """
    v = np.ascontiguousarray(v, dtype=np.float32)
    C = v.shape[-1]
    assert C % g == 0
    vg = v.reshape(v.shape[:-1] + (C // g, g))
    mn = np.min(vg, axis=-1)
    mx = np.max(vg, axis=-1)
    z16 = np.clip(mn, -FP16_MAX, FP16_MAX).astype(np.float16)        # RNE
    zf = z16.astype(np.float32)
    s32 = ((mx - mn).astype(np.float32) / np.float32(UQMAX)).astype(np.float32)
    s32 = np.minimum(s32, FP16_MAX)
    s16 = s32.astype(np.float16)
    sf = s16.astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = (np.float32(1.0) / sf).astype(np.float32)
    inv = np.where(sf == 0, np.float32(0.0), inv).astype(np.float32)
    t = ((vg - zf[..., None]).astype(np.float32) * inv[..., None]).astype(np.float32)
    q = np.clip(np.rint(t), 0, UQMAX).astype(np.uint8)
    return q.reshape(v.shape), s16, z16


def dequantize_groups_asym(codes, scales, zeros, g: int) -> np.ndarray:
    """codes * scale + zero, in float64."""
    c = np.asarray(codes).astype(np.float64)
    s = np.repeat(np.asarray(scales).astype(np.float64), g, axis=-1)
    z = np.repeat(np.asarray(zeros).astype(np.float64), g, axis=-1)
    return c * s + z


# --------------------------------------------------------------------------
# offline: fuse the rotation into the weights, split, quantize
# (weight-fusion step of Section 4.2, just before the forward-computation
#  equation; RTN stands in for GPTQ on the residual weights)
# --------------------------------------------------------------------------
def fuse_weights(W: np.ndarray, Q32: np.ndarray) -> np.ndarray:
    """W' = W Q: W float32 [N,K], Q32 float32 [K,K]; float64 accumulation, one rounding to fp32."""
    return (np.asarray(W, np.float64) @ np.asarray(Q32, np.float64)).astype(np.float32)


def split_quantize_weights(Wp: np.ndarray, r: int, g: int):
    """Fused weights W' fp32 [N,K] -> (Wh float32 bf16-valued [N,r], qw int8 [N,K-r], sw float16 [N,G]):
    the first r input channels in 16 bits, the rest per output channel and group with the quantizer."""
    Wh = round_to_bf16(Wp[:, :r])
    if r < Wp.shape[1]:
        qw, sw = quantize_groups(Wp[:, r:], g)
    else:
        qw = np.zeros((Wp.shape[0], 0), np.int8)
        sw = np.zeros((Wp.shape[0], 0), np.float16)
    return Wh, qw, sw


def prepare_weights(W: np.ndarray, Q32: np.ndarray, r: int, g: int):
    """W float32 [N,K], Q32 float32 [K,K] -> (Wh float32 bf16-valued [N,r],
    qw int8 [N,K-r], sw float16 [N,G]).  W' = W Q in float64, rounded to fp32."""
    return split_quantize_weights(fuse_weights(W, Q32), r, g)


# --------------------------------------------------------------------------
# online: rotate, split, quantize   (rotation / split equation; quantizer)
# --------------------------------------------------------------------------
def rotate(x: np.ndarray, Q: np.ndarray) -> np.ndarray:
    """x_hat = x Q.  x float32 (bf16-valued) [M,K]; Q float32 (bf16-valued) [K,K];
    float64 accumulation, result rounded once to float32."""
    return (np.asarray(x, np.float64) @ np.asarray(Q, np.float64)).astype(np.float32)


def split_quantize(xhat: np.ndarray, r: int, g: int):
    """First r rotated channels -> BF16; the rest -> per-token per-group INT4.
    Returns (xh float32 bf16-valued [M,r], qx int8 [M,K-r], sx float16 [M,G])."""
    xh = round_to_bf16(xhat[:, :r])
    if r < xhat.shape[1]:
        qx, sx = quantize_groups(xhat[:, r:], g)
    else:
        qx = np.zeros((xhat.shape[0], 0), np.int8)
        sx = np.zeros((xhat.shape[0], 0), np.float16)
    return xh, qx, sx


def rotate_quantize(x, Q, r, g):
    return split_quantize(rotate(x, Q), r, g)


# --------------------------------------------------------------------------
# online: mixed-precision product  (forward-computation equation)
# --------------------------------------------------------------------------
def group_int_dots(qx: np.ndarray, qw: np.ndarray, g: int) -> np.ndarray:
    """I[m,n,j] = sum over group j of qx[m,k] qw[n,k]; exact int64 [M,N,G]."""
    M, C = qx.shape
    N = qw.shape[0]
    G = C // g
    a = qx.astype(np.int64).reshape(M, G, g)
    b = qw.astype(np.int64).reshape(N, G, g)
    return np.einsum("mjk,njk->mnj", a, b)


def combine(xh, qx, sx, Wh, qw, sw, g, bias=None):
    """y32[m,n] = sum_{k<r} xh[m,k] Wh[n,k] + sum_j sx[m,j] sw[n,j] I[m,n,j] (+bias)
    in float64, rounded once to float32; y = bf16(y32).  Returns (y32, y_bf16_valued)."""
    M = xh.shape[0]
    N = Wh.shape[0]
    acc = np.asarray(xh, np.float64) @ np.asarray(Wh, np.float64).T if xh.shape[1] else np.zeros((M, N))
    C = qx.shape[1]
    G = C // g if C else 0
    sx64 = np.asarray(sx).astype(np.float64)
    sw64 = np.asarray(sw).astype(np.float64)
    for j in range(G):
        a = qx[:, j * g:(j + 1) * g].astype(np.float64)      # integers: products and
        b = qw[:, j * g:(j + 1) * g].astype(np.float64)      # sums exact in float64
        I = a @ b.T
        acc = acc + (sx64[:, j][:, None] * sw64[:, j][None, :]) * I
    if bias is not None:
        acc = acc + np.asarray(bias, np.float64)[None, :]
    y32 = acc.astype(np.float32)
    return y32, round_to_bf16(y32)


def linear(x, Q, Wh, qw, sw, r, g, bias=None):
    """The whole online layer on prepared weights.  Returns a dict of every
    intermediate so that tests can compare stage by stage."""
    xhat = rotate(x, Q)
    xh, qx, sx = split_quantize(xhat, r, g)
    y32, y = combine(xh, qx, sx, Wh, qw, sw, g, bias)
    return dict(xhat=xhat, xh=xh, qx=qx, sx=sx, y32=y32, y=y)


# --------------------------------------------------------------------------
# asymmetric activations: the same layer with the quantizer's z term kept
# ("the asymmetric case follows analogously with an additional z term";
#  weights stay symmetric)
# --------------------------------------------------------------------------
def split_quantize_asym(xhat: np.ndarray, r: int, g: int):
    """Returns (xh float32 bf16-valued [M,r], qx uint8 [M,K-r] in [0,15],
    sx float16 [M,G], zx float16 [M,G])."""
    xh = round_to_bf16(xhat[:, :r])
    if r < xhat.shape[1]:
        qx, sx, zx = quantize_groups_asym(xhat[:, r:], g)
    else:
        qx = np.zeros((xhat.shape[0], 0), np.uint8)
        sx = np.zeros((xhat.shape[0], 0), np.float16)
        zx = np.zeros((xhat.shape[0], 0), np.float16)
    return xh, qx, sx, zx


def weight_group_sums(qw: np.ndarray, g: int) -> np.ndarray:
    """sum of the weight codes of each group: int64 [N, G]."""
    N, C = qw.shape
    return qw.astype(np.int64).reshape(N, C // g, g).sum(axis=-1)


def combine_asym(xh, qx, sx, zx, Wh, qw, sw, g, bias=None):
    """With x~[m,k] = sx[m,j] qx[m,k] + zx[m,j] and w~[n,k] = sw[n,j] qw[n,k]:
    sum_k x~ w~ = sum_j ( sx sw I[m,n,j] + zx[m,j] sw[n,j] sum_{k in j} qw[n,k] ).
    y32 = sum_{k<r} xh Wh + that (+ bias), float64, rounded once to float32."""
    M = xh.shape[0]
    N = Wh.shape[0]
    acc = np.asarray(xh, np.float64) @ np.asarray(Wh, np.float64).T if xh.shape[1] else np.zeros((M, N))
    C = qx.shape[1]
    G = C // g if C else 0
    sx64 = np.asarray(sx).astype(np.float64)
    zx64 = np.asarray(zx).astype(np.float64)
    sw64 = np.asarray(sw).astype(np.float64)
    wsum = weight_group_sums(qw, g).astype(np.float64) if G else np.zeros((N, 0))
    for j in range(G):
        a = qx[:, j * g:(j + 1) * g].astype(np.float64)
        b = qw[:, j * g:(j + 1) * g].astype(np.float64)
        I = a @ b.T
        acc = acc + (sx64[:, j][:, None] * sw64[:, j][None, :]) * I
        acc = acc + zx64[:, j][:, None] * (sw64[:, j] * wsum[:, j])[None, :]
    if bias is not None:
        acc = acc + np.asarray(bias, np.float64)[None, :]
    y32 = acc.astype(np.float32)
    return y32, round_to_bf16(y32)


def linear_asym(x, Q, Wh, qw, sw, r, g, bias=None):
    xhat = rotate(x, Q)
    xh, qx, sx, zx = split_quantize_asym(xhat, r, g)
    y32, y = combine_asym(xh, qx, sx, zx, Wh, qw, sw, g, bias)
    return dict(xhat=xhat, xh=xh, qx=qx, sx=sx, zx=zx, y32=y32, y=y)


# --------------------------------------------------------------------------
# W4A8: 8-bit per-token activations (the paper's "per-token dynamic activation
# quantization" for 8-bit settings), 4-bit per-group weights
# --------------------------------------------------------------------------
def quantize_tokens_int8(v: np.ndarray):
    """Symmetric INT8 quantization of each row (token) with one scale.

    v: float32 [M, C].  Returns (codes int8 [M, C] in [-127,127], scales float16 [M]).
    Same fixed fp32 sequence as `quantize_groups` with q_max = 127:  amax = max|v|;
    s32 = amax / 127;  s16 = fp16(min(s32, 65504));  sf = float32(s16);  sf == 0 -> codes 0;
    inv = 1 / sf;  code = clip(rint(v * inv), -127, 127).
    """
    v = np.ascontiguousarray(v, dtype=np.float32)
    if v.shape[1] == 0:
        return np.zeros(v.shape, np.int8), np.zeros((v.shape[0],), np.float16)
    amax = np.max(np.abs(v), axis=1)
    s32 = np.minimum((amax / np.float32(QMAX8)).astype(np.float32), FP16_MAX)
    s16 = s32.astype(np.float16)
    sf = s16.astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = (np.float32(1.0) / sf).astype(np.float32)
    inv = np.where(sf == 0, np.float32(0.0), inv).astype(np.float32)
    t = (v * inv[:, None]).astype(np.float32)
    q = np.clip(np.rint(t), -QMAX8, QMAX8).astype(np.int8)
    return q, s16


def split_quantize_a8(xhat: np.ndarray, r: int):
    """Returns (xh float32 bf16-valued [M,r], qx int8 [M,K-r], sx float16 [M])."""
    xh = round_to_bf16(xhat[:, :r])
    qx, sx = quantize_tokens_int8(xhat[:, r:])
    return xh, qx, sx


def combine_a8(xh, qx, sx, Wh, qw, sw, g, bias=None):
    """y32[m,n] = sum_{k<r} xh Wh + sx[m] * sum_j sw[n,j] I[m,n,j] (+ bias), I the exact integer
    dot of the INT8 activation codes with the INT4 weight codes of group j; float64, one
    rounding to float32."""
    M = xh.shape[0]
    N = Wh.shape[0]
    acc = np.asarray(xh, np.float64) @ np.asarray(Wh, np.float64).T if xh.shape[1] else np.zeros((M, N))
    C = qx.shape[1]
    G = C // g if C else 0
    sx64 = np.asarray(sx).astype(np.float64)
    sw64 = np.asarray(sw).astype(np.float64)
    low = np.zeros((M, N))
    for j in range(G):
        a = qx[:, j * g:(j + 1) * g].astype(np.float64)
        b = qw[:, j * g:(j + 1) * g].astype(np.float64)
        low = low + (a @ b.T) * sw64[:, j][None, :]
    acc = acc + sx64[:, None] * low
    if bias is not None:
        acc = acc + np.asarray(bias, np.float64)[None, :]
    y32 = acc.astype(np.float32)
    return y32, round_to_bf16(y32)


def linear_a8(x, Q, Wh, qw, sw, r, g, bias=None):
    xhat = rotate(x, Q)
    xh, qx, sx = split_quantize_a8(xhat, r)
    y32, y = combine_a8(xh, qx, sx, Wh, qw, sw, g, bias)
    return dict(xhat=xhat, xh=xh, qx=qx, sx=sx, y32=y32, y=y)


# --------------------------------------------------------------------------
# W4A16: layers whose input activations stay in 16 bits (appendix "Quantization
# details"); weights quantized per group with the Section 3 quantizer, no rotation
# --------------------------------------------------------------------------
def linear_w4a16(x, qw, sw, g, bias=None):
    """y32[m,n] = sum_k x[m,k] * (qw[n,k] * sw[n, k // g]) (+ bias[n]) in float64, rounded once to
    float32; y = bf16(y32).  x: bf16-valued float32 [M,K]; qw int8 [N,K]; sw float16 [N,K/g].
    Returns (y32, y_bf16_valued)."""
    Wd = dequantize_groups(qw, sw, g)                       # float64, exact
    acc = np.asarray(x, np.float64) @ Wd.T
    if bias is not None:
        acc = acc + np.asarray(bias, np.float64)[None, :]
    y32 = acc.astype(np.float32)
    return y32, round_to_bf16(y32)


# --------------------------------------------------------------------------
# exact mode: the identity behind the method, no storage rounding
# --------------------------------------------------------------------------
def linear_exact(x, Q, W, r):
    """[x Q_h, x Q_l] [ (W Q)_h ; (W Q)_l ]^T in float64 with nothing rounded:
    equals x W^T for an orthogonal Q whatever the split point r."""
    x = np.asarray(x, np.float64)
    Q = np.asarray(Q, np.float64)
    W = np.asarray(W, np.float64)
    xhat = x @ Q
    Wp = W @ Q
    return xhat[:, :r] @ Wp[:, :r].T + xhat[:, r:] @ Wp[:, r:].T


def qsnr_db(ref: np.ndarray, approx: np.ndarray) -> float:
    ref = np.asarray(ref, np.float64)
    err = ref - np.asarray(approx, np.float64)
    return float(10.0 * np.log10(np.sum(ref * ref) / max(np.sum(err * err), 1e-300)))
