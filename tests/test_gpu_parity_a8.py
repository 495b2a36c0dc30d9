"""GPU parity of the 8-bit-activation variant (per-token INT8 activations against 4-bit per-group
weights) with the oracle, through the C ABI.  Same rules as test_gpu_parity.py: integer work
bit-exact, the end-to-end codes statistically (boundary cases only), the output within 1e-2."""
import sys

import numpy as np
import pytest
import torch

from oracle import dirotq_oracle as O
from paper_2605_16732_amd import binding as B
from paper_2605_16732_amd import inputs as I

from gpu_util import (accumulation_slack, check_flips_near_midpoint, check_output, dev, dev_bf16, host_bf16_bits, host_f16,
                      import_blob, oracle_fused_weights, oracle_rotation)

gpu = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


def _positions(C):
    """byte position of channel c in the library's x8 rows: per 32-channel block, evens then odds."""
    c = np.arange(C)
    return (c // 32) * 32 + (c % 2) * 16 + (c % 32) // 2


def pack_i8(q: np.ndarray) -> np.ndarray:
    """int codes [rows, C] in [-127, 127] -> sign-magnitude bytes in the library's channel order."""
    q = np.asarray(q).astype(np.int16)
    assert q.min(initial=0) >= -127 and q.max(initial=0) <= 127 and q.shape[-1] % 32 == 0
    b = (np.abs(q) | np.where(q < 0, 0x80, 0)).astype(np.uint8)
    out = np.empty_like(b)
    out[..., _positions(q.shape[-1])] = b
    return np.ascontiguousarray(out)


def unpack_i8(b: np.ndarray) -> np.ndarray:
    b = np.asarray(b, dtype=np.uint8)
    assert not np.any(b == 0x80), "sign bit set on a zero code"
    nat = b[..., _positions(b.shape[-1])]
    mag = (nat & 0x7F).astype(np.int16)
    return np.where(nat & 0x80, -mag, mag).astype(np.int8)


def test_pack_roundtrip_host():        # no GPU needed: checks the helpers above
    q = np.random.default_rng(0).integers(-127, 128, size=(3, 96)).astype(np.int8)
    np.testing.assert_array_equal(unpack_i8(pack_i8(q)), q)
    assert pack_i8(np.arange(32)[None, :])[0, :4].tolist() == [0, 2, 4, 6]
    assert pack_i8(np.arange(32)[None, :])[0, 16:20].tolist() == [1, 3, 5, 7]


def gpu_rq_a8(x_bits, Qt_dev, r):
    xh, x8, sx = B.rotate_quantize_a8(dev_bf16(x_bits), Qt_dev, r)
    torch.cuda.synchronize()
    M, K = x_bits.shape
    xh_h = O.from_bf16_bits(host_bf16_bits(xh)) if r else np.zeros((M, 0), np.float32)
    if r < K:
        return (xh, x8, sx), (xh_h, unpack_i8(x8.cpu().numpy()), host_f16(sx))
    return (xh, x8, sx), (xh_h, np.zeros((M, 0), np.int8), np.zeros((M,), np.float16))


def _signed_perm(K, seed):
    rng = np.random.default_rng(seed)
    Q = np.zeros((K, K), np.float32)
    Q[rng.permutation(K), np.arange(K)] = rng.choice([-1.0, 1.0], size=K)
    return Q


# ------------------------------------------------------------------ rotation + per-token quantizer, exact
@pytest.mark.parametrize("M,K,r,perm", [
    (300, 256, 64, False), (300, 256, 32, True), (129, 384, 0, True), (1, 128, 32, False),
    (257, 1152, 64, True), (64, 96, 96, True), (130, 448, 64, True), (700, 3072, 128, True), (40, 96, 64, True),
])
@gpu
def test_rotate_quantize_a8_exact_with_permutation_basis(M, K, r, perm):
    """With Q a (signed) permutation the rotation is exact, so the bf16 part, the INT8 codes and the
    per-token scales must equal the oracle's bit for bit (all tile shapes of the launcher are hit)."""
    _say(f"rotate_quantize_a8 exact M={M} K={K} r={r} perm={perm}")
    rng = np.random.default_rng(31)
    Q = _signed_perm(K, 6) if perm else np.eye(K, dtype=np.float32)
    x = O.round_to_bf16((rng.standard_normal((M, K)) * rng.lognormal(0, 1.5, size=(1, K))).astype(np.float32))
    x[M // 2, :] = 0.0                                   # all-zero token: scale 0, codes 0
    Qt = B.prepare_rotation(dev(Q))
    xhat = O.rotate(x, Q)
    xh_r, qx_r, sx_r = O.split_quantize_a8(xhat, r)
    _, (xh_g, qx_g, sx_g) = gpu_rq_a8(O.bf16_bits(x), Qt, r)
    np.testing.assert_array_equal(xh_g, xh_r)
    np.testing.assert_array_equal(sx_g.view(np.uint16), sx_r.view(np.uint16))
    np.testing.assert_array_equal(qx_g, qx_r)


@gpu
def test_rotate_quantize_a8_hand_rows():
    """The hand-worked tokens of tests/golden/quantizer_int8_cases.txt laid into rows (zero padded)."""
    K = 64
    rows = [([127, 0.5, 1.5, 2.5, -126.5, -127], 0x3C00, [127, 0, 2, 2, -126, -127]),
            ([-63.5, 1, 0.25, 0.75, 63], 0x3800, [-127, 2, 0, 2, 126]),
            ([254, 3, 5, -253], 0x4000, [127, 2, 2, -126]),
            ([0, 0, 0], 0x0000, [0, 0, 0])]
    x = np.zeros((len(rows), K), np.float32)
    for i, (vals, _, _) in enumerate(rows):
        x[i, 7:7 + len(vals)] = vals                      # odd start: both halves of a block are hit
    assert np.array_equal(O.round_to_bf16(x), x)
    Qt = B.prepare_rotation(dev(np.eye(K, dtype=np.float32)))
    _, (_, qx_g, sx_g) = gpu_rq_a8(O.bf16_bits(x), Qt, 0)
    for i, (vals, bits, codes) in enumerate(rows):
        assert int(sx_g.view(np.uint16)[i]) == bits
        assert qx_g[i, 7:7 + len(vals)].tolist() == codes
        assert not qx_g[i, :7].any() and not qx_g[i, 7 + len(vals):].any()


# ------------------------------------------------------------------ GEMM
@pytest.mark.parametrize("M,N,K,g", [(130, 200, 256, 32), (257, 136, 448, 64), (64, 129, 384, 128), (5, 8, 64, 32),
                                     (70, 40, 96, 32), (33, 130, 32, 32), (129, 257, 1152, 64)])
@gpu
def test_w4a8_integer_exact(M, N, K, g):
    """Unit scales: y = sum_k q_x q_w with |q_x| <= 127, |q_w| <= 7 is an integer below 2^24, exact in
    fp32 (covers the extreme codes, odd 32-channel counts and every group size)."""
    _say(f"w4a8 integer M={M} N={N} K={K} g={g}")
    rng = np.random.default_rng(32)
    G = K // g
    qx = rng.integers(-127, 128, size=(M, K)).astype(np.int8)
    qw = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    qx[0, :] = 127
    qw[0, :] = -7
    if M > 1 and N > 1:
        qx[1, :] = -127
        qw[1, :] = 7
    blob = import_blob(np.zeros((N, 0), np.float32), qw, np.ones((N, G), np.float16), N, K, 0, g)
    y = B.w4a8_gemm(None, dev(pack_i8(qx)), dev(np.ones((M,), np.float16)), blob, M, N, K, 0, g,
                    out_dtype=torch.float32)
    torch.cuda.synchronize()
    want = (qx.astype(np.int64) @ qw.astype(np.int64).T).astype(np.float32)
    np.testing.assert_array_equal(y.cpu().numpy(), want)


@gpu
def test_w4a8_one_hot_codes_address_every_channel():
    """A single nonzero activation code per token picks out one weight code: any slip in the
    even/odd byte order or in the plane split shows up as a wrong element."""
    K, N, g = 128, 64, 32
    M = 2 * K
    rng = np.random.default_rng(33)
    qw = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    qx = np.zeros((M, K), np.int8)
    qx[np.arange(K), np.arange(K)] = 1                    # low plane only
    qx[K + np.arange(K), np.arange(K)] = -112             # high plane only (7 * 16)
    blob = import_blob(np.zeros((N, 0), np.float32), qw, np.ones((N, K // g), np.float16), N, K, 0, g)
    y = B.w4a8_gemm(None, dev(pack_i8(qx)), dev(np.ones((M,), np.float16)), blob, M, N, K, 0, g,
                    out_dtype=torch.float32).cpu().numpy()
    np.testing.assert_array_equal(y[:K], qw.T.astype(np.float32))
    np.testing.assert_array_equal(y[K:], -112.0 * qw.T.astype(np.float32))


@pytest.mark.parametrize("M,N,K,r,g,use_bias", [
    (200, 136, 320, 64, 64, True), (130, 129, 288, 32, 32, False), (64, 64, 256, 128, 128, True),
    (300, 264, 1152, 64, 64, False), (140, 72, 3072, 0, 64, False), (77, 50, 160, 64, 32, True),
])
@gpu
def test_w4a8_matches_oracle_on_identical_inputs(M, N, K, r, g, use_bias):
    """Same inputs on both sides: only the fp32 accumulation order differs (1e-5 of the largest output)."""
    _say(f"w4a8 vs oracle M={M} N={N} K={K} r={r} g={g} bias={use_bias}")
    rng = np.random.default_rng(34)
    G = (K - r) // g
    xh = O.round_to_bf16(rng.standard_normal((M, r)).astype(np.float32) * 20)
    Wh = O.round_to_bf16(rng.standard_normal((N, r)).astype(np.float32) * 0.05)
    qx = rng.integers(-127, 128, size=(M, K - r)).astype(np.int8)
    qw = rng.integers(-7, 8, size=(N, K - r)).astype(np.int8)
    sx = rng.lognormal(-3, 1, size=(M,)).astype(np.float16)
    sw = rng.lognormal(-5, 1, size=(N, G)).astype(np.float16)
    bias = O.round_to_bf16(rng.standard_normal(N).astype(np.float32)) if use_bias else None
    y32, ybf = O.combine_a8(xh, qx, sx, Wh, qw, sw, g, bias)
    blob = import_blob(Wh, qw, sw, N, K, r, g)
    args = (dev_bf16(O.bf16_bits(xh)) if r else None, dev(pack_i8(qx)), dev(sx), blob, M, N, K, r, g)
    bias_d = dev_bf16(O.bf16_bits(bias)) if use_bias else None
    yf = B.w4a8_gemm(*args, bias=bias_d, out_dtype=torch.float32).cpu().numpy()
    yb = B.w4a8_gemm(*args, bias=bias_d, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    scale = np.abs(y32).max()
    assert np.abs(yf - y32).max() <= 1e-5 * scale
    assert np.abs(O.from_bf16_bits(host_bf16_bits(yb)) - ybf).max() <= 2.0 ** -7 * scale


# ------------------------------------------------------------------ end to end
def check_codes_a8(xhat, qx_gpu, sx_gpu, qx_ref, sx_ref, min_agree=0.999, band=1e-3, x=None, Q=None, col0=0):
    """>= 99.9% of the INT8 codes equal the oracle's.  A token whose stored scale differs must differ by
    one fp16 ulp, and only because the oracle's unrounded amax / 127 lies next to the fp16 rounding midpoint,
    closer than the fp32 accumulation noise of the absmax channel allows; every code is judged
    against the oracle's fp32 rotated value re-quantized with the GPU's stored scale and may differ,
    by one, only within `band` steps of a rounding boundary."""
    M, C = qx_ref.shape
    worst = 0.0
    d = sx_gpu.view(np.uint16) != sx_ref.view(np.uint16)
    if d.any():
        ulps = np.abs(sx_gpu.view(np.int16).astype(np.int32) - sx_ref.view(np.int16).astype(np.int32))
        assert ulps[d].max() == 1, "a scale differs by more than one fp16 ulp"
        assert d.sum() <= max(2, 5e-3 * M), f"{int(d.sum())} scale flips of {M}"
        if x is not None:
            mi = np.nonzero(d)[0]
            cpos = np.argmax(np.abs(xhat[mi]), axis=1)
            amax = np.abs(xhat[mi, cpos])
            s32 = (amax / np.float32(127.0)).astype(np.float32)
            slack = accumulation_slack(x[mi], Q, col0 + cpos, x.shape[1]) / 127.0
            worst = check_flips_near_midpoint(s32, sx_gpu[mi], sx_ref[mi], slack, "token scale")
    sf = sx_gpu.astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(sf == 0, np.float32(0), (np.float32(1.0) / sf).astype(np.float32))
    t = (xhat * inv[:, None]).astype(np.float32)
    want = np.clip(np.rint(t), -127, 127).astype(np.int8)
    diff = qx_gpu != want
    if diff.any():
        tt = t[diff].astype(np.float64)
        frac = np.abs(tt - np.floor(tt) - 0.5)
        assert np.all(frac <= band), f"code flip {frac.max():.3g} steps away from a boundary"
        assert np.all(np.abs(qx_gpu[diff].astype(np.int32) - want[diff]) == 1)
    same_scale = ~d
    agree = float((qx_gpu[same_scale] == qx_ref[same_scale]).mean()) if same_scale.any() else 1.0
    assert agree >= min_agree, f"only {agree:.5f} of the codes agree with the oracle"
    return dict(agree=agree, code_flips=int(diff.sum()), scale_flips=int(d.sum()), worst_flip_slack=worst)


def _end_to_end_a8(shape, y_rows=None):
    """Every token through rotation + per-token INT8 quantization against the oracle; the output of the fused
    layer (and the GEMM on identical inputs) on `y_rows` (default: every token)."""
    L, x, Q, xhat = oracle_rotation(shape)
    K, N, r, g = shape.K, shape.N, shape.r, shape.g
    Mx = x.shape[0]
    Wh, qw, sw = O.split_quantize_weights(oracle_fused_weights(shape), r, g)
    xh_r, qx_r, sx_r = O.split_quantize_a8(xhat, r)
    sel = slice(None) if y_rows is None else np.asarray(y_rows)
    Qt = B.prepare_rotation(dev(L.Q32))
    blob = import_blob(Wh, qw, sw, N, K, r, g)
    (xh_d, x8_d, sx_d), (xh_g, qx_g, sx_g) = gpu_rq_a8(L.x_bits, Qt, r)
    stats = check_codes_a8(xhat[:, r:], qx_g, sx_g, qx_r, sx_r, x=x, Q=Q, col0=r)
    # GEMM on the GPU's own intermediates against the oracle's combine of the same
    y32_same, _ = O.combine_a8(xh_g[sel], qx_g[sel], sx_g[sel], Wh, qw, sw, g)
    yf = B.w4a8_gemm(xh_d if r else None, x8_d, sx_d, blob, Mx, N, K, r, g, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert np.abs(yf.cpu().numpy()[sel] - y32_same).max() <= 1e-5 * np.abs(y32_same).max()
    del yf
    # the fused entry point against the oracle end to end
    y32, _ = O.combine_a8(xh_r[sel], qx_r[sel], sx_r[sel], Wh, qw, sw, g)
    y = B.linear_a8(dev_bf16(L.x_bits), Qt, blob, N, r, g)
    torch.cuda.synchronize()
    row_err, max_err = check_output(O.from_bf16_bits(host_bf16_bits(y))[sel], y32, tol=1e-2)
    y2 = B.w4a8_gemm(xh_d if r else None, x8_d, sx_d, blob, Mx, N, K, r, g, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    _say(f"{shape.name} a8: {Mx} tokens, codes agree {stats['agree']:.6f}, code flips {stats['code_flips']}, scale flips "
         f"{stats['scale_flips']} (worst at {stats['worst_flip_slack']:.2f} of the allowed distance), "
         f"out row-rel {row_err:.2e} max-rel {max_err:.2e}")


@gpu
def test_end_to_end_a8_small_and_ragged():
    _end_to_end_a8(I.SMALL)
    _end_to_end_a8(I.LayerShape("ragged_8", 333, 384, 200, 0, 32, 4, 7, 0))
    _end_to_end_a8(I.LayerShape("ragged128_8", 141, 640, 264, 128, 128, 4, 7, 1))
    _end_to_end_a8(I.LayerShape("odd32_8", 100, 224, 72, 64, 32, 4, 7, 2))


@gpu
def test_end_to_end_a8_flux_fc1_full_launch_every_token():
    # every token quantized and compared; the output on every 8th token
    shp = I.FLUX[2]
    _end_to_end_a8(shp, y_rows=np.arange(0, shp.M, 8))


@gpu
def test_end_to_end_a8_flux_fc2_full_launch_every_token():
    shp = I.FLUX[3]
    _end_to_end_a8(shp, y_rows=np.arange(0, shp.M, 8))


@gpu
def test_a8_rank_equals_K_and_empty():
    shp = I.LayerShape("allhigh_8", 150, 256, 96, 256, 32, 4, 7, 2)
    L = I.make_layer(shp)
    x, Q = I.bf16_bits_to_f32(L.x_bits), I.bf16_bits_to_f32(L.Q_bits)
    Wh, qw, sw = O.prepare_weights(L.W, L.Q32, shp.r, shp.g)
    ref = O.linear_a8(x, Q, Wh, qw, sw, shp.r, shp.g)
    Qt = B.prepare_rotation(dev(L.Q32))
    blob = import_blob(Wh, qw, sw, shp.N, shp.K, shp.r, shp.g)
    y = B.linear_a8(dev_bf16(L.x_bits), Qt, blob, shp.N, shp.r, shp.g)
    torch.cuda.synchronize()
    check_output(O.from_bf16_bits(host_bf16_bits(y)), ref["y32"], tol=1e-2)
    y0 = B.linear_a8(dev_bf16(L.x_bits)[:0], Qt, blob, shp.N, shp.r, shp.g)
    assert y0.shape == (0, shp.N)
