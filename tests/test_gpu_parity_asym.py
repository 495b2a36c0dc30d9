"""GPU parity of the asymmetric-activation variant (zero-point min, 16 unsigned levels) against
the oracle, through the C ABI.  Same rules as test_gpu_parity.py: integer work bit-exact, the
end-to-end codes statistically (boundary cases only), the output within 1e-2 relative."""
import sys

import numpy as np
import pytest
import torch

from oracle import dirotq_oracle as O
from paper_2605_16732_amd import binding as B
from paper_2605_16732_amd import inputs as I

from gpu_util import (accumulation_slack, check_flips_near_midpoint, check_output, dev, dev_bf16, host_bf16_bits, host_f16,
                      import_blob, oracle_fused_weights, oracle_rotation)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


def pack_u4(q: np.ndarray) -> np.ndarray:
    """unsigned codes [rows, C] in [0, 15] -> two nibbles per byte, even channel low."""
    q = np.asarray(q, dtype=np.uint8)
    assert q.max(initial=0) <= 15
    return np.ascontiguousarray(q[..., 0::2] | (q[..., 1::2] << 4))


def unpack_u4(b: np.ndarray) -> np.ndarray:
    b = np.asarray(b, dtype=np.uint8)
    return np.stack([b & 15, b >> 4], axis=-1).reshape(*b.shape[:-1], b.shape[-1] * 2)


def gpu_rq_asym(x_bits, Qt_dev, r, g):
    xh, xl, sx, zx = B.rotate_quantize_asym(dev_bf16(x_bits), Qt_dev, r, g)
    torch.cuda.synchronize()
    M, K = x_bits.shape
    xh_h = O.from_bf16_bits(host_bf16_bits(xh)) if r else np.zeros((M, 0), np.float32)
    if r < K:
        return (xh, xl, sx, zx), (xh_h, unpack_u4(xl.cpu().numpy()), np.ascontiguousarray(host_f16(sx).T),
                                  np.ascontiguousarray(host_f16(zx).T))
    z = np.zeros((M, 0), np.float16)
    return (xh, xl, sx, zx), (xh_h, np.zeros((M, 0), np.uint8), z, z)


def _signed_perm(K, seed):
    rng = np.random.default_rng(seed)
    Q = np.zeros((K, K), np.float32)
    Q[rng.permutation(K), np.arange(K)] = rng.choice([-1.0, 1.0], size=K)
    return Q


# ------------------------------------------------------------------ kernel A, exact
@pytest.mark.parametrize("M,K,r,g,perm", [
    (300, 256, 64, 64, False), (300, 256, 32, 32, True), (129, 384, 0, 128, True), (1, 128, 32, 32, False),
    (257, 1152, 64, 64, True), (64, 96, 96, 32, True), (130, 448, 64, 128, True), (700, 3072, 128, 64, True),
])
def test_rotate_quantize_asym_exact_with_permutation_basis(M, K, r, g, perm):
    """With Q a (signed) permutation the rotation is exact, so bf16 part, codes, scales and
    zero-points must equal the oracle's bit for bit (all tile shapes of the launcher are hit)."""
    _say(f"rotate_quantize_asym exact M={M} K={K} r={r} g={g} perm={perm}")
    rng = np.random.default_rng(13)
    Q = _signed_perm(K, 5) if perm else np.eye(K, dtype=np.float32)
    x = O.round_to_bf16((rng.standard_normal((M, K)) * rng.lognormal(0, 1.5, size=(1, K)) +
                         rng.normal(0, 2, size=(1, K))).astype(np.float32))
    x[M // 2, :] = 0.0                                   # all-zero token: s = 0, z = 0
    if M > 3:
        x[3, :] = O.round_to_bf16(np.float32(1.75))      # constant token: s = 0, z = +-1.75
    Qt = B.prepare_rotation(dev(Q))
    xhat = O.rotate(x, Q)
    xh_r, qx_r, sx_r, zx_r = O.split_quantize_asym(xhat, r, g)
    _, (xh_g, qx_g, sx_g, zx_g) = gpu_rq_asym(O.bf16_bits(x), Qt, r, g)
    np.testing.assert_array_equal(xh_g, xh_r)
    np.testing.assert_array_equal(sx_g.view(np.uint16), sx_r.view(np.uint16))
    np.testing.assert_array_equal(zx_g.view(np.uint16), zx_r.view(np.uint16))
    np.testing.assert_array_equal(qx_g, qx_r)


def test_rotate_quantize_asym_hand_rows():
    """The hand-worked groups of tests/golden/quantizer_asym_cases.txt laid into rows."""
    K, r, g = 64, 0, 32
    x = np.zeros((3, K), np.float32)
    x[0, :32] = -3.0
    x[0, :5] = [-3, 4.5, 0, 1, -2.75]
    x[0, 32:] = 0.0
    x[0, 32:38] = [0, 15, 0.5, 1.5, 2.5, 14.5]
    x[1, :32] = 2.0
    x[1, :5] = [2, 32, 3, 5, 31]
    x[1, 32:] = 2.5                                       # constant group
    x[2, :32] = -8.0
    x[2, :4] = [-8, -0.5, -4, -7.75]
    assert np.array_equal(O.round_to_bf16(x), x)
    Qt = B.prepare_rotation(dev(np.eye(K, dtype=np.float32)))
    _, (_, qx_g, sx_g, zx_g) = gpu_rq_asym(O.bf16_bits(x), Qt, r, g)
    assert list(qx_g[0, :5]) == [0, 15, 6, 8, 0] and float(sx_g[0, 0]) == 0.5 and float(zx_g[0, 0]) == -3.0
    assert list(qx_g[0, 32:38]) == [0, 15, 0, 2, 2, 14] and float(sx_g[0, 1]) == 1.0 and float(zx_g[0, 1]) == 0.0
    assert list(qx_g[1, :5]) == [0, 15, 0, 2, 14] and float(sx_g[1, 0]) == 2.0 and float(zx_g[1, 0]) == 2.0
    assert not qx_g[1, 32:].any() and float(sx_g[1, 1]) == 0.0 and float(zx_g[1, 1]) == 2.5
    assert list(qx_g[2, :4]) == [0, 15, 8, 0] and float(sx_g[2, 0]) == 0.5 and float(zx_g[2, 0]) == -8.0
    _, qx_r, sx_r, zx_r = O.split_quantize_asym(x, r, g)
    np.testing.assert_array_equal(qx_g, qx_r)


# ------------------------------------------------------------------ kernel B
@pytest.fixture(params=["tile", "ws"])
def asym_schedule(request, monkeypatch):
    """Asymmetric layers run on two schedules of kernel B (128 x 128 tiles with the zero-point passes in the tail;
    wave-specialised workgroups whose staging waves add zero-point stages to the stage stream); the library picks by
    problem size and the environment switch forces one, so that both run on the same inputs."""
    monkeypatch.setenv("DIROTQ_W4A4_KERNEL", request.param)
    return request.param


@pytest.mark.parametrize("M,N,K,g", [(130, 200, 256, 32), (257, 136, 448, 64), (64, 129, 384, 128), (5, 8, 64, 32),
                                     (300, 520, 832, 64)])
def test_w4a4_asym_integer_exact(M, N, K, g, asym_schedule):
    """Unit scales, integer zero-points: y = sum_k (q_x + z) q_w is a small integer, exact in fp32."""
    _say(f"w4a4_asym integer M={M} N={N} K={K} g={g}")
    rng = np.random.default_rng(14)
    G = K // g
    qx = rng.integers(0, 16, size=(M, K)).astype(np.uint8)
    qw = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    qx[0, :] = 15
    qw[0, :] = -7
    zx = rng.integers(-8, 9, size=(M, G)).astype(np.float16)
    ones = np.ones((G, M), np.float16)
    blob = import_blob(np.zeros((N, 0), np.float32), qw, np.ones((N, G), np.float16), N, K, 0, g)
    y = B.w4a4_gemm_asym(None, dev(pack_u4(qx)), dev(ones), dev(np.ascontiguousarray(zx.T)), blob, M, N, K, 0, g,
                         out_dtype=torch.float32)
    torch.cuda.synchronize()
    xt = qx.astype(np.int64) + np.repeat(zx.astype(np.int64), g, axis=1)
    want = (xt @ qw.astype(np.int64).T).astype(np.float32)
    np.testing.assert_array_equal(y.cpu().numpy(), want)


@pytest.mark.parametrize("M,N,K,r,g,use_bias", [
    (200, 136, 320, 64, 64, True), (130, 129, 288, 32, 32, False), (64, 64, 256, 128, 128, True),
    (300, 264, 1152, 64, 64, False), (140, 72, 3072, 0, 64, False), (260, 515, 224, 96, 32, True),
    (150, 300, 416, 32, 128, True),
])
def test_w4a4_asym_matches_oracle_on_identical_inputs(M, N, K, r, g, use_bias, asym_schedule):
    """Same inputs on both sides.  The zero-point term is summed from bf16 splits that drop
    less than 2^-16 of it, the rest is fp32 accumulation: 2e-5 of the largest output magnitude."""
    _say(f"w4a4_asym vs oracle M={M} N={N} K={K} r={r} g={g} bias={use_bias}")
    rng = np.random.default_rng(15)
    G = (K - r) // g
    xh = O.round_to_bf16(rng.standard_normal((M, r)).astype(np.float32) * 20)
    Wh = O.round_to_bf16(rng.standard_normal((N, r)).astype(np.float32) * 0.05)
    qx = rng.integers(0, 16, size=(M, K - r)).astype(np.uint8)
    qw = rng.integers(-7, 8, size=(N, K - r)).astype(np.int8)
    sx = rng.lognormal(-1, 1, size=(M, G)).astype(np.float16)
    zx = (rng.standard_normal((M, G)) * 5).astype(np.float16)
    sw = rng.lognormal(-5, 1, size=(N, G)).astype(np.float16)
    bias = O.round_to_bf16(rng.standard_normal(N).astype(np.float32)) if use_bias else None
    y32, ybf = O.combine_asym(xh, qx, sx, zx, Wh, qw, sw, g, bias)
    blob = import_blob(Wh, qw, sw, N, K, r, g)
    args = (dev_bf16(O.bf16_bits(xh)) if r else None, dev(pack_u4(qx)), dev(np.ascontiguousarray(sx.T)),
            dev(np.ascontiguousarray(zx.T)), blob, M, N, K, r, g)
    bias_d = dev_bf16(O.bf16_bits(bias)) if use_bias else None
    yf = B.w4a4_gemm_asym(*args, bias=bias_d, out_dtype=torch.float32).cpu().numpy()
    yb = B.w4a4_gemm_asym(*args, bias=bias_d, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    scale = np.abs(y32).max()
    assert np.abs(yf - y32).max() <= 2e-5 * scale
    assert np.abs(O.from_bf16_bits(host_bf16_bits(yb)) - ybf).max() <= 2.0 ** -7 * scale
    # without the zero-points the call reduces to ... a different answer (the term is live)
    y0 = B.w4a4_gemm_asym(*args[:3], dev(np.zeros((G, M), np.float16)), *args[4:], bias=bias_d,
                          out_dtype=torch.float32).cpu().numpy()
    assert np.abs(y0 - y32).max() > 1e-2 * scale


def test_w4a4_asym_persistent_workgroups_take_several_tiles(monkeypatch):
    """300 tiles of 256 x 128 on 256 CUs in the wave-specialised schedule: some workgroups run two tiles back to
    back, so a tile's zero-point stages are followed by the next tile's regular ones.  Ragged in both directions,
    a rank-32 branch, 8 groups (two zero-point stages of which the second is partly padding, plus two empty ones)."""
    monkeypatch.setenv("DIROTQ_W4A4_KERNEL", "ws")
    M, N, K, r, g = 2500, 3592, 544, 32, 64
    _say(f"w4a4_asym persistent M={M} N={N} K={K} r={r} g={g}")
    rng = np.random.default_rng(17)
    G = (K - r) // g
    xh = O.round_to_bf16(rng.standard_normal((M, r)).astype(np.float32) * 20)
    Wh = O.round_to_bf16(rng.standard_normal((N, r)).astype(np.float32) * 0.05)
    qx = rng.integers(0, 16, size=(M, K - r)).astype(np.uint8)
    qw = rng.integers(-7, 8, size=(N, K - r)).astype(np.int8)
    sx = rng.lognormal(-1, 1, size=(M, G)).astype(np.float16)
    zx = (rng.standard_normal((M, G)) * 5).astype(np.float16)
    sw = rng.lognormal(-5, 1, size=(N, G)).astype(np.float16)
    bias = O.round_to_bf16(rng.standard_normal(N).astype(np.float32))
    y32, ybf = O.combine_asym(xh, qx, sx, zx, Wh, qw, sw, g, bias)
    blob = import_blob(Wh, qw, sw, N, K, r, g)
    args = (dev_bf16(O.bf16_bits(xh)), dev(pack_u4(qx)), dev(np.ascontiguousarray(sx.T)),
            dev(np.ascontiguousarray(zx.T)), blob, M, N, K, r, g)
    bias_d = dev_bf16(O.bf16_bits(bias))
    yf = B.w4a4_gemm_asym(*args, bias=bias_d, out_dtype=torch.float32).cpu().numpy()
    torch.cuda.synchronize()
    scale = np.abs(y32).max()
    assert np.abs(yf - y32).max() <= 2e-5 * scale


def test_prepared_blob_carries_the_code_sums():
    """dirotq_prepare_weights and dirotq_import_weights must produce the same zero-point term."""
    rng = np.random.default_rng(16)
    N, K, r, g, M = 96, 256, 32, 32, 40
    Q64, _ = np.linalg.qr(rng.standard_normal((K, K)))
    Q32 = Q64.astype(np.float32)
    W = (rng.standard_normal((N, K)) / np.sqrt(K) + 0.02).astype(np.float32)
    blob_p = B.prepare_weights(dev(W), dev(Q32), r, g)
    Wh2, qw2, sw2 = B.export_weights(blob_p, N, K, r, g)
    torch.cuda.synchronize()
    blob_i = B.import_weights(Wh2, qw2, sw2, N, K, r, g)
    G = (K - r) // g
    qx = rng.integers(0, 16, size=(M, K - r)).astype(np.uint8)
    sx = dev(np.ones((G, M), np.float16))
    zx = dev((rng.standard_normal((G, M)) * 3).astype(np.float16))
    xh = dev_bf16(O.bf16_bits(O.round_to_bf16(rng.standard_normal((M, r)).astype(np.float32))))
    ya = B.w4a4_gemm_asym(xh, dev(pack_u4(qx)), sx, zx, blob_p, M, N, K, r, g, out_dtype=torch.float32)
    yb = B.w4a4_gemm_asym(xh, dev(pack_u4(qx)), sx, zx, blob_i, M, N, K, r, g, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert torch.equal(ya, yb)


# ------------------------------------------------------------------ end to end
def check_codes_asym(xhat, qx_gpu, sx_gpu, zx_gpu, qx_ref, sx_ref, zx_ref, g, min_agree=0.999, band=1e-3, x=None,
                     Q=None, col0=0):
    """>= 99.9% of the codes equal the oracle's.  A group whose stored scale or zero-point differs must
    differ by one fp16 ulp, and only because the oracle's unrounded value (min, or (max - min) / 15) lies
    next to the fp16 rounding midpoint, closer than the fp32 accumulation noise of the min / max channels
    allows; every code is judged against the oracle's fp32 rotated value re-quantized with the GPU's stored
    (s, z), and may differ only within `band` steps of a rounding boundary."""
    M, C = qx_ref.shape
    G = C // g
    xg = xhat.reshape(M, G, g)
    worst = 0.0
    for a, b, what in ((sx_gpu, sx_ref, "scale"), (zx_gpu, zx_ref, "zero-point")):
        d = a.view(np.uint16) != b.view(np.uint16)
        if d.any():
            ulps = np.abs(a.view(np.int16).astype(np.int32) - b.view(np.int16).astype(np.int32))
            assert ulps[d].max() == 1, f"a {what} differs by more than one fp16 ulp"
            assert d.sum() <= max(2, 5e-3 * M * G), f"{int(d.sum())} {what} flips of {M * G}"
            if x is not None:
                mi, ji = np.nonzero(d)
                grp = xg[mi, ji]
                cmin, cmax = np.argmin(grp, axis=1), np.argmax(grp, axis=1)
                mn, mx = grp[np.arange(len(mi)), cmin], grp[np.arange(len(mi)), cmax]
                s_min = accumulation_slack(x[mi], Q, col0 + ji * g + cmin, x.shape[1])
                s_max = accumulation_slack(x[mi], Q, col0 + ji * g + cmax, x.shape[1])
                if what == "scale":
                    unrounded = ((mx - mn).astype(np.float32) / np.float32(15.0)).astype(np.float32)
                    slack = (s_min + s_max) / 15.0
                else:
                    unrounded, slack = mn, s_min
                worst = max(worst, check_flips_near_midpoint(unrounded, a[mi, ji], b[mi, ji], slack, f"activation {what}"))
    sf, zf = sx_gpu.astype(np.float32), zx_gpu.astype(np.float32)
    with np.errstate(divide="ignore"):
        inv = np.where(sf == 0, np.float32(0), (np.float32(1.0) / sf).astype(np.float32))
    t = ((xg - zf[..., None]).astype(np.float32) * inv[..., None]).astype(np.float32)
    want = np.clip(np.rint(t), 0, 15).astype(np.uint8).reshape(M, C)
    diff = qx_gpu != want
    if diff.any():
        tt = t.reshape(M, C)[diff].astype(np.float64)
        frac = np.abs(tt - np.floor(tt) - 0.5)
        assert np.all(frac <= band), f"code flip {frac.max():.3g} steps away from a boundary"
        assert np.all(np.abs(qx_gpu[diff].astype(np.int32) - want[diff]) == 1)
    agree = float((qx_gpu == qx_ref).mean())
    assert agree >= min_agree, f"only {agree:.5f} of the codes agree with the oracle"
    return dict(agree=agree, code_flips=int(diff.sum()), worst_flip_slack=worst)


def _end_to_end_asym(shape, y_rows=None):
    """Every token through rotation + asymmetric quantization against the oracle; the output of the fused
    layer (and the GEMM on identical inputs) on `y_rows` (default: every token)."""
    L, x, Q, xhat = oracle_rotation(shape)
    K, N, r, g = shape.K, shape.N, shape.r, shape.g
    Mx = x.shape[0]
    Wh, qw, sw = O.split_quantize_weights(oracle_fused_weights(shape), r, g)
    xh_r, qx_r, sx_r, zx_r = O.split_quantize_asym(xhat, r, g)
    sel = slice(None) if y_rows is None else np.asarray(y_rows)
    Qt = B.prepare_rotation(dev(L.Q32))
    blob = import_blob(Wh, qw, sw, N, K, r, g)
    (xh_d, xl_d, sx_d, zx_d), (xh_g, qx_g, sx_g, zx_g) = gpu_rq_asym(L.x_bits, Qt, r, g)
    stats = check_codes_asym(xhat[:, r:], qx_g, sx_g, zx_g, qx_r, sx_r, zx_r, g, x=x, Q=Q, col0=r)
    # GEMM on the GPU's own intermediates against the oracle's combine of the same
    y32_same, _ = O.combine_asym(xh_g[sel], qx_g[sel], sx_g[sel], zx_g[sel], Wh, qw, sw, g)
    yf = B.w4a4_gemm_asym(xh_d if r else None, xl_d, sx_d, zx_d, blob, Mx, N, K, r, g, out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert np.abs(yf.cpu().numpy()[sel] - y32_same).max() <= 2e-5 * np.abs(y32_same).max()
    del yf
    # the fused entry point against the oracle end to end
    y32, _ = O.combine_asym(xh_r[sel], qx_r[sel], sx_r[sel], zx_r[sel], Wh, qw, sw, g)
    y = B.linear_asym(dev_bf16(L.x_bits), Qt, blob, N, r, g)
    torch.cuda.synchronize()
    row_err, max_err = check_output(O.from_bf16_bits(host_bf16_bits(y))[sel], y32, tol=1e-2)
    y2 = B.w4a4_gemm_asym(xh_d if r else None, xl_d, sx_d, zx_d, blob, Mx, N, K, r, g, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    _say(f"{shape.name} asym: {Mx} tokens, codes agree {stats['agree']:.6f}, code flips {stats['code_flips']}, worst "
         f"scale / zero-point flip at {stats['worst_flip_slack']:.2f} of the allowed distance, "
         f"out row-rel {row_err:.2e} max-rel {max_err:.2e}")


def test_end_to_end_asym_small_and_ragged():
    _end_to_end_asym(I.SMALL)
    _end_to_end_asym(I.LayerShape("ragged_a", 333, 384, 200, 0, 32, 4, 7, 0))
    _end_to_end_asym(I.LayerShape("ragged128_a", 141, 640, 264, 128, 128, 4, 7, 1))


@pytest.mark.parametrize("idx", range(4))
def test_end_to_end_asym_flux_layers_full_launch_every_token(idx):
    # the four FLUX-shaped layers in the launch configuration bench.py --asym times (kernel B: the wave-specialised
    # schedule with its zero-point stages); every token quantized and compared, the output on every 8th token
    shp = I.FLUX[idx]
    _end_to_end_asym(shp, y_rows=np.arange(0, shp.M, 8))


def test_asym_rank_equals_K_and_empty():
    shp = I.LayerShape("allhigh_a", 150, 256, 96, 256, 32, 4, 7, 2)
    L = I.make_layer(shp)
    x, Q = I.bf16_bits_to_f32(L.x_bits), I.bf16_bits_to_f32(L.Q_bits)
    Wh, qw, sw = O.prepare_weights(L.W, L.Q32, shp.r, shp.g)
    ref = O.linear_asym(x, Q, Wh, qw, sw, shp.r, shp.g)
    Qt = B.prepare_rotation(dev(L.Q32))
    blob = import_blob(Wh, qw, sw, shp.N, shp.K, shp.r, shp.g)
    y = B.linear_asym(dev_bf16(L.x_bits), Qt, blob, shp.N, shp.r, shp.g)
    torch.cuda.synchronize()
    check_output(O.from_bf16_bits(host_bf16_bits(y)), ref["y32"], tol=1e-2)
    y0 = B.linear_asym(dev_bf16(L.x_bits)[:0], Qt, blob, shp.N, shp.r, shp.g)
    assert y0.shape == (0, shp.N)
