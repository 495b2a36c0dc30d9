"""GPU parity: the HIP path (through the C-ABI) against the CPU oracle on the same
seeded inputs.  Integer / byte / index results are compared bit for bit; floating
point within tolerances stated at each test."""
import numpy as np
import pytest
import torch

from oracle import dirotq_oracle as O
from paper_2605_16732_amd import binding as B
from paper_2605_16732_amd import inputs as I

from gpu_util import (pack_codes, unpack_codes, check_codes_statistical, check_output, check_xh, dev, dev_bf16,
                      gpu_rotate_quantize, host_bf16_bits, host_f16, import_blob, layer_with_oracle, oracle_rotation,
                      oracle_fused_weights)

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[case] {msg}", flush=True)


# ------------------------------------------------------------------ offline side
def test_prepare_rotation_is_bf16_transpose():
    rng = np.random.default_rng(0)
    K = 160
    Q = rng.standard_normal((K, K)).astype(np.float32)
    Qt = B.prepare_rotation(dev(Q))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(host_bf16_bits(Qt), O.bf16_bits(O.round_to_bf16(Q.T)))


@pytest.mark.parametrize("N,K,r,g", [(70, 128, 32, 32), (129, 256, 0, 64), (64, 256, 128, 128), (33, 96, 96, 32)])
def test_import_export_roundtrip(N, K, r, g):
    _say(f"import/export N={N} K={K} r={r} g={g}")
    rng = np.random.default_rng(1)
    G = (K - r) // g
    Wh = O.round_to_bf16(rng.standard_normal((N, r)).astype(np.float32))
    qw = rng.integers(-7, 8, size=(N, K - r)).astype(np.int8)
    sw = rng.lognormal(-3, 1, size=(N, G)).astype(np.float16)
    blob = import_blob(Wh, qw, sw, N, K, r, g)
    Wh2, qw2, sw2 = B.export_weights(blob, N, K, r, g)
    torch.cuda.synchronize()
    if r:
        np.testing.assert_array_equal(host_bf16_bits(Wh2), O.bf16_bits(Wh))
    if r < K:
        np.testing.assert_array_equal(qw2.cpu().numpy(), qw)
        np.testing.assert_array_equal(host_f16(sw2).view(np.uint16), sw.view(np.uint16))


@pytest.mark.parametrize("N,K,r,g", [(100, 256, 32, 32), (192, 1152, 64, 64), (65, 384, 0, 128)])
def test_prepare_weights_matches_oracle(N, K, r, g):
    """W' = W Q in fp64 on both sides: stored scales, codes and the bf16 part agree bit
    for bit except where an fp64 sum lands within rounding noise of an fp32 tie (allow
    1e-5 of the elements, each off by one code / one bf16 ulp)."""
    _say(f"prepare_weights N={N} K={K} r={r} g={g}")
    rng = np.random.default_rng(2)
    Q64, _ = np.linalg.qr(rng.standard_normal((K, K)))
    Q32 = Q64.astype(np.float32)
    W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    Wh, qw, sw = O.prepare_weights(W, Q32, r, g)
    blob = B.prepare_weights(dev(W), dev(Q32), r, g)
    Wh2, qw2, sw2 = B.export_weights(blob, N, K, r, g)
    torch.cuda.synchronize()
    if r:
        a, b = host_bf16_bits(Wh2).astype(np.int32), O.bf16_bits(Wh).astype(np.int32)
        assert np.abs(a - b).max() <= 1 and (a != b).mean() <= 1e-5
    if r < K:
        q2 = qw2.cpu().numpy()
        assert (q2 != qw).mean() <= 1e-5 and np.abs(q2.astype(np.int32) - qw).max() <= 1
        assert (host_f16(sw2).view(np.uint16) != sw.view(np.uint16)).mean() <= 1e-4


# ------------------------------------------------------------------ kernel A, exact
def _signed_perm(K, seed):
    rng = np.random.default_rng(seed)
    Q = np.zeros((K, K), np.float32)
    Q[rng.permutation(K), np.arange(K)] = rng.choice([-1.0, 1.0], size=K)
    return Q


@pytest.mark.parametrize("M,K,r,g,perm", [
    (300, 256, 64, 64, False), (300, 256, 32, 32, True), (129, 384, 0, 128, True),
    (1, 128, 32, 32, False), (257, 1152, 64, 64, True), (64, 96, 96, 32, True), (130, 448, 64, 128, True),
])
def test_rotate_quantize_exact_with_permutation_basis(M, K, r, g, perm):
    """With Q a (signed) permutation the rotation is exact in any summation order, so
    bf16 part, codes and scales must equal the oracle's bit for bit."""
    _say(f"rotate_quantize exact M={M} K={K} r={r} g={g} perm={perm}")
    rng = np.random.default_rng(3)
    Q = _signed_perm(K, 5) if perm else np.eye(K, dtype=np.float32)
    x = O.round_to_bf16((rng.standard_normal((M, K)) * rng.lognormal(0, 1.5, size=(1, K))).astype(np.float32))
    x[M // 2, :] = 0.0                                   # an all-zero token: scale 0, codes 0
    x[0, :32] = O.round_to_bf16(np.float32(2.0 ** -26) * rng.integers(-9, 10, 32).astype(np.float32))
    Qt = B.prepare_rotation(dev(Q))
    xh_r, qx_r, sx_r = O.rotate_quantize(x, Q, r, g)
    _, (xh_g, qx_g, sx_g) = gpu_rotate_quantize(O.bf16_bits(x), Qt, r, g)
    np.testing.assert_array_equal(xh_g, xh_r)
    np.testing.assert_array_equal(sx_g.view(np.uint16), sx_r.view(np.uint16))
    np.testing.assert_array_equal(qx_g, qx_r)


def test_rotate_quantize_ties_and_clip():
    """Hand-built rows: ties at .5 (round half to even), a negative absmax, a scale
    that is an fp16 subnormal so that the top code clips."""
    K, r, g = 64, 0, 32
    x = np.zeros((4, K), np.float32)
    x[0, :4] = [7, -3.5, 0.5, 1.5]
    x[0, 32:36] = [2.5, -2.5, 3.5, -7]
    x[1, :4] = [14, 1, -3, 5]
    x[1, 32:36] = [-3.5, 3.25, 0.25, -0.75]
    x[2, :3] = np.array([9.75, -1.375, 1.0], np.float32) * np.float32(2.0 ** -24)   # amax/7 ~ 1.39 * 2^-24
    x[3, :2] = [7 * 2.0 ** -25, 2.0 ** -26]                                          # scale ties down to 0
    assert np.array_equal(O.round_to_bf16(x), x)
    Qt = B.prepare_rotation(dev(np.eye(K, dtype=np.float32)))
    _, qx_r, sx_r = O.rotate_quantize(x, np.eye(K, dtype=np.float32), r, g)
    _, (_, qx_g, sx_g) = gpu_rotate_quantize(O.bf16_bits(x), Qt, r, g)
    assert list(qx_r[0, :4]) == [7, -4, 0, 2] and list(qx_r[0, 32:36]) == [2, -2, 4, -7]
    assert list(qx_r[2, :3]) == [7, -1, 1] and int(sx_r.view(np.uint16)[2, 0]) == 1
    assert not qx_r[3].any() and int(sx_r.view(np.uint16)[3, 0]) == 0
    np.testing.assert_array_equal(sx_g.view(np.uint16), sx_r.view(np.uint16))
    np.testing.assert_array_equal(qx_g, qx_r)


# ------------------------------------------------------------------ kernel B, exact
@pytest.fixture(params=["tile", "ws", "skinny"])
def schedule(request, monkeypatch):
    """Kernel B has three schedules of the same arithmetic (128 x 128 tiles, two workgroups per CU; persistent
    wave-specialised workgroups on 256 x 128 tiles; 64 x 64 outputs per workgroup with the K axis split over its
    waves, for few tokens); the library picks by problem size.  The environment switch read at every launch
    forces one, so that all of them run on the same inputs."""
    monkeypatch.setenv("DIROTQ_W4A4_KERNEL", request.param)
    return request.param


@pytest.mark.parametrize("M,N,K,g", [(130, 200, 256, 32), (257, 136, 448, 64), (64, 129, 384, 128), (5, 8, 64, 32),
                                     (140, 520, 96, 32)])
def test_w4a4_integer_dot_is_exact(M, N, K, g, schedule):
    """Unit scales, no 16-bit branch: the fp32 output is the plain integer dot product
    (< 2^24), so it must be exact -- the int32 group accumulators are bit-exact."""
    _say(f"w4a4 integer M={M} N={N} K={K} g={g}")
    rng = np.random.default_rng(4)
    G = K // g
    qx = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    qw = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    qx[0, :] = 7
    qw[0, :] = -7                                         # extreme: I = -49 g per group
    blob = import_blob(np.zeros((N, 0), np.float32), qw, np.ones((N, G), np.float16), N, K, 0, g)
    xl = dev(pack_codes(qx))
    sx = dev(np.ones((G, M), np.float16))
    y = B.w4a4_gemm(None, xl, sx, blob, M, N, K, 0, g, out_dtype=torch.float32)
    torch.cuda.synchronize()
    want = (qx.astype(np.int64) @ qw.astype(np.int64).T).astype(np.float32)
    np.testing.assert_array_equal(y.cpu().numpy(), want)
    assert want[0, 0] == -49 * K


def test_w4a4_power_of_two_scales_exact(schedule):
    """Power-of-two scales keep every product and partial sum exact in fp32."""
    rng = np.random.default_rng(6)
    M, N, K, g = 96, 72, 256, 64
    G = K // g
    qx = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    qw = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    sx = (2.0 ** rng.integers(-3, 3, size=(M, G))).astype(np.float16)
    sw = (2.0 ** rng.integers(-4, 2, size=(N, G))).astype(np.float16)
    blob = import_blob(np.zeros((N, 0), np.float32), qw, sw, N, K, 0, g)
    y = B.w4a4_gemm(None, dev(pack_codes(qx)), dev(np.ascontiguousarray(sx.T)), blob, M, N, K, 0, g,
                    out_dtype=torch.float32)
    torch.cuda.synchronize()
    want, _ = O.combine(np.zeros((M, 0), np.float32), qx, sx, np.zeros((N, 0), np.float32), qw, sw, g)
    np.testing.assert_array_equal(y.cpu().numpy(), want)


@pytest.mark.parametrize("M,N,K,r,g,use_bias", [
    (200, 136, 320, 64, 64, True), (130, 129, 288, 32, 32, False), (64, 64, 256, 128, 128, True),
    (77, 40, 128, 128, 32, False), (300, 264, 1152, 64, 64, False), (150, 300, 416, 32, 128, True),
    (260, 515, 224, 96, 32, True),
])
def test_w4a4_gemm_matches_oracle_on_identical_inputs(M, N, K, r, g, use_bias, schedule):
    """Same x_h, codes, scales and weights on both sides.  fp32 accumulation of at most
    G + r/16 partial terms against a float64 sum: 1e-5 of the largest output magnitude
    per element is ample (observed ~1e-6); bf16 output equals the rounded fp32 output
    except where the fp32 values straddle a bf16 tie (allow one bf16 ulp)."""
    _say(f"w4a4 vs oracle M={M} N={N} K={K} r={r} g={g} bias={use_bias}")
    rng = np.random.default_rng(7)
    G = (K - r) // g
    xh = O.round_to_bf16(rng.standard_normal((M, r)).astype(np.float32) * 20)
    Wh = O.round_to_bf16(rng.standard_normal((N, r)).astype(np.float32) * 0.05)
    qx = rng.integers(-7, 8, size=(M, K - r)).astype(np.int8)
    qw = rng.integers(-7, 8, size=(N, K - r)).astype(np.int8)
    sx = rng.lognormal(-1, 1, size=(M, G)).astype(np.float16)
    sw = rng.lognormal(-5, 1, size=(N, G)).astype(np.float16)
    bias = O.round_to_bf16(rng.standard_normal(N).astype(np.float32)) if use_bias else None
    y32, ybf = O.combine(xh, qx, sx, Wh, qw, sw, g, bias)
    blob = import_blob(Wh, qw, sw, N, K, r, g)
    args = (dev_bf16(O.bf16_bits(xh)) if r else None, dev(pack_codes(qx)) if r < K else None,
            dev(np.ascontiguousarray(sx.T)) if r < K else None, blob, M, N, K, r, g)
    bias_d = dev_bf16(O.bf16_bits(bias)) if use_bias else None
    yf = B.w4a4_gemm(*args, bias=bias_d, out_dtype=torch.float32).cpu().numpy()
    yb = B.w4a4_gemm(*args, bias=bias_d, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    scale = np.abs(y32).max()
    assert np.abs(yf - y32).max() <= 1e-5 * scale
    a = host_bf16_bits(yb).astype(np.int32)
    np.testing.assert_array_equal(a, O.bf16_bits(O.round_to_bf16(yf)).astype(np.int32))   # own rounding is RNE
    assert np.abs(O.from_bf16_bits(host_bf16_bits(yb)) - ybf).max() <= 2.0 ** -7 * scale


def test_w4a4_persistent_workgroups_take_several_tiles(monkeypatch):
    """300 tiles of 256 x 128 on 256 CUs: some workgroups of the persistent schedule run two tiles back to back
    (the stage stream crosses the tile boundary).  Ragged in both directions; a rank-32 branch, so the 16-bit
    phase has padding stages."""
    monkeypatch.setenv("DIROTQ_W4A4_KERNEL", "ws")
    M, N, K, r, g = 2500, 3592, 224, 32, 64
    _say(f"w4a4 persistent M={M} N={N} K={K} r={r} g={g}")
    rng = np.random.default_rng(11)
    G = (K - r) // g
    xh = O.round_to_bf16(rng.standard_normal((M, r)).astype(np.float32) * 20)
    Wh = O.round_to_bf16(rng.standard_normal((N, r)).astype(np.float32) * 0.05)
    qx = rng.integers(-7, 8, size=(M, K - r)).astype(np.int8)
    qw = rng.integers(-7, 8, size=(N, K - r)).astype(np.int8)
    sx = rng.lognormal(-1, 1, size=(M, G)).astype(np.float16)
    sw = rng.lognormal(-5, 1, size=(N, G)).astype(np.float16)
    bias = O.round_to_bf16(rng.standard_normal(N).astype(np.float32))
    y32, ybf = O.combine(xh, qx, sx, Wh, qw, sw, g, bias)
    blob = import_blob(Wh, qw, sw, N, K, r, g)
    args = (dev_bf16(O.bf16_bits(xh)), dev(pack_codes(qx)), dev(np.ascontiguousarray(sx.T)), blob, M, N, K, r, g)
    bias_d = dev_bf16(O.bf16_bits(bias))
    yf = B.w4a4_gemm(*args, bias=bias_d, out_dtype=torch.float32).cpu().numpy()
    yb = B.w4a4_gemm(*args, bias=bias_d, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    scale = np.abs(y32).max()
    assert np.abs(yf - y32).max() <= 1e-5 * scale
    np.testing.assert_array_equal(host_bf16_bits(yb).astype(np.int32),
                                  O.bf16_bits(O.round_to_bf16(yf)).astype(np.int32))


# ------------------------------------------------------------------ end to end
def _end_to_end(shape, M=None, y_rows=None, residual_rotation=False, same_rows=None, blob_from="import", base=None):
    """Rotation + quantization of EVERY token against the oracle (codes, scales, bf16 part), then the
    fused layer's output against the oracle's on `y_rows` (default: every token).  `same_rows` (default:
    y_rows) are the tokens on which the GEMM is also checked on identical inputs.  `base` names the layer
    whose draws are used (shapes that differ only in r and g share them)."""
    draws = shape if base is None else base
    L, x, Q, xhat = oracle_rotation(draws, M, residual_rotation)
    Wp = oracle_fused_weights(draws, M, residual_rotation)
    Mx, K, N, r, g = L.x_bits.shape[0], shape.K, shape.N, shape.r, shape.g
    Wh, qw, sw = O.split_quantize_weights(Wp, r, g)
    xh_r, qx_r, sx_r = O.split_quantize(xhat, r, g)
    Qt = B.prepare_rotation(dev(L.Q32))
    np.testing.assert_array_equal(host_bf16_bits(Qt), np.ascontiguousarray(L.Q_bits.T))
    if blob_from == "import":
        blob = import_blob(Wh, qw, sw, N, K, r, g)
    else:                                        # the library's own offline fusion (fp64 on both sides)
        blob = B.prepare_weights(dev(L.W), dev(L.Q32), r, g)
    # stage 1: rotation + quantization of every token against the oracle's
    (xh_d, xl_d, sx_d), (xh_g, qx_g, sx_g) = gpu_rotate_quantize(L.x_bits, Qt, r, g)
    stats = dict(agree=1.0, code_flips=0, scale_flips=0, groups=0, worst_flip_slack=0.0)
    if r < K:
        stats = check_codes_statistical(xhat[:, r:], qx_g, sx_g, qx_r, sx_r, g, x=x, Q=Q, col0=r)
    xh_frac = check_xh(xh_g, xh_r, x, K) if r else 0.0
    # stage 2: GEMM on the GPU's own intermediates against the oracle's combine of the same
    sel = slice(None) if y_rows is None else np.asarray(y_rows)
    ssel = sel if same_rows is None else np.asarray(same_rows)
    yf = B.w4a4_gemm(xh_d if r else None, xl_d, sx_d, blob, Mx, N, K, r, g, out_dtype=torch.float32)
    torch.cuda.synchronize()
    if blob_from == "import":
        y32_same, _ = O.combine(xh_g[ssel], qx_g[ssel], sx_g[ssel], Wh, qw, sw, g)
        assert np.abs(yf.cpu().numpy()[ssel] - y32_same).max() <= 1e-5 * np.abs(y32_same).max()
    del yf
    # the fused entry point, bf16 out, against the oracle end to end
    y32, _ = O.combine(xh_r[sel], qx_r[sel], sx_r[sel], Wh, qw, sw, g)
    y = B.linear(dev_bf16(L.x_bits), Qt, blob, N, r, g)
    torch.cuda.synchronize()
    yg = O.from_bf16_bits(host_bf16_bits(y))
    row_err, max_err = check_output(yg[sel], y32, tol=1e-2)
    # and it is exactly the two-step path
    y2 = B.w4a4_gemm(xh_d if r else None, xl_d, sx_d, blob, Mx, N, K, r, g, out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    n_y = Mx if y_rows is None else len(y_rows)
    _say(f"{shape.name}: {Mx} tokens, codes agree {stats['agree']:.6f}, code flips {stats['code_flips']}, scale flips "
         f"{stats['scale_flips']}/{stats['groups']} (worst {stats['worst_flip_slack']:.2f} of the allowed distance), "
         f"bf16 part differs on {xh_frac:.4f}, out ({n_y} tokens) row-rel {row_err:.2e} max-rel {max_err:.2e}")
    return stats


def test_end_to_end_small_config():
    _end_to_end(I.SMALL)


def test_end_to_end_small_config_with_library_prepared_weights():
    # configs[0] with the blob from dirotq_prepare_weights (W Q in fp64 on the GPU) instead of the oracle's
    _end_to_end(I.SMALL, blob_from="prepare")


def test_end_to_end_ragged_tokens_and_outputs():
    # ragged M (several tiles + tail) and N not a multiple of the tile, r = 0 and g = 32
    shp = I.LayerShape("ragged", 333, 384, 200, 0, 32, 4, 7, 0)
    _end_to_end(shp)
    shp = I.LayerShape("ragged128", 141, 640, 264, 128, 128, 4, 7, 1)
    _end_to_end(shp)


def _random_shapes(n, seed):
    """Seeded draw of layer shapes that straddle the launchers' decisions: token counts on both sides of every
    tile size, K with and without the factors 64 and 128 (stage length, the small launch's split of K), every
    group size, r from 0 up, N off the tile grid."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < n:
        g = int(rng.choice([32, 64, 128]))
        K = 32 * int(rng.integers(2, 29))                      # 64 .. 896
        r_choices = [r for r in range(0, K, 32) if (K - r) % g == 0]
        if not r_choices:
            continue
        r = int(rng.choice(r_choices))
        M = int(rng.choice([1, 31, 33, 63, 65, 127, 129, 200, 257, 300, 513, 640]))
        N = int(rng.integers(8, 700))
        out.append(I.LayerShape(f"rand{len(out)}_M{M}_K{K}_N{N}_r{r}_g{g}", M, K, N, r, g, 3, 9, len(out)))
    return out


@pytest.mark.parametrize("shp", _random_shapes(16, 20260516), ids=lambda s: s.name)
def test_end_to_end_random_shapes(shp):
    _end_to_end(shp)


def _every(M, step):
    return np.arange(0, M, step)


@pytest.mark.parametrize("idx", range(4))
def test_end_to_end_pixart_layers_every_token(idx):
    # the four PixArt-shaped layers at full size (M = 4096): every token through rotation, quantization and
    # the fused layer; the identical-input GEMM check on every 8th token
    shp = I.PIXART[idx]
    _end_to_end(shp, same_rows=_every(shp.M, 8))


@pytest.mark.parametrize("idx", range(4))
def test_end_to_end_flux_layers_every_token(idx):
    # the launch configurations bench.py times (M = 4608; QKV, out-projection, fc1 with K = 3072, fc2 with
    # K = 12288: two rotation launches, 190 groups): every token against the oracle
    shp = I.FLUX[idx]
    _end_to_end(shp, same_rows=_every(shp.M, 8))


@pytest.mark.parametrize("M", [1024, 16384, 16461, 32768])
def test_end_to_end_token_sweep(M):
    # the token sweep on the PixArt fc1 shape; 16384 and 32768 tokens take the two-launch rotation (full rounds
    # of 256 x 256 tiles, then half-size tiles) with the short-K threshold.  Every token is quantized and
    # compared; the output is compared on every 4th token.
    # (16461 is not a benchmark size: a token count off every tile size whose second launch starts mid-way.)
    named = [s for s in I.TOKEN_SWEEP if s.M == M]
    shp = named[0] if named else I.LayerShape(f"pixart_fc1_M{M}", M, 1152, 4608, 64, 64, 8, 3, 9)
    _end_to_end(shp, y_rows=_every(M, 4) if M > 4096 else None, same_rows=_every(M, 16))


@pytest.mark.parametrize("r,g", [(s.r, s.g) for s in I.ABLATION])
def test_end_to_end_rank_group_ablation_full_shape(r, g):
    # the 12 (r, g) pairs of the rank/group ablation at the full fc2 shape (M = 4608, K = 12288, N = 3072), on
    # the draws of the FLUX fc2 layer (as bench.py does): one oracle rotation and one fused weight matrix serve
    # all pairs.  Codes, scales and the bf16 part of every token; the output on every 8th token.
    shp = [s for s in I.ABLATION if (s.r, s.g) == (r, g)][0]
    _end_to_end(shp, y_rows=_every(shp.M, 8), same_rows=_every(shp.M, 32), base=I.FLUX[3])


@pytest.mark.parametrize("r,g", [(0, 32), (32, 32), (0, 128), (256, 128), (256, 64)])
def test_end_to_end_rank_group_grid(r, g):
    # (r, g) pairs on a reduced fc2-like shape with a ragged M
    shp = I.LayerShape(f"abl_r{r}_g{g}", 200, 1536, 384, r, g, 8, 8, r * 4 + g)
    _end_to_end(shp)


def test_end_to_end_with_residual_rotation():
    """Q = [U_h, U_l R] with a random orthogonal R on the 4-bit subspace (Section 4.2): a data
    variant of the same kernels.  R equalises the 4-bit channels, so the oracle's own error
    against the unquantized product must not get worse."""
    shp = I.LayerShape("resrot", 384, 768, 512, 64, 64, 8, 8, 77)
    _end_to_end(shp, residual_rotation=True)
    errs = {}
    for rr in (False, True):
        L, (Wh, qw, sw), ref = layer_with_oracle(shp, residual_rotation=rr)
        x = I.bf16_bits_to_f32(L.x_bits).astype(np.float64)
        errs[rr] = O.qsnr_db(x @ L.W.astype(np.float64).T, ref["y32"])
    _say(f"QSNR vs unquantized product: PCA only {errs[False]:.2f} dB, PCA + R {errs[True]:.2f} dB")
    assert errs[True] > errs[False] - 0.5


def test_rank_equals_K_is_a_bf16_gemm():
    shp = I.LayerShape("allhigh", 150, 256, 96, 256, 32, 4, 7, 2)
    L, (Wh, qw, sw), ref = layer_with_oracle(shp)
    Qt = B.prepare_rotation(dev(L.Q32))
    blob = import_blob(Wh, qw, sw, shp.N, shp.K, shp.r, shp.g)
    y = B.linear(dev_bf16(L.x_bits), Qt, blob, shp.N, shp.r, shp.g)
    torch.cuda.synchronize()
    check_output(O.from_bf16_bits(host_bf16_bits(y)), ref["y32"], tol=1e-2)


def test_deterministic_and_empty():
    L, (Wh, qw, sw), _ = layer_with_oracle(I.SMALL)
    shp = I.SMALL
    Qt = B.prepare_rotation(dev(L.Q32))
    blob = import_blob(Wh, qw, sw, shp.N, shp.K, shp.r, shp.g)
    x = dev_bf16(L.x_bits)
    y1 = B.linear(x, Qt, blob, shp.N, shp.r, shp.g)
    y2 = B.linear(x, Qt, blob, shp.N, shp.r, shp.g)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    y0 = B.linear(x[:0], Qt, blob, shp.N, shp.r, shp.g)          # M == 0: a no-op
    assert y0.shape == (0, shp.N)
    # out-of-bounds canary: outputs sit inside a larger buffer that must stay untouched
    M = 100
    big = torch.full((M + 2, shp.N), 1.0, dtype=torch.bfloat16, device="cuda")
    B.linear(x[:M], Qt, blob, shp.N, shp.r, shp.g, out=big[1:M + 1])
    torch.cuda.synchronize()
    assert torch.all(big[0] == 1.0) and torch.all(big[M + 1] == 1.0)
    assert torch.equal(big[1:M + 1], y1[:M])


def test_shared_input_layers_equal_separate_calls():
    """dirotq_linear_shared = one rotation + quantization feeding several GEMMs: bit-identical to
    separate dirotq_linear calls (and therefore within the oracle's tolerance like them)."""
    shp = I.LayerShape("shared", 300, 512, 0, 64, 64, 8, 8, 5)
    rng = np.random.default_rng(31)
    Ns = [192, 333, 64]
    L = I.make_layer(I.LayerShape("shared", 300, 512, max(Ns), 64, 64, 8, 8, 5))
    Qt = B.prepare_rotation(dev(L.Q32))
    x = dev_bf16(L.x_bits)
    blobs, biases, refs = [], [], []
    for N in Ns:
        W = (rng.standard_normal((N, shp.K)) / np.sqrt(shp.K)).astype(np.float32)
        Wh, qw, sw = O.prepare_weights(W, L.Q32, shp.r, shp.g)
        bias = O.round_to_bf16(rng.standard_normal(N).astype(np.float32))
        blobs.append(import_blob(Wh, qw, sw, N, shp.K, shp.r, shp.g))
        biases.append(dev_bf16(O.bf16_bits(bias)))
        refs.append(O.linear(I.bf16_bits_to_f32(L.x_bits), I.bf16_bits_to_f32(L.Q_bits), Wh, qw, sw, shp.r, shp.g, bias))
    ys = B.linear_shared(x, Qt, blobs, Ns, shp.r, shp.g, biases=biases)
    torch.cuda.synchronize()
    for N, blob, bias, y, ref in zip(Ns, blobs, biases, ys, refs):
        y1 = B.linear(x, Qt, blob, N, shp.r, shp.g, bias=bias)
        torch.cuda.synchronize()
        assert torch.equal(y, y1)
        check_output(O.from_bf16_bits(host_bf16_bits(y)), ref["y32"], tol=1e-2)
