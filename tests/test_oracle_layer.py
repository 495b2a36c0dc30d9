"""Pins for the oracle's layer arithmetic (CPU only): brute force in pure Python on
tiny shapes, the rotation identity of the paper, special cases that reduce to a
library GEMM, and planted mistakes that the pins must catch."""
import struct
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import dirotq_oracle as O


def _f32(x):
    return struct.unpack("f", struct.pack("f", x))[0]


def _f16(x):
    return struct.unpack("e", struct.pack("e", x))[0]


def _bf16(x):
    """Python-float bf16 rounding, ties to even, via the fp32 bit pattern."""
    u = struct.unpack("I", struct.pack("f", x))[0]
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return struct.unpack("f", struct.pack("I", u))[0]


def _quant(vals):
    amax = max(abs(v) for v in vals)
    sf = _f16(min(_f32(amax / 7.0), 65504.0))
    if sf == 0.0:
        return [0] * len(vals), 0.0
    inv = _f32(1.0 / sf)
    return [max(-7, min(7, round(_f32(v * inv)))) for v in vals], sf


def _brute_layer(x, Q, Q32, W, r, g, bias=None):
    """Whole layer with Python loops and exact rational sums.  x, Q: bf16-valued
    floats; Q32, W: fp32-valued floats.  Returns y32 as Fractions rounded to fp32."""
    M, K, N = len(x), len(x[0]), len(W)
    G = (K - r) // g
    # offline: W' = W Q32 (exact sum, one rounding to fp32), split, quantize
    Wp = [[_f32(float(sum(Fraction(W[n][k]) * Fraction(Q32[k][c]) for k in range(K))))
           for c in range(K)] for n in range(N)]
    Wh = [[_bf16(Wp[n][c]) for c in range(r)] for n in range(N)]
    qw, sw = [], []
    for n in range(N):
        cs, ss = [], []
        for j in range(G):
            c, s = _quant(Wp[n][r + j * g: r + (j + 1) * g])
            cs += c
            ss.append(s)
        qw.append(cs)
        sw.append(ss)
    y = []
    for m in range(M):
        xhat = [_f32(float(sum(Fraction(x[m][k]) * Fraction(Q[k][c]) for k in range(K))))
                for c in range(K)]
        xh = [_bf16(v) for v in xhat[:r]]
        qx, sx = [], []
        for j in range(G):
            c, s = _quant(xhat[r + j * g: r + (j + 1) * g])
            qx += c
            sx.append(s)
        row = []
        for n in range(N):
            acc = sum(Fraction(xh[k]) * Fraction(Wh[n][k]) for k in range(r))
            for j in range(G):
                I = sum(qx[j * g + k] * qw[n][j * g + k] for k in range(g))
                assert abs(I) <= 49 * g
                acc += Fraction(sx[j]) * Fraction(sw[n][j]) * I
            if bias is not None:
                acc += Fraction(bias[n])
            row.append(_f32(float(acc)))
        y.append(row)
    return np.array(y, np.float32)


def _tiny(seed, M, K, N):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((K, K))
    Q64, _ = np.linalg.qr(A)
    Q32 = Q64.astype(np.float32)
    Q = O.round_to_bf16(Q32)
    s = rng.lognormal(0, 0.5, K)
    s[rng.integers(0, K)] *= 80
    x = O.round_to_bf16((rng.standard_normal((M, K)) * s).astype(np.float32))
    W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    return x, Q, Q32, W


@pytest.mark.parametrize("M,K,N,r,g", [(3, 16, 5, 0, 4), (3, 16, 5, 4, 4), (2, 12, 4, 4, 8),
                                        (2, 8, 3, 8, 4), (4, 20, 3, 4, 16)])
def test_brute_force_tiny(M, K, N, r, g):
    x, Q, Q32, W = _tiny(100 + K + r, M, K, N)
    bias = np.linspace(-1, 1, N).astype(np.float32)
    want = _brute_layer(x.tolist(), Q.tolist(), Q32.tolist(), W.tolist(), r, g, bias.tolist())
    Wh, qw, sw = O.prepare_weights(W, Q32, r, g)
    got = O.linear(x, Q, Wh, qw, sw, r, g, bias)
    # float64 sums vs exact sums: at most one fp32 ulp apart after the final rounding
    np.testing.assert_allclose(got["y32"], want, rtol=2.0 ** -22, atol=1e-30)
    assert np.array_equal(got["y"], O.round_to_bf16(got["y32"]))


def test_group_int_dots_is_a_plain_integer_sum():
    rng = np.random.default_rng(3)
    qx = rng.integers(-7, 8, size=(3, 16)).astype(np.int8)
    qw = rng.integers(-7, 8, size=(5, 16)).astype(np.int8)
    I = O.group_int_dots(qx, qw, 4)
    assert I.shape == (3, 5, 4)
    for m in range(3):
        for n in range(5):
            for j in range(4):
                assert I[m, n, j] == sum(int(qx[m, 4 * j + k]) * int(qw[n, 4 * j + k]) for k in range(4))
    # unit scales and r = 0: the layer output is the plain integer dot product
    sx = np.ones((3, 4), np.float16)
    sw = np.ones((5, 4), np.float16)
    y32, _ = O.combine(np.zeros((3, 0), np.float32), qx, sx, np.zeros((5, 0), np.float32), qw, sw, 4)
    np.testing.assert_array_equal(y32, (qx.astype(np.int64) @ qw.astype(np.int64).T).astype(np.float32))
    # extreme codes: the bound |I| <= 49 g is attained
    a = np.full((1, 64), 7, np.int8)
    assert O.group_int_dots(a, -a, 64)[0, 0, 0] == -49 * 64


@pytest.mark.parametrize("r", [0, 5, 24, 48])
def test_rotation_identity_exact_mode(r):
    """X W = X V V^T W (the derivation before the forward-computation equation):
    with nothing rounded the split point does not matter."""
    rng = np.random.default_rng(7)
    K, M, N = 48, 9, 11
    Qm, _ = np.linalg.qr(rng.standard_normal((K, K)))
    x = rng.standard_normal((M, K)) * rng.lognormal(0, 1, K)
    W = rng.standard_normal((N, K))
    got = O.linear_exact(x, Qm, W, r)
    np.testing.assert_allclose(got, x @ W.T, rtol=1e-10, atol=1e-10)
    # a planted mistake (the rotation applied transposed on one side) breaks it
    bad = (x @ Qm.T) @ (W @ Qm).T
    assert np.abs(bad - x @ W.T).max() > 1e-2


def test_r_equals_K_is_a_bf16_gemm():
    """No INT4 part: the layer is bf16(xQ) times bf16(WQ) with wide accumulation --
    compare with torch.matmul on the same rounded operands."""
    rng = np.random.default_rng(21)
    M, K, N = 16, 64, 24
    x, Q, Q32, W = _tiny(21, M, K, N)
    Wh, qw, sw = O.prepare_weights(W, Q32, K, 32)
    out = O.linear(x, Q, Wh, qw, sw, K, 32)
    assert qw.shape == (N, 0) and out["qx"].shape == (M, 0)
    xh_t = (torch.from_numpy(x).double() @ torch.from_numpy(Q).double()).float().to(torch.bfloat16)
    Wp_t = (torch.from_numpy(W).double() @ torch.from_numpy(Q32).double()).float().to(torch.bfloat16)
    ref = (xh_t.double() @ Wp_t.double().T).float().numpy()
    np.testing.assert_allclose(out["y32"], ref, rtol=1e-6, atol=1e-6)
    # and it is close to the unrotated product (bf16 storage only)
    full = x.astype(np.float64) @ W.astype(np.float64).T
    assert np.abs(out["y32"] - full).max() / np.abs(full).max() < 2e-2


def test_identity_rotation_is_plain_group_rtn():
    """Q = I, r = 0: plain per-group round-to-nearest W4A4 -- dequantise both sides
    and multiply."""
    rng = np.random.default_rng(4)
    M, K, N, g = 6, 64, 7, 32
    x = O.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    W = rng.standard_normal((N, K)).astype(np.float32)
    I = np.eye(K, dtype=np.float32)
    Wh, qw, sw = O.prepare_weights(W, I, 0, g)
    out = O.linear(x, I, Wh, qw, sw, 0, g)
    np.testing.assert_array_equal(out["xhat"], x)
    qx, sx = O.quantize_groups(x, g)
    np.testing.assert_array_equal(out["qx"], qx)
    xd = O.dequantize_groups(qx, sx, g)
    qw2, sw2 = O.quantize_groups(W, g)
    wd = O.dequantize_groups(qw2, sw2, g)
    np.testing.assert_allclose(out["y32"], (xd @ wd.T).astype(np.float32), rtol=1e-6, atol=1e-7)


def test_single_group_is_per_token_per_channel_scaling():
    """g = K - r: one scale per token and one per output channel, so the scales
    factor out of the sum."""
    rng = np.random.default_rng(8)
    M, K, N = 5, 32, 6
    x, Q, Q32, W = _tiny(8, M, K, N)
    Wh, qw, sw = O.prepare_weights(W, Q32, 0, K)
    out = O.linear(x, Q, Wh, qw, sw, 0, K)
    I = out["qx"].astype(np.int64) @ qw.astype(np.int64).T
    ref = out["sx"].astype(np.float64) * sw.astype(np.float64).T * I
    np.testing.assert_allclose(out["y32"], ref.astype(np.float32), rtol=1e-6)


def test_rotate_orientation_and_split_order():
    """x_hat[m, c] = sum_k x[m, k] Q[k, c]: a permutation matrix Q with Q[k, c] = 1
    moves input channel k to rotated channel c; the first r rotated channels are the
    BF16 part."""
    K = 8
    perm = np.array([3, 0, 7, 1, 2, 6, 5, 4])
    Q = np.zeros((K, K), np.float32)
    Q[perm, np.arange(K)] = 1.0          # rotated channel c reads input channel perm[c]
    x = np.arange(1, K + 1, dtype=np.float32)[None, :] * np.array([[1.0], [-2.0]], np.float32)
    xhat = O.rotate(x, Q)
    np.testing.assert_array_equal(xhat, x[:, perm])
    xh, qx, sx = O.split_quantize(xhat, 2, 6)
    np.testing.assert_array_equal(xh, x[:, perm[:2]])
    assert qx.shape == (2, 6) and sx.shape == (2, 1)
    # codes of row 0: channels perm[2:] = 8,2,3,7,6,5 over scale 8/7
    s = float(np.float16(np.float32(8.0) / np.float32(7.0)))
    want = [max(-7, min(7, round(_f32(v * _f32(1.0 / s))))) for v in [8, 2, 3, 7, 6, 5]]
    assert list(qx[0]) == want and list(qx[1]) == [-w for w in want]


def test_quantization_error_trend_on_outlier_activations():
    """Sanity trend from the paper (not a number of the paper): keeping the top
    principal directions in BF16 helps, and more of them helps more; the PCA
    rotation beats no rotation on channel-outlier activations."""
    from paper_2605_16732_amd import inputs as I
    shp = I.LayerShape("t", 128, 256, 96, 32, 32, 4, 9, 0)
    L = I.make_layer(shp)
    x = I.bf16_bits_to_f32(L.x_bits)
    Q = I.bf16_bits_to_f32(L.Q_bits)
    ref = x.astype(np.float64) @ L.W.astype(np.float64).T
    q = {}
    for r in (0, 32, 64):
        Wh, qw, sw = O.prepare_weights(L.W, L.Q32, r, 32)
        q[r] = O.qsnr_db(ref, O.linear(x, Q, Wh, qw, sw, r, 32)["y32"])
    assert q[0] < q[32] < q[64]
    eye = np.eye(256, dtype=np.float32)
    Wh, qw, sw = O.prepare_weights(L.W, eye, 0, 32)
    plain = O.qsnr_db(ref, O.linear(x, eye, Wh, qw, sw, 0, 32)["y32"])
    assert q[32] > plain + 3.0


# ---------------------------------------------------------------------------
# asymmetric activations
# ---------------------------------------------------------------------------
def _quant_asym(vals):
    mn, mx = min(vals), max(vals)
    zf = _f16(max(-65504.0, min(65504.0, mn)))
    sf = _f16(min(_f32(_f32(mx - mn) / 15.0), 65504.0))
    if sf == 0.0:
        return [0] * len(vals), 0.0, zf
    inv = _f32(1.0 / sf)
    return [max(0, min(15, round(_f32(_f32(v - zf) * inv)))) for v in vals], sf, zf


def _brute_layer_asym(x, Q, Q32, W, r, g, bias=None):
    """The layer with asymmetric activations written as the quantizer equation says: every
    activation is replaced by its dequantised value q s + z, every weight by q_w s_w, and
    the products are summed exactly -- no zero-point algebra here."""
    M, K, N = len(x), len(x[0]), len(W)
    G = (K - r) // g
    Wp = [[_f32(float(sum(Fraction(W[n][k]) * Fraction(Q32[k][c]) for k in range(K))))
           for c in range(K)] for n in range(N)]
    Wh = [[_bf16(Wp[n][c]) for c in range(r)] for n in range(N)]
    wt = []                                  # dequantised 4-bit weights, exact
    for n in range(N):
        row = []
        for j in range(G):
            c, s = _quant(Wp[n][r + j * g: r + (j + 1) * g])
            row += [Fraction(ci) * Fraction(s) for ci in c]
        wt.append(row)
    y = []
    for m in range(M):
        xhat = [_f32(float(sum(Fraction(x[m][k]) * Fraction(Q[k][c]) for k in range(K))))
                for c in range(K)]
        xh = [_bf16(v) for v in xhat[:r]]
        xt = []
        for j in range(G):
            c, s, z = _quant_asym(xhat[r + j * g: r + (j + 1) * g])
            xt += [Fraction(ci) * Fraction(s) + Fraction(z) for ci in c]
        row = []
        for n in range(N):
            acc = sum(Fraction(xh[k]) * Fraction(Wh[n][k]) for k in range(r))
            acc += sum(xt[k] * wt[n][k] for k in range(K - r))
            if bias is not None:
                acc += Fraction(bias[n])
            row.append(_f32(float(acc)))
        y.append(row)
    return np.array(y, np.float32)


@pytest.mark.parametrize("M,K,N,r,g", [(3, 16, 5, 0, 4), (3, 16, 5, 4, 4), (2, 12, 4, 4, 8), (4, 20, 3, 4, 16)])
def test_asym_brute_force_tiny(M, K, N, r, g):
    x, Q, Q32, W = _tiny(200 + K + r, M, K, N)
    x = O.round_to_bf16(x + np.float32(1.5))          # shifted: the zero-points matter
    bias = np.linspace(-1, 1, N).astype(np.float32)
    want = _brute_layer_asym(x.tolist(), Q.tolist(), Q32.tolist(), W.tolist(), r, g, bias.tolist())
    Wh, qw, sw = O.prepare_weights(W, Q32, r, g)
    got = O.linear_asym(x, Q, Wh, qw, sw, r, g, bias)
    np.testing.assert_allclose(got["y32"], want, rtol=2.0 ** -22, atol=1e-30)
    assert got["qx"].dtype == np.uint8 and got["qx"].max() <= 15
    # the zero-point term is not small here: dropping it must be visible
    no_z, _ = O.combine_asym(got["xh"], got["qx"], got["sx"], np.zeros_like(got["zx"]), Wh, qw, sw, g, bias)
    assert np.abs(no_z - want).max() > 1e-3 * np.abs(want).max()


def test_asym_equals_symmetric_layer_on_dequantised_inputs():
    # combine_asym on (q, s, z) == a plain float64 GEMM of the dequantised operands
    rng = np.random.default_rng(8)
    M, N, C, g = 6, 5, 32, 8
    xhat = (rng.standard_normal((M, C)) * 3 + 2).astype(np.float32)
    Wp = rng.standard_normal((N, C)).astype(np.float32)
    qx, sx, zx = O.quantize_groups_asym(xhat, g)
    qw, sw = O.quantize_groups(Wp, g)
    y32, _ = O.combine_asym(np.zeros((M, 0), np.float32), qx, sx, zx, np.zeros((N, 0), np.float32), qw, sw, g)
    want = O.dequantize_groups_asym(qx, sx, zx, g) @ O.dequantize_groups(qw, sw, g).T
    np.testing.assert_allclose(y32, want.astype(np.float32), rtol=2.0 ** -22, atol=1e-30)


def test_asym_is_closer_than_symmetric_on_shifted_activations():
    # activations with a per-group offset: the asymmetric grid spends its 16 levels on the range actually used
    rng = np.random.default_rng(9)
    v = (rng.standard_normal((64, 128)) + 4.0).astype(np.float32)
    qs, ss = O.quantize_groups(v, 64)
    qa, sa, za = O.quantize_groups_asym(v, 64)
    err_sym = np.abs(O.dequantize_groups(qs, ss, 64) - v).mean()
    err_asym = np.abs(O.dequantize_groups_asym(qa, sa, za, 64) - v).mean()
    assert err_asym < 0.5 * err_sym


# ---------------------------------------------------------------------------
# W4A8: 8-bit per-token activations
# ---------------------------------------------------------------------------
def _quant8(vals):
    amax = max(abs(v) for v in vals)
    sf = _f16(min(_f32(amax / 127.0), 65504.0))
    if sf == 0.0:
        return [0] * len(vals), 0.0
    inv = _f32(1.0 / sf)
    return [max(-127, min(127, round(_f32(v * inv)))) for v in vals], sf


def _brute_layer_a8(x, Q, Q32, W, r, g, bias=None):
    """Every activation replaced by q8 * s_token, every weight by q4 * s_group, exact sums."""
    M, K, N = len(x), len(x[0]), len(W)
    G = (K - r) // g
    Wp = [[_f32(float(sum(Fraction(W[n][k]) * Fraction(Q32[k][c]) for k in range(K))))
           for c in range(K)] for n in range(N)]
    Wh = [[_bf16(Wp[n][c]) for c in range(r)] for n in range(N)]
    wt = []
    for n in range(N):
        row = []
        for j in range(G):
            c, s = _quant(Wp[n][r + j * g: r + (j + 1) * g])
            row += [Fraction(ci) * Fraction(s) for ci in c]
        wt.append(row)
    y = []
    for m in range(M):
        xhat = [_f32(float(sum(Fraction(x[m][k]) * Fraction(Q[k][c]) for k in range(K))))
                for c in range(K)]
        xh = [_bf16(v) for v in xhat[:r]]
        c8, s8 = _quant8(xhat[r:]) if K > r else ([], 0.0)
        xt = [Fraction(ci) * Fraction(s8) for ci in c8]
        row = []
        for n in range(N):
            acc = sum(Fraction(xh[k]) * Fraction(Wh[n][k]) for k in range(r))
            acc += sum(xt[k] * wt[n][k] for k in range(K - r))
            if bias is not None:
                acc += Fraction(bias[n])
            row.append(_f32(float(acc)))
        y.append(row)
    return np.array(y, np.float32)


@pytest.mark.parametrize("M,K,N,r,g", [(3, 16, 5, 0, 4), (3, 16, 5, 4, 4), (2, 12, 4, 4, 8), (4, 20, 3, 4, 16)])
def test_a8_brute_force_tiny(M, K, N, r, g):
    x, Q, Q32, W = _tiny(300 + K + r, M, K, N)
    bias = np.linspace(-1, 1, N).astype(np.float32)
    want = _brute_layer_a8(x.tolist(), Q.tolist(), Q32.tolist(), W.tolist(), r, g, bias.tolist())
    Wh, qw, sw = O.prepare_weights(W, Q32, r, g)
    got = O.linear_a8(x, Q, Wh, qw, sw, r, g, bias)
    np.testing.assert_allclose(got["y32"], want, rtol=2.0 ** -22, atol=1e-30)
    assert got["qx"].dtype == np.int8 and got["sx"].shape == (M,)


def test_a8_is_closer_than_a4_on_the_same_layer():
    x, Q, Q32, W = _tiny(77, 8, 64, 12)
    Wh, qw, sw = O.prepare_weights(W, Q32, 8, 8)
    ref = O.linear_exact(x, Q, W, 8)
    e4 = np.abs(O.linear(x, Q, Wh, qw, sw, 8, 8)["y32"] - ref).mean()
    e8 = np.abs(O.linear_a8(x, Q, Wh, qw, sw, 8, 8)["y32"] - ref).mean()
    assert e8 < e4


# --------------------------------------------------------------------------
# W4A16: 16-bit activations against the 4-bit per-group weights, no rotation
# --------------------------------------------------------------------------
@pytest.mark.parametrize("M,K,N,g", [(3, 16, 5, 4), (2, 24, 4, 8), (4, 16, 3, 16)])
def test_w4a16_brute_force_tiny(M, K, N, g):
    """Python loops, exact rational sums: every weight is code * stored scale of its group."""
    x, _, _, W = _tiny(500 + K + g, M, K, N)
    bias = np.linspace(-2, 1, N).astype(np.float32)
    qw, sw = O.quantize_groups(W, g)
    want = np.zeros((M, N), np.float32)
    for m in range(M):
        for n in range(N):
            acc = Fraction(float(bias[n]))
            for k in range(K):
                c, s = _quant([float(v) for v in W[n, (k // g) * g:(k // g + 1) * g]])
                acc += Fraction(float(x[m, k])) * Fraction(c[k % g]) * Fraction(s)
            want[m, n] = _f32(float(acc))
    y32, y = O.linear_w4a16(x, qw, sw, g, bias)
    np.testing.assert_allclose(y32, want, rtol=2.0 ** -22, atol=1e-30)
    np.testing.assert_array_equal(y, O.round_to_bf16(y32))


def test_w4a16_integer_and_power_of_two_cases():
    """Unit scales and integer activations: a plain integer matrix product; power-of-two scales
    per group scale exactly that group's share (a wrong group index or a transposed scale fails)."""
    rng = np.random.default_rng(5)
    M, K, N, g = 5, 32, 6, 8
    x = rng.integers(-20, 21, size=(M, K)).astype(np.float32)
    qw = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    one = np.ones((N, K // g), np.float16)
    y32, _ = O.linear_w4a16(x, qw, one, g)
    np.testing.assert_array_equal(y32, (x.astype(np.int64) @ qw.astype(np.int64).T).astype(np.float32))
    sw = (2.0 ** rng.integers(-3, 4, size=(N, K // g))).astype(np.float16)
    y32, _ = O.linear_w4a16(x, qw, sw, g)
    want = np.zeros((M, N))
    for n in range(N):
        for j in range(K // g):
            want[:, n] += float(sw[n, j]) * (x[:, j * g:(j + 1) * g].astype(np.int64) @ qw[n, j * g:(j + 1) * g].astype(np.int64))
    np.testing.assert_array_equal(y32, want.astype(np.float32))


def test_w4a16_agrees_with_the_w4a4_combine_on_code_times_scale_activations():
    """If the 16-bit activations happen to be code * scale per group (exactly representable), the
    W4A16 product equals the W4A4 combine of those codes and scales: two separately written sums."""
    rng = np.random.default_rng(6)
    M, K, N, g = 7, 48, 9, 16
    qx = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    sx = (2.0 ** rng.integers(-4, 3, size=(M, K // g))).astype(np.float16)
    x = O.dequantize_groups(qx, sx, g).astype(np.float32)
    assert np.array_equal(O.round_to_bf16(x), x)
    qw = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    sw = rng.lognormal(-3, 1, size=(N, K // g)).astype(np.float16)
    y_a, _ = O.linear_w4a16(x, qw, sw, g)
    y_b, _ = O.combine(np.zeros((M, 0), np.float32), qx, sx, np.zeros((N, 0), np.float32), qw, sw, g)
    np.testing.assert_array_equal(y_a, y_b)


def test_qsnr_hand_value():
    """QSNR = 10 log10(|ref|^2 / |ref - approx|^2): ref (3, 4), approx (3, 3.5) -> 25 / 0.25 = 100 -> 20 dB.
    (20 log10 would give 40; swapped arguments 10 log10(21.25 / 0.25) = 19.29.)"""
    assert abs(O.qsnr_db(np.array([3.0, 4.0]), np.array([3.0, 3.5])) - 20.0) < 1e-12
    assert abs(O.qsnr_db(np.array([3.0, 3.5]), np.array([3.0, 4.0])) - 10.0 * np.log10(85.0)) < 1e-12
    assert O.qsnr_db(np.array([1.0, -2.0]), np.array([1.0, -2.0])) > 200.0          # exact: capped, not infinite
