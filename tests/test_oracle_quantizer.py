"""Pins for the oracle's quantizer and storage formats (CPU only).

Everything here checks `oracle/` against something other than itself: hand-worked
cases of the paper's quantizer equation, explicit bytes, error bounds that follow
from the definition, and a pure-Python re-derivation with exact rational arithmetic.
"""
import os
import struct
from fractions import Fraction

import numpy as np
import pytest

from oracle import dirotq_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quantizer_cases.txt")


def _cases():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            vals, scale_hex, codes = [p.strip() for p in line.split("|")]
            out.append((np.array([float(v) for v in vals.split()], np.float32),
                        int(scale_hex, 16),
                        np.array([int(c) for c in codes.split()], np.int8)))
    return out


def test_qmax_is_the_papers():
    # quantizer equation: q_max = 2^(k-1) - 1 for k-bit symmetric integers
    assert O.QMAX == 2 ** (4 - 1) - 1 == 7


@pytest.mark.parametrize("vals,scale_bits,codes", _cases())
def test_hand_worked_cases(vals, scale_bits, codes):
    q, s = O.quantize_groups(vals[None, :], g=len(vals))
    assert s.dtype == np.float16 and q.dtype == np.int8
    assert int(s.view(np.uint16)[0, 0]) == scale_bits
    np.testing.assert_array_equal(q[0], codes)


def test_hand_cases_as_two_groups_of_one_row():
    # groups are consecutive channels along the last axis: two 4-element cases
    # side by side in one row give the two cases' answers side by side.
    cs = _cases()
    a, b = cs[0], cs[2]
    row = np.concatenate([a[0], b[0]])[None, :]
    q, s = O.quantize_groups(row, g=4)
    np.testing.assert_array_equal(q[0], np.concatenate([a[2], b[2]]))
    assert [int(v) for v in s.view(np.uint16)[0]] == [a[1], b[1]]


def _f32(x):
    return struct.unpack("f", struct.pack("f", x))[0]


def _f16(x):
    return struct.unpack("e", struct.pack("e", x))[0]


def _quant_group_python(vals):
    """The same op sequence with Python floats: fp32 results obtained by rounding an
    fp64 result once (innocuous for +,*,/ of fp32 operands since 53 >= 2*24+2)."""
    amax = max(abs(v) for v in vals)
    s32 = min(_f32(amax / 7.0), 65504.0)
    sf = _f16(s32)
    if sf == 0.0:
        return [0] * len(vals), 0.0
    inv = _f32(1.0 / sf)
    codes = []
    for v in vals:
        t = _f32(v * inv)
        n = round(t)              # Python's round(): ties to even
        codes.append(max(-7, min(7, n)))
    return codes, sf


def test_against_pure_python_sequence():
    rng = np.random.default_rng(11)
    v = (rng.standard_normal((64, 128)) * rng.lognormal(0, 2, size=(64, 1))).astype(np.float32)
    v[3, 5:9] = 0.0
    v[7, :32] = 0.0                              # one all-zero group
    q, s = O.quantize_groups(v, g=32)
    for m in range(64):
        for j in range(4):
            codes, sf = _quant_group_python([float(x) for x in v[m, 32 * j:32 * j + 32]])
            assert float(s[m, j]) == sf
            assert list(q[m, 32 * j:32 * j + 32]) == codes


@pytest.mark.parametrize("g", [32, 64, 128])
def test_invariants(g):
    rng = np.random.default_rng(5)
    v = (rng.standard_normal((200, 4 * g)) * rng.lognormal(0, 1.5, size=(200, 1))).astype(np.float32)
    q, s = O.quantize_groups(v, g)
    sf = s.astype(np.float64)
    assert q.min() >= -7 and q.max() <= 7
    vg = v.reshape(200, 4, g).astype(np.float64)
    qg = q.reshape(200, 4, g)
    amax = np.abs(vg).max(-1)
    # the largest-magnitude element gets code +-7 with the sign of the element
    pos = np.abs(vg).argmax(-1)
    top = np.take_along_axis(qg, pos[..., None], -1)[..., 0]
    vtop = np.take_along_axis(vg, pos[..., None], -1)[..., 0]
    np.testing.assert_array_equal(top, 7 * np.sign(vtop).astype(np.int8))
    # stored scale is amax/7 to within fp16 rounding (2^-11 relative)
    assert np.all(np.abs(sf * 7 - amax) <= amax * 2.0 ** -11 * (1 + 1e-6))
    # dequantisation error at most half a step (+ the clip at the top code, where the
    # fp16 rounding of the scale can leave amax up to 7 * 2^-11 steps above 7 s)
    err = np.abs(vg - qg * sf[..., None])
    assert np.all(err <= sf[..., None] * (0.5 + 7 * 2.0 ** -11 + 1e-6))
    # dequantize_groups is codes * scale
    np.testing.assert_array_equal(O.dequantize_groups(q, s, g).reshape(200, 4, g), qg * sf[..., None])


def test_exact_rational_rounding_agrees_away_from_ties():
    """The real-arithmetic definition round(v / s) agrees with the fp32 sequence
    except within ~1 ulp of a rounding boundary."""
    rng = np.random.default_rng(9)
    v = rng.standard_normal((40, 64)).astype(np.float32)
    q, s = O.quantize_groups(v, 64)
    for m in range(40):
        sf = Fraction(float(s[m, 0]))
        for k in range(64):
            t = Fraction(float(v[m, k])) / sf
            frac = t - (t.numerator // t.denominator)
            if abs(frac - Fraction(1, 2)) < Fraction(1, 10 ** 5):
                continue
            assert int(q[m, k]) == max(-7, min(7, round(t)))


def test_pack_bytes_and_roundtrip():
    # byte i = channel 2i in bits 0-3, channel 2i+1 in bits 4-7, two's complement
    assert O.pack_int4(np.array([-7, 7], np.int8))[0] == 0x79
    assert O.pack_int4(np.array([7, -7], np.int8))[0] == 0x97
    assert O.pack_int4(np.array([1, 0], np.int8))[0] == 0x01
    assert O.pack_int4(np.array([0, 1], np.int8))[0] == 0x10
    assert O.pack_int4(np.array([-1, -1], np.int8))[0] == 0xFF
    pairs = np.array([[a, b] for a in range(-7, 8) for b in range(-7, 8)], np.int8)
    packed = O.pack_int4(pairs)
    assert packed.shape == (225, 1) and packed.dtype == np.uint8
    np.testing.assert_array_equal(O.unpack_int4(packed), pairs)
    row = np.arange(-7, 7, dtype=np.int8)[None, :]                 # 14 channels -> 7 bytes
    np.testing.assert_array_equal(O.unpack_int4(O.pack_int4(row)), row)


def test_bf16_rounding():
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: even mantissa wins (1.0);
    # 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6: goes to 1 + 2^-6.
    a = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                  -3.0, 0.0, 2.0 ** -130], np.float32)
    r = O.round_to_bf16(a)
    np.testing.assert_array_equal(
        r, np.array([1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7, -3.0, 0.0, 2.0 ** -130], np.float32))
    np.testing.assert_array_equal(O.bf16_bits(r)[:2], np.array([0x3F80, 0x3F82], np.uint16))
    np.testing.assert_array_equal(O.from_bf16_bits(O.bf16_bits(r)), r)
    # agrees with torch's cast on random data
    import torch
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 37.0
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(O.round_to_bf16(x), t)


# ---------------------------------------------------------------------------
# asymmetric variant (z = min X, s = (max X - min X) / 15, codes in [0, 15])
# ---------------------------------------------------------------------------
GOLDEN_ASYM = os.path.join(os.path.dirname(__file__), "golden", "quantizer_asym_cases.txt")


def _asym_cases():
    out = []
    with open(GOLDEN_ASYM) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            vals, s_hex, z_hex, codes = [p.strip() for p in line.split("|")]
            out.append((np.array([float(v) for v in vals.split()], np.float32), int(s_hex, 16), int(z_hex, 16),
                        np.array([int(c) for c in codes.split()], np.uint8)))
    return out


def test_asym_qmax_is_the_papers():
    # quantizer equation: q_min = 0, q_max = 2^k - 1 for k-bit asymmetric integers
    assert O.UQMAX == 2 ** 4 - 1 == 15


@pytest.mark.parametrize("vals,s_bits,z_bits,codes", _asym_cases())
def test_asym_hand_worked_cases(vals, s_bits, z_bits, codes):
    q, s, z = O.quantize_groups_asym(vals[None, :], g=len(vals))
    assert s.dtype == np.float16 and z.dtype == np.float16 and q.dtype == np.uint8
    assert int(s.view(np.uint16)[0, 0]) == s_bits
    assert int(z.view(np.uint16)[0, 0]) == z_bits
    np.testing.assert_array_equal(q[0], codes)


def _f16(x):
    return struct.unpack("e", struct.pack("e", x))[0]


def test_asym_against_pure_python_sequence():
    # the documented fp32 operation sequence, re-done with Python floats rounded by struct
    rng = np.random.default_rng(11)
    v = (rng.standard_normal((40, 24)) * rng.lognormal(0, 2, (40, 1)) + rng.normal(0, 3, (40, 1))).astype(np.float32)
    q, s, z = O.quantize_groups_asym(v, 8)
    for i in range(v.shape[0]):
        for j in range(3):
            grp = [float(t) for t in v[i, j * 8:(j + 1) * 8]]
            mn, mx = min(grp), max(grp)
            zf = _f16(max(-65504.0, min(65504.0, mn)))
            sf = _f16(min(_f32(_f32(mx - mn) / 15.0), 65504.0))
            assert float(s[i, j]) == sf and float(z[i, j]) == zf
            if sf == 0.0:
                want = [0] * 8
            else:
                inv = _f32(1.0 / sf)
                want = [max(0, min(15, round(_f32(_f32(t - zf) * inv)))) for t in grp]
            assert list(q[i, j * 8:(j + 1) * 8]) == want


@pytest.mark.parametrize("g", [4, 32, 64])
def test_asym_invariants(g):
    rng = np.random.default_rng(5 + g)
    v = (rng.standard_normal((64, 2 * g)) * rng.lognormal(0, 1.5, (64, 1)) + rng.normal(0, 2, (64, 1))).astype(np.float32)
    q, s, z = O.quantize_groups_asym(v, g)
    assert q.min() >= 0 and q.max() <= 15
    vg = v.reshape(64, 2, g).astype(np.float64)
    sf, zf = s.astype(np.float64), z.astype(np.float64)
    # the stored pair is the definition's pair up to fp16 rounding (relative 2^-11)
    np.testing.assert_allclose(zf, vg.min(-1), rtol=2.0 ** -11, atol=2.0 ** -25)
    np.testing.assert_allclose(sf, (vg.max(-1) - vg.min(-1)) / 15, rtol=2.0 ** -10, atol=2.0 ** -25)
    # error of the dequantised value: half a step, plus what the fp16 roundings of z and s move the grid
    # (at most |z - min| at the bottom and 15 |s - s_exact| + |z - min| at the top)
    deq = O.dequantize_groups_asym(q, s, z, g).reshape(64, 2, g)
    slack = np.abs(zf - vg.min(-1)) + 15 * np.abs(sf - (vg.max(-1) - vg.min(-1)) / 15)
    bound = sf / 2 * (1 + 2.0 ** -20) + slack + 1e-30
    assert np.all(np.abs(deq - vg) <= bound[..., None])
    # the smallest element gets code 0 and the largest 15 (unless the group is constant)
    live = sf > 0
    amin = np.take_along_axis(q.reshape(64, 2, g), vg.argmin(-1)[..., None], -1)[..., 0]
    amax = np.take_along_axis(q.reshape(64, 2, g), vg.argmax(-1)[..., None], -1)[..., 0]
    assert np.all(amin[live] == 0) and np.all(amax[live] >= 14)


def test_asym_shift_equivariance_on_a_dyadic_grid():
    # values on a coarse dyadic grid: adding a grid constant moves z by it and leaves s and the codes alone
    rng = np.random.default_rng(3)
    v = (rng.integers(-40, 41, (50, 16)) * 0.25).astype(np.float32)
    q0, s0, z0 = O.quantize_groups_asym(v, 16)
    q1, s1, z1 = O.quantize_groups_asym(v + np.float32(6.5), 16)
    np.testing.assert_array_equal(q0, q1)
    np.testing.assert_array_equal(s0.view(np.uint16), s1.view(np.uint16))
    np.testing.assert_array_equal(z1.astype(np.float32), z0.astype(np.float32) + np.float32(6.5))


def test_asym_of_a_symmetric_two_point_group():
    # {-a, +a}: z = -a, s = 2a/15, codes 0 and 15; dequantised ends are -a and -a + 15 s
    a = np.float32(3.75)
    q, s, z = O.quantize_groups_asym(np.array([[-a, a, -a, a]], np.float32), 4)
    np.testing.assert_array_equal(q[0], [0, 15, 0, 15])
    assert float(z[0, 0]) == -3.75 and float(s[0, 0]) == 0.5


# ---------------------------------------------------------------------------
# 8-bit per-token variant (W4A8)
# ---------------------------------------------------------------------------
GOLDEN_INT8 = os.path.join(os.path.dirname(__file__), "golden", "quantizer_int8_cases.txt")


def _int8_cases():
    out = []
    with open(GOLDEN_INT8) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            vals, s_hex, codes = [p.strip() for p in line.split("|")]
            out.append((np.array([float(v) for v in vals.split()], np.float32), int(s_hex, 16),
                        np.array([int(c) for c in codes.split()], np.int8)))
    return out


@pytest.mark.parametrize("vals,s_bits,codes", _int8_cases())
def test_int8_hand_worked_cases(vals, s_bits, codes):
    assert O.QMAX8 == 2 ** (8 - 1) - 1 == 127
    q, s = O.quantize_tokens_int8(vals[None, :])
    assert q.dtype == np.int8 and s.dtype == np.float16 and s.shape == (1,)
    assert int(s.view(np.uint16)[0]) == s_bits
    np.testing.assert_array_equal(q[0], codes)


def test_int8_against_pure_python_sequence_and_bounds():
    rng = np.random.default_rng(21)
    v = (rng.standard_normal((30, 200)) * rng.lognormal(0, 2, (30, 1))).astype(np.float32)
    v[:, 7] *= 50                                            # an outlier channel
    q, s = O.quantize_tokens_int8(v)
    for i in range(v.shape[0]):
        row = [float(t) for t in v[i]]
        sf = _f16(min(_f32(max(abs(t) for t in row) / 127.0), 65504.0))
        assert float(s[i]) == sf
        inv = _f32(1.0 / sf)
        assert list(q[i]) == [max(-127, min(127, round(_f32(t * inv)))) for t in row]
    # one scale per token: error at most half a step (plus what fp16 rounding of s moves the top code)
    deq = q.astype(np.float64) * s.astype(np.float64)[:, None]
    amax = np.abs(v).max(1).astype(np.float64)
    bound = s.astype(np.float64) / 2 * (1 + 2.0 ** -20) + 127 * np.abs(s.astype(np.float64) - amax / 127)
    assert np.all(np.abs(deq - v) <= bound[:, None] + 1e-30)
    assert np.all(np.abs(q).max(1) >= 126)


# --------------------------------------------------------------------------
# symmetries the quantizer equation implies (hold exactly in the fixed fp32 sequence)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("which", ["int4", "int8"])
def test_sign_power_of_two_and_permutation_symmetries(which):
    """Q(-v) = -Q(v); Q(2^k v) has the same codes and the scale times 2^k (every step of the
    sequence commutes with an exact power-of-two factor while the stored fp16 scale stays a normal
    number: the exponents below keep it between 2^-14 and 65504); permuting the channels of a group
    permutes its codes and leaves the scale alone."""
    rng = np.random.default_rng(77)
    g = 16
    v = (rng.standard_normal((64, g)) * rng.lognormal(0, 1, size=(64, 1))).astype(np.float32)
    quant = (lambda a: O.quantize_groups(a, g)) if which == "int4" else O.quantize_tokens_int8
    q, s = quant(v)
    qn, sn = quant(-v)
    np.testing.assert_array_equal(qn, -q)
    np.testing.assert_array_equal(sn.view(np.uint16), s.view(np.uint16))
    assert float(s.astype(np.float32).min()) * 2.0 ** -2 >= 2.0 ** -14
    for k in (-2, -1, 3, 9):
        qk, sk = quant((v * np.float32(2.0 ** k)).astype(np.float32))
        np.testing.assert_array_equal(qk, q)
        np.testing.assert_array_equal(sk.astype(np.float64).ravel(), s.astype(np.float64).ravel() * 2.0 ** k)
    perm = rng.permutation(g)
    qp, sp = quant(np.ascontiguousarray(v[:, perm]))
    np.testing.assert_array_equal(qp, q[:, perm])
    np.testing.assert_array_equal(sp.view(np.uint16), s.view(np.uint16))


def test_asym_sign_flip_mirrors_the_codes():
    """Negating a group swaps min and max: codes become 15 - q only where the stored zero-point and
    scale are exact, so the test uses a dyadic grid (values k / 8, range a multiple of 15 / 8)."""
    g = 8
    base = np.array([[0, 15, 1, 7, 8, 14, 3, 12]], np.float32) / np.float32(8.0) - np.float32(0.5)
    q, s, z = O.quantize_groups_asym(base, g)
    qn, sn, zn = O.quantize_groups_asym(-base, g)
    np.testing.assert_array_equal(qn, 15 - q)
    assert float(sn[0, 0]) == float(s[0, 0]) == 0.125
    assert float(z[0, 0]) == -0.5 and float(zn[0, 0]) == -(15 / 8 - 0.5)
