"""The acceptance rules of the GPU parity tests, exercised on the CPU with planted deviations: a stored fp16
scale may differ from the oracle's only next to a rounding midpoint."""
import numpy as np
import pytest

from oracle import dirotq_oracle as O

import gpu_util as U


def test_accumulation_slack_formula():
    rng = np.random.default_rng(0)
    K = 48
    x = rng.standard_normal((3, K)).astype(np.float32)
    Q = rng.standard_normal((K, K)).astype(np.float32)
    cols = np.array([5, 0, 47])
    got = U.accumulation_slack(x, Q, cols, K)
    for i in range(3):
        b2 = np.sqrt(sum((float(x[i, k]) * float(Q[k, cols[i]])) ** 2 for k in range(K)))
        assert abs(got[i] - 4 * np.sqrt(K) * 2.0 ** -24 * b2) <= 1e-12 * b2


def test_flip_next_to_the_midpoint_is_accepted_and_elsewhere_rejected():
    lo, hi = np.float16(0.4375), np.float16(0.4377)            # adjacent fp16 numbers
    assert int(hi.view(np.uint16)) - int(lo.view(np.uint16)) == 1
    mid = 0.5 * (float(lo) + float(hi))
    ulp = float(hi) - float(lo)
    slack = np.array([0.02 * ulp])
    # the oracle rounded down (value a hair below the midpoint), the other side rounded up: fine
    U.check_flips_near_midpoint(np.array([mid - 0.01 * ulp], np.float32), np.array([hi]), np.array([lo]), slack, "scale")
    # a value a third of an ulp away from the midpoint cannot flip by accumulation noise
    with pytest.raises(AssertionError):
        U.check_flips_near_midpoint(np.array([mid - 0.3 * ulp], np.float32), np.array([hi]), np.array([lo]), slack, "scale")
    # two ulps apart is never accepted
    hi2 = np.array([int(lo.view(np.uint16)) + 2], np.uint16).view(np.float16)
    with pytest.raises(AssertionError):
        U.check_flips_near_midpoint(np.array([mid], np.float32), hi2, np.array([lo]), slack, "scale")


def test_code_check_rejects_a_wrongly_rounded_scale():
    """A planted one-ulp scale error in a group whose amax / 7 is nowhere near a midpoint must fail the
    statistical check even though it is a single group in thousands."""
    rng = np.random.default_rng(1)
    M, K, g = 64, 256, 64
    x = O.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    Q = np.eye(K, dtype=np.float32)
    xhat = O.rotate(x, Q)
    qx, sx = O.quantize_groups(xhat, g)
    st = U.check_codes_statistical(xhat, qx, sx, qx, sx, g, x=x, Q=Q)
    assert st["scale_flips"] == 0 and st["agree"] == 1.0
    # find a group whose unrounded scale sits well inside its rounding interval, then bump its stored scale
    amax = np.abs(xhat.reshape(M, K // g, g)).max(-1)
    s32 = (amax / np.float32(7)).astype(np.float32)
    dist = np.abs(s32.astype(np.float64) - sx.astype(np.float64)) / np.spacing(sx.astype(np.float16)).astype(np.float64)
    m, j = np.unravel_index(np.argmin(dist), dist.shape)            # closest to its fp16 value: farthest from a midpoint
    bad = sx.copy()
    bad.view(np.uint16)[m, j] += 1
    qbad, _ = O.quantize_groups(xhat, g)
    with pytest.raises(AssertionError):
        U.check_codes_statistical(xhat, qbad, bad, qx, sx, g, x=x, Q=Q)
