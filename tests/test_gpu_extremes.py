"""Extreme magnitudes through the three activation quantizers (Q = I, so the rotation is exact and
the GPU must reproduce the oracle bit for bit): scales that saturate at the largest fp16 number,
scales that are fp16 subnormals or round to zero, and a token that mixes both ranges."""
import sys

import numpy as np
import pytest
import torch

from oracle import dirotq_oracle as O
from paper_2605_16732_amd import binding as B

from gpu_util import dev, gpu_rotate_quantize
from test_gpu_parity_a8 import gpu_rq_a8
from test_gpu_parity_asym import gpu_rq_asym

pytestmark = pytest.mark.gpu


def _rows(K):
    rng = np.random.default_rng(71)
    x = np.zeros((6, K), np.float32)
    x[0] = rng.standard_normal(K) * 1e37                       # amax / 7 far above 65504: scale saturates
    x[1] = rng.standard_normal(K) * 2.0 ** -22                 # fp16-subnormal scales
    x[2] = rng.standard_normal(K) * 2.0 ** -27                 # scales round to zero: all codes 0
    x[3] = rng.standard_normal(K)
    x[3, ::37] = 3e4 * 7                                       # a few channels right at the saturation edge
    x[4, : K // 2] = rng.standard_normal(K // 2) * 1e30        # huge and tiny groups in one token
    x[4, K // 2:] = rng.standard_normal(K // 2) * 2.0 ** -20
    x[5] = np.abs(rng.standard_normal(K)) * 1e36 + 1e36        # one-sided huge values (asymmetric zero-point saturates)
    return O.round_to_bf16(x)


@pytest.mark.parametrize("g", [32, 128])
def test_extreme_magnitudes_symmetric(g):
    K, r = 256, 0
    x = _rows(K)
    Qt = B.prepare_rotation(dev(np.eye(K, dtype=np.float32)))
    _, qx_r, sx_r = O.split_quantize(x, r, g)
    _, (_, qx_g, sx_g) = gpu_rotate_quantize(O.bf16_bits(x), Qt, r, g)
    assert float(sx_r[0].astype(np.float32).max()) == 65504.0 and not qx_r[2].any()
    np.testing.assert_array_equal(sx_g.view(np.uint16), sx_r.view(np.uint16))
    np.testing.assert_array_equal(qx_g, qx_r)


@pytest.mark.parametrize("g", [32, 64])
def test_extreme_magnitudes_asymmetric(g):
    K, r = 256, 0
    x = _rows(K)
    Qt = B.prepare_rotation(dev(np.eye(K, dtype=np.float32)))
    _, qx_r, sx_r, zx_r = O.split_quantize_asym(x, r, g)
    _, (_, qx_g, sx_g, zx_g) = gpu_rq_asym(O.bf16_bits(x), Qt, r, g)
    assert float(zx_r[5].astype(np.float32).min()) == 65504.0            # zero-point saturates
    np.testing.assert_array_equal(sx_g.view(np.uint16), sx_r.view(np.uint16))
    np.testing.assert_array_equal(zx_g.view(np.uint16), zx_r.view(np.uint16))
    np.testing.assert_array_equal(qx_g, qx_r)


def test_extreme_magnitudes_int8_tokens():
    K, r = 256, 0
    x = _rows(K)
    Qt = B.prepare_rotation(dev(np.eye(K, dtype=np.float32)))
    _, qx_r, sx_r = O.split_quantize_a8(x, r)
    _, (_, qx_g, sx_g) = gpu_rq_a8(O.bf16_bits(x), Qt, r)
    assert float(sx_r[0]) == 65504.0 and not qx_r[2].any()
    np.testing.assert_array_equal(sx_g.view(np.uint16), sx_r.view(np.uint16))
    np.testing.assert_array_equal(qx_g, qx_r)
