"""Element offsets beyond 2^31: the output of the GEMM and the input of the rotation are larger than a
32-bit index can address.  Inputs are drawn on the GPU (they are gigabytes); the oracle recomputes
sampled tokens, including the last ones."""
import sys

import numpy as np
import pytest
import torch

from oracle import dirotq_oracle as O
from paper_2605_16732_amd import binding as B

from gpu_util import dev, host_bf16_bits, host_f16, import_blob, unpack_codes

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


def _bf16_rows_to_f32(t):
    return O.from_bf16_bits(host_bf16_bits(t))


def test_gemm_output_beyond_2_31_elements():
    M, N, K, g = 65536 + 128, 36864, 64, 32                 # M * N = 2.42e9 elements (4.8 GB of bf16)
    _say(f"w4a4_gemm with {M * N / 2**31:.2f} x 2^31 output elements")
    rng = np.random.default_rng(61)
    G = K // g
    qw = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    sw = (2.0 ** rng.integers(-4, 1, size=(N, G))).astype(np.float16)
    blob = import_blob(np.zeros((N, 0), np.float32), qw, sw, N, K, 0, g)
    gen = torch.Generator(device="cuda").manual_seed(61)
    nib = torch.randint(0, 8, (M, K), generator=gen, device="cuda", dtype=torch.uint8)      # magnitudes 0..7
    sgn = torch.randint(0, 2, (M, K), generator=gen, device="cuda", dtype=torch.uint8)
    nib = torch.where(nib == 0, nib, nib | (sgn << 3))                                        # no "minus zero"
    xl = (nib[:, 0::2] | (nib[:, 1::2] << 4)).contiguous()
    sx = torch.ones((G, M), dtype=torch.float16, device="cuda")
    y = B.w4a4_gemm(None, xl, sx, blob, M, N, K, 0, g)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([rng.choice(M, size=20, replace=False), [0, 58254, 58255, M - 129, M - 1]]))
    qx = unpack_codes(xl[torch.from_numpy(rows).cuda()].cpu().numpy())
    y32, ybf = O.combine(np.zeros((len(rows), 0), np.float32), qx, np.ones((len(rows), G), np.float16),
                         np.zeros((N, 0), np.float32), qw, sw, g)
    got = _bf16_rows_to_f32(y[torch.from_numpy(rows).cuda()])
    np.testing.assert_array_equal(got, ybf)                  # integers times powers of two: exact


def test_rotation_input_beyond_2_31_elements():
    M, K, r, g = 524288 + 256, 4096, 128, 64                 # M * K = 2.15e9 elements (4.3 GB of bf16)
    _say(f"rotate_quantize with {M * K / 2**31:.2f} x 2^31 input elements")
    rng = np.random.default_rng(62)
    Q = np.zeros((K, K), np.float32)
    Q[rng.permutation(K), np.arange(K)] = rng.choice([-1.0, 1.0], size=K)                    # exact rotation
    Qt = B.prepare_rotation(dev(Q))
    gen = torch.Generator(device="cuda").manual_seed(62)
    x = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    step = 65536
    for m0 in range(0, M, step):                             # drawn in slices to bound the fp32 temporary
        m1 = min(m0 + step, M)
        x[m0:m1] = (torch.randn((m1 - m0, K), generator=gen, device="cuda") * 3).to(torch.bfloat16)
    xh, xl, sx = B.rotate_quantize(x, Qt, r, g)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([rng.choice(M, size=12, replace=False), [0, 524287, 524288, M - 1]]))
    idx = torch.from_numpy(rows).cuda()
    xs = _bf16_rows_to_f32(x[idx])
    xh_r, qx_r, sx_r = O.split_quantize(O.rotate(xs, Q), r, g)
    np.testing.assert_array_equal(_bf16_rows_to_f32(xh[idx]), xh_r)
    np.testing.assert_array_equal(unpack_codes(xl[idx].cpu().numpy()), qx_r)
    np.testing.assert_array_equal(host_f16(sx[:, idx].contiguous()).T.view(np.uint16), sx_r.view(np.uint16))
