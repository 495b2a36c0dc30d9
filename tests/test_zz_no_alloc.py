"""dirotq_linear_static (intermediates in the library's fixed device array, nothing allocated)
against dirotq_linear (caller-supplied workspace): the two run the same kernels, so the outputs
must be bit-identical.  Two calls in a row share the array, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2605_16732_amd import binding as B
from paper_2605_16732_amd import inputs as I

from gpu_util import dev, dev_bf16

pytestmark = pytest.mark.gpu


def _layer(M, K, N, r, g, seed):
    rng = np.random.default_rng(seed)
    Q64, _ = np.linalg.qr(rng.standard_normal((K, K)))
    Q32 = Q64.astype(np.float32)
    W = (rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32)
    s = rng.lognormal(0, 0.5, size=K)
    s[rng.choice(K, 4, replace=False)] *= 80
    x_bits = I.to_bf16_bits((rng.standard_normal((M, K)) * s).astype(np.float32))
    bias = I.to_bf16_bits(rng.standard_normal(N).astype(np.float32))
    return x_bits, Q32, W, bias


def test_static_scratch_entry_point_matches_workspace_entry_point():
    print("[case] dirotq_linear_static: 700x512->384 then 130x256->200", flush=True)
    calls = [(700, 512, 384, 64, 64, 11), (130, 256, 200, 32, 32, 12)]     # the second is smaller in every size
    prepared = []
    for (M, K, N, r, g, seed) in calls:
        x_bits, Q32, W, bias = _layer(M, K, N, r, g, seed)
        Qt = B.prepare_rotation(dev(Q32))
        blob = B.prepare_weights(dev(W), dev(Q32), r, g)
        x = dev_bf16(x_bits)
        b = dev_bf16(bias)
        want = B.linear(x, Qt, blob, N, r, g, bias=b)
        out = torch.full((M + 1, N), 3.0, dtype=torch.bfloat16, device=x.device)     # last row: canary
        prepared.append((x, Qt, blob, b, N, r, g, want, out))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for (x, Qt, blob, b, N, r, g, want, out) in prepared:                           # back to back, one stream
        B.linear_static(x, Qt, blob, N, r, g, out[:-1], bias=b)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for (x, Qt, blob, b, N, r, g, want, out) in prepared:
        assert torch.equal(out[:-1].view(torch.int16), want.view(torch.int16))
        assert bool((out[-1] == 3.0).all())
    # and once more in the opposite order (the larger call after the smaller one)
    for (x, Qt, blob, b, N, r, g, want, out) in reversed(prepared):
        out.fill_(3.0)
        B.linear_static(x, Qt, blob, N, r, g, out[:-1], bias=b)
        torch.cuda.synchronize()
        assert torch.equal(out[:-1].view(torch.int16), want.view(torch.int16))


def test_static_scratch_limit_is_enforced_on_the_host():
    a = torch.zeros(64, dtype=torch.uint8, device="cuda")
    st = B.lib().dirotq_linear_static(a.data_ptr(), a.data_ptr(), a.data_ptr(), None, 16384, 8, 12288, 128, 64,
                                      a.data_ptr(), None)
    assert st == B.ERR_STATIC_LIMIT
