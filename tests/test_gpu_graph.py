"""The online entry points only enqueue kernels on the caller's stream (no allocation, no
synchronisation, no host round trip), so they can be recorded into a HIP graph.  Each graph is
replayed several times with eager work and synchronisations in between, and every replay must
equal the eager result on the same inputs bit for bit."""
import sys

import numpy as np
import pytest
import torch

from paper_2605_16732_amd import binding as B
from paper_2605_16732_amd import inputs as I

from gpu_util import dev, dev_bf16

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


def _layer(shape):
    L = I.make_layer(shape)
    Qt = B.prepare_rotation(dev(L.Q32))
    blob = B.prepare_weights(dev(L.W), dev(L.Q32), shape.r, shape.g)
    xs = [dev_bf16(I.make_activations(shape, shape.M, seed=s)) for s in (1, 2, 3)]
    return L, Qt, blob, xs


@pytest.mark.parametrize("variant", ["sym", "asym", "a8"])
def test_fused_layer_in_a_graph_replays_equal_eager(variant):
    shp = I.LayerShape("graph", 300, 384, 200, 64, 64, 4, 7, 3)
    _say(f"graph capture of the fused layer, variant {variant}")
    _, Qt, blob, xs = _layer(shp)
    fn = {"sym": B.linear, "asym": B.linear_asym, "a8": B.linear_a8}[variant]
    nws = B.a8_workspace_bytes(shp.M, shp.K, shp.r) if variant == "a8" else B.workspace_bytes(shp.M, shp.K, shp.r, shp.g)
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    x_static = xs[0].clone()
    y_static = torch.empty((shp.M, shp.N), dtype=torch.bfloat16, device="cuda")
    eager = [fn(x, Qt, blob, shp.N, shp.r, shp.g).clone() for x in xs]       # also the warm-up of every kernel
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn(x_static, Qt, blob, shp.N, shp.r, shp.g, workspace=ws, out=y_static)
    for rep in range(6):
        i = rep % 3
        x_static.copy_(xs[i])
        y_static.zero_()
        ws.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_static, eager[i]), f"replay {rep} differs from the eager result"
        # unrelated eager work between replays
        _ = fn(xs[(i + 1) % 3], Qt, blob, shp.N, shp.r, shp.g)
        torch.cuda.synchronize()


@pytest.mark.parametrize("M", [4, 160])
def test_w4a16_in_a_graph_replays_equal_eager(M):
    shp = I.LayerShape("graph16", M, 384, 200, 0, 64, 4, 7, 4)
    _say(f"graph capture of the W4A16 GEMM, M={M}")
    L = I.make_layer(shp)
    blob = B.prepare_weights(dev(L.W), dev(np.eye(shp.K, dtype=np.float32)), 0, shp.g)
    xs = [dev_bf16(I.make_activations(shp, M, seed=s)) for s in (1, 2, 3)]
    eager = [B.w4a16_gemm(x, blob, shp.N, shp.g).clone() for x in xs]
    torch.cuda.synchronize()
    x_static = xs[0].clone()
    y_static = torch.empty((M, shp.N), dtype=torch.bfloat16, device="cuda")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        B.w4a16_gemm(x_static, blob, shp.N, shp.g, out=y_static)
    for rep in range(6):
        i = rep % 3
        x_static.copy_(xs[i])
        y_static.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_static, eager[i]), f"replay {rep} differs from the eager result"
        _ = B.w4a16_gemm(xs[(i + 1) % 3], blob, shp.N, shp.g)
        torch.cuda.synchronize()
