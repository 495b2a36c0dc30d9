"""Seeded synthetic inputs for the rotation-aware W4A4 linear layer.

This module only *draws* inputs: outlier-heavy DiT-like activations, a
calibration-derived orthogonal basis Q, and dense weights.  It contains none of
the layer's arithmetic (no quantizer, no packing, no GEMM of the method), so the
CPU oracle and the HIP path can both be fed from it without sharing code.

The structure follows what the paper describes for DiT activations: a few input
channels carry outliers about two orders of magnitude above the median channel
(Fig. 1b), and the basis is the eigenvector matrix of the uncentered second
moment of calibration activations, eigenvalues descending (Appendix "PCA-based
activation quantization", the eigendecomposition equation).  The paper's real
calibration data (prompts run through trained DiTs) is not available here; these
draws stand in for it.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import scipy.linalg
import torch

N_CALIB = 2048          # calibration rows used to estimate the second moment
OUTLIER_GAIN = 80.0     # outlier channels are this many times the log-normal scale


@dataclass(frozen=True)
class LayerShape:
    """One linear layer: M tokens, K input channels, N output channels,
    r coefficients kept in BF16, g channels per INT4 scale group."""
    name: str
    M: int
    K: int
    N: int
    r: int
    g: int
    n_outliers: int
    config_id: int
    layer_id: int

    @property
    def G(self) -> int:
        return (self.K - self.r) // self.g


def _mk(name, M, K, N, r, g, n_out, cfg, lid):
    assert (K - r) % g == 0
    return LayerShape(name, M, K, N, r, g, n_out, cfg, lid)


# configs[0]: the small case the oracle finishes in seconds.
SMALL = _mk("small", 256, 1152, 1152, 64, 64, 8, 0, 0)

# configs[1]: PixArt-Sigma-shaped block linears, 1024 px, batch 1.
PIXART = [
    _mk("pixart_qkv", 4096, 1152, 3456, 64, 64, 8, 1, 0),
    _mk("pixart_out", 4096, 1152, 1152, 64, 64, 8, 1, 1),
    _mk("pixart_fc1", 4096, 1152, 4608, 64, 64, 8, 1, 2),
    _mk("pixart_fc2", 4096, 4608, 1152, 64, 64, 8, 1, 3),
]

# configs[2]: FLUX.1-dev-shaped linears (4096 image + 512 text tokens).
FLUX = [
    _mk("flux_qkv", 4608, 3072, 9216, 128, 64, 16, 2, 0),
    _mk("flux_out", 4608, 3072, 3072, 128, 64, 16, 2, 1),
    _mk("flux_fc1", 4608, 3072, 12288, 128, 64, 16, 2, 2),
    _mk("flux_fc2", 4608, 12288, 3072, 128, 64, 16, 2, 3),
]

# configs[3]: token sweep on the PixArt fc1 shape.
TOKEN_SWEEP = [
    _mk(f"pixart_fc1_M{M}", M, 1152, 4608, 64, 64, 8, 3, i)
    for i, M in enumerate((1024, 4096, 16384, 32768))
]

# configs[4]: rank / group ablation on the FLUX fc2 shape; the pairs of the
# r x g grid for which K - r is a multiple of g.
ABLATION = [
    _mk(f"flux_fc2_r{r}_g{g}", 4608, 12288, 3072, r, g, 16, 4, i)
    for i, (r, g) in enumerate(
        (r, g) for r in (0, 32, 64, 128, 256) for g in (32, 64, 128)
        if (12288 - r) % g == 0)
]


def _rng(seed: int, shape: LayerShape, stream: int) -> np.random.Generator:
    return np.random.default_rng([seed, shape.config_id, shape.layer_id, stream])


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 array of bfloat16 bit patterns (torch's cast)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float32 values (exact)."""
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def channel_scales(shape: LayerShape, seed: int = 0, K: int | None = None,
                   n_outliers: int | None = None) -> np.ndarray:
    """Per-channel magnitudes: LogNormal(0, 0.5) with a few channels x80."""
    K = shape.K if K is None else K
    n_out = shape.n_outliers if n_outliers is None else n_outliers
    s = _rng(seed, shape, 0).lognormal(0.0, 0.5, size=K)
    idx = _rng(seed, shape, 1).choice(K, size=min(n_out, K), replace=False)
    s[idx] *= OUTLIER_GAIN
    return s.astype(np.float32)


def _sign_fix(Q: np.ndarray) -> np.ndarray:
    """Make each column's largest-magnitude entry positive (reproducible signs)."""
    piv = np.argmax(np.abs(Q), axis=0)
    sgn = np.sign(Q[piv, np.arange(Q.shape[1])])
    sgn[sgn == 0] = 1.0
    return Q * sgn[None, :]


def pca_basis(Xc: np.ndarray) -> tuple[np.ndarray, np.ndarray]:
    """Orthogonal eigenvector matrix of the uncentered second moment
    Sigma = Xc^T Xc / n (float64), eigenvalues descending.

    Returns (Q float64 [K,K], eigenvalues float64 [K]).  When there are fewer
    calibration rows than channels, Sigma has a null space whose eigenvectors are
    arbitrary; then the nonzero-eigenvalue eigenvectors are taken from the n x n
    Gram matrix and completed to an orthogonal matrix with a full QR, which avoids
    a K^3 eigensolve at K = 12288.
    """
    Xc = np.asarray(Xc, dtype=np.float64)
    n, K = Xc.shape
    if n >= K:
        sigma = Xc.T @ Xc / n
        lam, U = np.linalg.eigh(sigma)
        order = np.argsort(lam)[::-1]
        return _sign_fix(U[:, order]), lam[order]
    gram = Xc @ Xc.T / n
    mu, P = np.linalg.eigh(gram)
    order = np.argsort(mu)[::-1]
    mu, P = mu[order], P[:, order]
    V = (Xc.T @ P) / np.sqrt(np.maximum(mu, 1e-300) * n)[None, :]
    Qfull, _ = scipy.linalg.qr(V, mode="full")     # first n columns = +-V
    lam = np.concatenate([mu, np.zeros(K - n)])
    return _sign_fix(Qfull), lam


def random_orthogonal(dim: int, seed: int) -> np.ndarray:
    """Haar-distributed orthogonal matrix (QR of a seeded Gaussian, R's diagonal
    made positive).  Stands for the data-independent rotation of the 4-bit
    subspace, one per distinct dimension, drawn once with a fixed seed."""
    A = np.random.default_rng([seed, 0x52, dim]).standard_normal((dim, dim))
    Qm, Rm = np.linalg.qr(A)
    d = np.sign(np.diag(Rm))
    d[d == 0] = 1.0
    return Qm * d[None, :]


@dataclass
class LayerInputs:
    shape: LayerShape
    x_bits: np.ndarray     # [M,K] uint16, bfloat16 activations
    Q32: np.ndarray        # [K,K] float32 orthogonal basis, column j = j-th direction
    Q_bits: np.ndarray     # [K,K] uint16, bfloat16 cast of Q32
    W: np.ndarray          # [N,K] float32 weights (y = W x)
    eigenvalues: np.ndarray  # [K] float64, descending


def make_layer(shape: LayerShape, seed: int = 0, residual_rotation: bool = False,
               M: int | None = None) -> LayerInputs:
    """Draw all inputs of one layer.  `M` overrides the token count (the draws of
    the first rows do not depend on it).  With `residual_rotation` the last K-r
    basis columns are mixed by a random orthogonal matrix, Q = [U_h, U_l R]."""
    K, N = shape.K, shape.N
    M = shape.M if M is None else M
    s = channel_scales(shape, seed)
    Zc = _rng(seed, shape, 2).standard_normal((N_CALIB, K), dtype=np.float32)
    Q, lam = pca_basis(Zc * s[None, :])
    del Zc
    if residual_rotation and shape.r < K:
        R = random_orthogonal(K - shape.r, seed)
        Q = np.concatenate([Q[:, :shape.r], Q[:, shape.r:] @ R], axis=1)
    Q32 = np.ascontiguousarray(Q, dtype=np.float32)
    del Q
    Z = _rng(seed, shape, 3).standard_normal((M, K), dtype=np.float32)
    x_bits = to_bf16_bits(Z * s[None, :])
    del Z
    W = (_rng(seed, shape, 4).standard_normal((N, K), dtype=np.float32)
         / np.float32(np.sqrt(K)))
    return LayerInputs(shape, x_bits, Q32, to_bf16_bits(Q32), W, lam)


def make_activations(shape: LayerShape, M: int, seed: int = 0) -> np.ndarray:
    """Only the activations of `make_layer` (same draws), as bf16 bits [M,K]."""
    s = channel_scales(shape, seed)
    Z = _rng(seed, shape, 3).standard_normal((M, shape.K), dtype=np.float32)
    return to_bf16_bits(Z * s[None, :])
