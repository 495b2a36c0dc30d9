"""The synthetic input generators (CPU only): the basis is orthogonal, sorted by
variance, and the activations have the channel-outlier structure the paper shows."""
import numpy as np
import pytest

from paper_2605_16732_amd import inputs as I


def test_small_config_basis_is_orthogonal_and_sorted():
    L = I.make_layer(I.SMALL)
    K = I.SMALL.K
    Q = L.Q32.astype(np.float64)
    assert np.abs(Q.T @ Q - np.eye(K)).max() < 1e-5          # max-abs entry, fp64 evaluation
    assert np.all(np.diff(L.eigenvalues) <= 1e-9 * L.eigenvalues[0])
    # rotated calibration channels have variance = eigenvalue, descending
    # (appendix on PCA: Var(x_hat_j) = lambda_j)
    s = I.channel_scales(I.SMALL)
    Zc = np.random.default_rng([0, 0, 0, 2]).standard_normal((I.N_CALIB, K), dtype=np.float32)
    Xc = (Zc * s[None, :]).astype(np.float64)
    var = ((Xc @ Q) ** 2).mean(0)
    np.testing.assert_allclose(var, L.eigenvalues, rtol=1e-4, atol=1e-6 * L.eigenvalues[0])
    # rotation preserves token norms
    x = I.bf16_bits_to_f32(L.x_bits).astype(np.float64)
    np.testing.assert_allclose(np.linalg.norm(x @ Q, axis=1), np.linalg.norm(x, axis=1), rtol=1e-5)
    # bf16 copies are the casts of the fp32 arrays
    np.testing.assert_array_equal(L.Q_bits, I.to_bf16_bits(L.Q32))
    assert L.x_bits.shape == (256, K) and L.W.shape == (1152, K)
    # channel outliers: a few channels far above the median (paper, Fig. 1b: ~83x)
    col = np.abs(x).max(0)
    assert 40 < col.max() / np.median(col) < 400
    # after rotation the 4-bit part is far more uniform than the raw channels
    xr = np.abs(x @ Q)[:, I.SMALL.r:].max(0)
    assert xr.max() / np.median(xr) < 0.25 * col.max() / np.median(col)


def test_rank_deficient_calibration_completes_to_an_orthogonal_matrix():
    rng = np.random.default_rng(1)
    n, K = 24, 40
    Xc = rng.standard_normal((n, K)) * rng.lognormal(0, 1, K)
    Q, lam = I.pca_basis(Xc)
    assert np.abs(Q.T @ Q - np.eye(K)).max() < 1e-12
    sigma = Xc.T @ Xc / n
    # first n columns are eigenvectors with the listed eigenvalues, the rest span the null space
    np.testing.assert_allclose(sigma @ Q[:, :n], Q[:, :n] * lam[:n], atol=1e-9 * lam[0])
    assert np.abs(sigma @ Q[:, n:]).max() < 1e-9 * lam[0]
    assert np.all(np.diff(lam) <= 0)
    # and agrees with the direct route where both apply
    Xc2 = rng.standard_normal((64, 16))
    Qa, la = I.pca_basis(Xc2)
    lb, Ub = np.linalg.eigh(Xc2.T @ Xc2 / 64)
    np.testing.assert_allclose(la, lb[::-1], rtol=1e-10)
    np.testing.assert_allclose(np.abs(Qa.T @ Ub[:, ::-1]), np.eye(16), atol=1e-8)


def test_residual_rotation_keeps_orthogonality():
    # lemma of the paper: U_l R has orthonormal columns; [U_h, U_l R] stays orthogonal
    shp = I.LayerShape("t", 8, 96, 16, 16, 16, 2, 9, 1)
    L0 = I.make_layer(shp)
    L1 = I.make_layer(shp, residual_rotation=True)
    Q = L1.Q32.astype(np.float64)
    assert np.abs(Q.T @ Q - np.eye(96)).max() < 1e-5
    np.testing.assert_array_equal(L0.Q32[:, :16], L1.Q32[:, :16])
    assert np.abs(L0.Q32[:, 16:] - L1.Q32[:, 16:]).max() > 0.1
    R = I.random_orthogonal(80, 0)
    assert np.abs(R.T @ R - np.eye(80)).max() < 1e-12


def test_shapes_tables():
    assert [s.G for s in I.PIXART] == [17, 17, 17, 71]
    assert [s.G for s in I.FLUX] == [46, 46, 46, 190]
    assert len(I.ABLATION) == 12 and all((s.K - s.r) % s.g == 0 for s in I.ABLATION)
    assert [s.M for s in I.TOKEN_SWEEP] == [1024, 4096, 16384, 32768]


def test_seeded_and_prefix_stable():
    a = I.make_activations(I.SMALL, 8)
    b = I.make_activations(I.SMALL, 4)
    np.testing.assert_array_equal(a[:4], b)
    c = I.make_activations(I.SMALL, 4, seed=1)
    assert not np.array_equal(b, c)


def _max_orthogonality_defect(Q32: np.ndarray, block: int = 2048) -> float:
    """max |Q^T Q - I| with the fp32 matrix evaluated in fp64, upper triangle by blocks of columns."""
    K = Q32.shape[0]
    worst = 0.0
    for i0 in range(0, K, block):
        Qi = Q32[:, i0:i0 + block].astype(np.float64)
        for j0 in range(i0, K, block):
            Qj = Qi if j0 == i0 else Q32[:, j0:j0 + block].astype(np.float64)
            Gm = Qi.T @ Qj
            if j0 == i0:
                Gm -= np.eye(Gm.shape[0])
            worst = max(worst, float(np.abs(Gm).max()))
    return worst


@pytest.mark.parametrize("idx", [2, 3])
def test_benchmark_bases_are_orthogonal(idx):
    """The fp32 bases the benchmark and the full-size parity tests use -- K = 3072 (eigendecomposition of the
    second moment) and K = 12288 (2048 calibration rows: Gram-matrix eigenvectors completed by a full QR) --
    satisfy max |Q^T Q - I| < 1e-5 in fp64, as the small config's does."""
    shp = I.FLUX[idx]
    s = I.channel_scales(shp)
    Zc = np.random.default_rng([0, shp.config_id, shp.layer_id, 2]).standard_normal((I.N_CALIB, shp.K), dtype=np.float32)
    Q, lam = I.pca_basis(Zc * s[None, :])
    Q32 = np.ascontiguousarray(Q, dtype=np.float32)
    del Q, Zc
    assert Q32.shape == (shp.K, shp.K)
    assert _max_orthogonality_defect(Q32) < 1e-5
    assert np.all(np.diff(lam) <= 1e-9 * lam[0])
    # the same draws as make_layer: spot-check against it on the smaller basis
    if shp.K <= 4096:
        np.testing.assert_array_equal(I.make_layer(shp).Q32, Q32)
