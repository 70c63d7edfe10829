"""Pins for the compensator construction (Section 3.2.3, Eq. compensate / Eq. UV)."""
import numpy as np

from oracle import quantize_rtn, dequantize, svd_compensator, randomized_svd_compensator


def _residual(N=96, K=128, seed=0):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    q, s, z = quantize_rtn(W)
    Wdq = dequantize(q, s, z)
    return W.astype(np.float64), Wdq


def test_full_rank_reconstructs_weight():
    W, Wdq = _residual()
    U, V, S = svd_compensator(W - Wdq, min(W.shape))
    assert np.allclose(Wdq + U @ V, W, rtol=0, atol=1e-15)


def test_eckart_young_and_balance():
    W, Wdq = _residual()
    E = W - Wdq
    for r in (1, 8, 32):
        U, V, S = svd_compensator(E, r)
        assert U.shape == (96, r) and V.shape == (r, 128)
        err2 = np.linalg.norm(E - U @ V, "fro") ** 2
        assert np.isclose(err2, np.sum(S[r:] ** 2), rtol=1e-10)
        # Eq. UV splits the singular values evenly: U^T U = V V^T = diag(S_r)
        assert np.allclose(U.T @ U, np.diag(S[:r]), atol=1e-12)
        assert np.allclose(V @ V.T, np.diag(S[:r]), atol=1e-12)
        assert np.linalg.norm(E - U @ V) < np.linalg.norm(E)
    # no rank-r matrix does better than the truncated SVD (spot check with random ones)
    rng = np.random.default_rng(1)
    U, V, S = svd_compensator(E, 4)
    best = np.linalg.norm(E - U @ V)
    for _ in range(5):
        A = U + 1e-3 * rng.standard_normal(U.shape)
        assert np.linalg.norm(E - A @ V) >= best


def test_randomized_matches_exact_on_small():
    W, Wdq = _residual(N=128, K=192, seed=4)
    E = W - Wdq
    # a residual with a clear low-rank part on top of the quantization noise
    rng = np.random.default_rng(2)
    E = E + 0.05 * rng.standard_normal((128, 6)) @ rng.standard_normal((6, 192))
    U, V, S = svd_compensator(E, 6)
    Ur, Vr = randomized_svd_compensator(E, 6, seed=7)
    assert np.allclose(Ur @ Vr, U @ V, atol=1e-6)
    assert np.linalg.norm(E - Ur @ Vr) <= np.linalg.norm(E - U @ V) * (1 + 1e-6)
    U0, V0 = randomized_svd_compensator(E, 0, seed=1)
    assert U0.shape == (128, 0) and V0.shape == (0, 192)
