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


# ---------------------------------------------------------------- INT3 compensator (Eq. symm_int3)

def _factors(N=128, K=192, r=20, seed=3):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((N, r)) * 0.05).astype(np.float32), (rng.standard_normal((r, K)) * 0.05).astype(np.float32)


def test_quantized_compensator_is_the_printed_equation_per_group():
    # exact rationals on a dyadic example: q = round(7 w / (2 s)) + 4 with s the group's largest
    # magnitude, groups of 64 along N for U and along K for V; dequantization (q - 4) * 2 s / 7
    from fractions import Fraction
    from oracle import quantize_compensator, dequantize_compensator
    N, K, r = 64, 64, 2
    U = np.zeros((N, r), np.float32)
    V = np.zeros((r, K), np.float32)
    U[:, 0] = np.linspace(-1.75, 1.75, N)          # s = 1.75 -> step 0.5, exact in fp16
    U[:, 1] = 3.5                                  # s = 3.5 -> step 1: all codes clamp to 7
    V[0] = np.linspace(1.75, -1.75, K)
    V[1, 5] = -7.0                                 # s = 7 -> step 2
    (qu, su, zu), (qv, sv, zv) = quantize_compensator(U, V)
    assert qu.shape == (16, N) and qv.shape == (16, K)                  # rank padded to 16 rows
    assert np.all(zu == 4) and np.all(zv == 4)
    for mat, q, s in ((U.T, qu, su), (V, qv, sv)):
        for j in range(r):
            smax = max(abs(Fraction(float(x))) for x in mat[j])
            assert Fraction(float(s[j, 0])) == 2 * smax / 7
            for n in range(64):
                t = Fraction(7) * Fraction(float(mat[j, n])) / (2 * smax)
                want = min(max(round(t) + 4, 0), 7)                      # Python rounds halves to even
                assert int(q[j, n]) == want, (j, n)
    assert np.all(qu[2:] == 4) and np.all(qv[2:] == 4)                  # padded ranks dequantize to zero
    Ud, Vd = dequantize_compensator((qu, su, zu), (qv, sv, zv), r)
    assert Ud.shape == (N, r) and Vd.shape == (r, K)
    # -s maps to round(-3.5) + 4 = 0 (four steps below zero), +s to 8, clamped to 7 (three steps above)
    assert Ud[0, 0] == -2.0 and Ud[-1, 0] == 1.5 and np.all(Ud[:, 1] == 3.0) and Vd[1, 5] == -8.0


def test_quantized_compensator_groups_run_along_the_long_dimension():
    # one huge entry coarsens only the 64 features (U) / columns (V) of its own rank and group
    from oracle import quantize_compensator, dequantize_compensator
    U, V = _factors()
    U2, V2 = U.copy(), V.copy()
    U2[70, 3] = 50.0
    V2[3, 130] = 50.0
    a = dequantize_compensator(*quantize_compensator(U, V), U.shape[1])
    b = dequantize_compensator(*quantize_compensator(U2, V2), U.shape[1])
    du, dv = a[0] != b[0], a[1] != b[1]
    assert du[64:128, 3].any() and not du[:64].any() and not np.delete(du, 3, axis=1).any()
    assert dv[3, 128:192].any() and not dv[:, :128].any() and not np.delete(dv, 3, axis=0).any()


def test_quantized_compensator_error_bound_and_size():
    from oracle import quantize_compensator, dequantize_compensator, pack_w3
    U, V = _factors(N=256, K=320, r=32, seed=9)
    uq, vq = quantize_compensator(U, V)
    Ud, Vd = dequantize_compensator(uq, vq, 32)
    stepU = np.repeat(uq[1].astype(np.float64)[:32], 64, axis=1).T      # [N, r]
    stepV = np.repeat(vq[1].astype(np.float64)[:32], 64, axis=1)
    # half a step; at the positive extreme the clamp to code 7 costs half a step too, and the fp16
    # rounding of the step moves w / d by up to 3.5 * 2^-11 there
    assert np.all(np.abs(U - Ud) <= stepU * (0.5 + 3.5 * 2.0 ** -11) + 1e-12)
    assert np.all(np.abs(V - Vd) <= stepV * (0.5 + 3.5 * 2.0 ** -11) + 1e-12)
    # 3.5 bits per element (3-bit codes + two fp16 words per 64), against 16 for fp16 factors
    assert pack_w3(*uq).size + pack_w3(*vq).size == 32 * (256 + 320) * 7 // 16
