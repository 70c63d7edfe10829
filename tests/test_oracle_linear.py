"""Pins for the compensated linear (Section 3.1.2: W~ = Q^-1(W_q) + U V) in the oracle."""
import numpy as np

from oracle import quantize_rtn, dequantize, w3lr_linear, linear_from_dense


def _case(M=3, N=16, K=128, r=2, seed=0):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    q, s, z = quantize_rtn(W)
    X = rng.standard_normal((M, K)).astype(np.float16)
    U = (rng.standard_normal((N, r)) * 0.05).astype(np.float16)
    V = (rng.standard_normal((r, K)) * 0.05).astype(np.float16)
    return X, q, s, z, U, V


def test_triple_loop_brute_force():
    X, q, s, z, U, V = _case()
    M, K = X.shape
    N, r = U.shape
    Y = w3lr_linear(X, q, s, z, U, V)
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                w = float(s[n, k // 64]) * (int(q[n, k]) - float(z[n, k // 64]))
                for j in range(r):
                    w += float(U[n, j]) * float(V[j, k])
                acc += float(X[m, k]) * w
            assert abs(acc - Y[m, n]) <= 1e-12 * max(1.0, abs(acc))


def test_rank_zero_is_plain_matmul():
    X, q, s, z, _, _ = _case(M=5, N=32, K=192)
    ref = np.matmul(X.astype(np.float64), dequantize(q, s, z).T)
    assert np.array_equal(w3lr_linear(X, q, s, z), ref)
    U0 = np.zeros((32, 0), np.float16)
    V0 = np.zeros((0, 192), np.float16)
    assert np.array_equal(w3lr_linear(X, q, s, z, U0, V0), ref)


def test_one_hot_activations_return_compensated_weight():
    X, q, s, z, U, V = _case(N=32, K=128, r=3)
    K = 128
    I = np.eye(K, dtype=np.float16)
    Y = w3lr_linear(I, q, s, z, U, V)                       # [K, N]
    Wt = dequantize(q, s, z) + U.astype(np.float64) @ V.astype(np.float64)
    assert np.allclose(Y, Wt.T, rtol=0, atol=1e-15)
    # a transposed or swapped compensator would not survive this
    assert not np.allclose(Y, (dequantize(q, s, z)).T, atol=1e-6)


def test_integer_special_case_exact():
    rng = np.random.default_rng(3)
    N, K, M = 16, 256, 7
    q = rng.integers(0, 8, size=(N, K), dtype=np.uint8)
    s = np.ones((N, K // 64), np.float16)
    z = np.zeros((N, K // 64), np.float16)
    X = rng.integers(-1, 2, size=(M, K)).astype(np.float16)
    Y = w3lr_linear(X, q, s, z)
    ref = X.astype(np.int64) @ q.astype(np.int64).T
    assert np.array_equal(Y, ref.astype(np.float64))


def test_linearity_and_low_rank_part():
    X, q, s, z, U, V = _case(M=4, N=16, K=128, r=4, seed=9)
    X2 = np.random.default_rng(1).standard_normal(X.shape).astype(np.float16)
    f = lambda A: w3lr_linear(A, q, s, z, U, V)
    a, b = 0.5, -2.0            # exact in fp16, so a*X + b*X2 stays exact in fp64
    lhs = linear_from_dense(a * X.astype(np.float64) + b * X2.astype(np.float64),
                            dequantize(q, s, z), U, V)
    assert np.allclose(lhs, a * f(X) + b * f(X2), rtol=1e-12, atol=1e-12)
    # difference between rank-r and rank-0 output is exactly X (UV)^T
    d = f(X) - w3lr_linear(X, q, s, z)
    ref = X.astype(np.float64) @ (U.astype(np.float64) @ V.astype(np.float64)).T
    assert np.allclose(d, ref, rtol=1e-10, atol=1e-12)
