"""Pins for the oracle's MoE layer (SwiGLU experts, top-k gate-weighted combine)."""
import numpy as np

from oracle import quantize_rtn, w3lr_linear, moe_forward, silu


def _weight(N, K, r, rng):
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    q, s, z = quantize_rtn(W)
    U = (rng.standard_normal((N, r)) * 0.05).astype(np.float16)
    V = (rng.standard_normal((r, K)) * 0.05).astype(np.float16)
    return dict(codes=q, scales=s, zeros=z, U=U, V=V)


def _expert(H, F, r, rng):
    return dict(w1=_weight(F, H, r, rng), w3=_weight(F, H, r, rng), w2=_weight(H, F, r, rng))


def test_silu_closed_values():
    assert silu(np.float64(0.0)) == 0.0
    x = np.array([-3.0, -0.5, 0.7, 4.0])
    assert np.allclose(silu(x) - silu(-x), x)            # x*sig(x) - (-x)*sig(-x) = x
    assert np.isclose(silu(np.float64(1.0)), 1.0 / (1.0 + np.exp(-1.0)))
    assert np.isclose(silu(np.float64(40.0)), 40.0)


def test_single_expert_is_three_chained_linears():
    rng = np.random.default_rng(0)
    H, F, T = 64, 128, 5
    ex = _expert(H, F, 2, rng)
    X = rng.standard_normal((T, H)).astype(np.float16)
    ids = np.zeros((T, 1), np.int32)
    g = np.ones((T, 1), np.float32)
    Y = moe_forward(X, [ex], ids, g)
    a = w3lr_linear(X, **ex["w1"])
    b = w3lr_linear(X, **ex["w3"])
    h = a / (1 + np.exp(-a)) * b
    ref = w3lr_linear(h, **ex["w2"])
    assert np.allclose(Y, ref, rtol=1e-13, atol=1e-13)


def test_identical_experts_sum_gates_and_permutation():
    rng = np.random.default_rng(1)
    H, F, T, E, k = 64, 64, 12, 4, 2
    ex = _expert(H, F, 1, rng)
    X = rng.standard_normal((T, H)).astype(np.float16)
    ids = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    g = rng.random((T, k)).astype(np.float32)
    Y = moe_forward(X, [ex] * E, ids, g)
    one = moe_forward(X, [ex], np.zeros((T, 1), np.int32), np.ones((T, 1), np.float32))
    assert np.allclose(Y, g.astype(np.float64).sum(1, keepdims=True) * one, rtol=1e-12, atol=1e-12)
    # distinct experts: permuting tokens permutes outputs
    exs = [_expert(H, F, 2, rng) for _ in range(E)]
    Y1 = moe_forward(X, exs, ids, g)
    perm = rng.permutation(T)
    Y2 = moe_forward(X[perm], exs, ids[perm], g[perm])
    assert np.allclose(Y2, Y1[perm], rtol=1e-12, atol=1e-12)
    # swapping the slot order of a token does not change its output
    Y3 = moe_forward(X, exs, ids[:, ::-1], g[:, ::-1])
    assert np.allclose(Y3, Y1, rtol=1e-12, atol=1e-12)


def test_empty_expert_and_lazy_experts():
    rng = np.random.default_rng(2)
    H, F, T = 64, 64, 6
    exs = [_expert(H, F, 1, rng) for _ in range(3)]
    X = rng.standard_normal((T, H)).astype(np.float16)
    ids = np.array([[0, 2]] * T, np.int32)             # expert 1 receives nothing
    g = np.full((T, 2), 0.5, np.float32)
    called = []

    def lazy(i):
        def make():
            called.append(i)
            return exs[i]
        return make

    Y = moe_forward(X, [lazy(0), lazy(1), lazy(2)], ids, g)
    assert called == [0, 2]
    ref = 0.5 * moe_forward(X, [exs[0]], np.zeros((T, 1), np.int32), np.ones((T, 1), np.float32)) \
        + 0.5 * moe_forward(X, [exs[2]], np.zeros((T, 1), np.int32), np.ones((T, 1), np.float32))
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-12)
