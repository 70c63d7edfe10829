"""Pins for the oracle of the MiLo compression loop (Algorithm 1; Section 3.2 Eq. update_We, update_z,
UV, epsilon, stop_condition)."""
import numpy as np

import oracle
from oracle import (milo_compress, hqq_zero_points, shrink_lp, fixed_scales, quantize_with, stop_rule,
                    quantize_rtn, dequantize, svd_compensator)


def _weight(N=64, K=256, seed=0, outliers=True):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    if outliers:
        W[:, rng.choice(K, 3, replace=False)] *= 8
    return W


def test_shrink_closed_forms():
    x = np.array([-3.0, -0.5, 0.0, 0.2, 4.0])
    # p = 1 is the soft threshold 1 / beta
    assert np.allclose(shrink_lp(x, 2.0, 1.0), np.sign(x) * np.maximum(np.abs(x) - 0.5, 0))
    # printed form, evaluated by hand at p = 0.5, beta = 4: |x| - |x|^-0.5 / 4
    assert np.isclose(shrink_lp(4.0, 4.0, 0.5), 4.0 - 0.5 / 4)
    assert shrink_lp(0.01, 4.0, 0.5) == 0.0                    # 0.01 - 10 / 4 < 0 -> relu
    assert np.all(shrink_lp(x, 1e30, 0.7) == x)                # beta -> infinity: identity
    assert np.all(np.sign(shrink_lp(x, 3.0, 0.7)) * np.sign(x) >= 0)
    assert np.all(np.abs(shrink_lp(x, 3.0, 0.7)) <= np.abs(x))


def test_fixed_scales_are_the_round_to_nearest_scales():
    W = _weight()
    q, s_rtn, z_rtn = quantize_rtn(W)
    s, z0 = fixed_scales(W)
    assert np.array_equal(s.view(np.uint16), s_rtn.view(np.uint16))
    # the starting zero-point is the unrounded -min / s; rounded it is the round-to-nearest zero-point
    assert np.array_equal(np.rint(z0).astype(np.float16), z_rtn)


def test_zero_point_update_by_hand_and_fixed_point():
    # one group, one update, written out element by element (Eq. update_We, update_z)
    rng = np.random.default_rng(5)
    R = (rng.standard_normal((1, 64)) * 0.03)
    s = np.array([[0.011]]); z = np.array([[3.3]]); beta, p = 10.0, 0.7
    want = 0.0
    for k in range(64):
        q = min(max(round(R[0, k] / 0.011 + 3.3), 0), 7)
        e = R[0, k] - 0.011 * (q - 3.3)
        m = np.sign(e) * max(abs(e) - abs(e) ** (p - 1) / beta, 0.0) if e != 0 else 0.0
        want += q - (R[0, k] - m) / 0.011
    got = hqq_zero_points(R, s, z, iters=1, p=p, beta=beta)
    assert np.isclose(got[0, 0], want / 64, rtol=1e-12)
    # with the shrinkage switched off (beta -> infinity, M = R - W_dq) z is a fixed point:
    # < W_q - (R - M) / s > = < W_q - W_dq / s > = z
    assert np.allclose(hqq_zero_points(R, s, z, iters=3, p=p, beta=1e300), z, rtol=1e-12)


def test_first_iteration_without_inner_loop_is_plain_quantize_then_compensate():
    # zero inner iterations and one outer one: real-valued zero-point -min / s, codes from Eq. wq with
    # U = V = 0, compensator = truncated SVD of the residual (the pinned svd_compensator)
    W = _weight(seed=2)
    out = milo_compress(W, r=8, iters=1, hqq_iters=0)
    s, z0 = fixed_scales(W)
    _, Wdq = quantize_with(W.astype(np.float64), s.astype(np.float64), z0)
    U, V, S = svd_compensator(W.astype(np.float64) - Wdq, 8)
    assert np.allclose(out["U"] @ out["V"], U @ V, atol=1e-12)
    assert np.isclose(out["eps"][0], np.sqrt(np.sum(S[8:] ** 2)), rtol=1e-9)       # Eckart-Young
    # stored form: fp16 zero-point, codes recomputed with it from W - U V
    q, _ = quantize_with(W.astype(np.float64) - out["U"] @ out["V"], s.astype(np.float64),
                         out["zeros"].astype(np.float64))
    assert np.array_equal(out["codes"], q.astype(np.uint8)) and out["codes"].max() <= 7


def test_inner_loop_lowers_the_lp_error_and_outer_loop_the_frobenius_error():
    W = _weight(N=96, K=512, seed=3)
    s16, z0 = fixed_scales(W)
    s = s16.astype(np.float64)
    R = W.astype(np.float64)
    lp = lambda z: np.sum(np.abs(R - quantize_with(R, s, z)[1]) ** 0.7)
    z20 = hqq_zero_points(R, s, z0, iters=20)
    assert lp(z20) < lp(z0)                                       # what the half-quadratic solver minimises
    one = milo_compress(W, r=16, iters=1)
    many = milo_compress(W, r=16, iters=12, tol=-1.0)             # (tol < 0: never stop early)
    assert len(many["eps"]) == 12
    assert many["eps"][-1] < one["eps"][0]                        # the alternation pays (Fig. of eps_t)
    rtn_q, rtn_s, rtn_z = quantize_rtn(W)
    assert many["eps"][-1] < np.linalg.norm(W - dequantize(rtn_q, rtn_s, rtn_z))
    # rank 0: pure zero-point optimisation, no compensator
    z_only = milo_compress(W, r=0, iters=3, tol=-1.0)
    assert z_only["U"].shape == (96, 0) and len(z_only["eps"]) == 3


def test_stop_rule_on_printed_sequences():
    assert not stop_rule([1.0])
    assert not stop_rule([1.0, 0.9])                              # mean 0.95 against 1.0: still improving
    assert stop_rule([1.0, 1.0])                                  # no improvement
    assert stop_rule([1.0, 1.2])                                  # diverging
    seq = [1.0, 0.9, 0.85, 0.84, 0.8399, 0.83989, 0.839889]
    fired = [stop_rule(seq[:n]) for n in range(1, len(seq) + 1)]
    # sixth: windows (0.85, 0.84, 0.8399) -> (0.84, 0.8399, 0.83989), relative gain 4.0e-3: go on;
    # seventh: (0.84, 0.8399, 0.83989) -> (0.8399, 0.83989, 0.839889), relative gain 4.4e-5 < 1e-4: stop
    assert fired == [False, False, False, False, False, False, True]


def test_output_is_self_consistent_and_balanced():
    W = _weight(N=80, K=320, seed=7)
    out = milo_compress(W, r=12, iters=5)
    U, V = out["U"], out["V"]
    assert np.allclose(U.T @ U, V @ V.T, atol=1e-10)              # Eq. UV: both carry sqrt(S)
    assert out["zeros"].dtype == np.float16 and out["scales"].dtype == np.float16
    Wt = dequantize(out["codes"], out["scales"], out["zeros"]) + U @ V
    assert np.linalg.norm(W - Wt) <= out["eps"][-1] * 1.05       # (fp16 zero-points cost a little)
