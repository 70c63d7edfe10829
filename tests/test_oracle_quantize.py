"""Pins for the oracle's quantizer (Section 3.2, Eq. wq / wdq) against things other than itself."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import quantize_rtn, quantize_sym, dequantize


def _half_even(fr: Fraction) -> int:
    return round(fr)        # Python rounds exact rationals half-to-even


def test_dyadic_worked_example_exact_rationals():
    # One group whose values are multiples of 1/16 in [-1, 0.75]: every quantity is a
    # dyadic rational, so binary32 arithmetic is exact and the expected result follows
    # from Eq. wq by hand: range 1.75 -> s = 1.75/7 = 0.25, z = round(1/0.25) = 4,
    # code = round_half_even(w/0.25 + 4) = round_half_even(j/4 + 4) for w = j/16.
    js = list(range(-16, 13)) + [0] * 35           # 29 distinct values + padding, 64 total
    w = np.array([j / 16 for j in js], dtype=np.float32)[None, :].repeat(16, axis=0)
    q, s, z = quantize_rtn(w)
    assert s.dtype == np.float16 and z.dtype == np.float16 and q.dtype == np.uint8
    assert float(s[0, 0]) == 0.25 and float(z[0, 0]) == 4.0
    expect = [min(7, max(0, _half_even(Fraction(j, 4) + 4))) for j in js]
    assert q[0].tolist() == expect
    # ties really occur in this example and go to even: w=2/16 -> 4.5 -> 4 ; w=6/16 -> 5.5 -> 6
    assert expect[js.index(2)] == 4 and expect[js.index(6)] == 6
    # Eq. wdq
    wdq = dequantize(q, s, z)
    assert np.array_equal(wdq[0], 0.25 * (np.array(expect, dtype=np.float64) - 4.0))


def _scalar_reference(w_group):
    """Element-at-a-time binary32 evaluation of the same definition (independent code path)."""
    f = np.float32
    mn = f(min(w_group)); mx = f(max(w_group))
    s16 = np.float16(f(f(mx - mn) / f(7)))
    sf = f(s16)
    z16 = np.float16(np.rint(f(f(-mn) / sf)))
    zf = f(z16)
    out = []
    for w in w_group:
        t = f(f(f(w) / sf) + zf)
        out.append(int(min(7, max(0, np.rint(t)))))
    return out, s16, z16


def test_against_scalar_loop():
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((16, 256)) * 0.02).astype(np.float32)
    W[3, 64:128] += 0.5          # an all-positive group: zero-point goes negative
    W[5, 0:64] -= 0.7            # an all-negative group: zero-point above 7
    q, s, z = quantize_rtn(W)
    for n in (0, 3, 5, 15):
        for g in range(4):
            cq, cs, cz = _scalar_reference(W[n, 64 * g: 64 * g + 64])
            assert q[n, 64 * g: 64 * g + 64].tolist() == cq
            assert s[n, g] == cs and z[n, g] == cz
    assert z[3, 1] < 0 and z[5, 0] > 7      # the zero-point is not clamped to the code range


def test_closed_form_properties_gaussian():
    rng = np.random.default_rng(11)
    W = (rng.standard_normal((64, 1024)) * 0.02).astype(np.float32)
    q, s, z = quantize_rtn(W)
    assert q.min() == 0 and q.max() == 7
    Wg = W.reshape(64, 16, 64)
    qg = q.reshape(64, 16, 64)
    # the group minimum maps to code 0 and the maximum to 7 (6 only through fp16 rounding of s)
    amin = np.take_along_axis(qg, Wg.argmin(-1)[..., None], -1)[..., 0]
    amax = np.take_along_axis(qg, Wg.argmax(-1)[..., None], -1)[..., 0]
    assert np.all(amin == 0)
    assert np.all(amax >= 6) and np.mean(amax == 7) > 0.95
    # s is (max-min)/7 up to fp16 rounding; z is -min/s up to rounding to an integer
    sf = s.astype(np.float64)
    rng_ = (Wg.max(-1) - Wg.min(-1)).astype(np.float64)
    assert np.all(np.abs(sf * 7 - rng_) <= rng_ * 2.0 ** -11 * 1.01)
    zf = z.astype(np.float64)
    assert np.all(zf == np.rint(zf))
    assert np.all(np.abs(zf + Wg.min(-1) / sf) <= 0.5 + 1e-6)
    # elementwise error bound of round-to-nearest inside the clamp range, and the
    # uniform-noise closed form E[(err/s)^2] = 1/12
    err = (W.astype(np.float64) - dequantize(q, s, z)).reshape(64, 16, 64) / sf[..., None]
    assert np.max(np.abs(err)) <= 0.5 + 0.01
    assert 0.075 < np.mean(err ** 2) < 0.092


def test_clamp_is_needed_and_applied():
    # min = -0.875, max = 0.875: s = 1.75/7 = 0.25 exactly, -min/s = 3.5 rounds (half-even)
    # to z = 4, so the maximum maps to 0.875/0.25 + 4 = 7.5 which rounds to 8: the unclamped
    # Eq. wq leaves the 3-bit range and the clamp has to bring it back to 7.
    w = np.zeros((16, 64), dtype=np.float32)
    w[:, 0] = -0.875
    w[:, 1] = 0.875
    q, s, z = quantize_rtn(w)
    assert float(s[0, 0]) == 0.25 and float(z[0, 0]) == 4.0
    assert q[0, 1] == 7 and q[0, 0] == 0          # -3.5 + 4 = 0.5 -> 0 (half-even)
    assert q[0, 2] == 4
    assert q.max() == 7


def test_degenerate_groups():
    w = np.zeros((16, 128), dtype=np.float32)
    w[:, :64] = 0.3125                                # constant group
    w[:, 64:] = np.linspace(1.0, 1.0 + 1e-7, 64, dtype=np.float32)[None, :]  # range below fp16 resolution
    q, s, z = quantize_rtn(w)
    assert np.all(q == 0)
    assert np.all(s == np.float16(1))
    assert np.all(z[:, 0] == np.float16(-0.3125))
    wdq = dequantize(q, s, z)
    assert np.allclose(wdq[:, :64], 0.3125)
    assert np.allclose(wdq[:, 64:], 1.0, atol=1e-3)


def test_subnormal_scale_is_kept():
    # range 7 * 2^-20: the fp16 scale 2^-20 is subnormal but non-zero, so the group is
    # quantized normally and the codes of an exact ramp are exact.
    step = np.float32(2.0 ** -20)
    w = (np.arange(64) % 8).astype(np.float32) * step
    w = np.tile(w, (16, 1))
    q, s, z = quantize_rtn(w)
    assert float(s[0, 0]) == 2.0 ** -20 and float(z[0, 0]) == 0.0
    assert np.array_equal(q[0], (np.arange(64) % 8).astype(np.uint8))


def test_rejects_bad_shapes():
    with pytest.raises(ValueError):
        quantize_rtn(np.zeros((16, 100), np.float32))
    with pytest.raises(ValueError):
        quantize_rtn(np.zeros((16, 128), np.float32), group=128)


# ---- symmetric INT3 quantizer (Section 3.2.3, Eq. symm_int3) -------------------------------------

def test_sym_dyadic_worked_example_is_the_papers_equation():
    # Values j/16 with largest magnitude 14/16: s = 0.875, so 7 w / (2 s) = 4 w = j/4 exactly and the
    # step 2 s / 7 = 0.25 is exact in fp16.  Eq. symm_int3 evaluated with exact rationals must give
    # the oracle's codes; +s maps to round(3.5) + 4 = 8 and is clamped, -s to round(-3.5) + 4 = 0.
    js = list(range(-14, 15)) + [0] * 35
    w = np.array([j / 16 for j in js], dtype=np.float32)[None, :].repeat(16, axis=0)
    q, d, z = quantize_sym(w)
    assert q.dtype == np.uint8 and d.dtype == np.float16 and z.dtype == np.float16
    assert float(d[0, 0]) == 0.25 and np.all(z == np.float16(4))
    s_max = Fraction(14, 16)
    expect = [min(7, max(0, _half_even(7 * Fraction(j, 16) / (2 * s_max)) + 4)) for j in js]
    assert q[0].tolist() == expect
    assert expect[js.index(14)] == 7 and expect[js.index(-14)] == 0 and expect[js.index(0)] == 4
    assert expect[js.index(2)] == 4 and expect[js.index(6)] == 6        # ties go to even
    wdq = dequantize(q, d, z)
    assert np.array_equal(wdq[0], 0.25 * (np.array(expect, dtype=np.float64) - 4.0))


def test_sym_against_scalar_loop():
    f = np.float32
    rng = np.random.default_rng(15)
    W = (rng.standard_normal((16, 256)) * 0.02).astype(np.float32)
    W[2, 0:64] += 0.1
    q, d, z = quantize_sym(W)
    for n in (0, 2, 9):
        for g in range(4):
            grp = W[n, 64 * g: 64 * g + 64]
            amax = f(max(abs(float(v)) for v in grp))
            d16 = np.float16(f(f(amax + amax) / f(7)))
            df = f(d16)
            codes = [int(min(7, max(0, f(np.rint(f(f(v) / df)) + f(4))))) for v in grp]
            assert q[n, 64 * g: 64 * g + 64].tolist() == codes
            assert d[n, g] == d16


def test_sym_properties():
    rng = np.random.default_rng(16)
    W = (rng.standard_normal((64, 512)) * 0.02).astype(np.float32)
    q, d, z = quantize_sym(W)
    assert q.min() >= 0 and q.max() <= 7 and np.all(z == np.float16(4))
    Wg = W.reshape(64, 8, 64)
    qg = q.reshape(64, 8, 64)
    # the weight of largest magnitude sits 3.5 steps from zero, up to the fp16 rounding of the
    # step: code 7 when it is positive (from 7 or from the clamped 8), 0 or 1 when negative
    arg = np.abs(Wg).argmax(axis=-1)
    ext_w = np.take_along_axis(Wg, arg[..., None], -1)[..., 0]
    ext_q = np.take_along_axis(qg, arg[..., None], -1)[..., 0]
    assert np.all(np.where(ext_w > 0, ext_q == 7, ext_q <= 1))
    assert np.any((ext_w < 0) & (ext_q == 0))
    # rounding error at most half a step everywhere (largest magnitude is 3.5 steps, within fp16
    # rounding of the step), and about step^2 / 12 on average
    err = (W.astype(np.float64) - dequantize(q, d, z)).reshape(64, 8, 64)
    step = d.astype(np.float64)[..., None]
    assert np.all(np.abs(err) <= step * (0.5 + 4e-3))
    assert 0.07 < np.mean((err / step) ** 2) < 0.095
    # odd symmetry wherever the clamp is not involved: q(-w) = 8 - q(w)
    qn, dn, _ = quantize_sym(-W)
    assert np.array_equal(dn, d)
    inner = (q >= 1) & (q <= 7) & (qn >= 1)
    assert inner.mean() > 0.95
    assert np.array_equal(qn[inner].astype(int), 8 - q[inner].astype(int))
    # zero weights get code 4 and dequantize to exactly 0
    W0 = W.copy(); W0[:, ::7] = 0.0
    q0, d0, z0 = quantize_sym(W0)
    assert np.all(q0[:, ::7] == 4) and np.all(dequantize(q0, d0, z0)[:, ::7] == 0.0)


def test_sym_degenerate_group():
    W = np.zeros((16, 128), dtype=np.float32)
    W[:, 64:] = 1e-9                      # step below fp16 resolution
    q, d, z = quantize_sym(W)
    assert np.all(q == 4) and np.all(d == np.float16(1)) and np.all(dequantize(q, d, z) == 0.0)
