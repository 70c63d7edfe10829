"""Group-wise asymmetric round-to-nearest 3-bit quantizer and its inverse.

Test infrastructure only (see the package docstring).

Follows the paper's quantizer definition (Section 3.2, Eq. wq / wdq, taken with
U = V = 0, i.e. the first pass of Algorithm 1 before any compensator exists):

    W_q  = round(W / s + z)          W_dq = s * (W_q - z)

with one scale s and one zero-point z per group of 64 consecutive weights along
the input (K) dimension of a row of W (group size 64 is what the paper uses
throughout its experiments and what its kernel accepts).

Readings where the paper is silent (all listed in the design notes):
  * s = (max - min) / 7 of the group, rounded to fp16 *before* z and the codes
    are computed, so that the stored parameters are self-consistent;
  * z = round(-min / s), kept as a real-valued fp16 number (not clamped to 0..7);
    the codes are computed with the stored (fp16-rounded) z;
  * round = round-half-to-even; codes are clamped to 0..7;
  * all arithmetic is IEEE binary32, one rounding per operation, no fused
    multiply-add (numpy evaluates each ufunc separately, so this holds);
  * a group whose fp16 scale is zero or non-finite (constant group, or a range
    below fp16 resolution) stores s = 1, z = fp16(-min), codes 0, which
    dequantizes to the group minimum.
"""
import numpy as np

GROUP = 64
QMAX = 7
F16_MAX = np.float32(65504.0)


def quantize_rtn(W, group=GROUP):
    """W: float32 [N, K] -> (codes uint8 [N, K], scales fp16 [N, K/64], zeros fp16 [N, K/64])."""
    if group != GROUP:
        raise ValueError("group size must be 64")
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    if K % GROUP:
        raise ValueError("K must be a multiple of 64")
    Wg = W.reshape(N, K // GROUP, GROUP)
    mn = Wg.min(axis=-1)
    mx = Wg.max(axis=-1)
    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        s32 = (mx - mn) / np.float32(QMAX)
        s16 = s32.astype(np.float16)
        degenerate = ~(np.isfinite(s16) & (s16 > 0))
        sf = np.where(degenerate, np.float32(1), s16.astype(np.float32))
        z = np.rint(-mn / sf)
        z = np.clip(z, -F16_MAX, F16_MAX)
        z16 = z.astype(np.float16)
        zf = z16.astype(np.float32)
        t = Wg / sf[..., None]
        t = t + zf[..., None]
        q = np.clip(np.rint(t), 0, QMAX)
    q = np.where(degenerate[..., None], np.float32(0), q).astype(np.uint8)
    s16 = np.where(degenerate, np.float16(1), s16)
    with np.errstate(over="ignore"):
        z16 = np.where(degenerate, (-mn).astype(np.float16), z16)
    return q.reshape(N, K), s16, z16


def quantize_sym(W, group=GROUP):
    """Symmetric INT3 quantizer (Section 3.2.3, Eq. symm_int3): q = round(7 w / (2 s)) + 4 with s the
    largest magnitude of the group.  Returned in the same (codes, scales, zeros) form as
    quantize_rtn: the scale is the step d = 2 s / 7 and every zero-point is 4, so dequantize()
    gives d * (q - 4).

    Readings: the step is rounded to fp16 before the codes are computed (q = round(w / d) + 4 with
    the stored d, as for the asymmetric quantizer); round-half-to-even; the codes are clamped to
    0..7, which the equation needs because w = +s maps to round(3.5) + 4 = 8; a group whose fp16
    step is zero or not finite stores d = 1 and codes 4 (dequantizes to zero); binary32, one
    rounding per operation.
    """
    if group != GROUP:
        raise ValueError("group size must be 64")
    W = np.ascontiguousarray(W, dtype=np.float32)
    N, K = W.shape
    if K % GROUP:
        raise ValueError("K must be a multiple of 64")
    Wg = W.reshape(N, K // GROUP, GROUP)
    amax = np.abs(Wg).max(axis=-1)
    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        d32 = (amax + amax) / np.float32(QMAX)
        d16 = d32.astype(np.float16)
        degenerate = ~(np.isfinite(d16) & (d16 > 0))
        df = np.where(degenerate, np.float32(1), d16.astype(np.float32))
        t = np.rint(Wg / df[..., None])
        t = t + np.float32(4)
        q = np.clip(t, 0, QMAX)
    q = np.where(degenerate[..., None], np.float32(4), q).astype(np.uint8)
    d16 = np.where(degenerate, np.float16(1), d16)
    z16 = np.full(d16.shape, 4, dtype=np.float16)
    return q.reshape(N, K), d16, z16


def dequantize(codes, scales, zeros):
    """Eq. wdq in fp64: W_dq[n, k] = s[n, g] * (q[n, k] - z[n, g]), g = k // 64."""
    N, K = codes.shape
    q = codes.reshape(N, K // GROUP, GROUP).astype(np.float64)
    s = scales.astype(np.float64)[..., None]
    z = zeros.astype(np.float64)[..., None]
    return (s * (q - z)).reshape(N, K)
