"""The MiLo compression loop (Algorithm 1 of the paper) in fp64.

Test infrastructure only (see the package docstring).

Algorithm 1 alternates two steps on one weight W [N x K] until a stop rule fires:

  quantization step (Section 3.2, "Optimizing W_q with U, V fixed"): with the target
      R = W - U V and the scales s kept fixed, a few half-quadratic iterations move the zero-points z:
          W_q  = clamp(round(R / s + z), 0, 7)                       (Eq. update_z, second line; Eq. wq)
          W_dq = s (W_q - z)                                          (Eq. wdq)
          M    = shrink_lp(R - W_dq, beta)                            (Eq. update_We)
          z    = < W_q - (R - M) / s >   (mean over the group)        (Eq. update_z)
      with shrink_lp(x, beta) = sign(x) relu(|x| - |x|^(p-1) / beta);
  compensation step ("Solving U, V with W_q fixed"): E = W - W_dq, truncated SVD, U = U^ S^(1/2),
      V = S^(1/2) V^ (Eq. UV);
  error eps_t = || W - W_dq - U V ||_F (Eq. epsilon) and the stop rule on its three-iteration sliding
      mean (Eq. stop_condition), with the early stop at 20 iterations.

Readings where the paper is silent (it refers to the HQQ solver for the details of the inner loop):
  - s is the round-to-nearest scale of W itself, fp16((max - min) / 7) per group of 64, computed once
    and never changed ("we fix the scaling parameter"); a group whose scale is zero or not finite takes
    s = 1, as in quantize_rtn;
  - z starts at -min / s of W's group, real-valued, and is carried from one outer iteration to the next;
  - the inner loop runs a fixed number of iterations (default 20) with p = 0.7, beta = 10 growing by
    the factor 1.01 per iteration, restarted at every outer iteration; no early exit;
  - the sliding mean uses the iterations available so far (one, then two, then three), and the rule is
    first applied at the second iteration;
  - the outputs are the codes recomputed with z rounded to fp16 (what the packed format stores), that z,
    s, and U, V in fp64 (to be quantized by quantize_compensator, Algorithm 1's last line).
"""
import numpy as np

from .compensator import svd_compensator

GROUP = 64
QMAX = 7


def shrink_lp(x, beta, p):
    """Generalized soft-thresholding operator of Eq. update_We."""
    x = np.asarray(x, dtype=np.float64)
    ax = np.abs(x)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.where(ax > 0, ax ** (p - 1.0), 0.0) / beta
    return np.sign(x) * np.maximum(ax - t, 0.0)


def fixed_scales(W):
    """fp16 scales of the round-to-nearest quantizer of W (the ones Algorithm 1 keeps fixed) and the
    matching real-valued starting zero-points -min / s.  Both [N, K / 64]."""
    W = np.asarray(W, dtype=np.float32)
    N, K = W.shape
    Wg = W.reshape(N, K // GROUP, GROUP)
    mn, mx = Wg.min(axis=-1), Wg.max(axis=-1)
    with np.errstate(over="ignore", invalid="ignore"):
        s16 = ((mx - mn) / np.float32(QMAX)).astype(np.float16)
    bad = ~(np.isfinite(s16) & (s16 > 0))
    s16 = np.where(bad, np.float16(1), s16)
    z0 = -mn.astype(np.float64) / s16.astype(np.float64)
    return s16, z0


def quantize_with(R, s, z):
    """Codes and dequantized weight of the target R for given scales and zero-points (Eq. wq / wdq)."""
    N, K = R.shape
    Rg = R.reshape(N, K // GROUP, GROUP)
    q = np.clip(np.rint(Rg / s[..., None] + z[..., None]), 0, QMAX)
    return q.reshape(N, K), (s[..., None] * (q - z[..., None])).reshape(N, K)


def hqq_zero_points(R, s, z, iters=20, p=0.7, beta=10.0, kappa=1.01):
    """The inner loop: `iters` half-quadratic updates of z for the target R with fixed scales s."""
    N, K = R.shape
    s = np.asarray(s, dtype=np.float64)
    z = np.array(z, dtype=np.float64)
    Rg = R.reshape(N, K // GROUP, GROUP)
    for _ in range(iters):
        q = np.clip(np.rint(Rg / s[..., None] + z[..., None]), 0, QMAX)
        Wdq = s[..., None] * (q - z[..., None])
        M = shrink_lp(Rg - Wdq, beta, p)
        z = np.mean(q - (Rg - M) / s[..., None], axis=-1)
        beta *= kappa
    return z


def stop_rule(eps, tol=1e-4):
    """True if the three-iteration sliding mean of the errors so far has stopped improving
    (Eq. stop_condition) or has started to grow."""
    if len(eps) < 2:
        return False
    cur = np.mean(eps[-3:])
    prev = np.mean(eps[-4:-1]) if len(eps) >= 4 else np.mean(eps[:-1])
    return (prev - cur) / prev < tol


def milo_compress(W, r, iters=20, hqq_iters=20, p=0.7, beta=10.0, kappa=1.01, tol=1e-4):
    """Algorithm 1.  Returns a dict with codes (uint8), scales and zeros (fp16), U [N, r], V [r, K]
    (fp64), and eps, the list of errors eps_t of the iterations run."""
    W64 = np.asarray(W, dtype=np.float64)
    N, K = W64.shape
    s16, z = fixed_scales(W)
    s = s16.astype(np.float64)
    U = np.zeros((N, r))
    V = np.zeros((r, K))
    eps = []
    for _ in range(iters):
        R = W64 - U @ V
        z = hqq_zero_points(R, s, z, hqq_iters, p, beta, kappa)
        _, Wdq = quantize_with(R, s, z)
        if r > 0:
            U, V, _ = svd_compensator(W64 - Wdq, r)
        eps.append(float(np.linalg.norm(W64 - Wdq - U @ V)))
        if stop_rule(eps, tol):
            break
    z16 = np.clip(z, -65504, 65504).astype(np.float16)
    q, _ = quantize_with(W64 - U @ V, s, z16.astype(np.float64))
    return dict(codes=q.astype(np.uint8), scales=s16, zeros=z16, U=U, V=V, eps=eps)
