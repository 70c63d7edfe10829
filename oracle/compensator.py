"""Low-rank compensator of the quantization residual (workload preparation).

Test infrastructure only (see the package docstring).

Section 3.2.3, Eq. compensate / Eq. UV: with E = W - W_dq = U^ S V^ (SVD),
    U = U^[:, :r] sqrt(S_r),     V = sqrt(S_r) V^[:r, :],
which is the best rank-r approximation of E in the Frobenius norm
(Eckart-Young-Mirsky).  The result is cast to fp16 by the caller; U, V are
*inputs* to both the oracle linear and the GPU kernel.

`randomized_svd_compensator` is the approximate variant for the large shapes:
the paper's own implementation (appendix "Implementation") uses an approximate
randomized SVD routine as well.  It is a seeded range finder with oversampling
and power iterations followed by an exact SVD of the small projected matrix.
"""
import numpy as np


def _split(Uh, S, Vh, r):
    rs = np.sqrt(S[:r])
    return Uh[:, :r] * rs[None, :], rs[:, None] * Vh[:r, :]


def svd_compensator(E, r):
    """Exact truncated SVD factors of E (fp64): returns U [N,r], V [r,K], singular values."""
    E = np.asarray(E, dtype=np.float64)
    Uh, S, Vh = np.linalg.svd(E, full_matrices=False)
    U, V = _split(Uh, S, Vh, r)
    return U, V, S


def randomized_svd_compensator(E, r, seed, oversample=10, power_iters=2):
    E = np.asarray(E, dtype=np.float64)
    N, K = E.shape
    if r == 0:
        return np.zeros((N, 0)), np.zeros((0, K))
    rng = np.random.default_rng(seed)
    k = min(r + oversample, min(N, K))
    Q, _ = np.linalg.qr(E @ rng.standard_normal((K, k)))
    for _ in range(power_iters):
        Q, _ = np.linalg.qr(E.T @ Q)
        Q, _ = np.linalg.qr(E @ Q)
    B = Q.T @ E
    Ub, S, Vh = np.linalg.svd(B, full_matrices=False)
    return _split(Q @ Ub, S, Vh, r)


def quantize_compensator(U, V):
    """INT3 compensator (Section 3.2.3, Eq. symm_int3; the last step of Algorithm 1): both factors go
    through the symmetric INT3 quantizer in groups of 64 along their long dimension, U [N x r] along N
    and V [r x K] along K.  (The paper does not print the group axis; its memory table grows in exact
    proportion to the rank, which a group along the rank would not, and 64 is the group size of all its
    kernels.)  Returned in the stored form: (codes, scales, zeros) of U^T [rp x N] and of V [rp x K],
    rp = r rounded up to a multiple of 16 with zero rows added.
    """
    from .quantize import quantize_sym
    U = np.asarray(U, dtype=np.float32)
    V = np.asarray(V, dtype=np.float32)
    N, r = U.shape
    rp = (r + 15) // 16 * 16
    Ut = np.zeros((rp, N), np.float32)
    Ut[:r] = U.T
    Vp = np.zeros((rp, V.shape[1]), np.float32)
    Vp[:r] = V
    return quantize_sym(Ut), quantize_sym(Vp)


def dequantize_compensator(uq, vq, r):
    """fp64 U [N x r] and V [r x K] of a quantized compensator."""
    from .quantize import dequantize
    return dequantize(*uq)[:r].T.copy(), dequantize(*vq)[:r].copy()
