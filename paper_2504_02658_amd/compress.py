"""Workload preparation on the GPU: fit the low-rank compensator to a packed weight.

Not on the inference hot path.  Section 3.2.3 (Eq. compensate / Eq. UV): with the residual
E = W - W_dq, U = U^_r sqrt(S_r) and V = sqrt(S_r) V^_r from a truncated SVD.  As in the
paper's own implementation (appendix "Implementation") the SVD is the randomized routine
torch.svd_lowrank; W_dq comes from the library's own dequantization kernel.
"""
import torch

from . import api


def fit_compensator(W, pw, r, niter=2, oversample=10, seed=0):
    """W fp32 CUDA [N, K], pw = api.pack_w3(W)  ->  PackedWeight with fp16 U [N, r], V [r, K]."""
    if r == 0:
        return pw
    E = W - api.dequant_w3(pw).float()
    gen_state = torch.random.get_rng_state()
    torch.manual_seed(seed)
    try:
        Uh, S, Vh = torch.svd_lowrank(E, q=min(r + oversample, min(E.shape)), niter=niter)
    finally:
        torch.random.set_rng_state(gen_state)
    rs = torch.sqrt(S[:r])
    U = (Uh[:, :r] * rs[None, :]).to(torch.float16).contiguous()
    V = (rs[:, None] * Vh[:, :r].T).to(torch.float16).contiguous()
    return pw.with_compensator(U, V)


def clone_weight(pw):
    """A byte-identical copy at new addresses (used to rotate weights through HBM in benchmarks)."""
    return api.PackedWeight(pw.N, pw.K, pw.q3.clone(),
                            None if pw.U is None else pw.U.clone(),
                            None if pw.V is None else pw.V.clone())
