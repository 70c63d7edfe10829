"""Shared plumbing of the GPU parity tests: build one workload on both sides and compare."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import oracle
from paper_2504_02658_amd import workloads as wl

REL_FRO_TOL = 1e-3          # relative Frobenius error against the fp64 oracle
MAX_ABS_TOL = 2e-2          # max |err| as a fraction of max |Y_ref|


def assert_close(Y_gpu, Y_ref, what=""):
    Y = np.asarray(Y_gpu, dtype=np.float64)
    R = np.asarray(Y_ref, dtype=np.float64)
    assert Y.shape == R.shape, (Y.shape, R.shape)
    assert np.all(np.isfinite(Y)), f"{what}: non-finite output"
    denom = np.linalg.norm(R)
    rel = np.linalg.norm(Y - R) / denom if denom > 0 else np.linalg.norm(Y - R)
    mx = np.max(np.abs(Y - R)) / max(np.max(np.abs(R)), 1e-30)
    assert rel <= REL_FRO_TOL, f"{what}: relative Frobenius error {rel:.3e} > {REL_FRO_TOL}"
    assert mx <= MAX_ABS_TOL, f"{what}: max abs error {mx:.3e} of max|Y_ref| > {MAX_ABS_TOL}"
    return rel, mx


def oracle_weight(W, r, seed=0, exact_svd_limit=1024 * 1024, symmetric=False):
    """Quantize W on the CPU and fit the rank-r compensator to the residual."""
    q, s, z = oracle.quantize_sym(W) if symmetric else oracle.quantize_rtn(W)
    if r > 0:
        E = W.astype(np.float64) - oracle.dequantize(q, s, z)
        if W.size <= exact_svd_limit:
            U, V, _ = oracle.svd_compensator(E, r)
        else:
            U, V = oracle.randomized_svd_compensator(E, r, seed=seed)
        U, V = U.astype(np.float16), V.astype(np.float16)
    else:
        U = np.zeros((W.shape[0], 0), np.float16)
        V = np.zeros((0, W.shape[1]), np.float16)
    return dict(codes=q, scales=s, zeros=z, U=U, V=V)


def gpu_weight(W, ow, check_pack=True, symmetric=False):
    """Pack W with the library; the compensator comes from the oracle side as an input."""
    import torch
    from paper_2504_02658_amd import api
    pw = api.pack_w3(torch.from_numpy(W).cuda(), symmetric=symmetric)
    if check_pack:
        N, K = W.shape
        assert np.array_equal(pw.q3.cpu().numpy(), oracle.pack_w3(ow["codes"], ow["scales"], ow["zeros"])), \
            "packed weight differs"
    if ow["U"].shape[1] > 0:
        pw = pw.with_compensator(torch.from_numpy(ow["U"]).cuda(), torch.from_numpy(ow["V"]).cuda())
    return pw


def int3_weight(W, ow):
    """The same weight with its compensator INT3-quantized on both sides (Section 3.2.3, Eq. symm_int3):
    returns (oracle dict with the dequantized fp64 factors, library PackedWeight with the two blobs)."""
    import torch
    from paper_2504_02658_amd import api
    r = ow["U"].shape[1]
    pw = gpu_weight(W, dict(ow, U=np.zeros((W.shape[0], 0), np.float16)))
    if r == 0:
        return ow, pw
    U32, V32 = ow["U"].astype(np.float32), ow["V"].astype(np.float32)
    uq, vq = oracle.quantize_compensator(U32, V32)
    Ud, Vd = oracle.dequantize_compensator(uq, vq, r)
    u3, v3 = api.pack_lr3(torch.from_numpy(U32).cuda(), torch.from_numpy(V32).cuda())
    assert np.array_equal(u3.cpu().numpy(), oracle.pack_w3(*uq)) and np.array_equal(v3.cpu().numpy(), oracle.pack_w3(*vq))
    return dict(ow, U=Ud, V=Vd), pw.with_int3_compensator(u3, v3, r)


def to_bf16(x):
    """Round to bfloat16 (a torch CPU tensor; numpy has no such type)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(np.asarray(x, np.float32))).to(torch.bfloat16)


def build_moe(case, threads=8, int3=False, bf16=False):
    """Both sides of an MoE layer: list of oracle expert dicts and the library's MoELayer.
    int3: every compensator is INT3-quantized (on both sides).  bf16: the layer runs on bfloat16
    activations; the compensators are rounded to bfloat16 on both sides."""
    from paper_2504_02658_amd import api
    ranks = wl.expert_ranks(case)
    n_exp = case.E + case.n_shared

    def one(e):
        out = {}
        for which in ("w1", "w3", "w2"):
            W = wl.expert_weight(case, e, which)
            out[which] = (W, oracle_weight(W, ranks[e], seed=case.seed + 7 * e))
        return out

    with ThreadPoolExecutor(max_workers=threads) as pool:
        built = list(pool.map(one, range(n_exp)))
    o_experts, g_experts = [], []
    for b in built:
        if int3:
            pairs = {k: int3_weight(b[k][0], b[k][1]) for k in ("w1", "w3", "w2")}
            o_experts.append({k: pairs[k][0] for k in pairs})
            g_experts.append(tuple(pairs[k][1] for k in ("w1", "w3", "w2")))
        elif bf16:
            oe, ge = {}, []
            for k in ("w1", "w3", "w2"):
                W, ow = b[k]
                Ub, Vb = to_bf16(ow["U"]), to_bf16(ow["V"])
                oe[k] = dict(ow, U=Ub.float().numpy(), V=Vb.float().numpy())
                pw = gpu_weight(W, dict(ow, U=np.zeros((W.shape[0], 0), np.float16)))
                ge.append(pw.with_compensator(Ub.cuda(), Vb.cuda()) if ow["U"].shape[1] else pw)
            o_experts.append(oe)
            g_experts.append(tuple(ge))
        else:
            o_experts.append({k: b[k][1] for k in b})
            g_experts.append(tuple(gpu_weight(b[k][0], b[k][1]) for k in ("w1", "w3", "w2")))
        for k in b:
            b[k] = None
    layer = api.MoELayer(g_experts, case.H, case.F, bf16=bf16)
    return o_experts, layer
