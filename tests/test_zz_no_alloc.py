"""milo_w3lr_gemm_static (the entry point for callers that cannot allocate) against milo_w3lr_gemm:
same kernels on the library's own scratch array, so the outputs must agree bit for bit, also on a
second call with a smaller problem right after a larger one (the array keeps the last call's contents)."""
import numpy as np
import pytest

from paper_2504_02658_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _weight(N, K, r, seed):
    import torch
    from paper_2504_02658_amd import api
    rng = np.random.default_rng(seed)
    pw = api.pack_w3(torch.from_numpy(wl.gen_weight(N, K, seed=seed)).cuda())
    if r:
        U = torch.from_numpy((0.02 * rng.standard_normal((N, r))).astype(np.float16)).cuda()
        V = torch.from_numpy((0.02 * rng.standard_normal((r, K))).astype(np.float16)).cuda()
        pw = pw.with_compensator(U, V)
    return pw


def test_static_scratch_entry_matches_the_workspace_entry():
    import torch
    from paper_2504_02658_amd import api
    # two calls in a row, the second with a smaller input; decode kernel, then tiled kernel
    for shapes in (((16, 1024, 4096, 32), (4, 272, 1408, 8)),
                   ((96, 512, 2048, 24), (40, 256, 832, 0)),
                   ((16, 1024, 4096, 32), (48, 512, 4096, 24))):
        outs = []
        for (M, N, K, r) in shapes:
            pw = _weight(N, K, r, seed=M + N + K + r)
            X = torch.from_numpy(wl.gen_activations(M, K, seed=7 + M)).cuda()
            outs.append((X, pw, api.w3lr_gemm_static(X, pw)))
        torch.cuda.synchronize()
        for X, pw, Ys in outs:
            Yw = api.w3lr_gemm(X, pw)
            assert torch.equal(Ys, Yw), "static-scratch result differs from the workspace result"
            assert torch.isfinite(Ys.float()).all() and (Ys != 0).any()


def test_static_scratch_entry_rejects_what_does_not_fit():
    import torch
    from paper_2504_02658_amd import api
    M, N, K, r = 512, 4096, 14336, 0            # K split: fp32 partial sums far beyond the array
    assert api.gemm_workspace_bytes(M, N, K, r) > 4 << 20
    pw = api.PackedWeight(N, K, torch.zeros(api.packed_bytes(N, K), dtype=torch.uint8, device="cuda"))
    X = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    with pytest.raises(api.MiloError) as ei:
        api.w3lr_gemm_static(X, pw)
    assert ei.value.status == 5
    with pytest.raises(api.MiloError) as ei:
        api.lib()                                  # (argument errors come back like the other entry's)
        api._check(api.lib().milo_w3lr_gemm_static(None, 4, 64, 64, None, None, None, 0, None, None), "static")
    assert ei.value.status == 1
