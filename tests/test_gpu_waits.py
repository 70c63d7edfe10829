"""The GEMM kernels wait for their memory requests with hand-counted `s_waitcnt vmcnt(N)`.  The build
also makes a library in which every such wait is a wait for everything; both must agree bit for bit,
whatever the compiler did with the instruction order."""
import ctypes

import numpy as np
import pytest

from paper_2504_02658_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _gemm(L, X, q3, U, V, r, N):
    import torch
    M, K = X.shape
    need = int(L.milo_w3lr_gemm_workspace(M, N, K, r))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    assert L.milo_workspace_init(ctypes.c_void_p(ws.data_ptr()), ws.numel(), None) == 0
    Y = torch.empty((M, N), dtype=torch.float16, device="cuda")
    p = lambda t: ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)
    st = L.milo_w3lr_gemm(p(X), M, N, K, p(q3), p(U), p(V), r, p(Y), p(ws), ws.numel(), None)
    assert st == 0
    torch.cuda.synchronize()
    return Y.cpu().numpy()


@pytest.mark.parametrize("M,N,K,r", [
    (16, 1024, 4096, 32), (1, 528, 2112, 16), (4, 272, 14336, 32), (7, 20480, 256, 16), (16, 272, 1408, 20),
    (48, 512, 4096, 24), (130, 528, 1024, 64), (512, 1024, 2048, 8),
])
def test_counted_waits_equal_full_waits(M, N, K, r):
    import torch
    from paper_2504_02658_amd import api
    counted, full = api.lib(), api.bind(api.FULLWAITS_LIB_PATH)
    rng = np.random.default_rng(M + N + K + r)
    W = torch.from_numpy(wl.gen_weight(N, K, seed=M + N + K)).cuda()
    q3 = api.pack_w3(W).q3
    X = torch.from_numpy(wl.gen_activations(M, K, seed=r + 1)).cuda()
    U = torch.from_numpy((0.02 * rng.standard_normal((N, r))).astype(np.float16)).cuda()
    V = torch.from_numpy((0.02 * rng.standard_normal((r, K))).astype(np.float16)).cuda()
    a = _gemm(counted, X, q3, U, V, r, N)
    b = _gemm(full, X, q3, U, V, r, N)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    assert np.all(np.isfinite(a)) and np.any(a != 0)


def test_moe_layer_counted_waits_equal_full_waits(monkeypatch):
    # the grouped kernels of the MoE call share the K loop with its counted waits: the same layer through
    # both builds, tile heights 32 and 128, must agree bit for bit
    import torch
    from paper_2504_02658_amd import api
    from helpers import build_moe
    for T in (24, 400):
        case = wl.MoECase("waits", T=T, H=256, F=384, E=4, topk=2, seed=41, rank_choices=(0, 8, 40))
        _, layer = build_moe(case)
        X = torch.from_numpy(wl.moe_activations(case)).cuda()
        ids_np, gates_np = wl.moe_routing(case)
        ids, gates = torch.from_numpy(ids_np).cuda(), torch.from_numpy(gates_np).cuda()
        Y1 = layer.forward(X, ids, gates).clone()
        assert layer.routing_status() == 0
        with monkeypatch.context() as m:
            m.setattr(api, "_lib", api.bind(api.FULLWAITS_LIB_PATH))
            layer2 = api.MoELayer(layer.experts, case.H, case.F)
            Y2 = layer2.forward(X, ids, gates).clone()
            assert layer2.routing_status() == 0
        assert torch.equal(Y1, Y2), f"the two builds differ at {T} tokens"
        assert bool(torch.isfinite(Y1.float()).all()) and bool((Y1 != 0).any())
