"""GPU parity of milo_w3lr_gemm against the fp64 oracle (decode kernel for M <= 16, tiled above)."""
import numpy as np
import pytest

import oracle
from paper_2504_02658_amd import workloads as wl
from helpers import assert_close, oracle_weight, gpu_weight

pytestmark = pytest.mark.gpu


def _run(X, pw):
    import torch
    from paper_2504_02658_amd import api
    return api.w3lr_gemm(torch.from_numpy(X).cuda(), pw).cpu().numpy()


def _check_case(M, N, K, r, seed, outlier_frac=0.0):
    case = wl.LinearCase("t", M=M, N=N, K=K, r=r, seed=seed, outlier_frac=outlier_frac)
    X, W = wl.linear_inputs(case)
    ow = oracle_weight(W, r, seed=seed)
    pw = gpu_weight(W, ow)
    ref = oracle.w3lr_linear(X, **ow)
    Y = _run(X, pw)
    return assert_close(Y, ref, f"M{M} N{N} K{K} r{r}")


def test_c0_small_config():
    c = wl.C0
    _check_case(c.M, c.N, c.K, c.r, c.seed)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 7, 15, 16])
def test_decode_rows(M):
    _check_case(M, 272, 1408, 8, seed=40 + M)          # ragged N (not a multiple of 32), K = 22 groups


@pytest.mark.parametrize("N,K,r", [(16, 64, 0), (48, 192, 8), (1024, 4096, 32), (272, 2112, 24),
                                   (64, 1024, 40), (528, 3136, 16)])
def test_decode_shapes(N, K, r):
    _check_case(16, N, K, r, seed=N + K + r)
    _check_case(5, N, K, r, seed=N + K + r + 1)


@pytest.mark.parametrize("N,K,r", [
    (256, 14336, 32),      # K > 4096: several pieces of 16 chunks per workgroup; staged low-rank path
    (256, 14336, 64),      # the same with more T fragments than the staged path holds: plain loads
    (20480, 256, 16),      # more row blocks than resident workgroups: second turn of the block loop
    (272, 1408, 20),       # rank not a multiple of 8 at decode: element-wise U loads
    (4096, 14336, 32),     # Mixtral's own down projection at decode (Section 4 shapes)
])
@pytest.mark.parametrize("M", [1, 16])
def test_decode_long_k_many_blocks_odd_rank(N, K, r, M):
    _check_case(M, N, K, r, seed=N + K + r + M)


def test_decode_block_loop_second_turn_with_staged_low_rank():
    # many row blocks with a rank the staged path takes (U fragments are re-copied per turn), and
    # a long K on top of it
    _check_case(16, 36864, 512, 32, seed=811)
    _check_case(3, 16400, 4352, 24, seed=812)


@pytest.mark.parametrize("M", [17, 32, 33, 64, 100, 130, 257])
def test_tiled_rows(M):
    _check_case(M, 272, 1408, 8, seed=60 + M)


@pytest.mark.parametrize("N,K,r", [(16, 64, 0), (48, 192, 8), (528, 1024, 64), (1408, 2048, 128),
                                   (256, 832, 20), (2048, 1408, 136)])
def test_tiled_shapes(N, K, r):
    _check_case(96, N, K, r, seed=N + K + r)


@pytest.mark.parametrize("M,N,K,r", [(8, 1024, 1024, 512), (12, 528, 2112, 136), (200, 1024, 1024, 512),
                                     (96, 512, 2048, 300)])
def test_high_rank_compensators(M, N, K, r):
    # ranks of the size the paper gives dense layers (Section 3.2.2, "Dense-512"): beyond what the
    # staged low-rank paths hold at once, so the generic path / several passes over the ranks run
    _check_case(M, N, K, r, seed=500 + M)


@pytest.mark.parametrize("M,N,K,r", [(512, 4096, 4096, 512), (300, 2048, 4096, 1024), (512, 4096, 4096, 200)])
def test_dense_layer_ranks_in_a_split_gemm(M, N, K, r):
    # Dense-512 / Dense-1024 on an attention-sized projection: too few tiles for the chip, so K is split
    # over workgroups; the parts of T share the addition of their partial sums and every K split applies
    # a share of the ranks.  Two runs on one workspace agree bit for bit.
    import torch
    from paper_2504_02658_amd import api
    case = wl.LinearCase("dense", M=M, N=N, K=K, r=r, seed=700 + r)
    X, W = wl.linear_inputs(case)
    ow = oracle_weight(W, r, seed=case.seed)
    pw = gpu_weight(W, ow, check_pack=False)
    ref = oracle.w3lr_linear(X, **ow)
    ws = api.new_workspace(api.gemm_workspace_bytes(M, N, K, r))
    Xd = torch.from_numpy(X).cuda()
    Y1 = api.w3lr_gemm(Xd, pw, workspace=ws).cpu().numpy()
    Y2 = api.w3lr_gemm(Xd, pw, workspace=ws).cpu().numpy()
    assert api.workspace_status(ws) == 0
    assert_close(Y1, ref, f"M{M} N{N} K{K} r{r}")
    assert np.array_equal(Y1.view(np.uint16), Y2.view(np.uint16)), "two runs differ"


def test_rank_zero_equals_no_compensator_and_is_deterministic():
    import torch
    from paper_2504_02658_amd import api
    case = wl.LinearCase("t", M=40, N=512, K=1024, r=16, seed=9)
    X, W = wl.linear_inputs(case)
    ow = oracle_weight(W, 16)
    pw = gpu_weight(W, ow)
    pw0 = api.PackedWeight(pw.N, pw.K, pw.q3)
    for Xm in (X, X[:9]):
        Y0 = _run(Xm, pw0)
        assert_close(Y0, oracle.w3lr_linear(Xm, ow["codes"], ow["scales"], ow["zeros"]), "rank 0")
        Y1a, Y1b = _run(Xm, pw), _run(Xm, pw)
        assert np.array_equal(Y1a.view(np.uint16), Y1b.view(np.uint16)), "two runs differ"
        assert not np.array_equal(Y0, Y1a)


@pytest.mark.parametrize("M", [8, 48])
def test_integer_case_is_exact(M):
    import torch
    from paper_2504_02658_amd import api
    rng = np.random.default_rng(3)
    N, K = 64, 256
    q = rng.integers(0, 8, size=(N, K), dtype=np.uint8)
    s = np.ones((N, K // 64), np.float16)
    z = np.zeros((N, K // 64), np.float16)
    X = rng.integers(-1, 2, size=(M, K)).astype(np.float16)
    pw = api.PackedWeight(N, K, torch.from_numpy(oracle.pack_w3(q, s, z)).cuda())
    Y = _run(X, pw).astype(np.float64)
    assert np.array_equal(Y, oracle.w3lr_linear(X, q, s, z))


@pytest.mark.parametrize("M", [16, 64])
def test_one_hot_activations_expose_the_layout(M):
    # X = rows of the identity: output row k is column k of W_dq + U V, so any permutation of k
    # inside a unit, any swapped plane or transposed compensator shows up element by element.
    N, K, r = 48, 192, 8
    case = wl.LinearCase("t", M=M, N=N, K=K, r=r, seed=77)
    _, W = wl.linear_inputs(case)
    ow = oracle_weight(W, r)
    pw = gpu_weight(W, ow)
    Wt = oracle.dequantize(ow["codes"], ow["scales"], ow["zeros"]) + \
        ow["U"].astype(np.float64) @ ow["V"].astype(np.float64)
    for k0 in range(0, K, M):
        X = np.zeros((M, K), np.float16)
        X[np.arange(M), k0 + np.arange(M)] = 1.0
        Y = _run(X, pw).astype(np.float64)
        ref = Wt[:, k0:k0 + M].T
        assert np.max(np.abs(Y - ref)) <= 2.0 ** -10 * np.max(np.abs(ref)) + 1e-6, f"k0={k0}"


def test_real_valued_zero_points():
    import torch
    from paper_2504_02658_amd import api
    rng = np.random.default_rng(12)
    N, K, r = 128, 512, 0
    q = rng.integers(0, 8, size=(N, K), dtype=np.uint8)
    s = rng.uniform(0.005, 0.03, size=(N, K // 64)).astype(np.float16)
    z = rng.uniform(1.5, 5.5, size=(N, K // 64)).astype(np.float16)
    pw = api.PackedWeight(N, K, torch.from_numpy(oracle.pack_w3(q, s, z)).cuda())
    for M in (4, 40):
        X = rng.standard_normal((M, K)).astype(np.float16)
        assert_close(_run(X, pw), oracle.w3lr_linear(X, q, s, z), f"real z, M={M}")


def test_gpu_argument_errors():
    import torch
    from paper_2504_02658_amd import api
    X = torch.zeros((4, 128), dtype=torch.float16, device="cuda")
    W = torch.zeros((32, 128), dtype=torch.float32, device="cuda")
    pw = api.pack_w3(W)
    with pytest.raises(api.MiloError) as ei:
        api.pack_w3(W, group_size=128)
    assert ei.value.status == 3
    with pytest.raises(api.MiloError) as ei:
        api.w3lr_gemm(X, pw, workspace=torch.zeros(16, dtype=torch.uint8, device="cuda"))
    assert ei.value.status == 5
    with pytest.raises(ValueError):
        api.w3lr_gemm(torch.zeros((4, 64), dtype=torch.float16, device="cuda"), pw)


# ------------------------------------------------------------------ full-size configurations

@pytest.fixture(scope="module")
def c1_weight():
    c = wl.C1[16]
    W = wl.gen_weight(c.N, c.K, c.seed, c.outlier_frac, c.outlier_gain)
    ow = oracle_weight(W, c.r, seed=c.seed)
    pw = gpu_weight(W, ow)
    return ow, pw


@pytest.mark.parametrize("M", [1, 4, 16])
def test_c1_mixtral_up_projection_decode(c1_weight, M):
    ow, pw = c1_weight
    c = wl.C1[M]
    X = wl.gen_activations(c.M, c.K, c.seed)
    assert_close(_run(X, pw), oracle.w3lr_linear(X, **ow), c.name)


def test_c2_mixtral_down_projection_prefill():
    c = wl.C2
    X, W = wl.linear_inputs(c)
    ow = oracle_weight(W, c.r, seed=c.seed)
    pw = gpu_weight(W, ow)
    assert_close(_run(X, pw), oracle.w3lr_linear(X, **ow), c.name)


def test_k_splits_and_t_parts_many_chunks():
    # few tiles and a long K: the tiled kernel splits K over workgroups (partial sums added in
    # order by a second kernel) and forms X V^T in several parts; odd number of groups as well
    _check_case(48, 512, 4096, 24, seed=301)
    _check_case(200, 256, 8256, 72, seed=302)           # 129 groups


@pytest.mark.parametrize("M,N,K,r", [(16, 528, 2112, 16), (5, 272, 1408, 0), (200, 512, 2048, 24)])
def test_symmetric_weights(M, N, K, r):
    # weights packed by milo_pack_w3_sym (Eq. symm_int3) go through the same kernels
    case = wl.LinearCase("t", M=M, N=N, K=K, r=r, seed=400 + M)
    X, W = wl.linear_inputs(case)
    ow = oracle_weight(W, r, seed=400 + M, symmetric=True)
    pw = gpu_weight(W, ow, symmetric=True)
    assert_close(_run(X, pw), oracle.w3lr_linear(X, **ow), f"symmetric M{M} N{N} K{K} r{r}")


def test_many_m_tiles_take_the_xcd_placement_path():
    # from 128 M-tiles on the tiled kernel renumbers its workgroups (a contiguous share of the
    # tile rows per XCD); with one column tile K is split as well, ragged last tile included
    _check_case(128 * 129 + 40, 256, 2048, 8, seed=303)
    _check_case(128 * 128, 320, 192, 24, seed=304)


def test_graph_replay_matches_eager_and_needs_no_reset():
    # the kernels leave their control words clean: a captured graph of calls that share one
    # workspace per shape can be replayed with eager work in between, bit for bit
    import torch
    from paper_2504_02658_amd import api
    cases = []
    for M, N, K, r, seed in ((16, 1024, 4096, 32, 71), (7, 272, 1408, 8, 72), (96, 512, 4096, 24, 73)):
        case = wl.LinearCase("t", M=M, N=N, K=K, r=r, seed=seed)
        X, W = wl.linear_inputs(case)
        pw = gpu_weight(W, oracle_weight(W, r, seed=seed), check_pack=False)
        Xd = torch.from_numpy(X).cuda()
        ws = api.new_workspace(api.gemm_workspace_bytes(M, N, K, r), Xd.device)
        out = torch.empty((M, N), dtype=torch.float16, device=Xd.device)
        cases.append((Xd, pw, ws, out))
    eager = [api.w3lr_gemm(Xd, pw, workspace=ws).clone() for Xd, pw, ws, _ in cases]
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for Xd, pw, ws, out in cases:
            api.w3lr_gemm(Xd, pw, out=out, workspace=ws)
    torch.cuda.current_stream().wait_stream(stream)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(2):                     # back-to-back calls on the same workspaces
            for Xd, pw, ws, out in cases:
                api.w3lr_gemm(Xd, pw, out=out, workspace=ws)
    for rep in range(3):
        for _, _, _, out in cases:
            out.zero_()
        g.replay()
        torch.cuda.synchronize()
        for (_, _, _, out), ref in zip(cases, eager):
            assert torch.equal(out, ref), f"replay {rep} differs from the eager result"
        # eager work and a synchronisation between the replays
        again = api.w3lr_gemm(cases[0][0], cases[0][1], workspace=cases[0][2])
        torch.cuda.synchronize()
        assert torch.equal(again, eager[0])


def test_workspace_status_reports_a_wait_that_gave_up():
    # The give-up word is forced from the host (no kernel spins): status turns to MILO_ERR_WAIT and
    # stays there until the workspace is prepared again; a clean run reports MILO_OK.
    import torch
    from paper_2504_02658_amd import api
    for M in (16, 96):                                  # decode and tiled workspaces
        case = wl.LinearCase("t", M=M, N=512, K=1024, r=16, seed=31)
        X, W = wl.linear_inputs(case)
        ow = oracle_weight(W, 16)
        pw = gpu_weight(W, ow, check_pack=False)
        ws = api.new_workspace(api.gemm_workspace_bytes(M, 512, 1024, 16))
        Xd = torch.from_numpy(X).cuda()
        Y = api.w3lr_gemm(Xd, pw, workspace=ws)
        assert api.workspace_status(ws) == 0
        assert_close(Y.cpu().numpy(), oracle.w3lr_linear(X, **ow), "before")
        ws.view(torch.int32)[3] = 1                     # what a kernel writes when its wait runs out
        assert api.workspace_status(ws) == 8
        api.w3lr_gemm(Xd, pw, workspace=ws)
        assert api.workspace_status(ws) == 8            # sticky for a GEMM workspace
        api.lib().milo_workspace_init(ws.data_ptr(), ws.numel(), None)
        Y = api.w3lr_gemm(Xd, pw, workspace=ws)
        assert api.workspace_status(ws) == 0
        assert_close(Y.cpu().numpy(), oracle.w3lr_linear(X, **ow), "after re-init")


# ------------------------------------------------------------------ INT3 compensators, weight flags

def _int3_case(M, N, K, r, seed, symmetric=False):
    """Both sides of a linear whose compensator is INT3-quantized (Section 3.2.3, Eq. symm_int3)."""
    import torch
    from paper_2504_02658_amd import api
    case = wl.LinearCase("t", M=M, N=N, K=K, r=r, seed=seed)
    X, W = wl.linear_inputs(case)
    ow = oracle_weight(W, r, seed=seed, symmetric=symmetric)
    U32, V32 = ow["U"].astype(np.float32), ow["V"].astype(np.float32)
    uq, vq = oracle.quantize_compensator(U32, V32)
    Ud, Vd = oracle.dequantize_compensator(uq, vq, r)
    ref = oracle.w3lr_linear(X, ow["codes"], ow["scales"], ow["zeros"], Ud, Vd)
    pw = gpu_weight(W, dict(ow, U=np.zeros((N, 0), np.float16)), symmetric=symmetric)
    u3, v3 = api.pack_lr3(torch.from_numpy(U32).cuda(), torch.from_numpy(V32).cuda())
    assert np.array_equal(u3.cpu().numpy(), oracle.pack_w3(*uq)), "U blob differs from the oracle's"
    assert np.array_equal(v3.cpu().numpy(), oracle.pack_w3(*vq)), "V blob differs from the oracle's"
    return X, pw.with_int3_compensator(u3, v3, r), ref


@pytest.mark.parametrize("M,N,K,r", [
    (16, 1024, 4096, 32), (1, 256, 1408, 8), (5, 320, 2112, 20), (16, 4096, 14336, 64), (7, 20480, 256, 16),
    (16, 128, 128, 128), (3, 192, 512, 100),
    (96, 512, 1024, 32), (40, 256, 832, 8), (200, 1024, 2048, 128), (130, 320, 1408, 20), (512, 1024, 4096, 64),
])
def test_int3_compensator(M, N, K, r):
    X, pw, ref = _int3_case(M, N, K, r, seed=M + N + K + r)
    assert pw.flags == 2 and pw.weight_bytes() == (N * K + ((r + 15) // 16 * 16) * (N + K)) * 7 // 16
    assert_close(_run(X, pw), ref, f"INT3 compensator M{M} N{N} K{K} r{r}")


def test_int3_and_bf16_compensators_in_a_split_gemm():
    # rank 128 as INT3 blobs and rank 200 in bf16 on a projection whose K is split over workgroups: the
    # K splits share the ranks, the parts of T share their sums
    import torch
    from paper_2504_02658_amd import api
    X, pw, ref = _int3_case(512, 4096, 4096, 128, seed=901)
    assert_close(_run(X, pw), ref, "INT3 rank 128, split GEMM")
    case = wl.LinearCase("t", M=512, N=4096, K=4096, r=200, seed=902)
    X, W = wl.linear_inputs(case)
    ow = oracle_weight(W, 200, seed=902)
    Xb, Ub, Vb = _to_bf16(X), _to_bf16(ow["U"]), _to_bf16(ow["V"])
    ref = oracle.w3lr_linear(Xb.float().numpy(), ow["codes"], ow["scales"], ow["zeros"], Ub.float().numpy(), Vb.float().numpy())
    pw = gpu_weight(W, dict(ow, U=np.zeros((4096, 0), np.float16)), check_pack=False).with_compensator(Ub.cuda(), Vb.cuda())
    Yf = api.w3lr_gemm(Xb.cuda(), pw).float().cpu().numpy().astype(np.float64)
    rel = np.linalg.norm(Yf - ref) / np.linalg.norm(ref)
    mx = np.max(np.abs(Yf - ref)) / np.max(np.abs(ref))
    assert rel <= BF16_REL_FRO_TOL and mx <= BF16_MAX_ABS_TOL, (rel, mx)


def test_int3_compensator_full_size_c1_and_a_symmetric_weight():
    c = wl.C1[16]
    X, pw, ref = _int3_case(c.M, c.N, c.K, c.r, seed=c.seed)
    assert_close(_run(X, pw), ref, "c1 with INT3 compensator")
    X, pw, ref = _int3_case(16, 1024, 4096, 32, seed=5, symmetric=True)
    assert pw.flags == 3
    assert_close(_run(X, pw), ref, "symmetric weight + INT3 compensator")


@pytest.mark.parametrize("M,N,K,r", [(16, 14336, 4096, 32), (4, 4096, 4096, 0), (16, 272, 1408, 8), (200, 512, 2048, 24)])
def test_symmetric_flag_changes_nothing_but_the_kernel(M, N, K, r):
    # MILO_W3_SYMMETRIC selects the conversion without zero-point arithmetic (Section 3.3): same bits
    import torch
    from paper_2504_02658_amd import api
    case = wl.LinearCase("t", M=M, N=N, K=K, r=r, seed=600 + M)
    X, W = wl.linear_inputs(case)
    rng = np.random.default_rng(M + r)
    pw = api.pack_w3(torch.from_numpy(W).cuda(), symmetric=True)
    assert pw.flags == api.W3_SYMMETRIC
    if r:
        pw = pw.with_compensator(torch.from_numpy((0.02 * rng.standard_normal((N, r))).astype(np.float16)).cuda(),
                                 torch.from_numpy((0.02 * rng.standard_normal((r, K))).astype(np.float16)).cuda())
    plain = api.PackedWeight(pw.N, pw.K, pw.q3, pw.U, pw.V, flags=0)
    a, b = _run(X, pw), _run(X, plain)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


# ------------------------------------------------------------------ bf16 activations (MILO_ACT_BF16)

# Tolerance for the bf16 variant, from its arithmetic: every dequantized weight is rounded once to
# bf16 (relative 2^-9 at most, 2^-9 / sqrt(12) rms; the errors of the K products are independent, so
# they appear undiminished in the relative error of a sum), the output once more, T = X V^T once in
# between: about 1e-3 rms in all, bounded here by 4e-3; single elements by 3e-2 of the largest output.
BF16_REL_FRO_TOL, BF16_MAX_ABS_TOL = 4e-3, 3e-2


def _to_bf16(x):
    import torch
    return torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16)


@pytest.mark.parametrize("M,N,K,r", [(16, 1024, 4096, 32), (1, 272, 1408, 0), (5, 528, 14336, 64), (7, 256, 1408, 20),
                                     (96, 512, 1024, 24), (512, 1024, 4096, 64), (40, 4096, 14336, 16), (130, 272, 832, 136)])
def test_bf16_activations(M, N, K, r):
    import torch
    from paper_2504_02658_amd import api
    case = wl.LinearCase("t", M=M, N=N, K=K, r=r, seed=700 + M + r)
    X, W = wl.linear_inputs(case)
    ow = oracle_weight(W, r, seed=case.seed)
    Xb, Ub, Vb = _to_bf16(X), _to_bf16(ow["U"]), _to_bf16(ow["V"])
    ref = oracle.w3lr_linear(Xb.float().numpy(), ow["codes"], ow["scales"], ow["zeros"],
                             Ub.float().numpy(), Vb.float().numpy())
    pw = gpu_weight(W, dict(ow, U=np.zeros((N, 0), np.float16)))
    if r:
        pw = pw.with_compensator(Ub.cuda(), Vb.cuda())
    Y = api.w3lr_gemm(Xb.cuda(), pw)
    assert Y.dtype == torch.bfloat16
    Yf = Y.float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(Yf))
    rel = np.linalg.norm(Yf - ref) / np.linalg.norm(ref)
    mx = np.max(np.abs(Yf - ref)) / np.max(np.abs(ref))
    assert rel <= BF16_REL_FRO_TOL and mx <= BF16_MAX_ABS_TOL, (rel, mx)
    Y2 = api.w3lr_gemm(Xb.cuda(), pw)
    assert torch.equal(Y, Y2)


def test_bf16_integer_case_is_exact():
    # small integers are exact in bf16 too: codes 0..7, scale 1, zero 0, activations in {-1, 0, 1}
    import torch
    from paper_2504_02658_amd import api
    rng = np.random.default_rng(4)
    N, K = 64, 256
    q = rng.integers(0, 8, size=(N, K), dtype=np.uint8)
    s = np.ones((N, K // 64), np.float16)
    z = np.zeros((N, K // 64), np.float16)
    pw = api.PackedWeight(N, K, torch.from_numpy(oracle.pack_w3(q, s, z)).cuda())
    for M in (8, 48):
        X = rng.integers(-1, 2, size=(M, K)).astype(np.float32)
        Y = api.w3lr_gemm(_to_bf16(X).cuda(), pw).float().cpu().numpy().astype(np.float64)
        ref = oracle.w3lr_linear(X, q, s, z)
        assert np.array_equal(Y, np.asarray(_to_bf16(ref).float().numpy(), np.float64))
