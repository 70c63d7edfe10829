"""GPU parity of milo_moe_w3lr_forward against the fp64 oracle."""
import numpy as np
import pytest

import oracle
from paper_2504_02658_amd import workloads as wl
from helpers import assert_close, build_moe

pytestmark = pytest.mark.gpu


def _forward(layer, X, ids, gates):
    import torch
    Y = layer.forward(torch.from_numpy(X).cuda(), torch.from_numpy(ids).cuda(),
                      torch.from_numpy(gates).cuda())
    return Y.cpu().numpy()


def _check(case, what=None, int3=False):
    o_experts, layer = build_moe(case, int3=int3)
    X = wl.moe_activations(case)
    ids, gates = wl.moe_routing(case)
    ref = oracle.moe_forward(X, o_experts, ids, gates)
    Y = _forward(layer, X, ids, gates)
    res = assert_close(Y, ref, what or case.name)
    assert layer.routing_status() == 0
    Y2 = _forward(layer, X, ids, gates)
    assert np.array_equal(Y.view(np.uint16), Y2.view(np.uint16)), "two runs differ"
    return res


def test_tiny_layer_all_tile_heights():
    base = wl.MoECase("tiny", T=40, H=256, F=384, E=4, topk=2, seed=11, rank_choices=(0, 8, 16))
    _check(base)                                              # ~20 rows per expert: 32-row tiles
    _check(wl.scaled(base, T=80, name="tiny64"))             # ~40 rows: 64-row tiles
    _check(wl.scaled(base, T=150, name="tiny128a"))          # ~75 rows: 128-row tiles, partly filled
    _check(wl.scaled(base, T=400, name="tiny128"))           # ~200 rows: 128-row tiles, several per expert


def test_int3_compensators_in_a_layer():
    # every expert's U, V as INT3 blobs (Section 3.2.3): the grouped kernels unpack them like weights
    base = wl.MoECase("int3", T=40, H=256, F=384, E=4, topk=2, seed=21, rank_choices=(0, 8, 16, 40))
    _check(base, int3=True)
    _check(wl.scaled(base, T=400, name="int3_128", rank_choices=(16, 32, 128)), int3=True)


# bfloat16 layer (MILO_ACT_BF16): on top of the single linear's roundings (every dequantized weight, T, the
# output: see test_gpu_gemm) the SwiGLU output and every routed pair's expert output are rounded to bf16
# (2^-9 relative at most, 5.6e-4 rms each) and the second linear sees the first one's error: about 1.3e-3
# rms in all, bounded here by 6e-3; single elements by 4e-2 of the largest output.
BF16_MOE_REL_FRO_TOL, BF16_MOE_MAX_ABS_TOL = 6e-3, 4e-2


def _check_bf16(case):
    import torch
    from helpers import to_bf16
    o_experts, layer = build_moe(case, bf16=True)
    Xb = to_bf16(wl.moe_activations(case))
    ids, gates = wl.moe_routing(case)
    ref = oracle.moe_forward(Xb.float().numpy(), o_experts, ids, gates)
    args = (Xb.cuda(), torch.from_numpy(ids).cuda(), torch.from_numpy(gates).cuda())
    Y = layer.forward(*args)
    assert Y.dtype == torch.bfloat16
    Yf = Y.float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(Yf))
    rel = np.linalg.norm(Yf - ref) / np.linalg.norm(ref)
    mx = np.max(np.abs(Yf - ref)) / np.max(np.abs(ref))
    assert rel <= BF16_MOE_REL_FRO_TOL and mx <= BF16_MOE_MAX_ABS_TOL, (case.name, rel, mx)
    assert layer.routing_status() == 0
    assert torch.equal(Y, layer.forward(*args)), "two runs differ"


def test_bf16_layer():
    base = wl.MoECase("bf16", T=40, H=256, F=384, E=4, topk=2, seed=31, rank_choices=(0, 8, 16, 40))
    _check_bf16(base)                                                           # 32-row tiles
    _check_bf16(wl.scaled(base, T=400, name="bf16_128"))                        # 128-row tiles, several per expert
    _check_bf16(wl.scaled(base, T=3, name="bf16_small"))                        # single-launch routing
    _check_bf16(wl.scaled(wl.C4, T=256, H=512, F=704, E=16, name="bf16_c4_reduced"))  # shared experts, K splits


def test_bf16_layer_rejects_int3_compensators():
    from paper_2504_02658_amd import api
    case = wl.MoECase("bf16_int3", T=8, H=256, F=384, E=2, topk=1, seed=32, rank_choices=(16,))
    _, layer = build_moe(case, int3=True)
    with pytest.raises(api.MiloError) as ei:
        api.MoELayer(layer.experts, case.H, case.F, bf16=True)
    assert ei.value.status == 2


def test_many_tiles_take_the_xcd_placement_path():
    # 16 800 routed rows -> more than 128 M-tiles: the grouped kernels renumber their workgroups
    # per XCD and the work list is dealt over the eight ranges
    case = wl.MoECase("many", T=4200, H=256, F=384, E=8, topk=4, seed=14, rank_choices=(0, 8, 24))
    _check(case)


def test_graph_replay_of_a_layer():
    # routing, flags and partial buffers are re-initialised by the kernels themselves: a captured
    # layer replays bit for bit with eager work on the same workspace in between
    import torch
    case = wl.MoECase("replay", T=150, H=256, F=384, E=4, topk=2, seed=15, rank_choices=(8, 16))
    _, layer = build_moe(case)
    X = torch.from_numpy(wl.moe_activations(case)).cuda()
    ids_np, gates_np = wl.moe_routing(case)
    ids, gates = torch.from_numpy(ids_np).cuda(), torch.from_numpy(gates_np).cuda()
    from paper_2504_02658_amd import api
    ws = api.new_workspace(layer.workspace_bytes(case.T, case.topk), X.device)
    out = torch.empty((case.T, case.H), dtype=torch.float16, device=X.device)
    eager = layer.forward(X, ids, gates, workspace=ws).clone()
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        layer.forward(X, ids, gates, out=out, workspace=ws)
    torch.cuda.current_stream().wait_stream(stream)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        layer.forward(X, ids, gates, out=out, workspace=ws)
        layer.forward(X, ids, gates, out=out, workspace=ws)
    for rep in range(3):
        out.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager result"
        again = layer.forward(X, ids, gates, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(again, eager)


def test_single_token_and_empty_experts():
    case = wl.MoECase("one", T=1, H=128, F=192, E=8, topk=2, seed=12, rank_choices=(8,))
    _check(case)                                              # six experts receive nothing


def test_shared_experts_and_skew():
    case = wl.scaled(wl.C4, T=200, H=256, F=320, E=16, topk=4, name="ds_small", shared_rank=24)
    _check(case)


def test_reduced_mixtral_and_deepseek_shapes():
    _check(wl.scaled(wl.C3, T=96, H=512, F=1792, name="c3_reduced"))
    _check(wl.scaled(wl.C4, T=512, H=512, F=704, E=24, name="c4_reduced"))


def test_out_of_range_expert_id_is_skipped_and_flagged():
    case = wl.MoECase("bad", T=24, H=128, F=192, E=4, topk=2, seed=13, rank_choices=(8,))
    o_experts, layer = build_moe(case)
    X = wl.moe_activations(case)
    ids, gates = wl.moe_routing(case)
    ids = ids.copy()
    ids[5, 1] = 4
    ids[7, 0] = -1
    good = (ids >= 0) & (ids < 4)
    ref = oracle.moe_forward(X, o_experts, np.where(good, ids, 0), np.where(good, gates, 0).astype(np.float32))
    Y = _forward(layer, X, ids, gates)
    assert_close(Y, ref, "bad ids skipped")
    assert layer.routing_status() == 6


def test_status_reports_a_wait_that_gave_up():
    # the give-up word of the layer's workspace, forced from the host (no kernel spins): the status call
    # reports MILO_ERR_WAIT for that forward; the next forward clears the word at its start
    import torch
    from paper_2504_02658_amd import api
    case = wl.MoECase("wait", T=24, H=128, F=192, E=4, topk=2, seed=16, rank_choices=(8,))
    _, layer = build_moe(case)
    X = torch.from_numpy(wl.moe_activations(case)).cuda()
    ids_np, gates_np = wl.moe_routing(case)
    ids, gates = torch.from_numpy(ids_np).cuda(), torch.from_numpy(gates_np).cuda()
    ws = api.new_workspace(layer.workspace_bytes(case.T, case.topk))
    Y = layer.forward(X, ids, gates, workspace=ws).clone()
    assert layer.routing_status() == 0
    ws.view(torch.int32)[3] = 1                         # what a kernel writes when its wait runs out
    assert layer.routing_status() == 8
    Y2 = layer.forward(X, ids, gates, workspace=ws)
    assert layer.routing_status() == 0
    assert torch.equal(Y, Y2)


@pytest.mark.timeout(900)
def test_c3_mixtral_layer_full_size():
    # the full layer at 512 tokens, then the same experts at decode-sized batches (16, 4 and 1 tokens:
    # routing and work list come from the single-launch kernel, tiles are 32 rows high)
    import dataclasses
    o_experts, layer = build_moe(wl.C3)
    for T in (512, 16, 4, 1):
        case = dataclasses.replace(wl.C3, T=T)
        X = wl.moe_activations(case)
        ids, gates = wl.moe_routing(case)
        ref = oracle.moe_forward(X, o_experts, ids, gates)
        Y = _forward(layer, X, ids, gates)
        assert_close(Y, ref, f"c3 at {T} tokens")
        assert layer.routing_status() == 0
        Y2 = _forward(layer, X, ids, gates)
        assert np.array_equal(Y.view(np.uint16), Y2.view(np.uint16)), "two runs differ"


def test_routing_of_small_batches_matches_the_general_kernels():
    # up to 256 routed pairs the routing and the work list come from one single-workgroup kernel; from
    # 257 on from the two general kernels: the same layer just below and just above the limit, many
    # experts empty, several tiles per expert
    base = wl.MoECase("small_route", T=64, H=128, F=192, E=24, topk=4, seed=23, rank_choices=(0, 8, 40))
    _check(base)                                              # 256 pairs
    _check(wl.scaled(base, T=65, name="general_route"))      # 260 pairs
    _check(wl.scaled(base, T=3, name="three_tokens"))


@pytest.mark.timeout(900)
def test_c4_deepseek_layer_full_size():
    _check(wl.C4)
