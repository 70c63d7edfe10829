"""The synthetic input recipe: shapes, determinism and the structure the configs ask for."""
import numpy as np

from paper_2504_02658_amd import workloads as wl


def test_linear_inputs_shapes_and_determinism():
    case = wl.scaled(wl.C1[4], N=64, K=4096)
    X, W = wl.linear_inputs(case)
    X2, W2 = wl.linear_inputs(case)
    assert X.dtype == np.float16 and W.dtype == np.float32
    assert X.shape == (4, 4096) and W.shape == (64, 4096)
    assert np.array_equal(X, X2) and np.array_equal(W, W2)
    # 1 % outlier input channels: floor(0.01 * 4096) = 40 columns scaled by 8
    col_std = W.std(axis=0)
    assert int(np.sum(col_std > 0.08)) == 40
    assert abs(np.median(col_std) - 0.02) < 0.004
    assert abs(float(X.astype(np.float32).std()) - 1.0) < 0.02


def test_mixtral_style_routing():
    case = wl.scaled(wl.C3, T=256)
    ids, g = wl.moe_routing(case)
    assert ids.shape == (256, 2) and g.shape == (256, 2)
    assert ids.dtype == np.int32 and g.dtype == np.float32
    assert np.all(ids[:, 0] != ids[:, 1]) and ids.min() >= 0 and ids.max() < 8
    assert np.allclose(g.sum(1), 1.0, atol=1e-6) and np.all(g[:, 0] >= g[:, 1])
    ranks = wl.expert_ranks(case)
    assert len(ranks) == 8 and set(ranks) <= {16, 32, 64}


def test_deepseek_style_routing_is_skewed_with_shared_experts():
    ids, g = wl.moe_routing(wl.C4)
    assert ids.shape == (4096, 8)
    assert np.all(ids[:, 6] == 64) and np.all(ids[:, 7] == 65) and np.all(g[:, 6:] == 1.0)
    routed = ids[:, :6]
    assert all(len(set(row)) == 6 for row in routed[:64].tolist())
    counts = np.bincount(routed.reshape(-1), minlength=64)
    assert counts.sum() == 4096 * 6
    assert counts.max() / max(1, counts.min()) > 8          # popularity skew
    assert np.all(g[:, :6].sum(1) < 1.0)                     # top-6 of 64, not renormalised
    ranks = wl.expert_ranks(wl.C4)
    assert ranks[:64] == [8] * 64 and ranks[64:] == [128, 128]


def test_expert_weights_are_distinct_and_shaped():
    case = wl.scaled(wl.C4, H=128, F=192)
    a = wl.expert_weight(case, 0, "w1")
    b = wl.expert_weight(case, 0, "w3")
    c = wl.expert_weight(case, 1, "w2")
    assert a.shape == (192, 128) and c.shape == (128, 192)
    assert not np.array_equal(a, b)
    assert np.array_equal(a, wl.expert_weight(case, 0, "w1"))
