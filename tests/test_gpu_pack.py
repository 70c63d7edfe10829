"""GPU parity: milo_pack_w3 / milo_unpack_w3 / milo_dequant_w3 against the oracle, bit for bit."""
import numpy as np
import pytest

import oracle
from paper_2504_02658_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _pack_both(W, symmetric=False):
    import torch
    from paper_2504_02658_amd import api
    q, s, z = oracle.quantize_sym(W) if symmetric else oracle.quantize_rtn(W)
    pw = api.pack_w3(torch.from_numpy(W).cuda(), symmetric=symmetric)
    return (q, s, z), pw


def _assert_pack_equal(W, what, symmetric=False):
    (q, s, z), pw = _pack_both(W, symmetric)
    N, K = W.shape
    got = pw.q3.cpu().numpy()
    assert got.size == N * K * 7 // 16, what
    if not np.array_equal(got, oracle.pack_w3(q, s, z)):
        gq, gs, gz = oracle.unpack_w3(got, N, K)
        assert np.array_equal(gs.view(np.uint16), s.view(np.uint16)), f"{what}: scales"
        assert np.array_equal(gz.view(np.uint16), z.view(np.uint16)), f"{what}: zeros"
        bad = np.argwhere(gq != q)
        raise AssertionError(f"{what}: {len(bad)} codes differ, first at {bad[:5].tolist()}")
    return (q, s, z), pw


@pytest.mark.parametrize("N,K", [(16, 64), (48, 192), (272, 1408), (1024, 1024)])
def test_pack_bit_exact_gaussian(N, K):
    W = wl.gen_weight(N, K, seed=100 + N + K, outlier_frac=0.01 if K >= 1024 else 0.0)
    _assert_pack_equal(W, f"gaussian {N}x{K}")


def test_pack_bit_exact_edge_groups():
    rng = np.random.default_rng(7)
    W = (rng.standard_normal((64, 640)) * 0.02).astype(np.float32)
    W[:, 0:64] = 0.3125                                   # constant group -> degenerate rule
    W[:, 64:128] += 0.5                                   # all positive -> negative zero-point
    W[:, 128:192] -= 0.7                                  # all negative -> zero-point above 7
    W[:, 192:256] *= 1e-6                                 # tiny range: subnormal fp16 scale
    W[:, 256:320] = np.linspace(1.0, 1.0 + 1e-7, 64, dtype=np.float32)   # range below fp16 resolution
    W[:, 320:384] *= 3000.0                               # large values
    W[0, 384:448] = (np.arange(64) % 8 - 3.5).astype(np.float32) * 0.25  # exact half-way cases
    W[:, 448:512] = (np.arange(64, dtype=np.float32) / 16 - 1.0)[None, :].clip(-1, 0.75)
    (q, s, z), pw = _assert_pack_equal(W, "edge groups")
    assert np.all(q[:, 0:64] == 0) and np.all(s[:, 0] == np.float16(1))


def test_pack_bit_exact_many_seeds():
    for seed in range(5):
        rng = np.random.default_rng(1000 + seed)
        scale = 10.0 ** rng.uniform(-3, 1)
        W = (rng.standard_normal((96, 512)) * scale + rng.standard_normal((96, 1)) * scale * 0.3)
        _assert_pack_equal(W.astype(np.float32), f"seed {seed}")


def test_unpack_and_dequant():
    import torch
    from paper_2504_02658_amd import api
    W = wl.gen_weight(112, 448, seed=5)
    (q, s, z), pw = _assert_pack_equal(W, "unpack case")
    uq, us, uz = api.unpack_w3(pw)
    assert np.array_equal(uq.cpu().numpy(), q)
    assert np.array_equal(us.cpu().numpy().view(np.uint16), s.view(np.uint16))
    assert np.array_equal(uz.cpu().numpy().view(np.uint16), z.view(np.uint16))
    wdq = api.dequant_w3(pw).cpu().numpy()
    ref = oracle.dequantize(q, s, z)
    # the kernel rounds s*(q-z) once to fp16: compare with the correctly rounded oracle value
    ref16 = ref.astype(np.float16)
    diff_ulps = np.abs(wdq.view(np.int16).astype(np.int32) - ref16.view(np.int16).astype(np.int32))
    assert diff_ulps.max() <= 1, f"dequant differs by up to {diff_ulps.max()} fp16 ulps"
    assert np.mean(diff_ulps == 0) > 0.99
    # arbitrary codes with real-valued zero-points (the GEMM accepts those)
    rng = np.random.default_rng(3)
    N, K = 32, 256
    codes = rng.integers(0, 8, size=(N, K), dtype=np.uint8)
    s2 = (rng.uniform(0.001, 0.05, size=(N, K // 64))).astype(np.float16)
    z2 = (rng.uniform(-3.0, 9.0, size=(N, K // 64))).astype(np.float16)
    pw2 = api.PackedWeight(N, K, torch.from_numpy(oracle.pack_w3(codes, s2, z2)).cuda())
    assert np.array_equal(api.unpack_w3(pw2)[0].cpu().numpy(), codes)
    wdq2 = api.dequant_w3(pw2).cpu().numpy().astype(np.float64)
    ref2 = oracle.dequantize(codes, s2, z2)
    # one fp16 rounding of the result plus the fp32 cancellation of the 1024 bias (~2^-13 s)
    s_el = np.repeat(s2.astype(np.float64), 64, axis=1)
    tol = np.abs(ref2) * 2.0 ** -10 + s_el * 2.0 ** -12
    assert np.all(np.abs(wdq2 - ref2) <= tol)


def test_pack_sym_bit_exact():
    # milo_pack_w3_sym against the oracle's symmetric quantizer (Eq. symm_int3), same blob layout
    for N, K, seed in ((16, 64, 1), (272, 1408, 2), (1024, 1024, 3)):
        W = wl.gen_weight(N, K, seed=200 + seed, outlier_frac=0.01 if K >= 1024 else 0.0)
        (q, s, z), _ = _assert_pack_equal(W, f"symmetric gaussian {N}x{K}", symmetric=True)
        assert np.all(z == np.float16(4))
    rng = np.random.default_rng(8)
    W = (rng.standard_normal((64, 512)) * 0.02).astype(np.float32)
    W[:, 0:64] = 0.0                                      # all zero -> degenerate rule
    W[:, 64:128] *= 1e-7                                  # step below fp16 resolution
    W[:, 128:192] *= 3000.0
    W[0, 192:256] = (np.arange(64) % 8 - 3.5).astype(np.float32) * 0.25    # exact half-way cases, +max clamps
    W[:, 256:320] = np.abs(W[:, 256:320])                 # one-sided group
    (q, s, z), _ = _assert_pack_equal(W, "symmetric edge groups", symmetric=True)
    assert np.all(q[:, 0:64] == 4) and np.all(s[:, 0] == np.float16(1))
