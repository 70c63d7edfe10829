"""The C-ABI library loads on a machine without a GPU, exports every symbol of include/milo.h and
rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2504_02658_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    return api.lib()


def test_exports_match_header(L):
    header = open(os.path.join(ROOT, "include", "milo.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(milo_[a-z0-9_]+)\s*\(", header))
    assert declared == set(api.EXPORTS)
    for name in declared:
        assert getattr(L, name) is not None


def test_status_strings(L):
    for code in api.STATUS_NAMES:
        assert L.milo_status_string(code)
    assert L.milo_status_string(12345) == b"unknown status"
    assert L.milo_version() >= 100


def test_sizes(L):
    assert L.milo_w3_packed_bytes(1024, 1024) == 1024 * 1024 * 7 // 16
    assert L.milo_w3_packed_bytes(14336, 4096) == 25690112      # 22,020,096 of codes + 3,670,016 of parameters
    assert L.milo_w3_packed_bytes(16, 64) == 448
    assert L.milo_w3_packed_bytes(8, 64) == 0 and L.milo_w3_packed_bytes(16, 100) == 0
    assert L.milo_w3lr_gemm_workspace(16, 1024, 1024, 16) >= 16 * 16 * 2
    assert L.milo_w3lr_gemm_workspace(0, 1024, 1024, 16) == 0
    assert L.milo_moe_w3lr_workspace(512, 4096, 14336, 8, 2, 64) > 512 * 2 * (14336 * 2 + 4096 * 4)
    assert L.milo_moe_w3lr_workspace(512, 4096, 100, 8, 2, 64) == 0


def test_host_side_argument_errors(L):
    p = ctypes.c_void_p(0x10000)       # never dereferenced: validation fails first
    null = ctypes.c_void_p(0)
    odd = ctypes.c_void_p(0x10008)
    st = ctypes.c_void_p(0)
    assert L.milo_pack_w3(null, 16, 64, 64, p, st) == 1
    assert L.milo_pack_w3(p, 16, 64, 128, p, st) == 3          # group size must be 64
    assert L.milo_pack_w3(p, 16, 100, 64, p, st) == 2
    assert L.milo_pack_w3(p, 8, 64, 64, p, st) == 2
    assert L.milo_pack_w3(odd, 16, 64, 64, p, st) == 7
    assert L.milo_unpack_w3(null, 16, 64, p, p, p, st) == 1
    assert L.milo_unpack_w3(p, 16, 64, null, null, null, st) == 1
    assert L.milo_dequant_w3(p, 16, 65, p, st) == 2
    big = 1 << 20
    g = lambda **kw: L.milo_w3lr_gemm(kw.get("X", p), kw.get("M", 16), kw.get("N", 1024),
                                      kw.get("K", 1024), p, kw.get("U", p), kw.get("V", p),
                                      kw.get("r", 16), p, kw.get("ws", p), kw.get("wsb", big), st)
    assert g(X=null) == 1
    assert g(M=0) == 2 and g(K=1000) == 2 and g(N=1000) == 2
    assert g(r=-1) == 4 and g(r=2048) == 4 and g(U=null) == 4
    assert g(ws=null) == 5 and g(wsb=16) == 5
    assert g(X=odd) == 7
    # MoE
    experts = (api.Expert * 2)()
    assert L.milo_moe_w3lr_check_experts(experts, 2, 256, 512, None) == 1      # NULL weight pointers
    w = api.Weight(0x10000, 0, 0, 0, 0)
    for e in range(2):
        experts[e] = api.Expert(w, w, w)
    rmax = ctypes.c_int(-1)
    assert L.milo_moe_w3lr_check_experts(experts, 2, 256, 512, ctypes.byref(rmax)) == 0
    assert rmax.value == 0
    experts[1].w2.r = 8                                                          # rank without U, V
    assert L.milo_moe_w3lr_check_experts(experts, 2, 256, 512, None) == 4
    experts[1].w2.r = 0
    assert L.milo_moe_w3lr_check_experts(experts, 2, 250, 512, None) == 2
    f = lambda **kw: L.milo_moe_w3lr_forward(kw.get("X", p), kw.get("T", 32), 256, 512, p, 2,
                                             kw.get("r", 0), p, p, kw.get("topk", 2), p,
                                             kw.get("ws", p), kw.get("wsb", 1 << 30), st)
    assert f(X=null) == 1 and f(T=0) == 2 and f(topk=0) == 2
    assert f(ws=null) == 5 and f(wsb=1024) == 5
    assert f(r=1000) == 4
    # status query
    assert L.milo_workspace_status(null, st) == 1
    assert L.milo_workspace_status(odd, st) == 7


def test_compressor_argument_errors(L):
    # milo_compress_w3lr validates on the host before it touches the device
    p = ctypes.c_void_p(0x10000)
    null = ctypes.c_void_p(0)
    st = ctypes.c_void_p(0)
    eps = (ctypes.c_double * 32)()
    ran = ctypes.c_int(0)
    assert L.milo_compress_w3lr_workspace(14336, 4096, 32) > 14336 * 4096 * 4
    assert L.milo_compress_w3lr_workspace(1024, 1000, 8) == 0
    assert L.milo_compress_w3lr_workspace(1024, 1024, 129) == 0

    def call(W=p, N=1024, K=1024, ws=p, wsb=1 << 40, U=p, V=p, **kw):
        f = dict(rank=16, iters=20, hqq_iters=20, power_iters=2, refine_iters=0, p=0.7, beta=10.0, kappa=1.01,
                 tol=1e-4, seed=1)
        f.update(kw)
        prm = api.CompressParams(*(f[name] for name, _ in api.CompressParams._fields_))
        return L.milo_compress_w3lr(W, N, K, ctypes.byref(prm), p, U, V, eps, ctypes.byref(ran), ws, wsb, st)

    assert call(W=null) == 1 and call(U=null) == 1 and call(ws=null) == 1
    assert call(rank=-1) == 4 and call(rank=129) == 4 and call(N=16, K=64, rank=32) == 4
    assert call(K=1000) == 2 and call(N=1000) == 2
    assert call(iters=0) == 2 and call(hqq_iters=-1) == 2 and call(p=1.5) == 2 and call(beta=0.0) == 2
    assert call(wsb=1024) == 5
    assert call(W=ctypes.c_void_p(0x10008)) == 7


def test_bench_refuses_more_than_one_gpu():
    # the benchmark measures one GPU; asking for more ends with a message, before any GPU work
    import subprocess, sys, os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stderr + p.stdout)
