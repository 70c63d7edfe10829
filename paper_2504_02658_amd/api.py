"""ctypes binding over the C ABI of libmilo.so (see include/milo.h).

Argument marshalling only: every step of the path runs inside the HIP library.  PyTorch is
used for device memory and for the current stream, nothing else.  Importing this module
without a built library raises: there is no fallback path.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libmilo.so")
# the same library with every hand-counted memory wait replaced by a wait for everything (a check build)
FULLWAITS_LIB_PATH = os.path.join(_HERE, "lib", "libmilo_fullwaits.so")

STATUS_NAMES = {0: "MILO_OK", 1: "MILO_ERR_NULL", 2: "MILO_ERR_SHAPE", 3: "MILO_ERR_GROUP",
                4: "MILO_ERR_RANK", 5: "MILO_ERR_WORKSPACE", 6: "MILO_ERR_ROUTING",
                7: "MILO_ERR_ALIGN", 8: "MILO_ERR_WAIT", 100: "MILO_ERR_HIP"}

W3_SYMMETRIC = 1          # weight flags of include/milo.h
LR_INT3 = 2
ACT_BF16 = 4

# every symbol include/milo.h declares
EXPORTS = ("milo_status_string", "milo_version", "milo_w3_packed_bytes", "milo_pack_w3",
           "milo_pack_w3_sym", "milo_workspace_init", "milo_workspace_status",
           "milo_unpack_w3", "milo_dequant_w3", "milo_w3lr_gemm_workspace", "milo_w3lr_gemm",
           "milo_w3lr_gemm_static", "milo_w3lr_gemm_flags", "milo_lr3_packed_bytes", "milo_pack_lr3",
           "milo_moe_w3lr_check_experts", "milo_moe_w3lr_workspace", "milo_moe_w3lr_forward",
           "milo_moe_w3lr_routing_status", "milo_moe_w3lr_check_experts_flags", "milo_moe_w3lr_forward_flags",
           "milo_compress_w3lr_workspace", "milo_compress_w3lr")


class MiloError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        text = lib().milo_status_string(status).decode()
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({text})")


class Weight(ctypes.Structure):
    _fields_ = [("q3", ctypes.c_void_p), ("U", ctypes.c_void_p), ("V", ctypes.c_void_p), ("r", ctypes.c_int32),
                ("flags", ctypes.c_uint32)]


class CompressParams(ctypes.Structure):
    _fields_ = [("rank", ctypes.c_int32), ("iters", ctypes.c_int32), ("hqq_iters", ctypes.c_int32),
                ("power_iters", ctypes.c_int32), ("refine_iters", ctypes.c_int32), ("p", ctypes.c_float), ("beta", ctypes.c_float),
                ("kappa", ctypes.c_float), ("tol", ctypes.c_float), ("seed", ctypes.c_uint32)]


class Expert(ctypes.Structure):
    _fields_ = [("w1", Weight), ("w3", Weight), ("w2", Weight)]


_lib = None


def bind(path):
    """Load a build of the library and declare the C signatures of include/milo.h on it."""
    if not os.path.exists(path):
        raise ImportError(f"{path} is not built; run __graft_entry__.build() "
                          "(or paper_2504_02658_amd/csrc/build.sh)")
    L = ctypes.CDLL(path)
    vp, i64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    L.milo_status_string.restype = ctypes.c_char_p
    L.milo_status_string.argtypes = [ci]
    L.milo_version.restype = ci
    L.milo_w3_packed_bytes.restype = sz
    L.milo_w3_packed_bytes.argtypes = [i64, i64]
    L.milo_pack_w3.restype = ci
    L.milo_pack_w3.argtypes = [vp, i64, i64, ci, vp, vp]
    L.milo_pack_w3_sym.restype = ci
    L.milo_pack_w3_sym.argtypes = [vp, i64, i64, ci, vp, vp]
    L.milo_unpack_w3.restype = ci
    L.milo_unpack_w3.argtypes = [vp, i64, i64, vp, vp, vp, vp]
    L.milo_dequant_w3.restype = ci
    L.milo_dequant_w3.argtypes = [vp, i64, i64, vp, vp]
    L.milo_workspace_init.restype = ci
    L.milo_workspace_init.argtypes = [vp, sz, vp]
    L.milo_workspace_status.restype = ci
    L.milo_workspace_status.argtypes = [vp, vp]
    L.milo_w3lr_gemm_workspace.restype = sz
    L.milo_w3lr_gemm_workspace.argtypes = [i64, i64, i64, ci]
    L.milo_w3lr_gemm.restype = ci
    L.milo_w3lr_gemm.argtypes = [vp, i64, i64, i64, vp, vp, vp, ci, vp, vp, sz, vp]
    L.milo_w3lr_gemm_flags.restype = ci
    L.milo_w3lr_gemm_flags.argtypes = [vp, i64, i64, i64, vp, vp, vp, ci, ctypes.c_uint, vp, vp, sz, vp]
    L.milo_lr3_packed_bytes.restype = ci
    L.milo_lr3_packed_bytes.argtypes = [i64, i64, ci, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.milo_pack_lr3.restype = ci
    L.milo_pack_lr3.argtypes = [vp, vp, i64, i64, ci, vp, vp, vp]
    L.milo_w3lr_gemm_static.restype = ci
    L.milo_w3lr_gemm_static.argtypes = [vp, i64, i64, i64, vp, vp, vp, ci, vp, vp]
    L.milo_compress_w3lr_workspace.restype = sz
    L.milo_compress_w3lr_workspace.argtypes = [i64, i64, ci]
    L.milo_compress_w3lr.restype = ci
    L.milo_compress_w3lr.argtypes = [vp, i64, i64, ctypes.POINTER(CompressParams), vp, vp, vp,
                                     ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ci), vp, sz, vp]
    L.milo_moe_w3lr_check_experts.restype = ci
    L.milo_moe_w3lr_check_experts.argtypes = [ctypes.POINTER(Expert), ci, i64, i64,
                                              ctypes.POINTER(ci)]
    L.milo_moe_w3lr_check_experts_flags.restype = ci
    L.milo_moe_w3lr_check_experts_flags.argtypes = [ctypes.POINTER(Expert), ci, i64, i64, ctypes.c_uint,
                                                    ctypes.POINTER(ci)]
    L.milo_moe_w3lr_forward_flags.restype = ci
    L.milo_moe_w3lr_forward_flags.argtypes = [vp, i64, i64, i64, vp, ci, ci, vp, vp, ci, ctypes.c_uint, vp, vp, sz, vp]
    L.milo_moe_w3lr_workspace.restype = sz
    L.milo_moe_w3lr_workspace.argtypes = [i64, i64, i64, ci, ci, ci]
    L.milo_moe_w3lr_forward.restype = ci
    L.milo_moe_w3lr_forward.argtypes = [vp, i64, i64, i64, vp, ci, ci, vp, vp, ci, vp, vp, sz, vp]
    L.milo_moe_w3lr_routing_status.restype = ci
    L.milo_moe_w3lr_routing_status.argtypes = [vp, vp]
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = bind(LIB_PATH)
    return _lib


def _check(status, where):
    if status != 0:
        raise MiloError(status, where)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _dev(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous CUDA tensor of {dtype}")
    return t


class PackedWeight:
    """Device buffers of one packed [N x K] weight and its optional compensator (fp16 U [N, r] and
    V [r, K], or with the LR_INT3 flag the two blobs of pack_lr3)."""

    def __init__(self, N, K, q3, U=None, V=None, flags=0, r=None):
        self.N, self.K = int(N), int(K)
        self.q3 = q3                    # uint8 blob: codes, scales and zero-points
        self.U, self.V = U, V
        self.flags = int(flags)
        self._r = r

    @property
    def r(self):
        if self.U is None:
            return 0
        return int(self._r) if self._r is not None else int(self.U.shape[1])

    def with_compensator(self, U, V):
        """fp16 factors, or bf16 ones for calls with bf16 activations (MILO_ACT_BF16)."""
        dt = torch.bfloat16 if U.dtype == torch.bfloat16 else torch.float16
        U = _dev(U, dt, "U")
        V = _dev(V, dt, "V")
        assert U.shape[0] == self.N and V.shape[1] == self.K and U.shape[1] == V.shape[0]
        if U.shape[1] == 0:
            U = V = None
        return PackedWeight(self.N, self.K, self.q3, U, V, self.flags & ~LR_INT3)

    def with_int3_compensator(self, u3, v3, r):
        """u3, v3: the blobs written by pack_lr3 for this weight's shape and rank r."""
        return PackedWeight(self.N, self.K, self.q3, _dev(u3, torch.uint8, "u3"), _dev(v3, torch.uint8, "v3"),
                            self.flags | LR_INT3, r=int(r))

    def weight_bytes(self):
        n = self.q3.numel()
        if self.U is not None:
            n += self.U.numel() * self.U.element_size() + self.V.numel() * self.V.element_size()
        return n

    def c_struct(self):
        return Weight(self.q3.data_ptr(), 0 if self.U is None else self.U.data_ptr(),
                      0 if self.V is None else self.V.data_ptr(), self.r, self.flags)


def packed_bytes(N, K):
    return int(lib().milo_w3_packed_bytes(N, K))


def pack_w3(W, group_size=64, symmetric=False):
    """milo_pack_w3 (or milo_pack_w3_sym): fp32 CUDA weight [N, K] -> PackedWeight (no compensator)."""
    W = _dev(W, torch.float32, "W")
    N, K = W.shape
    nbytes = packed_bytes(N, K)
    q3 = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=W.device)
    fn, name = (lib().milo_pack_w3_sym, "milo_pack_w3_sym") if symmetric else (lib().milo_pack_w3, "milo_pack_w3")
    _check(fn(_ptr(W), N, K, group_size, _ptr(q3), _stream()), name)
    return PackedWeight(N, K, q3[:nbytes], flags=W3_SYMMETRIC if symmetric else 0)


def pack_lr3(U, V):
    """milo_pack_lr3: fp32 CUDA U [N, r], V [r, K] -> (u3, v3) uint8 blobs of the INT3 compensator."""
    U = _dev(U, torch.float32, "U")
    V = _dev(V, torch.float32, "V")
    N, r = U.shape
    K = V.shape[1]
    assert V.shape[0] == r
    ub, vb = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().milo_lr3_packed_bytes(N, K, r, ctypes.byref(ub), ctypes.byref(vb)), "milo_lr3_packed_bytes")
    u3 = torch.empty(ub.value, dtype=torch.uint8, device=U.device)
    v3 = torch.empty(vb.value, dtype=torch.uint8, device=U.device)
    _check(lib().milo_pack_lr3(_ptr(U), _ptr(V), N, K, r, _ptr(u3), _ptr(v3), _stream()), "milo_pack_lr3")
    return u3, v3


def compress_w3lr(W, r, iters=20, hqq_iters=20, power_iters=2, refine_iters=0, p=0.7, beta=10.0, kappa=1.01, tol=1e-4, seed=1):
    """milo_compress_w3lr (Algorithm 1): fp32 CUDA weight [N, K] -> (PackedWeight without compensator,
    U [N, r] fp32, V [r, K] fp32, list of the errors eps_t of the iterations run)."""
    W = _dev(W, torch.float32, "W")
    N, K = W.shape
    prm = CompressParams(r, iters, hqq_iters, power_iters, refine_iters, p, beta, kappa, tol, seed)
    nbytes = packed_bytes(N, K)
    q3 = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=W.device)
    U = torch.empty((N, max(r, 1)), dtype=torch.float32, device=W.device)[:, :r].contiguous()
    V = torch.empty((max(r, 1), K), dtype=torch.float32, device=W.device)[:r]
    wsb = int(lib().milo_compress_w3lr_workspace(N, K, r))
    if wsb == 0:
        _check(2 if 0 <= r <= min(N, K) else 4, "milo_compress_w3lr_workspace")
    ws = torch.empty(wsb, dtype=torch.uint8, device=W.device)
    eps = (ctypes.c_double * max(iters, 1))()
    ran = ctypes.c_int(0)
    _check(lib().milo_compress_w3lr(_ptr(W), N, K, ctypes.byref(prm), _ptr(q3), _ptr(U) if r else None,
                                    _ptr(V) if r else None, eps, ctypes.byref(ran), _ptr(ws), wsb, _stream()),
           "milo_compress_w3lr")
    return PackedWeight(N, K, q3[:nbytes]), U, V, [eps[i] for i in range(ran.value)]


def unpack_w3(pw):
    """milo_unpack_w3: (codes uint8 [N, K], scales fp16 [N, K/64], zeros fp16 [N, K/64])."""
    dev = pw.q3.device
    codes = torch.empty((pw.N, pw.K), dtype=torch.uint8, device=dev)
    scales = torch.empty((pw.N, pw.K // 64), dtype=torch.float16, device=dev)
    zeros = torch.empty((pw.N, pw.K // 64), dtype=torch.float16, device=dev)
    _check(lib().milo_unpack_w3(_ptr(pw.q3), pw.N, pw.K, _ptr(codes), _ptr(scales), _ptr(zeros),
                                _stream()), "milo_unpack_w3")
    return codes, scales, zeros


def dequant_w3(pw):
    out = torch.empty((pw.N, pw.K), dtype=torch.float16, device=pw.q3.device)
    _check(lib().milo_dequant_w3(_ptr(pw.q3), pw.N, pw.K, _ptr(out), _stream()), "milo_dequant_w3")
    return out


def new_workspace(nbytes, device="cuda"):
    """Allocate a workspace and prepare its control block (milo_workspace_init)."""
    ws = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
    _check(lib().milo_workspace_init(_ptr(ws), ws.numel(), _stream()), "milo_workspace_init")
    return ws


def workspace_status(workspace):
    """milo_workspace_status: 0, or MILO_ERR_WAIT (8) if a kernel's bounded wait gave up."""
    return int(lib().milo_workspace_status(_ptr(workspace), _stream()))


def gemm_workspace_bytes(M, N, K, r):
    return int(lib().milo_w3lr_gemm_workspace(M, N, K, r))


def w3lr_gemm(X, pw, out=None, workspace=None):
    """milo_w3lr_gemm: Y = X dequant(Q3)^T + (X V^T) U^T."""
    bf = isinstance(X, torch.Tensor) and X.dtype == torch.bfloat16
    X = _dev(X, torch.bfloat16 if bf else torch.float16, "X")
    M, K = X.shape
    if K != pw.K:
        raise ValueError("X and weight disagree on K")
    if pw.U is not None and not (pw.flags & LR_INT3) and pw.U.dtype != X.dtype:
        raise TypeError("the compensator and the activations must have the same 16-bit type")
    if out is None:
        out = torch.empty((M, pw.N), dtype=X.dtype, device=X.device)
    need = gemm_workspace_bytes(M, pw.N, K, pw.r)
    if workspace is None:
        workspace = new_workspace(need, X.device)
    flags = pw.flags | (ACT_BF16 if bf else 0)
    if flags == 0:
        _check(lib().milo_w3lr_gemm(_ptr(X), M, pw.N, K, _ptr(pw.q3), _ptr(pw.U), _ptr(pw.V), pw.r, _ptr(out),
                                    _ptr(workspace), workspace.numel(), _stream()), "milo_w3lr_gemm")
    else:
        _check(lib().milo_w3lr_gemm_flags(_ptr(X), M, pw.N, K, _ptr(pw.q3), _ptr(pw.U), _ptr(pw.V), pw.r, flags,
                                          _ptr(out), _ptr(workspace), workspace.numel(), _stream()),
               "milo_w3lr_gemm_flags")
    return out


def w3lr_gemm_static(X, pw, out=None):
    """milo_w3lr_gemm_static: the same linear on the library's own scratch array (no workspace)."""
    X = _dev(X, torch.float16, "X")
    M, K = X.shape
    if K != pw.K:
        raise ValueError("X and weight disagree on K")
    if out is None:
        out = torch.empty((M, pw.N), dtype=torch.float16, device=X.device)
    _check(lib().milo_w3lr_gemm_static(_ptr(X), M, pw.N, K, _ptr(pw.q3), _ptr(pw.U), _ptr(pw.V), pw.r, _ptr(out),
                                       _stream()), "milo_w3lr_gemm_static")
    return out


class MoELayer:
    """Expert table of one MoE layer: validates on the host, keeps the device copy of the table."""

    def __init__(self, experts, H, F, bf16=False):
        # experts: list of (w1, w3, w2) PackedWeight triples; bf16: the layer runs on bfloat16 activations
        # (compensators are bf16 arrays then)
        self.H, self.F, self.E = int(H), int(F), len(experts)
        self.flags = ACT_BF16 if bf16 else 0
        self.experts = experts                      # keeps the device buffers alive
        arr = (Expert * self.E)()
        for e, (w1, w3, w2) in enumerate(experts):
            arr[e] = Expert(w1.c_struct(), w3.c_struct(), w2.c_struct())
        rmax = ctypes.c_int(0)
        _check(lib().milo_moe_w3lr_check_experts_flags(arr, self.E, self.H, self.F, self.flags, ctypes.byref(rmax)),
               "milo_moe_w3lr_check_experts_flags")
        self.r_max = int(rmax.value)
        host = np.frombuffer(bytes(arr), dtype=np.uint8).copy()
        self.table = torch.from_numpy(host).cuda()
        self._ws = None

    def workspace_bytes(self, T, topk):
        return int(lib().milo_moe_w3lr_workspace(T, self.H, self.F, self.E, topk, self.r_max))

    def forward(self, X, ids, gates, out=None, workspace=None):
        dt = torch.bfloat16 if self.flags & ACT_BF16 else torch.float16
        X = _dev(X, dt, "X")
        ids = _dev(ids, torch.int32, "ids")
        gates = _dev(gates, torch.float32, "gates")
        T, H = X.shape
        topk = ids.shape[1]
        need = self.workspace_bytes(T, topk)
        if workspace is None:
            if self._ws is None or self._ws.numel() < need:
                self._ws = new_workspace(need, X.device)
            workspace = self._ws
        if out is None:
            out = torch.empty((T, H), dtype=dt, device=X.device)
        if self.flags:
            _check(lib().milo_moe_w3lr_forward_flags(_ptr(X), T, H, self.F, _ptr(self.table), self.E,
                                                     self.r_max, _ptr(ids), _ptr(gates), topk, self.flags, _ptr(out),
                                                     _ptr(workspace), workspace.numel(), _stream()),
                   "milo_moe_w3lr_forward_flags")
        else:
            _check(lib().milo_moe_w3lr_forward(_ptr(X), T, H, self.F, _ptr(self.table), self.E,
                                               self.r_max, _ptr(ids), _ptr(gates), topk, _ptr(out),
                                               _ptr(workspace), workspace.numel(), _stream()),
                   "milo_moe_w3lr_forward")
        self.last_workspace = workspace
        return out

    def routing_status(self):
        return int(lib().milo_moe_w3lr_routing_status(_ptr(self.last_workspace), _stream()))
