// Status text, version and the single-linear entry point milo_w3lr_gemm.
#include <stdlib.h>

#include "milo_host.h"
#include "milo_kernels.h"

using namespace milo;

extern "C" const char* milo_status_string(int status) {
    switch (status) {
        case MILO_OK: return "ok";
        case MILO_ERR_NULL: return "a required pointer is NULL";
        case MILO_ERR_SHAPE: return "invalid shape (need K % 64 == 0, N % 16 == 0, M >= 1, sizes in range)";
        case MILO_ERR_GROUP: return "group size must be 64";
        case MILO_ERR_RANK: return "invalid rank (need 0 <= r <= min(N, K), U and V given when r > 0)";
        case MILO_ERR_WORKSPACE: return "workspace missing or too small";
        case MILO_ERR_ROUTING: return "expert id out of range";
        case MILO_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case MILO_ERR_WAIT: return "a bounded wait inside a kernel gave up; re-initialise the workspace";
        case MILO_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

extern "C" int milo_version(void) { return 200; }

namespace milo {
__global__ void clear_kernel(u32x4* p, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        p[i] = u32x4{0u, 0u, 0u, 0u};
}
}  // namespace milo

extern "C" int milo_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
    if (!workspace) return MILO_ERR_NULL;
    if (workspace_bytes < 256) return MILO_ERR_WORKSPACE;
    if (!aligned16(workspace)) return MILO_ERR_ALIGN;
    const size_t n16 = workspace_bytes / 16;
    const size_t blocks = (n16 + 255) / 256;
    clear_kernel<<<dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, (hipStream_t)stream>>>(
        reinterpret_cast<u32x4*>(workspace), n16);
    return launch_status();
}

namespace milo {
bool gemm_takes_decode(int64_t M, int64_t N, int64_t K, int r) {
    // Up to 16 rows the weight-streaming kernel wins on every shape measured (the tiled kernel at a
    // 32-row tile needs K splits and a second kernel for so few tiles: 1.3 to 2 times slower).
    (void)N; (void)K; (void)r;
    return M <= 16;
}
}  // namespace milo

static int64_t rank_pad(int r) { return ((int64_t)r + 15) / 16 * 16; }

// Tile height (in blocks of 32 rows) and K splits of the tiled kernel for an [M x N x K] problem.
static int gemm_mb(int64_t M) {
    // tile height / 32; measured on N = 14336, K = 4096: up to 64 rows the shallow tile wins, up to
    // a few hundred rows two 64-row tiles beat one tall one
    int mb = M <= 64 ? 1 : (M <= 384 ? 2 : 4);
    // tuning override, read once per process so that the workspace query and the call agree
    static const int mb_override = [] {
        const char* e = getenv("MILO_GEMM_MB");
        const int v = e ? atoi(e) : 0;
        return (v == 1 || v == 2 || v == 4) ? v : 0;
    }();
    if (mb_override) mb = mb_override;
    return mb;
}
static int gemm_splits(int64_t M, int64_t N, int64_t K, int r) {
    const int bm = 32 * gemm_mb(M);
    const int64_t m_tiles = (M + bm - 1) / bm;
    return tiled_k_splits(m_tiles * ((N + 255) / 256), K, r > 0 ? m_tiles * tiled_t_parts(K) : 0);
}
// Parts of T = X V^T per M-tile for the single GEMM.  T must be there when the column tiles reach their
// epilogue: a part should take at most half as long as a column tile's share of K.  A part walks its
// chunks once per 256 ranks, and with K splits a column tile's share is short, so both call for more
// (shorter) parts than the default of eight chunks each.
static int gemm_t_parts(int64_t M, int64_t N, int64_t K, int r) {
    if (r <= 0) return 0;
    const int base = tiled_t_parts(K);
    const int64_t nchunks = (K / 64 + 1) / 2;
    const int64_t cps = (nchunks + gemm_splits(M, N, K, r) - 1) / gemm_splits(M, N, K, r);
    const int64_t passes = ((int64_t)r + 255) / 256;
    int64_t cpp = cps / (2 * passes);
    if (cpp < 1) cpp = 1;
    int64_t parts = (nchunks + cpp - 1) / cpp;
    if (parts > 16) parts = 16;
    return parts > base ? (int)parts : base;
}

// Adds the fp32 partial sums of the K splits in split order and rounds once.
template <bool BF>
__global__ __launch_bounds__(256) void splitk_sum_kernel(const float* __restrict__ part, int splits,
                                                         int64_t n4, int64_t stride, f16* __restrict__ Y) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n4) return;
    f32x4 sum = *reinterpret_cast<const f32x4*>(part + 4 * i);
    for (int s = 1; s < splits; ++s) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(part + (int64_t)s * stride + 4 * i);
#pragma unroll
        for (int e = 0; e < 4; ++e) sum[e] += v[e];
    }
    if (BF) {
        *reinterpret_cast<u32x2*>(Y + 4 * i) = u32x2{pack_bf16(sum[0], sum[1]), pack_bf16(sum[2], sum[3])};
        return;
    }
    f16x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (f16)sum[e];
    *reinterpret_cast<f16x4*>(Y + 4 * i) = o;
}

static bool gemm_shape_ok(int64_t M, int64_t N, int64_t K) {
    return M >= 1 && M <= (int64_t)0x3fffffff && weight_shape_ok(N, K);
}

extern "C" size_t milo_w3lr_gemm_workspace(int64_t M, int64_t N, int64_t K, int r) {
    if (!gemm_shape_ok(M, N, K) || r < 0) return 0;
    if (gemm_takes_decode(M, N, K, r)) return decode_workspace_bytes(r, K);
    // control words | four flag words per 32-row tile | T = X V^T, fp16 [M x pad16(r)] | its fp32
    // partials per part of K | with K splits, their fp32 partial sums [M x N] each
    const size_t parts = (size_t)gemm_t_parts(M, N, K, r);
    const int splits = gemm_splits(M, N, K, r);
    return 256 + align_up((size_t)((M + 31) / 32) * 16, 256) +
           align_up((size_t)M * (size_t)rank_pad(r) * 2 + 256, 256) +
           align_up(parts * (size_t)M * (size_t)rank_pad(r) * 4 + 256, 256) +
           (splits > 1 ? align_up((size_t)splits * (size_t)M * (size_t)N * 4, 256) : 0);
}

extern "C" int milo_w3lr_gemm(const milo_half* X, int64_t M, int64_t N, int64_t K, const void* q3,
                              const milo_half* U, const milo_half* V, int r, milo_half* Y, void* workspace,
                              size_t workspace_bytes, void* stream_) {
    return milo_w3lr_gemm_flags(X, M, N, K, q3, U, V, r, 0u, Y, workspace, workspace_bytes, stream_);
}

extern "C" int milo_w3lr_gemm_flags(const milo_half* X, int64_t M, int64_t N, int64_t K, const void* q3,
                                    const void* U, const void* V, int r, unsigned flags, milo_half* Y,
                                    void* workspace, size_t workspace_bytes, void* stream_) {
    if (!X || !q3 || !Y) return MILO_ERR_NULL;
    if (!gemm_shape_ok(M, N, K)) return MILO_ERR_SHAPE;
    if (flags & ~(MILO_W3_SYMMETRIC | MILO_LR_INT3 | MILO_ACT_BF16)) return MILO_ERR_SHAPE;
    if ((flags & MILO_ACT_BF16) && (flags & MILO_LR_INT3) && r > 0) return MILO_ERR_SHAPE;
    if (r < 0 || r > N || r > K) return MILO_ERR_RANK;
    if (r > 0 && (!U || !V)) return MILO_ERR_RANK;
    if (r == 0) flags &= ~MILO_LR_INT3;
    if (flags & MILO_LR_INT3) {
        if (r > MILO_LR3_MAX_RANK) return MILO_ERR_RANK;
        if ((N % kGroup) != 0) return MILO_ERR_SHAPE;
    }
    if (!workspace || workspace_bytes < milo_w3lr_gemm_workspace(M, N, K, r))
        return MILO_ERR_WORKSPACE;
    if (!aligned16(X) || !aligned16(q3) ||
        !aligned16(Y) || !aligned16(workspace) || (r > 0 && (!aligned16(U) || !aligned16(V))))
        return MILO_ERR_ALIGN;
    hipStream_t stream = (hipStream_t)stream_;

    WeightDev w;
    w.q3 = q3;
    w.U = reinterpret_cast<const f16*>(U);
    w.V = reinterpret_cast<const f16*>(V);
    w.r = r;
    w.flags = flags;
    const bool decode = gemm_takes_decode(M, N, K, r);
    if (decode) {
        // 32-bit buffer offsets in the decode kernel
        if ((uint64_t)M * K * 2 >= 0xFFFFFFF0ull || ((uint64_t)r + 128) * K * 2 >= 0xFFFFFFF0ull ||
            (uint64_t)N * (uint64_t)(r > 0 ? r : 1) * 2 >= 0xFFFFFFF0ull)
            return MILO_ERR_SHAPE;
        DecodeArgs da;
        da.X = reinterpret_cast<const f16*>(X); da.M = (int)M; da.N = N; da.K = K;
        da.w = w; da.Y = reinterpret_cast<f16*>(Y);
        return launch_decode(da, workspace, stream);
    }
    char* ws = reinterpret_cast<char*>(workspace);
    uint32_t* ctrl = reinterpret_cast<uint32_t*>(ws);
    uint32_t* tile_flags = reinterpret_cast<uint32_t*>(ws + 256);
    f16* T = reinterpret_cast<f16*>(ws + 256 + align_up((size_t)((M + 31) / 32) * 16, 256));
    const int64_t ldt = rank_pad(r);

    const int mb = gemm_mb(M);
    const int bm = 32 * mb;
    const int64_t m_tiles = (M + bm - 1) / bm;
    if (m_tiles > 65535) return MILO_ERR_SHAPE;
    const int parts = gemm_t_parts(M, N, K, r);
    const int splits = gemm_splits(M, N, K, r);
    if ((uint64_t)M * K * 2 >= 0x80000000ull || ((uint64_t)r + 256) * K * 2 >= 0xFFFFFFF0ull ||
        (uint64_t)(parts > 0 ? parts : 1) * M * ldt * 4 >= 0xFFFFFFF0ull || (N & 3) != 0)
        return MILO_ERR_SHAPE;                                          // 32-bit offsets in the kernel
    float* Tp = reinterpret_cast<float*>(reinterpret_cast<char*>(T) + align_up((size_t)M * (size_t)ldt * 2 + 256, 256));
    float* partial = reinterpret_cast<float*>(
        reinterpret_cast<char*>(Tp) + align_up((size_t)parts * (size_t)M * (size_t)ldt * 4 + 256, 256));

    RowSpace rs;
    rs.tiles = nullptr; rs.n_tiles = nullptr; rs.experts = nullptr;
    rs.which[0] = rs.which[1] = 0;
    rs.w[0] = rs.w[1] = w;
    rs.M = M; rs.x_rows = nullptr;

    TiledArgs ga;
    ga.rs = rs; ga.X = reinterpret_cast<const f16*>(X); ga.ldx = K; ga.x_bytes = (uint64_t)M * K * 2;
    ga.N = N; ga.K = K;
    ga.T[0] = ga.T[1] = T; ga.ldt = ldt; ga.t_bytes = (uint64_t)M * ldt * 2;
    ga.Tp[0] = ga.Tp[1] = Tp; ga.tp_bytes = (uint64_t)parts * M * ldt * 4;
    ga.t_part_stride = M * ldt; ga.t_parts = parts; ga.v_tiles = parts; ga.ksplit = splits;
    ga.flags = tile_flags; ga.flags_status = ctrl + 3; ga.weights_once = m_tiles == 1;
    ga.lr3_rank = (w.flags & MILO_LR_INT3) ? r : 0;
    ga.self_clean = 1;
    ga.act_bf16 = (flags & MILO_ACT_BF16) ? 1 : 0;
    // Ranks of the size the paper gives dense layers (Section 3.2.2, Dense-512, Dense-1024): the parts of T
    // share the addition of their partial sums, and with K splits every split applies a share of the
    // ranks (the fp32 partial sums of the splits are added anyway), in blocks of 64.
    ga.t_dist = r > 64 ? 1 : 0;
    ga.lr_splits = 1; ga.lr_step = 0;
    if (splits > 1 && r > 64) {
        const int nblk = (r + 63) / 64;
        const int per = (nblk + (splits < nblk ? splits : nblk) - 1) / (splits < nblk ? splits : nblk);
        ga.lr_step = 64 * per;
        ga.lr_splits = (nblk + per - 1) / per;
    }
    ga.out = splits > 1 ? static_cast<void*>(partial) : static_cast<void*>(Y);
    ga.ldo = N; ga.out_split_stride = M * N; ga.out_rows = nullptr; ga.out_scale = nullptr;
    int st = launch_tiled(ga, 1, mb, EPI_STORE, (int)m_tiles, stream);
    if (st != MILO_OK || splits == 1) return st;
    const int64_t n4 = M * N / 4;
    const int64_t blocks = (n4 + 255) / 256;
    if (blocks > 0x7fffffff) return MILO_ERR_SHAPE;
    if (flags & MILO_ACT_BF16)
        splitk_sum_kernel<true><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(partial, splits, n4, M * N,
                                                                              reinterpret_cast<f16*>(Y));
    else
        splitk_sum_kernel<false><<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(partial, splits, n4, M * N,
                                                                               reinterpret_cast<f16*>(Y));
    return launch_status();
}

// Word 3 of every workspace's control block is the "a wait gave up" word of the kernels that use it.
extern "C" int milo_workspace_status(const void* workspace, void* stream) {
    if (!workspace) return MILO_ERR_NULL;
    if (!aligned16(workspace)) return MILO_ERR_ALIGN;
    uint32_t words[4] = {0u, 0u, 0u, 0u};
    if (hipMemcpyAsync(words, workspace, sizeof(words), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess)
        return MILO_ERR_HIP;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return MILO_ERR_HIP;
    return words[3] != 0u ? MILO_ERR_WAIT : MILO_OK;
}
