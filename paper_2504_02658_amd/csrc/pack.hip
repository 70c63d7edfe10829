// milo_pack_w3 / milo_unpack_w3 / milo_dequant_w3: group quantizer (Eq. wq, round-to-nearest
// reading), the zero-waste 3-bit packer (Section 3.3) and the two test aids.
//
// This translation unit is compiled with -ffp-contract=off: the quantizer must perform one
// binary32 rounding per operation (no fused multiply-add) so that its codes are reproducible
// bit for bit.
#include "milo_device.h"
#include "milo_host.h"
#include "pack_device.h"

namespace milo {

// SYM = false: asymmetric quantizer (Eq. wq).  SYM = true: the symmetric INT3 quantizer (Eq.
// symm_int3) in the same storage: the scale word holds the step 2 * max|w| / 7, the zero word 4.
// The source is element (n, k) = W[n * row_stride + k * col_stride] for n < n_valid and zero for the
// rows from n_valid up to N (a plain row-major weight has row_stride = K, col_stride = 1, n_valid = N;
// the compensator factors of milo_pack_lr3 come transposed or with padded rows).
template <bool SYM>
__global__ __launch_bounds__(kPackThreads) void pack_w3_kernel(
    const float* __restrict__ W, int64_t N, int64_t K, int64_t row_stride, int64_t col_stride, int64_t n_valid,
    uint32_t* __restrict__ planeA, uint32_t* __restrict__ planeB) {
    const int64_t G = K / kGroup;
    const int64_t total = N * G;
    const int64_t gu = (int64_t)blockIdx.x * kUnitsPerBlock + (threadIdx.x >> 4);
    const int l16 = threadIdx.x & 15;
    if (gu >= total) return;          // whole 16-lane groups leave together
    const int64_t n = gu / G;
    const int64_t g = gu - n * G;

    float4 v = {0.0f, 0.0f, 0.0f, 0.0f};
    if (n < n_valid) {
        const float* src = W + n * row_stride + (g * kGroup + 4 * l16) * col_stride;
        if (col_stride == 1) {
            v = *reinterpret_cast<const float4*>(src);
        } else {
            v.x = src[0];
            v.y = src[col_stride];
            v.z = src[2 * col_stride];
            v.w = src[3 * col_stride];
        }
    }
    float mn = fminf(fminf(v.x, v.y), fminf(v.z, v.w));
    float mx = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) {
        mn = fminf(mn, shfl_xor16(mn, m));
        mx = fmaxf(mx, shfl_xor16(mx, m));
    }

    f16 s16, z16;
    uint32_t q[4];
    const float in[4] = {v.x, v.y, v.z, v.w};
    if (SYM) {
        const float amax = fmaxf(mx, -mn);              // largest magnitude of the group
        const float s32 = (amax + amax) / 7.0f;
        s16 = (f16)s32;
        const float sf = (float)s16;
        z16 = (f16)4.0f;
        if (!(sf > 0.0f && sf <= 65504.0f)) {           // zero, NaN or overflowed step: all codes 4
            s16 = (f16)1.0f;
            q[0] = q[1] = q[2] = q[3] = 4u;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float t = in[i] / sf;
                t = __builtin_rintf(t);
                t = t + 4.0f;
                t = fminf(fmaxf(t, 0.0f), 7.0f);
                q[i] = (uint32_t)t;
            }
        }
    } else {
        const float s32 = (mx - mn) / 7.0f;
        s16 = (f16)s32;
        const float sf = (float)s16;
        const bool degenerate = !(sf > 0.0f && sf <= 65504.0f);   // zero, NaN or overflowed scale
        if (degenerate) {
            s16 = (f16)1.0f;
            z16 = (f16)(-mn);
            q[0] = q[1] = q[2] = q[3] = 0u;
        } else {
            float z = __builtin_rintf((-mn) / sf);
            z = fminf(fmaxf(z, -65504.0f), 65504.0f);
            z16 = (f16)z;
            const float zf = (float)z16;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float t = in[i] / sf;
                t = t + zf;
                t = __builtin_rintf(t);
                t = fminf(fmaxf(t, 0.0f), 7.0f);
                q[i] = (uint32_t)t;
            }
        }
    }

    store_unit(q, l16, s16, z16, unit_index(n, g, G), planeA, planeB);
}

// One thread per unit: unpack to bytes / dequantize to fp16.  Test aids, not tuned.
__global__ __launch_bounds__(256) void unpack_w3_kernel(W3View w, int64_t N, int64_t K,
                                                        uint8_t* __restrict__ codes,
                                                        unsigned short* __restrict__ scales,
                                                        unsigned short* __restrict__ zeros) {
    const int64_t G = w.G;
    const int64_t gu = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gu >= N * G) return;
    const int64_t n = gu / G, g = gu - n * G;
    const int64_t u = unit_index(n, g, G);
    const RawUnit ru = load_unit(w, u);
    const uint32_t d[6] = {ru.a.x, ru.a.y, ru.a.z, ru.a.w, ru.b.x, ru.b.y};
    if (scales) scales[gu] = (unsigned short)(ru.sz & 0xffffu);
    if (zeros) zeros[gu] = (unsigned short)(ru.sz >> 16);
    if (!codes) return;
    uint8_t* out = codes + n * K + g * kGroup;
    for (int P = 0; P < 32; ++P) {
        uint32_t lo, hi;
        if (P < 30) {
            const int j = P / 5, c = P % 5;
            lo = (d[j] >> (3 * c)) & 7u;
            hi = (d[j] >> (16 + 3 * c)) & 7u;
        } else {
            const int base = (P == 30) ? 0 : 3;
            lo = hi = 0u;
            for (int i = 0; i < 3; ++i) {
                lo |= ((d[base + i] >> 15) & 1u) << i;
                hi |= ((d[base + i] >> 31) & 1u) << i;
            }
        }
        out[2 * P] = (uint8_t)lo;
        out[2 * P + 1] = (uint8_t)hi;
    }
}

__global__ __launch_bounds__(256) void dequant_w3_kernel(W3View w, int64_t N, int64_t K,
                                                         f16* __restrict__ Wdq) {
    const int64_t G = w.G;
    const int64_t gu = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gu >= N * G) return;
    const int64_t n = gu / G, g = gu - n * G;
    const RawUnit ru = load_unit(w, unit_index(n, g, G));
    uint32_t wv[32];
    dequant_unit(ru, wv);
    u32x4* out = reinterpret_cast<u32x4*>(Wdq + n * K + g * kGroup);
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = u32x4{wv[4 * i], wv[4 * i + 1], wv[4 * i + 2], wv[4 * i + 3]};
}

}  // namespace milo

using namespace milo;

extern "C" size_t milo_w3_packed_bytes(int64_t N, int64_t K) {
    if (!weight_shape_ok(N, K)) return 0;
    return (size_t)(N * K / 64 * 28);
}

template <bool SYM>
static int pack_launch(const float* W, int64_t N, int64_t K, int group_size, void* q3, void* stream) {
    if (!W || !q3) return MILO_ERR_NULL;
    if (group_size != kGroup) return MILO_ERR_GROUP;
    if (!weight_shape_ok(N, K)) return MILO_ERR_SHAPE;
    if (!aligned16(W) || !aligned16(q3)) return MILO_ERR_ALIGN;
    const int64_t units = N * (K / kGroup);
    const int64_t blocks = (units + kUnitsPerBlock - 1) / kUnitsPerBlock;
    if (blocks > 0x7fffffff) return MILO_ERR_SHAPE;
    uint32_t* planeA = reinterpret_cast<uint32_t*>(q3);
    uint32_t* planeB = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(q3) + (N * K) / 4);
    pack_w3_kernel<SYM><<<dim3((unsigned)blocks), dim3(kPackThreads), 0, (hipStream_t)stream>>>(W, N, K, K, 1, N, planeA,
                                                                                               planeB);
    return launch_status();
}

static int64_t rank_rows(int r) { return ((int64_t)r + 15) / 16 * 16; }

extern "C" int milo_lr3_packed_bytes(int64_t N, int64_t K, int r, size_t* u_bytes, size_t* v_bytes) {
    if (r <= 0 || r > MILO_LR3_MAX_RANK) return MILO_ERR_RANK;
    if (!weight_shape_ok(N, K) || (N % kGroup) != 0 || !weight_shape_ok(rank_rows(r), N) || !weight_shape_ok(rank_rows(r), K))
        return MILO_ERR_SHAPE;
    if (u_bytes) *u_bytes = (size_t)(rank_rows(r) * N / 64 * 28);
    if (v_bytes) *v_bytes = (size_t)(rank_rows(r) * K / 64 * 28);
    return MILO_OK;
}

extern "C" int milo_pack_lr3(const float* U, const float* V, int64_t N, int64_t K, int r, void* u3, void* v3,
                             void* stream) {
    if (!U || !V || !u3 || !v3) return MILO_ERR_NULL;
    const int st = milo_lr3_packed_bytes(N, K, r, nullptr, nullptr);
    if (st != MILO_OK) return st;
    if (!aligned16(U) || !aligned16(V) || !aligned16(u3) || !aligned16(v3)) return MILO_ERR_ALIGN;
    const int64_t rp = rank_rows(r);
    // U^T: [rp x N], element (j, n) = U[n * r + j], groups of 64 along N
    {
        const int64_t units = rp * (N / kGroup), blocks = (units + kUnitsPerBlock - 1) / kUnitsPerBlock;
        uint32_t* planeA = reinterpret_cast<uint32_t*>(u3);
        uint32_t* planeB = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(u3) + (rp * N) / 4);
        pack_w3_kernel<true><<<dim3((unsigned)blocks), dim3(kPackThreads), 0, (hipStream_t)stream>>>(U, rp, N, 1, r, r,
                                                                                                planeA, planeB);
        if (launch_status() != MILO_OK) return MILO_ERR_HIP;
    }
    // V: [rp x K], element (j, k) = V[j * K + k], groups of 64 along K
    {
        const int64_t units = rp * (K / kGroup), blocks = (units + kUnitsPerBlock - 1) / kUnitsPerBlock;
        uint32_t* planeA = reinterpret_cast<uint32_t*>(v3);
        uint32_t* planeB = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(v3) + (rp * K) / 4);
        pack_w3_kernel<true><<<dim3((unsigned)blocks), dim3(kPackThreads), 0, (hipStream_t)stream>>>(V, rp, K, K, 1, r,
                                                                                                planeA, planeB);
    }
    return launch_status();
}

extern "C" int milo_pack_w3(const float* W, int64_t N, int64_t K, int group_size, void* q3, void* stream) {
    return pack_launch<false>(W, N, K, group_size, q3, stream);
}

extern "C" int milo_pack_w3_sym(const float* W, int64_t N, int64_t K, int group_size, void* q3, void* stream) {
    return pack_launch<true>(W, N, K, group_size, q3, stream);
}

extern "C" int milo_unpack_w3(const void* q3, int64_t N, int64_t K, uint8_t* codes, milo_half* scales,
                              milo_half* zeros, void* stream) {
    if (!q3 || (!codes && !scales && !zeros)) return MILO_ERR_NULL;
    if (!weight_shape_ok(N, K)) return MILO_ERR_SHAPE;
    if (!aligned16(q3)) return MILO_ERR_ALIGN;
    const int64_t units = N * (K / kGroup);
    const int64_t blocks = (units + 255) / 256;
    if (blocks > 0x7fffffff) return MILO_ERR_SHAPE;
    W3View w = make_view(q3, N, K);
    unpack_w3_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>(w, N, K, codes, scales, zeros);
    return launch_status();
}

extern "C" int milo_dequant_w3(const void* q3, int64_t N, int64_t K, milo_half* W_dq, void* stream) {
    if (!q3 || !W_dq) return MILO_ERR_NULL;
    if (!weight_shape_ok(N, K)) return MILO_ERR_SHAPE;
    if (!aligned16(q3) || !aligned16(W_dq)) return MILO_ERR_ALIGN;
    const int64_t units = N * (K / kGroup);
    const int64_t blocks = (units + 255) / 256;
    if (blocks > 0x7fffffff) return MILO_ERR_SHAPE;
    W3View w = make_view(q3, N, K);
    dequant_w3_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>(
        w, N, K, reinterpret_cast<f16*>(W_dq));
    return launch_status();
}
