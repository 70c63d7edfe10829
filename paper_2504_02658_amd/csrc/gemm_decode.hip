// Weight-streaming kernel for the compensated W3A16 linear at M <= 16 (decode).
//
// The job is bound by reading the packed weight once from HBM, so the kernel is organised
// around the weight stream: a workgroup of four waves owns 32 output features (two 16-row
// blocks) over the whole K.  K is walked in stages of 1024; inside a stage wave w takes the
// 256-wide chunk w, so that one lane of one wave loads exactly one unit (24 bytes of codes,
// one scale, one zero-point) per row block and chunk with fully coalesced 16- and 8-byte
// loads, several stages ahead of their use.  The lane converts its unit in registers and
// feeds it as the A operand of v_mfma_f32_16x16x32_f16 (lane quad q = group 4c+q, eight steps
// of eight codes); the activations are the B operand, staged per stage in LDS in MFMA lane
// order (double buffered) and shared by both row blocks.  At the end the four waves' partial
// sums are added in a fixed order through LDS, the low-rank term T U^T is added with a few
// more MFMAs and the tile is rounded once to fp16.
#include "milo_host.h"
#include "milo_kernels.h"

namespace milo {

constexpr int kDecThreads = 256;
constexpr int kDecRows = 32;            // output features per workgroup
constexpr int kDecStageK = 1024;        // k per stage (4 waves x 256)
constexpr int kDecStageBytes = 16 * kDecStageK * 2;   // X stage for 16 rows
constexpr int kDecAhead = 2;            // stages of weights in flight beyond the current one

// 16-byte slice "chunk c (0..3), step t, k-quad q, row j" of an X stage.
__device__ __forceinline__ int dec_xs_offset(int c, int t, int q, int j) {
    return ((c * 8 + t) * 64 + q * 16 + (j ^ t ^ ((c & 1) << 3))) * 16;
}

struct DecTask {
    RawUnit u[2];
};

__global__ __launch_bounds__(kDecThreads) void w3lr_decode_kernel(const DecodeArgs a) {
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * kDecStageBytes];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int j16 = lane & 15, q = lane >> 4;
    const int M = a.M;
    const int64_t N = a.N, K = a.K;
    const int G = (int)(K / kGroup);
    const int nstages = (int)((K + kDecStageK - 1) / kDecStageK);
    const int64_t n0 = (int64_t)blockIdx.x * kDecRows;

    const W3View view = make_view(a.w.q3, a.w.scales, a.w.zeros, N, K);
    int64_t ubase[2];
    bool nvalid[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int64_t n = n0 + 16 * b + j16;
        nvalid[b] = n < N;
        ubase[b] = unit_index(nvalid[b] ? n : 0, 0, G);
    }

    auto load_w = [&](int stage, DecTask& t) {
        const int g = (stage * 4 + wave) * 4 + q;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            if (nvalid[b] && g < G)
                t.u[b] = load_unit<true>(view, ubase[b] + (int64_t)g * 16);
            else
                t.u[b] = zero_unit();
        }
    };

    // X staging: slice id = tid + 256*it over (row, 128 slices of 8 columns); only rows < M.
    constexpr int XIT = 16 * 128 / kDecThreads;   // 8 slices per thread at M = 16
    auto load_x = [&](int stage, u32x4 (&xr)[XIT]) {
#pragma unroll
        for (int it = 0; it < XIT; ++it) {
            const int id = tid + kDecThreads * it;
            const int row = id >> 7, seg = id & 127;
            const int64_t k = (int64_t)stage * kDecStageK + seg * 8;
            if (row < M && k < K)
                xr[it] = *reinterpret_cast<const u32x4*>(a.X + (int64_t)row * K + k);
            else
                xr[it] = u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto store_x = [&](int buf, const u32x4 (&xr)[XIT]) {
#pragma unroll
        for (int it = 0; it < XIT; ++it) {
            const int id = tid + kDecThreads * it;
            const int row = id >> 7, seg = id & 127;
            if (row < M)
                *reinterpret_cast<u32x4*>(smem + buf * kDecStageBytes +
                                          dec_xs_offset(seg >> 5, seg & 7, (seg >> 3) & 3, row)) = xr[it];
        }
    };

    f32x4 acc[2];
    acc[0] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    acc[1] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // Weight ring: stages s .. s+kDecAhead are in registers (slot = stage % ring size).
    DecTask ring[kDecAhead + 1];
#pragma unroll
    for (int i = 0; i <= kDecAhead; ++i) {
        if (i < nstages)
            load_w(i, ring[i]);
        else
            ring[i].u[0] = ring[i].u[1] = zero_unit();
    }
    {
        u32x4 xr[XIT];
        load_x(0, xr);
        store_x(0, xr);
    }
    __syncthreads();

    // The stage loop is unrolled by the ring depth so that ring slots are compile-time names
    // (no register shuffling): stage s lives in slot s % (kDecAhead + 1).
    for (int s0 = 0; s0 < nstages; s0 += kDecAhead + 1) {
#pragma unroll
        for (int slot = 0; slot <= kDecAhead; ++slot) {
            const int s = s0 + slot;
            if (s >= nstages) break;
            const int cur = s & 1;
            const bool more = (s + 1) < nstages;
            u32x4 xr[XIT];
            if (more) load_x(s + 1, xr);

            uint32_t wv[2][32];
            dequant_unit(ring[slot].u[0], wv[0]);
            dequant_unit(ring[slot].u[1], wv[1]);
            if (s + 1 + kDecAhead < nstages) load_w(s + 1 + kDecAhead, ring[slot]);

            const unsigned char* xs = smem + cur * kDecStageBytes;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                f16x8 b = zero_f16x8();
                if (j16 < M)
                    b = __builtin_bit_cast(
                        f16x8,
                        *reinterpret_cast<const u32x4*>(xs + dec_xs_offset(wave, t, q, j16)));
                acc[0] = mfma16(unit_frag(wv[0], t), b, acc[0]);
                acc[1] = mfma16(unit_frag(wv[1], t), b, acc[1]);
            }
            if (more) store_x(cur ^ 1, xr);
            __syncthreads();
        }
    }

    // Cross-wave reduction (fixed order) + low-rank term + store: wave b finishes row block b.
    f32x4* red = reinterpret_cast<f32x4*>(smem);          // [wave][block][lane]
    red[(wave * 2 + 0) * 64 + lane] = acc[0];
    red[(wave * 2 + 1) * 64 + lane] = acc[1];
    __syncthreads();
    if (wave < 2) {
        const int b = wave;
        f32x4 sum = red[(0 * 2 + b) * 64 + lane];
#pragma unroll
        for (int p = 1; p < 4; ++p) {
            const f32x4 v = red[(p * 2 + b) * 64 + lane];
#pragma unroll
            for (int e = 0; e < 4; ++e) sum[e] += v[e];
        }
        const int r = a.w.r;
        if (r > 0) {
            const bool ualigned = (r & 7) == 0;
            const f16* urow = a.w.U + (nvalid[b] ? (n0 + 16 * b + j16) : 0) * (int64_t)r;
            for (int ks = 0; ks < r; ks += 32) {
                const int k0 = ks + 8 * q;
                f16x8 av = zero_f16x8(), bv = zero_f16x8();
                if (nvalid[b] && k0 < r) av = load_row8(urow, k0, r, ualigned);
                if (j16 < M && k0 < a.ldt) bv = load_f16x8(a.T + (int64_t)j16 * a.ldt + k0);
                sum = mfma16(av, bv, sum);
            }
        }
        // D[v]: feature n0 + 16b + 4q + v, token j16
        const int64_t n = n0 + 16 * b + 4 * q;
        if (j16 < M && n < N) {
            f16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (f16)sum[e];
            *reinterpret_cast<f16x4*>(a.Y + (int64_t)j16 * N + n) = o;
        }
    }
}

int launch_decode(const DecodeArgs& a, hipStream_t stream) {
    const int64_t blocks = (a.N + kDecRows - 1) / kDecRows;
    if (blocks > 0x7fffffff) return MILO_ERR_SHAPE;
    w3lr_decode_kernel<<<dim3((unsigned)blocks), dim3(kDecThreads), 0, stream>>>(a);
    return launch_status();
}

}  // namespace milo
