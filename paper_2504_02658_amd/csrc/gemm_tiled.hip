// Tiled MFMA kernel for the compensated W3A16 linear at M > 16, single or grouped per expert,
// and the small kernel that forms T = X V^T for the low-rank term.
//
// Work split.  A workgroup of four waves owns BM = 32*MB rows of the (expert-sorted) row space
// and a band of output features.  Each wave keeps two 32-row blocks of weights ("streams")
// entirely in registers: it loads their packed units straight from HBM, converts them to fp16
// with the bit trick (milo_device.h) and feeds them as the A operand of v_mfma_f32_32x32x16_f16.
// Weights therefore never pass through LDS.  The activations are the B operand; the workgroup
// stages a [BM x 128] slice per step in LDS (double buffered) in exactly the order the MFMA
// lanes read it, so every ds_read_b128 is conflict free, and each B fragment read from LDS is
// used by both streams of the wave.
//   NW = 1: the two streams are rows n0+64*wave.. and +32 of one weight (band of 256 features).
//   NW = 2: the streams are the same 32 rows of two weights (gate and up projection, band of
//           128 features) and the epilogue applies SiLU(gate) * up.
// The low-rank term is appended as extra k-steps [X | T] [W_dq | U]^T with U read as plain fp16.
#include "milo_host.h"
#include "milo_kernels.h"

namespace milo {

constexpr int kTiledThreads = 256;

struct TileInfo {
    int row0;
    int rows;
    WeightDev w[2];
    bool valid;
};

template <int NW>
__device__ __forceinline__ TileInfo resolve_tile(const RowSpace& rs, int tile, int bm) {
    TileInfo ti;
    ti.valid = true;
    if (rs.tiles) {
        if (tile >= *rs.n_tiles) {
            ti.valid = false;
            ti.row0 = 0;
            ti.rows = 0;
            return ti;
        }
        const TileDesc td = rs.tiles[tile];
        ti.row0 = td.row0;
        ti.rows = td.rows;
        const WeightDev* ew = reinterpret_cast<const WeightDev*>(rs.experts + td.expert);
        ti.w[0] = ew[rs.which[0]];
        ti.w[1] = ew[rs.which[NW - 1]];
    } else {
        ti.row0 = tile * bm;
        const int64_t left = rs.M - (int64_t)ti.row0;
        ti.rows = left < bm ? (int)left : bm;
        ti.w[0] = rs.w[0];
        ti.w[1] = rs.w[NW - 1];
        if (ti.rows <= 0) ti.valid = false;
    }
    return ti;
}

__device__ __forceinline__ int64_t input_row(const RowSpace& rs, int64_t R) {
    return rs.x_rows ? (int64_t)(rs.x_rows[R] / rs.x_row_div) : R;
}

// LDS offset (bytes) of the 16-byte slice "row block mb, MFMA step t, k-half h, row j" inside a
// stage.  For a fixed (mb, t) the 64 lanes (h, j) read one contiguous KB; the xor spreads the
// writer's lanes (same row, different t and h) over all 16 bank groups.
__device__ __forceinline__ int xs_offset(int mb, int t, int h, int j) {
    return ((mb * 8 + t) * 64 + h * 32 + (j ^ t ^ (h << 3))) * 16;
}

__device__ __forceinline__ float silu(float a) { return a / (1.0f + __expf(-a)); }

template <int NW, int MB, int EPI>
__global__ __launch_bounds__(kTiledThreads) void w3lr_tiled_kernel(const TiledArgs a) {
    constexpr int BM = 32 * MB;
    constexpr int BN = (NW == 1) ? 256 : 128;
    constexpr int STAGE = MB * 8 * 1024;         // bytes of one X stage
    constexpr int IT = 2 * MB;                   // 16-byte X slices per thread per stage
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * STAGE];

    const TileInfo ti = resolve_tile<NW>(a.rs, blockIdx.y, BM);
    if (!ti.valid) return;

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int i32 = lane & 31;
    const int h = lane >> 5;
    const int64_t N = a.N, K = a.K;
    const int G = (int)(K / kGroup);
    const int nchunks = (G + 1) / 2;
    const int64_t n0 = (int64_t)blockIdx.x * BN;

    // Weight streams of this wave.
    W3View view[2];
    int64_t nrow[2];        // output feature this lane feeds into the A operand
    int64_t ubase[2];       // unit index of (nrow, group 0)
    bool nvalid[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const WeightDev& w = ti.w[NW == 1 ? 0 : s];
        view[s] = make_view(w.q3, w.scales, w.zeros, N, K);
        const int64_t nb = (NW == 1) ? n0 + 64 * wave + 32 * s : n0 + 32 * wave;
        nrow[s] = nb + i32;
        nvalid[s] = nrow[s] < N;
        ubase[s] = unit_index(nvalid[s] ? nrow[s] : 0, 0, G);
    }

    // Activation rows this thread stages: slice q = tid + 256*it -> row q/16, 8 columns (q%16)*8.
    const f16* xrow[IT];
    int xoff[IT];
    int xseg[IT];
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const int q = tid + kTiledThreads * it;
        const int row = q >> 4, seg = q & 15;
        xseg[it] = seg;
        xoff[it] = xs_offset(row >> 5, seg & 7, seg >> 3, row & 31);
        xrow[it] = (row < ti.rows) ? a.X + input_row(a.rs, ti.row0 + row) * a.ldx : nullptr;
    }

    f32x16 acc[2][MB];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][mb][v] = 0.0f;

    auto load_x = [&](int c, u32x4 (&xr)[IT]) {
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int64_t k = (int64_t)c * 128 + xseg[it] * 8;
            if (xrow[it] != nullptr && k < K)
                xr[it] = *reinterpret_cast<const u32x4*>(xrow[it] + k);
            else
                xr[it] = u32x4{0u, 0u, 0u, 0u};
        }
    };
    auto store_x = [&](int stage, const u32x4 (&xr)[IT]) {
#pragma unroll
        for (int it = 0; it < IT; ++it)
            *reinterpret_cast<u32x4*>(smem + stage * STAGE + xoff[it]) = xr[it];
    };
    auto load_w = [&](int c, RawUnit (&ru)[2]) {
        const int g = 2 * c + h;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            if (nvalid[s] && g < G)
                ru[s] = load_unit<false>(view[s], ubase[s] + (int64_t)g * 16);
            else
                ru[s] = zero_unit();
        }
    };

    RawUnit raw[2];
    {
        u32x4 xr[IT];
        load_x(0, xr);
        load_w(0, raw);
        store_x(0, xr);
    }
    __syncthreads();

    for (int c = 0; c < nchunks; ++c) {
        const int cur = c & 1;
        const bool more = (c + 1) < nchunks;
        u32x4 xr[IT];
        RawUnit rawn[2];
        if (more) {
            load_x(c + 1, xr);
            load_w(c + 1, rawn);
        }
        const unsigned char* xs = smem + cur * STAGE;
#pragma unroll
        for (int s = 0; s < 2; ++s)
            dequant_unit_steps(raw[s], [&](int t, f16x8 frag) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const f16x8 b = __builtin_bit_cast(
                        f16x8, *reinterpret_cast<const u32x4*>(xs + xs_offset(mb, t, h, i32)));
                    acc[s][mb] = mfma32(frag, b, acc[s][mb]);
                }
            });
        if (more) {
            store_x(cur ^ 1, xr);
            raw[0] = rawn[0];
            raw[1] = rawn[1];
        }
        __syncthreads();
    }

    // Low-rank term: r extra k-steps with A = U rows and B = T rows.
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const WeightDev& w = ti.w[NW == 1 ? 0 : s];
        const int r = w.r;
        if (r <= 0) continue;
        const f16* Tm = a.T[NW == 1 ? 0 : s];
        const f16* urow = w.U + (nvalid[s] ? nrow[s] : 0) * (int64_t)r;
        const bool ualigned = (r & 7) == 0;
        for (int ks = 0; ks < r; ks += 16) {
            const int k0 = ks + 8 * h;
            f16x8 av = zero_f16x8();
            if (nvalid[s] && k0 < r) av = load_row8(urow, k0, r, ualigned);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int m = 32 * mb + i32;
                f16x8 bv = zero_f16x8();
                if (m < ti.rows) bv = load_f16x8(Tm + (int64_t)(ti.row0 + m) * a.ldt + k0);
                acc[s][mb] = mfma32(av, bv, acc[s][mb]);
            }
        }
    }

    // Epilogue.  D[v] of block (s, mb): feature nb + 8*(v/4) + 4*h + v%4, row 32*mb + i32.
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = 32 * mb + i32;
        if (m >= ti.rows) continue;
        const int64_t R = (int64_t)ti.row0 + m;
        if (EPI == EPI_SWIGLU) {
            const int64_t nb = n0 + 32 * wave;
            f16* orow = reinterpret_cast<f16*>(a.out) + R * a.ldo;
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int64_t n = nb + 8 * vq + 4 * h;
                if (n >= N) continue;
                f16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    o[e] = (f16)(silu(acc[0][mb][4 * vq + e]) * acc[1][mb][4 * vq + e]);
                *reinterpret_cast<f16x4*>(orow + n) = o;
            }
        } else {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int64_t nb = n0 + 64 * wave + 32 * s;
                if (EPI == EPI_STORE) {
                    f16* orow = reinterpret_cast<f16*>(a.out) + R * a.ldo;
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const int64_t n = nb + 8 * vq + 4 * h;
                        if (n >= N) continue;
                        f16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (f16)acc[s][mb][4 * vq + e];
                        *reinterpret_cast<f16x4*>(orow + n) = o;
                    }
                } else {
                    const int64_t orow_i = a.out_rows ? (int64_t)a.out_rows[R] : R;
                    const float sc = a.out_scale ? a.out_scale[orow_i] : 1.0f;
                    float* orow = reinterpret_cast<float*>(a.out) + orow_i * a.ldo;
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const int64_t n = nb + 8 * vq + 4 * h;
                        if (n >= N) continue;
                        f32x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = sc * acc[s][mb][4 * vq + e];
                        *reinterpret_cast<f32x4*>(orow + n) = o;
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// T = X V^T, fp16 [rows x ldt], columns >= r written as zero up to the next multiple of 16.
// One workgroup per 32 rows and weight; its four waves split K (k-step 16*w, 16*(w+4), ...)
// and are summed in a fixed order through LDS.  Ranks are processed 128 at a time.
__global__ __launch_bounds__(kTiledThreads) void t_kernel(const TArgs a) {
    __shared__ __attribute__((aligned(16))) float red[4][64][16];

    const int s = blockIdx.x;                 // weight stream
    const TileInfo ti = resolve_tile<2>(a.rs, blockIdx.y, a.bm);
    if (!ti.valid) return;
    const int sub0 = 32 * blockIdx.z;
    const int rows = ti.rows - sub0 < 32 ? ti.rows - sub0 : 32;
    if (rows <= 0) return;
    const WeightDev w = (s == 0) ? ti.w[0] : ti.w[1];
    const int r = w.r;
    if (r <= 0) return;
    const int rpad = (r + 15) & ~15;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int i32 = lane & 31, h = lane >> 5;
    const int64_t K = a.K;
    const int64_t R0 = (int64_t)ti.row0 + sub0;
    const f16* xrow = (i32 < rows) ? a.X + input_row(a.rs, R0 + i32) * a.ldx : nullptr;
    f16* Tm = (s == 0) ? a.T[0] : a.T[1];

    for (int jc = 0; jc < r; jc += 128) {
        const int left = r - jc;
        const int nb = left >= 128 ? 4 : (left + 31) / 32;
        f32x16 acc[4];
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[b][v] = 0.0f;
        const f16* vrow[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int j = jc + 32 * b + i32;
            vrow[b] = (j < r) ? w.V + (int64_t)j * K : nullptr;
        }
        for (int64_t k0 = 16 * wave; k0 < K; k0 += 64) {
            const int64_t k = k0 + 8 * h;
            const f16x8 bv = xrow ? load_f16x8(xrow + k) : zero_f16x8();
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                if (b < nb) {
                    const f16x8 av = vrow[b] ? load_f16x8(vrow[b] + k) : zero_f16x8();
                    acc[b] = mfma32(av, bv, acc[b]);
                }
            }
        }
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            if (b >= nb) continue;
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 16; ++v) red[wave][lane][v] = acc[b][v];
            __syncthreads();
            // thread (wave, lane) sums quarter vq = wave of D: rank 32b + 8*wave + 4h + e, row i32
            f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int p = 0; p < 4; ++p)
#pragma unroll
                for (int e = 0; e < 4; ++e) sum[e] += red[p][lane][4 * wave + e];
            const int j = jc + 32 * b + 8 * wave + 4 * h;
            if (i32 < rows && j < rpad) {
                f16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (f16)sum[e];
                *reinterpret_cast<f16x4*>(Tm + (R0 + i32) * a.ldt + j) = o;
            }
        }
    }
}

int launch_t_kernel(const TArgs& a, int nw, int m_tiles, hipStream_t stream) {
    if (m_tiles <= 0) return MILO_OK;
    dim3 grid((unsigned)nw, (unsigned)m_tiles, (unsigned)(a.bm / 32));
    t_kernel<<<grid, dim3(kTiledThreads), 0, stream>>>(a);
    return launch_status();
}

template <int NW, int EPI>
static int launch_tiled_mb(const TiledArgs& a, int mb, dim3 grid, hipStream_t stream) {
    switch (mb) {
        case 1: w3lr_tiled_kernel<NW, 1, EPI><<<grid, dim3(kTiledThreads), 0, stream>>>(a); break;
        case 2: w3lr_tiled_kernel<NW, 2, EPI><<<grid, dim3(kTiledThreads), 0, stream>>>(a); break;
        case 4: w3lr_tiled_kernel<NW, 4, EPI><<<grid, dim3(kTiledThreads), 0, stream>>>(a); break;
        default: return MILO_ERR_SHAPE;
    }
    return launch_status();
}

int launch_tiled(const TiledArgs& a, int nw, int mb, int epi, int m_tiles, hipStream_t stream) {
    if (m_tiles <= 0) return MILO_OK;
    const int bn = (nw == 1) ? 256 : 128;
    const int64_t n_tiles = (a.N + bn - 1) / bn;
    if (n_tiles > 0x7fffffff || m_tiles > 65535) return MILO_ERR_SHAPE;
    dim3 grid((unsigned)n_tiles, (unsigned)m_tiles, 1);
    if (nw == 2 && epi == EPI_SWIGLU) return launch_tiled_mb<2, EPI_SWIGLU>(a, mb, grid, stream);
    if (nw == 1 && epi == EPI_STORE) return launch_tiled_mb<1, EPI_STORE>(a, mb, grid, stream);
    if (nw == 1 && epi == EPI_SCALE_SCATTER)
        return launch_tiled_mb<1, EPI_SCALE_SCATTER>(a, mb, grid, stream);
    return MILO_ERR_SHAPE;
}

}  // namespace milo
