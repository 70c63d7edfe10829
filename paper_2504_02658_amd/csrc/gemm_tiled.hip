// Tiled MFMA kernel for the compensated W3A16 linear at M > 16, single or grouped per expert,
// including the workgroups of the same launch that form T = X V^T for the low-rank term.
//
// Work split.  A workgroup of four waves owns BM = 32*MB rows of the (expert-sorted) row space
// and a band of output features.  Each wave keeps two 32-row blocks of weights ("streams")
// entirely in registers: it loads their packed units straight from HBM, converts them to fp16
// with the bit trick (milo_device.h) and feeds them as the A operand of v_mfma_f32_32x32x16_f16.
// Weights therefore never pass through LDS.  The activations are the B operand; the workgroup
// stages a [BM x 128] slice per step in LDS (double buffered) with coalesced buffer-to-LDS copies
// (no registers, no ds_write), swizzled so that every ds_read_b128 of a B fragment is conflict
// free, and each B fragment read from LDS is used by both streams of the wave.
//   NW = 1: the two streams are rows n0+64*wave.. and +32 of one weight (band of 256 features).
//   NW = 2: the streams are the same 32 rows of two weights (gate and up projection, band of
//           128 features) and the epilogue applies SiLU(gate) * up.
// The low-rank term is appended as extra k-steps [X | T] [W_dq | U]^T with U read as plain fp16.
#include <type_traits>

#include "milo_host.h"
#include "milo_kernels.h"

namespace milo {

constexpr int kTiledThreads = 256;
constexpr int kTiledStages = 3;      // chunks in flight per workgroup (LDS stages / register ring)

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
        if (td.rows <= 0) ti.valid = false;          // an empty slot of the tile list
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
    return rs.x_rows ? (int64_t)rs.x_rows[R] : R;
}

__device__ __forceinline__ float silu(float a) { return a / (1.0f + __expf(-a)); }

typedef __attribute__((address_space(3))) void* LdsPtr;
// Offset that lies outside every activation buffer (they are kept below 2 GiB) and stays outside
// when a column offset is added to it.
constexpr uint32_t kOobHalf = 0x80000000u;

// Spin until *flag reaches `target`.  The producers never wait and were dispatched earlier, so the
// wait ends; the bound only turns a broken assumption into an error code instead of a hang.
__device__ __forceinline__ void wait_flag(const uint32_t* flag, uint32_t target, uint32_t* status) {
    for (uint32_t spins = 0; __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target; ++spins) {
        __builtin_amdgcn_s_sleep(2);
        if (spins > (1u << 24)) {
            if (status) atomicOr(status, 1u);
            break;
        }
    }
}

// T = X V^T for one M-tile, computed with the same pipeline as the weight tiles: the activations
// are staged in LDS, the A operand is V read as plain fp16 (rank row = lane % 32, 64 columns per
// lane and chunk).  NW = 1: wave w, stream s take ranks 64w + 32s ..; NW = 2: stream s is weight s,
// ranks 32w ..; larger ranks take further passes.  T is written with device-coherent stores and
// published through the tile's flag.
template <int NW, int MB, bool BF>
__device__ __forceinline__ void v_tile_body(const TiledArgs& a, const TileInfo& ti, unsigned char* smem, int part,
                                            uint32_t by) {
    constexpr int BM = 32 * MB;
    constexpr int STAGE = BM * 256;
    constexpr int NCP = BM / 16;
    constexpr int PASS = (NW == 1) ? 256 : 128;     // ranks per weight covered by one pass

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int i32 = lane & 31, h = lane >> 5;
    const int64_t K = a.K;
    const int G = (int)(K / kGroup);
    const int nchunks = (G + 1) / 2;
    // this part's share of the chunks
    const int cpp = (nchunks + a.t_parts - 1) / a.t_parts;
    const int c_lo = part * cpp;
    const int c_hi = (c_lo + cpp < nchunks) ? c_lo + cpp : nchunks;

    const BufRsrc xb = make_rsrc(a.X, a.x_bytes);
    uint32_t xoff[NCP];
    bool xhi[NCP];
    {
        int32_t src[NCP];
#pragma unroll
        for (int i = 0; i < NCP; ++i) {
            const int row = 4 * (wave * NCP + i) + (lane >> 4);
            const int R = ti.row0 + (row < ti.rows ? row : 0);
            src[i] = a.rs.x_rows ? a.rs.x_rows[R] : R;
        }
#pragma unroll
        for (int i = 0; i < NCP; ++i) {
            const int row = 4 * (wave * NCP + i) + (lane >> 4);
            const int seg = (lane & 15) ^ (row & 15);
            xhi[i] = seg >= 8;
            xoff[i] = (row < ti.rows) ? (uint32_t)src[i] * (uint32_t)(a.ldx * 2) + (uint32_t)(seg * 16) : kOobHalf;
        }
    }
    const bool ktail = (G & 1) != 0;
    auto issue_x = [&](int c) {
        unsigned char* stage = smem + (c & 1) * STAGE;
        const bool last_half = ktail && c == nchunks - 1;
#pragma unroll
        for (int i = 0; i < NCP; ++i) {
            uint32_t off = xoff[i] + (uint32_t)c * 256u;
            if (last_half && xhi[i]) off = kOobHalf;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xb, (LdsPtr)(stage + (wave * NCP + i) * 1024), 16, off, 0, 0,
                                                     0);
        }
    };

    const int rmax = ti.w[0].r > ti.w[1].r ? ti.w[0].r : ti.w[1].r;
    // Ranks up to 32 (the experts' compensators) fit one 32-row MFMA stream.  Instead of one wave
    // multiplying every row block of the tile while three only copy, wave w then takes row block w
    // (waves past the tile's blocks only copy): the pass below is instantiated for MBT = MB row blocks
    // starting at block 0, or for MBT = 1 block starting at this wave's.
    const bool small = MB > 1 && rmax <= 32;
    auto pass = [&](auto mbt_c, const int blk0, const int pass0) {
        constexpr int MBT = decltype(mbt_c)::value;
        // rank row of each stream of this wave, and its V as a buffer (rows >= r read as zero)
        BufRsrc vb[2];
        uint32_t voff[2];
        int rank0[2];
        bool active[2];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const WeightDev& w = ti.w[NW == 1 ? 0 : s];
            rank0[s] = MBT != MB ? ((NW == 1) ? 32 * s : 0) : pass0 + ((NW == 1) ? 64 * wave + 32 * s : 32 * wave);
            active[s] = rank0[s] < w.r && (MBT == MB || wave < MB);
            vb[s] = make_rsrc(w.V, (uint64_t)(w.r > 0 ? w.r : 0) * (uint64_t)K * 2u);
            voff[s] = active[s] ? (uint32_t)(((int64_t)(rank0[s] + i32) * K + 64 * h) * 2) : kOobOffset;
        }
        f32x16 acc[2][MBT];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int mb = 0; mb < MBT; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[s][mb][v] = 0.0f;
        // one step of the product: A fragments a0, a1 (streams 0, 1) against the B fragments of this
        // wave's row blocks; xs points at row i32 of block 0 in the stage
        auto mfma_step = [&](const unsigned char* xs, int sx, int t, f16x8 a0, f16x8 a1) {
#pragma unroll
            for (int mb = 0; mb < MBT; ++mb) {
                const f16x8 b = __builtin_bit_cast(
                    f16x8, *reinterpret_cast<const u32x4*>(xs + (blk0 + mb) * 32 * 256 + (((8 * h + t) ^ sx) << 4)));
                if (BF) {       // (bf16 activations: V is bf16 as well, same bits in the fragments)
                    if (active[0])
                        acc[0][mb] = mfma32_bf16(__builtin_bit_cast(bf16x8, a0), __builtin_bit_cast(bf16x8, b), acc[0][mb]);
                    if (active[1])
                        acc[1][mb] = mfma32_bf16(__builtin_bit_cast(bf16x8, a1), __builtin_bit_cast(bf16x8, b), acc[1][mb]);
                } else {
                    if (active[0]) acc[0][mb] = mfma32(a0, b, acc[0][mb]);
                    if (active[1]) acc[1][mb] = mfma32(a1, b, acc[1][mb]);
                }
            }
        };

        // INT3 compensator (MILO_LR_INT3): V is a packed blob [pad16(r) x K] in the layout of a weight,
        // so lane (i32, h) loads the unit of rank rank0 + i32, group 2c + h, and converts it (symmetric
        // quantizer: no zero-point arithmetic) into the same eight fragments per chunk.
        const bool vq = ((ti.w[0].flags | ti.w[1].flags) & MILO_LR_INT3) != 0;     // (one setting per tile)
        if (vq) {
            W3Buf vqb[2];
            uint32_t vu[2];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const WeightDev& w = ti.w[NW == 1 ? 0 : s];
                const int rp = (w.r + 15) & ~15;
                vqb[s] = make_w3buf(w.V, rp, K);
                const int rank = rank0[s] + i32;
                vu[s] = (active[s] && rank < rp) ? (uint32_t)unit_index(rank, 0, G) : kOobUnit;
            }
            auto load_vq = [&](int c, int s) -> RawUnit {
                const bool out = vu[s] == kOobUnit || c >= c_hi || (ktail && c == nchunks - 1 && h == 1);
                return load_unit_buf(vqb[s], out ? (1u << 27) : vu[s] + (uint32_t)(2 * c + h) * 16u);
            };
            RawUnit cur[2], nxt[2];
            __syncthreads();            // a previous pass is done with the stages
            if (c_lo < c_hi) issue_x(c_lo);
            cur[0] = load_vq(c_lo, 0);
            cur[1] = load_vq(c_lo, 1);
            for (int c = c_lo; c < c_hi; ++c) {
                wait_vmem();
                pin_unit(cur[0]);
                pin_unit(cur[1]);
                __syncthreads();
                if (c + 1 < c_hi) issue_x(c + 1);
                nxt[0] = load_vq(c + 1, 0);
                nxt[1] = load_vq(c + 1, 1);
                const unsigned char* xs = smem + (c & 1) * STAGE + i32 * 256;
                const int sx = i32 & 15;
                if (active[0] || active[1]) {
                    dequant_units2_steps<true>(cur[0], cur[1],
                                               [&](int t, f16x8 a0, f16x8 a1) { mfma_step(xs, sx, t, a0, a1); });
                }
                cur[0] = nxt[0];
                cur[1] = nxt[1];
            }
        } else {
            // V fragment of step t of chunk c; out of range (inactive stream, ragged K tail) reads zero
            auto load_v = [&](int c, int s, int t) -> u32x4 {
                const bool out = !active[s] || c >= c_hi || (ktail && c == nchunks - 1 && h == 1);
                return buf_load16(vb[s], out ? kOobOffset : voff[s] + (uint32_t)c * 256u + 16u * t);
            };
            u32x4 va[2][8];
            __syncthreads();            // a previous pass is done with the stages
            if (c_lo < c_hi) issue_x(c_lo);
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int t = 0; t < 8; ++t) va[s][t] = load_v(c_lo, s, t);
            for (int c = c_lo; c < c_hi; ++c) {
                wait_vmem();
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int t = 0; t < 8; ++t)
                        asm volatile("" : "+v"(va[s][t].x), "+v"(va[s][t].y), "+v"(va[s][t].z), "+v"(va[s][t].w));
                __syncthreads();
                if (c + 1 < c_hi) issue_x(c + 1);
                const unsigned char* xs = smem + (c & 1) * STAGE + i32 * 256;
                const int sx = i32 & 15;
                // A wave without ranks or row blocks of its own only takes part in the copies and barriers.
                if (active[0] || active[1]) {
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        mfma_step(xs, sx, t, __builtin_bit_cast(f16x8, va[0][t]), __builtin_bit_cast(f16x8, va[1][t]));
                        // the registers of this step are free again: fetch the next chunk's fragment into them
                        va[0][t] = load_v(c + 1, 0, t);
                        va[1][t] = load_v(c + 1, 1, t);
                    }
                }
            }
        }
        // D[v] of (s, mb): rank rank0 + 8*(v/4) + 4*h + v%4, row 32*(blk0 + mb) + i32; ranks up to the
        // next multiple of 16 are written (they are exact zeros) because the consumers read that far.
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const WeightDev& w = ti.w[NW == 1 ? 0 : s];
            const int rpad = (w.r + 15) & ~15;
            const BufRsrc pb = make_rsrc(a.Tp[NW == 1 ? 0 : s], a.tp_bytes);
#pragma unroll
            for (int mb = 0; mb < MBT; ++mb) {
                const int m = 32 * (blk0 + mb) + i32;
#pragma unroll
                for (int vq4 = 0; vq4 < 4; ++vq4) {
                    const int rank = rank0[s] + 8 * vq4 + 4 * h;
                    f32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = acc[s][mb][4 * vq4 + e];
                    const bool ok = active[s] && m < ti.rows && rank < rpad;
                    __builtin_amdgcn_raw_buffer_store_b128(
                        __builtin_bit_cast(u32x4, o), pb,
                        ok ? (uint32_t)((part * a.t_part_stride + (ti.row0 + m) * a.ldt + rank) * 4) : kOobOffset, 0,
                        17);
                }
            }
        }
    };
    if (small) {
        pass(std::integral_constant<int, MB == 1 ? MB : 1>{}, wave, 0);
    } else {
        for (int pass0 = 0; pass0 < rmax; pass0 += PASS) pass(std::integral_constant<int, MB>{}, 0, pass0);
    }
    // This part is complete once its stores are; the last part of the tile to get here adds all
    // parts in part order (so the sum does not depend on which one that was), writes T as fp16
    // and raises the tile's flag.
    // With large ranks (t_dist) that sum is too much for one workgroup (t_parts x rows x ranks x 4 bytes
    // through a single CU): every part then waits until all parts are written, adds its share of the
    // elements, and the flag counts the parts that are done.  The parts of a tile are neighbours in
    // dispatch order and none of them waits for anything else, so that wait ends.
    wait_vmem();
    __syncthreads();
    int last = 0;
    if (tid == 0) {
        last = atomicAdd(a.flags + 4 * by, 1u) == (uint32_t)a.t_parts - 1u;
        if (a.t_dist) wait_flag(a.flags + 4 * by, (uint32_t)a.t_parts, a.flags_status);
    }
    if (!__syncthreads_or(last) && !a.t_dist) return;
#pragma unroll
    for (int s = 0; s < NW; ++s) {
        const WeightDev& w = ti.w[s];
        const int rquads = ((w.r + 15) & ~15) / 4;              // groups of four ranks
        if (rquads == 0) continue;
        const BufRsrc pb = make_rsrc(a.Tp[s], a.tp_bytes);
        const BufRsrc tb = make_rsrc(a.T[s], a.t_bytes);
        // all partials of two elements (up to NB parts at a time) are requested at once: the sum
        // costs a few memory round trips, not one per part
        const int all_items = ti.rows * rquads;
        const int share = a.t_dist ? (all_items + a.t_parts - 1) / a.t_parts : all_items;
        const int item_lo = a.t_dist ? part * share : 0;
        const int items = item_lo + share < all_items ? item_lo + share : all_items;
        auto sum_parts = [&](auto nb_c) {
            constexpr int NB = decltype(nb_c)::value;
            for (int item0 = item_lo + tid; item0 < items; item0 += 2 * kTiledThreads) {
                uint32_t at[2];
                f32x4 sum[2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int item = item0 + u * kTiledThreads;
                    const int m = item / rquads, rank = 4 * (item - m * rquads);
                    at[u] = item < items ? (uint32_t)((ti.row0 + m) * a.ldt + rank) : kOobOffset;
                    sum[u] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                }
                for (int p0 = 0; p0 < a.t_parts; p0 += NB) {
                    u32x4 v[2][NB];
#pragma unroll
                    for (int i = 0; i < NB; ++i)
#pragma unroll
                        for (int u = 0; u < 2; ++u)
                            v[u][i] = buf_load16_coherent(
                                pb, (p0 + i < a.t_parts && at[u] != kOobOffset)
                                        ? (uint32_t)(((p0 + i) * a.t_part_stride + at[u]) * 4)
                                        : kOobOffset);
#pragma unroll
                    for (int i = 0; i < NB; ++i)
#pragma unroll
                        for (int u = 0; u < 2; ++u) {
                            const f32x4 f = __builtin_bit_cast(f32x4, v[u][i]);
#pragma unroll
                            for (int e = 0; e < 4; ++e) sum[u][e] += f[e];
                        }
                }
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    u32x2 ob;
                    if (BF) {
                        ob = u32x2{pack_bf16(sum[u][0], sum[u][1]), pack_bf16(sum[u][2], sum[u][3])};
                    } else {
                        f16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (f16)sum[u][e];
                        ob = __builtin_bit_cast(u32x2, o);
                    }
                    __builtin_amdgcn_raw_buffer_store_b64(ob, tb,
                                                          at[u] != kOobOffset ? at[u] * 2u : kOobOffset, 0, 17);
                }
            }
        };
        if (a.t_parts <= 4) sum_parts(std::integral_constant<int, 4>{});
        else sum_parts(std::integral_constant<int, 16>{});
    }
    wait_vmem();
    __syncthreads();
    if (tid == 0) {
        if (a.t_dist) atomicAdd(a.flags + 4 * by + 1, 1u);
        else __hip_atomic_store(a.flags + 4 * by + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Lanes i and i + 32 hold, for the same row of a 32x32 accumulator block, interleaved groups of
// four features (group v of lane half h is features 8v + 4h ..).  Swapping groups 2, 3 of the lower
// half with groups 0, 1 of the upper half leaves every lane with 16 consecutive features, starting
// at 16h, in the order o[0], o[2], o[1], o[3]: two 16-byte stores instead of four scattered 8-byte
// ones.  Lane pairs are active together (they share the row).
__device__ __forceinline__ void gather16(u32x2 (&o)[4]) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const u32x2 r0 = __builtin_amdgcn_permlane32_swap(o[j].x, o[j + 2].x, false, false);
        const u32x2 r1 = __builtin_amdgcn_permlane32_swap(o[j].y, o[j + 2].y, false, false);
        o[j].x = r0.x; o[j + 2].x = r0.y;
        o[j].y = r1.x; o[j + 2].y = r1.y;
    }
}

// MODE 1: every weight of the launch is a symmetric blob (MILO_W3_SYMMETRIC): conversion without
// zero-point arithmetic.  MODE 2: bf16 activations, compensator and output (MILO_ACT_BF16).
template <int NW, int MB, int EPI, int MODE = 0>
__global__ __launch_bounds__(kTiledThreads, 2) void w3lr_tiled_kernel(const TiledArgs a) {
    constexpr bool SYM = MODE == 1, BF = MODE == 2;
    constexpr int BM = 32 * MB;
    constexpr int BN = (NW == 1) ? 256 : 128;
    constexpr int STAGE = BM * 256;              // bytes of one X stage: BM rows x 128 columns
    constexpr int NCP = BM / 16;                 // 1-KB copies per wave and stage (4 rows each)
    constexpr int PD = MB == 4 ? 2 : kTiledStages;   // chunks in flight, the one being computed included
    constexpr int PER = NCP + 4;                 // vector memory instructions a wave issues per chunk
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];      // PD stages

    // Placement.  The grid is one-dimensional; what a workgroup does follows from its index hw.
    // The hardware hands workgroups to the eight XCDs (each with its own L2) round robin in index
    // order.  A row is one M-tile in one K split: first the v_tiles workgroups that form T (first
    // split only), then the gxm column tiles.
    //   Few M-tiles: all T workgroups of the launch come first, then the column tiles of every
    //   (tile, split) row in order, nothing in between - so the working workgroups spread evenly
    //   over the XCDs and a launch sized for the chip is resident at once.
    //   Many M-tiles: the indices are read as eight sequences, hw mod 8, and sequence k works
    //   through a contiguous range of the rows, all workgroups of a row back to back: those that
    //   share an activation tile meet in one L2.  (With few tiles a fixed share per XCD balances
    //   worse than the common queue.)
    // Either way every logical workgroup is taken by exactly one hardware workgroup, whatever the
    // hardware does with the index, and the T workgroups of a tile have lower indices than (are
    // dispatched before) the workgroups that wait for them.
    const uint32_t gxm = (uint32_t)((a.N + BN - 1) / BN);
    const uint32_t gx = gxm + (uint32_t)a.v_tiles;
    const uint32_t n_act = a.rs.tiles ? (uint32_t)*a.rs.n_tiles : (uint32_t)((a.rs.M + BM - 1) / BM);
    const uint32_t hw = blockIdx.x;
    if (n_act == 0) return;
    uint32_t bx, by, bz;
    if (n_act >= kXcdPlacementTiles) {
        const uint32_t xcd = hw & 7u, seq = hw >> 3;
        const uint32_t n_rows = n_act * (uint32_t)a.ksplit, base = n_rows >> 3, rem = n_rows & 7u;
        const uint32_t cnt = base + (xcd < rem ? 1u : 0u), first = xcd * base + (xcd < rem ? xcd : rem);
        const uint32_t rl = seq / gx;
        if (rl >= cnt) return;
        bx = seq - rl * gx;
        bz = (first + rl) / n_act;
        by = (first + rl) - bz * n_act;
        if (bx < (uint32_t)a.v_tiles && bz != 0) return;        // T belongs to the first split
    } else {
        const uint32_t nv = (uint32_t)a.m_tiles * (uint32_t)a.v_tiles;
        if (hw < nv) {
            by = hw / (uint32_t)a.v_tiles;
            bx = hw - by * (uint32_t)a.v_tiles;
            bz = 0;
            if (by >= n_act) return;
        } else {
            const uint32_t m = hw - nv, t = m / gxm;
            bx = m - t * gxm + (uint32_t)a.v_tiles;
            // first split of every tile first (it also applies the low-rank term, so it is the
            // longest), then the other splits tile by tile: the list is ordered longest first,
            // and so is the grid
            if (t < n_act) {
                by = t;
                bz = 0;
            } else {
                const uint32_t rest = (uint32_t)a.ksplit - 1u, t2 = t - n_act;
                if (rest == 0) return;
                by = t2 / rest;
                bz = 1u + (t2 - by * rest);
                if (by >= n_act) return;
            }
        }
    }

    const TileInfo ti = resolve_tile<NW>(a.rs, (int)by, BM);
    if (!ti.valid) return;
    const bool any_rank = ti.w[0].r > 0 || ti.w[1].r > 0;
    if ((int)bx < a.v_tiles) {
        // forms one part of T = X V^T for this M-tile (see v_tile_body)
        if (any_rank && bz == 0) v_tile_body<NW, MB, BF>(a, ti, smem, (int)bx, by);
        return;
    }

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int i32 = lane & 31;
    const int h = lane >> 5;
    const int64_t N = a.N, K = a.K;
    const int G = (int)(K / kGroup);
    const int nchunks = (G + 1) / 2;
    // K split: this workgroup multiplies chunks [c_begin, c_end)
    const int cps = (nchunks + a.ksplit - 1) / a.ksplit;
    const int c_begin = (int)bz * cps;
    const int c_end = (c_begin + cps < nchunks) ? c_begin + cps : nchunks;
    const int64_t n0 = (int64_t)((int)bx - a.v_tiles) * BN;

    // Weight streams of this wave: lane (i32, h) feeds row nrow of the stream, group 2c + h.
    W3Buf wbuf[2];
    int64_t nrow[2];
    uint32_t ubase[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const WeightDev& w = ti.w[NW == 1 ? 0 : s];
        wbuf[s] = make_w3buf(w.q3, N, K);
        const int64_t nb = (NW == 1) ? n0 + 64 * wave + 32 * s : n0 + 32 * wave;
        nrow[s] = nb + i32;
        ubase[s] = (nrow[s] < N) ? (uint32_t)unit_index(nrow[s], 0, G) : kOobUnit;
    }

    // Activation staging.  A stage is [BM rows][256 bytes]; copy ci of the workgroup moves rows
    // 4ci .. 4ci+3 (1 KB, coalesced): lane l -> row 4ci + l/16, position p = l%16, which receives
    // segment p ^ (row%16) of the row's 16 segments of 8 columns.  The xor makes the per-lane
    // ds_read_b128 of the B fragments conflict free (16 lanes read 16 different rows).
    const BufRsrc xb = make_rsrc(a.X, a.x_bytes);
    uint32_t xoff[NCP];
    bool xhi[NCP];
    {
        // gather indices first, all loads in flight together (rows past the tile re-read row 0)
        int32_t src[NCP];
#pragma unroll
        for (int i = 0; i < NCP; ++i) {
            const int row = 4 * (wave * NCP + i) + (lane >> 4);
            const int R = ti.row0 + (row < ti.rows ? row : 0);
            src[i] = a.rs.x_rows ? a.rs.x_rows[R] : R;
        }
#pragma unroll
        for (int i = 0; i < NCP; ++i) {
            const int row = 4 * (wave * NCP + i) + (lane >> 4);
            const int seg = (lane & 15) ^ (row & 15);
            xhi[i] = seg >= 8;
            xoff[i] = (row < ti.rows) ? (uint32_t)src[i] * (uint32_t)(a.ldx * 2) + (uint32_t)(seg * 16) : kOobHalf;
        }
    }
    const bool ktail = (G & 1) != 0;            // the last chunk has only its first 64 columns

    f32x16 acc[2][MB];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[s][mb][v] = 0.0f;

    // One chunk's loads of this wave are always PER instructions: the two weight units (two loads
    // each), then the NCP activation copies into stage `slot`.  All are issued when a chunk starts:
    // the time a wave needs to get them out is best spent while the other workgroup on the CU
    // multiplies (spreading them over the steps of the chunk was slower).  The common case costs
    // an add per instruction: unit indices advance by 32 per chunk (a row without data starts at
    // 2^27, far past every weight, and stays there), copy offsets by 256 bytes.  Chunks past the
    // end of this workgroup's share are requested like any other: nobody looks at them, and a
    // request past the end of a buffer returns zeros.  Only the last chunk of a K that is an odd
    // number of groups takes the careful path, where the upper 64 columns must read as zero
    // instead of running into the next row.
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);        // known to be uniform
    uint32_t ucur[2];               // unit of this lane in the chunk to be requested next
#pragma unroll
    for (int s = 0; s < 2; ++s)
        ucur[s] = ubase[s] != kOobUnit ? ubase[s] + (uint32_t)(2 * c_begin + h) * 16u : (1u << 27);
    auto issue = [&](int c, int slot, RawUnit (&ru)[2]) {
        const bool ragged = ktail && c == nchunks - 1;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const uint32_t u = (ragged && h == 1) ? (1u << 27) : ucur[s];
            ru[s] = a.weights_once ? load_unit_buf_once(wbuf[NW == 1 ? 0 : s], u)
                                   : load_unit_buf(wbuf[NW == 1 ? 0 : s], u);
            ucur[s] += 32u;
        }
        asm volatile("" ::: "memory");
        unsigned char* const stage = smem + slot * STAGE + wave_s * NCP * 1024;
        const uint32_t cbytes = (uint32_t)c * 256u;
        // (the offset goes through a named variable: with an expression as the builtin's argument
        // the host pass of the compiler silently drops the kernel's launch stub)
        if (!ragged) {
#pragma unroll
            for (int i = 0; i < NCP; ++i) {
                const uint32_t off = xoff[i] + cbytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(xb, (LdsPtr)(stage + i * 1024), 16, off, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NCP; ++i) {
                uint32_t off = xoff[i] + cbytes;
                if (xhi[i]) off = kOobHalf;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(xb, (LdsPtr)(stage + i * 1024), 16, off, 0, 0, 0);
            }
        }
        asm volatile("" ::: "memory");
    };
    // Row blocks of 32 actually present in this tile.  The K loop is instantiated per count, so
    // that blocks past the tile's rows cost nothing and the loop body has no branches (the
    // instruction scheduler interleaves conversion, LDS reads and MFMAs only within a basic block).
    const int mb_used = (ti.rows + 31) / 32;
    // The tile's "T is ready" flag is asked for once, by every wave for itself, while the last chunk
    // is still being multiplied (a read of a word written during the launch takes about a
    // microsecond): the workgroups that form T were dispatched long before, so the answer is nearly
    // always yes, and the wave goes from its last chunk straight to the low-rank term.
    uint32_t early_flag = 0u;
    const bool wants_t = any_rank && bz < (uint32_t)a.lr_splits;
    const uint32_t t_ready = a.t_dist ? (uint32_t)a.t_parts : 1u;     // value of the tile's flag when T is complete
    auto k_loop = [&](auto mbu_c) {
        constexpr int MBU = decltype(mbu_c)::value;
        auto compute = [&](int slot, RawUnit (&ru)[2], auto&& between) {
            pin_unit(ru[0]);
            pin_unit(ru[1]);
            // B fragment of step t, row block mb: row 32mb + i32, segment 8h + t.
            const unsigned char* xs = smem + slot * STAGE + i32 * 256;
            const int sx = i32 & 15;
            auto bfrag = [&](int mb, int t) {
                return __builtin_bit_cast(
                    f16x8, *reinterpret_cast<const u32x4*>(xs + mb * 32 * 256 + (((8 * h + t) ^ sx) << 4)));
            };
            // the next step's B fragments are requested before this step's MFMAs are issued
            f16x8 bc[MBU], bn[MBU];
#pragma unroll
            for (int mb = 0; mb < MBU; ++mb) bc[mb] = bfrag(mb, 0);
            auto step = [&](int t, auto a0, auto a1) {
                between(t);
                if (t < 7) {
#pragma unroll
                    for (int mb = 0; mb < MBU; ++mb) bn[mb] = bfrag(mb, t + 1);
                }
#pragma unroll
                for (int mb = 0; mb < MBU; ++mb) {
                    if constexpr (BF) {
                        acc[0][mb] = mfma32_bf16(a0, __builtin_bit_cast(bf16x8, bc[mb]), acc[0][mb]);
                        acc[1][mb] = mfma32_bf16(a1, __builtin_bit_cast(bf16x8, bc[mb]), acc[1][mb]);
                    } else {
                        acc[0][mb] = mfma32(a0, bc[mb], acc[0][mb]);
                        acc[1][mb] = mfma32(a1, bc[mb], acc[1][mb]);
                    }
                }
                if (t < 7) {
#pragma unroll
                    for (int mb = 0; mb < MBU; ++mb) bc[mb] = bn[mb];
                }
            };
            if constexpr (BF) dequant_units2_steps_bf16(ru[0], ru[1], step);
            else dequant_units2_steps<SYM>(ru[0], ru[1], step);
        };

        // PD-deep pipeline: chunk c lives in ring slot c % PD (registers for the weights, LDS stage
        // for the activations).  Vector memory operations complete in order, so once at most the
        // (PD - 2) * PER instructions of the younger chunks are outstanding, chunk c has arrived.
        // (The count relies on the compiler adding no memory operation of its own, i.e. on the
        // kernel not using scratch memory; the build script checks that.)
        RawUnit ring[PD][2];
#pragma unroll
        for (int i = 0; i < PD - 1; ++i) issue(c_begin + i, i, ring[i]);
        for (int c0 = c_begin; c0 < c_end; c0 += PD) {
#pragma unroll
            for (int slot = 0; slot < PD; ++slot) {
                const int c = c0 + slot;
                if (c >= c_end) break;
                MILO_WAIT_VMEM((PD - 2) * PER);
                __syncthreads();        // everyone's copies of chunk c landed; everyone left chunk c-1
                issue(c + PD - 1, (slot + PD - 1) % PD, ring[(slot + PD - 1) % PD]);
                if (wants_t && c == c_end - 1 && lane == 0)
                    early_flag = __hip_atomic_load(a.flags + 4 * by + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                compute(slot, ring[slot], [](int) {});
            }
        }
    };
    if (MB >= 4 && mb_used >= 4) k_loop(std::integral_constant<int, MB >= 4 ? 4 : 1>{});
    else if (MB >= 4 && mb_used == 3) k_loop(std::integral_constant<int, MB >= 4 ? 3 : 1>{});
    else if (MB >= 2 && mb_used >= 2) k_loop(std::integral_constant<int, MB >= 2 ? 2 : 1>{});
    else k_loop(std::integral_constant<int, 1>{});

    bool nvalid[2];
    nvalid[0] = nrow[0] < N;
    nvalid[1] = nrow[1] < N;

    // Low-rank term: r extra k-steps with A = U rows and B = T rows.  T of this M-tile is formed
    // by other workgroups of this launch (see v_tile_body): wait for the tile's flag (they were
    // dispatched before this workgroup and never wait themselves), then read T coherently.
    if (wants_t) {
        const BufRsrc tb0 = make_rsrc(a.T[0], a.t_bytes);
        const BufRsrc tb1 = make_rsrc(a.T[1], a.t_bytes);
        // Two k-steps of 16 ranks at a time: their U fragments (which do not depend on T) and then
        // their T fragments are all requested before the first is used, so that a rank-128
        // compensator costs four memory round trips instead of forty.
        bool waited = false;
        // INT3 compensator: the U blob holds U^T [pad16(r) x N] with groups of 64 along N.  The band of
        // this workgroup is four groups (NW = 1) or two groups of each of the two weights (NW = 2):
        // thread (wave w, lane l) converts the unit of rank l (then l + 64) of the w-th of them and
        // writes its 64 features as a column of the LDS array UL[band feature][rank] (fp16, row length
        // ldu), from which every lane then reads the eight ranks of a k-step of its feature with one
        // 16-byte load.  The array takes the place of the activation stages, which are dead by now.
        const bool uq = ((ti.w[0].flags | ti.w[1].flags) & MILO_LR_INT3) != 0;
        const int ldu = (((ti.w[0].r > ti.w[1].r ? ti.w[0].r : ti.w[1].r) + 15) & ~15) + 8;     // (+8: rows on different banks)
        if (uq) {
            __syncthreads();                // every wave is done with the stages
            const int gsel = wave_s;
            const bool second = NW == 2 && gsel >= 2;       // (selected field by field: no indexing of ti.w)
            const int rp = ((second ? ti.w[1].r : ti.w[0].r) + 15) & ~15;
            const int GN = (int)(N >> 6);
            const int64_t g = (n0 >> 6) + (NW == 1 ? gsel : (gsel & 1));
            const W3Buf ub = make_w3buf(second ? ti.w[1].U : ti.w[0].U, rp, N);
            f16* const UL = reinterpret_cast<f16*>(smem);
            for (int j = lane; j < rp; j += 64) {
                const RawUnit u = load_unit_buf(ub, g < GN ? (uint32_t)unit_index(j, g, GN) : (1u << 27));
                uint32_t wv[32];
                dequant_unit<true>(u, wv);
                f16* col = UL + (int64_t)(64 * gsel) * ldu + j;
#pragma unroll
                for (int P = 0; P < 32; ++P) {
                    const f16x2 pr = __builtin_bit_cast(f16x2, wv[P]);
                    col[(2 * P) * ldu] = pr[0];
                    col[(2 * P + 1) * ldu] = pr[1];
                }
            }
            __syncthreads();
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const WeightDev& w = ti.w[NW == 1 ? 0 : s];
            const int r = w.r;
            if (r <= 0) continue;
            const BufRsrc tb = (NW == 1 || s == 0) ? tb0 : tb1;
            const f16* urow = w.U + (nvalid[s] ? nrow[s] : 0) * (int64_t)r;
            const bool ualigned = (r & 7) == 0;
            const int rpad = (r + 15) & ~15;            // T is written (with zeros) up to here
            // row of this lane's feature in UL: band feature index (NW = 2: the second weight's follow)
            const f16* ulrow = reinterpret_cast<const f16*>(smem) +
                               (int64_t)((NW == 1) ? (64 * wave + 32 * s + i32) : (128 * s + 32 * wave + i32)) * ldu;
            // One k-step pair (32 ranks): U fragments (they do not depend on T), T fragments.
            auto load_u = [&](int ks, f16x8 (&av)[2]) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int k0 = ks + 16 * j + 8 * h;
                    av[j] = zero_f16x8();
                    if (uq) {
                        if (k0 < rpad) av[j] = load_f16x8(ulrow + k0);
                    } else if (nvalid[s] && k0 < r) {
                        av[j] = load_row8(urow, k0, r, ualigned);
                    }
                }
            };
            auto load_t = [&](int ks, u32x4 (&bv)[2][MB]) {
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int k0 = ks + 16 * j + 8 * h;
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        const int m = 32 * mb + i32;
                        bv[j][mb] = buf_load16_coherent(
                            tb, (m < ti.rows && k0 < rpad) ? (uint32_t)(((ti.row0 + m) * a.ldt + k0) * 2) : kOobOffset);
                    }
                }
            };
            auto multiply = [&](const f16x8 (&av)[2], const u32x4 (&bv)[2][MB]) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        acc[s][mb] = BF ? mfma32_bf16(__builtin_bit_cast(bf16x8, av[j]), __builtin_bit_cast(bf16x8, bv[j][mb]),
                                                      acc[s][mb])
                                        : mfma32(av[j], __builtin_bit_cast(f16x8, bv[j][mb]), acc[s][mb]);
            };
            // Two sets of fragments: while one is multiplied the next 32 ranks are already on their
            // way, so a rank-512 compensator costs about two memory round trips, not sixteen.
            f16x8 avA[2], avB[2];
            u32x4 bvA[2][MB], bvB[2][MB];
            // ranks of this K split: all of them, or with lr_splits > 1 (large ranks in a split GEMM, whose
            // partial sums are added anyway) this split's lr_step ranks
            const int ks_lo = a.lr_splits > 1 ? (int)bz * a.lr_step : 0;
            const int ks_hi = a.lr_splits > 1 && ks_lo + a.lr_step < r ? ks_lo + a.lr_step : r;
            load_u(ks_lo, avA);
            if (!waited) {
                // every wave asks for itself (no barrier: a wave that is done early goes on early)
                if (lane == 0 && early_flag < t_ready) wait_flag(a.flags + 4 * by + 1, t_ready, a.flags_status);
                waited = true;
            }
            load_t(ks_lo, bvA);
            for (int ks = ks_lo; ks < ks_hi; ks += 64) {
                if (ks + 32 < ks_hi) {
                    load_u(ks + 32, avB);
                    load_t(ks + 32, bvB);
                }
                multiply(avA, bvA);
                if (ks + 64 < ks_hi) {
                    load_u(ks + 64, avA);
                    load_t(ks + 64, bvA);
                }
                if (ks + 32 < ks_hi) multiply(avB, bvB);
            }
        }
        if (!waited) {          // (not reached: some rank is positive)
            if (lane == 0 && early_flag < t_ready) wait_flag(a.flags + 4 * by + 1, t_ready, a.flags_status);
        }
        // the last reader of this M-tile's T clears its control words for the next launch (the MoE
        // call clears all of them before every forward instead: the returning atomic is a round
        // trip to memory per workgroup)
        if (a.self_clean) __syncthreads();
        if (a.self_clean && tid == 0) {
            const uint32_t readers = (gx - (uint32_t)a.v_tiles) * (uint32_t)a.lr_splits;
            if (atomicAdd(a.flags + 4 * by + 2, 1u) == readers - 1u) {
                __hip_atomic_store(a.flags + 4 * by, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(a.flags + 4 * by + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(a.flags + 4 * by + 2, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }

    // Epilogue.  D[v] of block (s, mb): feature nb + 8*(v/4) + 4*h + v%4, row 32*mb + i32.
    // fp16 results go out as 16 consecutive features per lane (see gather16).
    auto store16 = [&](f16* orow, int64_t nb, u32x2 (&o)[4]) {
        gather16(o);
        const int64_t n = nb + 16 * h;
        if (n < N) {
            *reinterpret_cast<u32x4*>(orow + n) = u32x4{o[0].x, o[0].y, o[2].x, o[2].y};
            *reinterpret_cast<u32x4*>(orow + n + 8) = u32x4{o[1].x, o[1].y, o[3].x, o[3].y};
        }
    };
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int m = 32 * mb + i32;
        if (m >= ti.rows) continue;
        const int64_t R = (int64_t)ti.row0 + m;
        if (EPI == EPI_SWIGLU) {
            f16* orow = reinterpret_cast<f16*>(a.out) + R * a.ldo;
            u32x2 o[4];
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                float g[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) g[e] = silu(acc[0][mb][4 * vq + e]) * acc[1][mb][4 * vq + e];
                if (BF) {
                    o[vq] = u32x2{pack_bf16(g[0], g[1]), pack_bf16(g[2], g[3])};
                } else {
                    f16x4 v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = (f16)g[e];
                    o[vq] = __builtin_bit_cast(u32x2, v);
                }
            }
            store16(orow, n0 + 32 * wave, o);
        } else {
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int64_t nb = n0 + 64 * wave + 32 * s;
                if (EPI == EPI_STORE && a.ksplit > 1) {
                    // partial sum of this K split, fp32; a small kernel adds the splits in order
                    float* orow = reinterpret_cast<float*>(a.out) + (int64_t)bz * a.out_split_stride + R * a.ldo;
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const int64_t n = nb + 8 * vq + 4 * h;
                        if (n >= N) continue;
                        f32x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = acc[s][mb][4 * vq + e];
                        *reinterpret_cast<f32x4*>(orow + n) = o;
                    }
                } else {
                    f16* orow;
                    float sc = 1.0f;
                    if (EPI == EPI_STORE) {
                        orow = reinterpret_cast<f16*>(a.out) + R * a.ldo;
                    } else {
                        const int64_t orow_i = a.out_rows ? (int64_t)a.out_rows[R] : R;
                        if (a.out_scale) sc = a.out_scale[orow_i];
                        orow = reinterpret_cast<f16*>(a.out) + (int64_t)bz * a.out_split_stride + orow_i * a.ldo;
                    }
                    u32x2 o[4];
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        if (BF) {
                            const float m = EPI == EPI_STORE ? 1.0f : sc;
                            o[vq] = u32x2{pack_bf16(m * acc[s][mb][4 * vq], m * acc[s][mb][4 * vq + 1]),
                                          pack_bf16(m * acc[s][mb][4 * vq + 2], m * acc[s][mb][4 * vq + 3])};
                        } else {
                            f16x4 v;
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                v[e] = (f16)(EPI == EPI_STORE ? acc[s][mb][4 * vq + e] : sc * acc[s][mb][4 * vq + e]);
                            o[vq] = __builtin_bit_cast(u32x2, v);
                        }
                    }
                    store16(orow, nb, o);
                }
            }
        }
    }
}

template <int NW, int MB, int EPI, int MODE = 0>
static int launch_one(const TiledArgs& a, dim3 grid, hipStream_t stream) {
    constexpr int lds_stages = (MB == 4 ? 2 : kTiledStages) * 32 * MB * 256;
    // room for the U array of an INT3 compensator: 256 band features x (pad16(rank) + 8) fp16
    const int lds_u = a.lr3_rank > 0 ? 256 * (((a.lr3_rank + 15) & ~15) + 8) * 2 : 0;
    const int lds = lds_u > lds_stages ? lds_u : lds_stages;
    static bool raised[64] = {false};
    if (lds > 64 * 1024) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MILO_ERR_HIP;
        if (!raised[dev]) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(w3lr_tiled_kernel<NW, MB, EPI, MODE>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024) != hipSuccess)
                return MILO_ERR_HIP;
            raised[dev] = true;
        }
    }
    w3lr_tiled_kernel<NW, MB, EPI, MODE><<<grid, dim3(kTiledThreads), lds, stream>>>(a);
    return launch_status();
}

template <int NW, int EPI, int MODE = 0>
static int launch_tiled_mb(const TiledArgs& a, int mb, dim3 grid, hipStream_t stream) {
    switch (mb) {
        case 1: return launch_one<NW, 1, EPI, MODE>(a, grid, stream);
        case 2: return launch_one<NW, 2, EPI, MODE>(a, grid, stream);
        case 4: return launch_one<NW, 4, EPI, MODE>(a, grid, stream);
        default: return MILO_ERR_SHAPE;
    }
}

int launch_tiled(const TiledArgs& a, int nw, int mb, int epi, int m_tiles, hipStream_t stream) {
    if (m_tiles <= 0) return MILO_OK;
    const int bn = (nw == 1) ? 256 : 128;
    const int64_t n_tiles = (a.N + bn - 1) / bn + a.v_tiles;
    if (n_tiles > 0x7fffffff || m_tiles > 65535) return MILO_ERR_SHAPE;
    if (a.ksplit < 1 || a.ksplit > 64 || a.v_tiles != a.t_parts || (epi == EPI_SWIGLU && a.ksplit != 1))
        return MILO_ERR_SHAPE;
    // every one of the eight sequences may need ceil(m_tiles * ksplit / 8) rows of n_tiles indices
    // (this also covers the other numbering: m_tiles * (v_tiles + columns * ksplit) indices)
    const int64_t rows8 = (((int64_t)m_tiles * a.ksplit + 7) / 8) * 8;
    if (n_tiles * rows8 > 0x7fffffff) return MILO_ERR_SHAPE;
    TiledArgs b = a;
    b.m_tiles = m_tiles;
    dim3 grid((unsigned)(n_tiles * rows8));
    if (nw == 2 && epi == EPI_SWIGLU)
        return a.act_bf16 ? launch_tiled_mb<2, EPI_SWIGLU, 2>(b, mb, grid, stream)
                          : launch_tiled_mb<2, EPI_SWIGLU>(b, mb, grid, stream);
    if (nw == 1 && epi == EPI_STORE) {
        if (a.act_bf16) return launch_tiled_mb<1, EPI_STORE, 2>(b, mb, grid, stream);
        // the single linear knows its one weight: a symmetric blob takes the zero-point-free conversion
        if (!a.rs.tiles && (a.rs.w[0].flags & MILO_W3_SYMMETRIC)) return launch_tiled_mb<1, EPI_STORE, 1>(b, mb, grid, stream);
        return launch_tiled_mb<1, EPI_STORE>(b, mb, grid, stream);
    }
    if (nw == 1 && epi == EPI_SCALE_SCATTER)
        return a.act_bf16 ? launch_tiled_mb<1, EPI_SCALE_SCATTER, 2>(b, mb, grid, stream)
                          : launch_tiled_mb<1, EPI_SCALE_SCATTER>(b, mb, grid, stream);
    return MILO_ERR_SHAPE;
}

// Parts of T = X V^T per M-tile: about eight 128-column chunks each, so that forming a part takes
// a fraction of the time a streaming workgroup needs for its tile.
int tiled_t_parts(int64_t K) {
    const int64_t nchunks = (K / kGroup + 1) / 2;
    int64_t p = (nchunks + 7) / 8;
    if (p < 1) p = 1;
    if (p > 16) p = 16;
    return (int)p;
}

}  // namespace milo
