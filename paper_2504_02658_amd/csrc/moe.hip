// milo_moe_w3lr_forward: top-k routed SwiGLU experts over compensated W3A16 linears.
//
// Launch sequence on the caller's stream (no host synchronisation in between):
//   route     group the (token, slot) pairs per expert: stable placement by counting and scans,
//             and each expert's M-tiles in its own slots of a tile list
//   order     work list = the filled slots, full tiles first, then the partly filled ones
//   gate/up   H = SiLU(lin_w1(x)) * lin_w3(x), both projections in one grouped launch, which
//             also forms T1 = X V1^T and T3 = X V3^T (low-rank inputs) in its leading columns
//   down      O[split][pair] = gate_weight * lin_w2(H) over the split's share of K (fp16, one row
//             per routed pair); T2 = H V2^T is formed inside this launch as well
//   combine   y_t = fp16( sum over the token's slots and the K splits, in a fixed order, of O )
#include <math.h>
#include <stdlib.h>

#include "milo_host.h"
#include "milo_kernels.h"

namespace milo {

constexpr int kRouteThreads = 1024;

struct RouteArgs {
    const int32_t* ids;     // [P] expert id per (token, slot) pair, pair index p = t*topk + j
    int32_t P;
    int32_t E;
    int32_t bm;             // rows per M-tile
    int32_t topk;
    int32_t* sorted;        // [P] pair indices grouped by expert, original order inside a group
    int32_t* sorted_token;  // [P] token of each sorted pair (pair / topk)
    TileDesc* tiles;
    int32_t* header;        // [0] routing status, [1] number of tiles, [3] wait status (a wait gave up)
    uint32_t* flags;        // per-tile control words of the GEMM kernels, cleared here
    int32_t n_flags;
    int32_t max_tiles;      // slots of the tile list: ceil(P / bm) + E
};

// One workgroup per expert; no workgroup depends on another one, so a single launch suffices.
// A thread owns a contiguous range of the pairs and counts the ids equal to its expert and the
// ids below it: the stable position of a pair inside its expert's group is the number of matches
// in the threads before it (one scan over the workgroup) plus the matches before it in its own
// range, and the group starts at the number of ids below the expert.  No histogram over all
// experts is needed (LDS atomics of a whole workgroup on the few popular experts serialize
// badly): expert e places its tiles from slot floor(start_e / bm) + e of the tile list, which
// never overlaps the next expert's first slot, and marks the slots up to there as empty.
__global__ __launch_bounds__(kRouteThreads) void route_kernel(const RouteArgs a) {
    __shared__ int32_t s_bad;
    __shared__ int32_t wsum_eq[kRouteThreads / 64], wsum_less[kRouteThreads / 64];

    const int e = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_bad = 0;
    __syncthreads();

    // a thread's range: a multiple of 16 pairs, read 16 at a time with four 16-byte loads in flight
    // (one id per load would pay the memory latency once per pair)
    const int per = ((a.P + kRouteThreads - 1) / kRouteThreads + 15) & ~15;
    const int lo = tid * per < a.P ? tid * per : a.P;
    const int hi = lo + per < a.P ? lo + per : a.P;
    int n_eq = 0, n_less = 0, bad = 0;
    auto load16 = [&](int i0, int32_t (&v)[16]) {
        if (i0 + 16 <= a.P) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int4 q = *reinterpret_cast<const int4*>(a.ids + i0 + 4 * j);
                v[4 * j] = q.x; v[4 * j + 1] = q.y; v[4 * j + 2] = q.z; v[4 * j + 3] = q.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) v[j] = i0 + j < a.P ? a.ids[i0 + j] : e + 1;   // padding: no match
        }
    };
    for (int i0 = lo; i0 < hi; i0 += 16) {
        int32_t v[16];
        load16(i0, v);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            if (i0 + j >= hi) break;
            const int id = v[j];
            if (id >= 0 && id < a.E) {
                n_eq += id == e;
                n_less += id < e;
            } else {
                bad = 1;
            }
        }
    }
    // inclusive scan of n_eq within the wave, wave totals to LDS
    int scan = n_eq;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int v = __shfl_up(scan, d, 64);
        if (lane >= d) scan += v;
    }
    int less = n_less;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) less += __shfl_xor(less, d, 64);
    if (lane == 63) wsum_eq[wave] = scan;
    if (lane == 0) wsum_less[wave] = less;
    __syncthreads();
    int before = 0, off_e = 0, count = 0;
    for (int w = 0; w < kRouteThreads / 64; ++w) {
        if (w < wave) before += wsum_eq[w];
        count += wsum_eq[w];
        off_e += wsum_less[w];
    }
    // stable scatter of the pairs routed to expert e
    int pos = off_e + before + scan - n_eq;
    if (n_eq) {
        for (int i0 = lo; i0 < hi; i0 += 16) {
            int32_t v[16];
            load16(i0, v);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                if (i0 + j < hi && v[j] == e) {
                    a.sorted[pos] = i0 + j;
                    a.sorted_token[pos] = (i0 + j) / a.topk;
                    ++pos;
                }
            }
        }
    }
    // this expert's slots of the tile list: its tiles, then empty slots up to the next expert's first
    const int tile0 = off_e / a.bm + e;
    const int tile1 = (e + 1 < a.E) ? (off_e + count) / a.bm + e + 1 : a.max_tiles;
    const int nt = (count + a.bm - 1) / a.bm;
    for (int i = tid; i < tile1 - tile0; i += kRouteThreads) {
        TileDesc td;
        td.expert = e;
        td.row0 = off_e + (i < nt ? i * a.bm : 0);
        td.rows = i < nt ? ((count - i * a.bm) < a.bm ? (count - i * a.bm) : a.bm) : 0;
        td.pad = 0;
        a.tiles[tile0 + i] = td;
    }
    if (e == 0) {
        // every workgroup has looked at all ids; this one reports the ones out of range
        if (bad) atomicOr(&s_bad, 1);
        for (int i = tid; i < a.n_flags; i += kRouteThreads) a.flags[i] = 0u;
        __syncthreads();
        if (tid == 0) {
            a.header[0] = s_bad ? MILO_ERR_ROUTING : MILO_OK;
            a.header[1] = a.max_tiles;
            a.header[3] = 0;
        }
    }
}

// Work list of the grouped GEMMs: the slots the experts filled, compacted (empty slots dropped) and
// put longest first: a tile costs about what its number of 32-row blocks says, and more with a
// compensator of high rank, so tiles go by that number, most blocks first, within it those of
// experts with a rank above 32 first, in expert order within a class.  The dispatcher hands out workgroups
// in list order, so the launch ends with the short items.  One workgroup; a thread owns a
// contiguous range of slots and a scan per class gives every tile its place.
__global__ __launch_bounds__(kRouteThreads) void order_tiles_kernel(const TileDesc* __restrict__ slots,
                                                                    int n_slots, int bm,
                                                                    TileDesc* __restrict__ tiles,
                                                                    int32_t* __restrict__ header,
                                                                    const milo_w3lr_expert* __restrict__ experts) {
    constexpr int NC = 8;                               // classes: bm / 32 blocks down to one, x rank
    __shared__ int32_t wsum[NC][kRouteThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (n_slots + kRouteThreads - 1) / kRouteThreads;
    const int lo = tid * per < n_slots ? tid * per : n_slots;
    const int hi = lo + per < n_slots ? lo + per : n_slots;
    const int mb = bm / 32;
    auto cls = [&](const TileDesc& td) {                // 0: as many blocks as a full tile, high rank
        const int nb = (td.rows + 31) / 32;
        const milo_w3lr_expert& ex = experts[td.expert];
        const int low = (ex.w1.r <= 32 && ex.w3.r <= 32 && ex.w2.r <= 32) ? 1 : 0;
        return 2 * (mb - (nb < mb ? nb : mb)) + low;
    };
    int cnt[NC] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = lo; i < hi; ++i) {
        const TileDesc td0 = slots[i];
        const int rows = td0.rows;
        if (rows > 0) {
            const int c = cls(td0);
#pragma unroll
            for (int k = 0; k < NC; ++k) cnt[k] += c == k;
        }
    }
    int scan[NC];                                       // inclusive scans within the wave
#pragma unroll
    for (int k = 0; k < NC; ++k) scan[k] = cnt[k];
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
#pragma unroll
        for (int k = 0; k < NC; ++k) {
            const int v = __shfl_up(scan[k], d, 64);
            if (lane >= d) scan[k] += v;
        }
    }
    if (lane == 63) {
#pragma unroll
        for (int k = 0; k < NC; ++k) wsum[k][wave] = scan[k];
    }
    __syncthreads();
    int before[NC], total[NC];
#pragma unroll
    for (int k = 0; k < NC; ++k) {
        before[k] = 0;
        total[k] = 0;
        for (int w = 0; w < kRouteThreads / 64; ++w) {
            if (w < wave) before[k] += wsum[k][w];
            total[k] += wsum[k][w];
        }
    }
    // From kXcdPlacementTiles tiles on, the tiled kernel reads the list as eight contiguous ranges,
    // one per sequence of workgroups (range k starts at k * (n / 8) + min(k, n % 8)).  Position p of
    // the order goes to range p % 8, place p / 8, so that every range gets the same mix and ends
    // with its short items.
    int n = 0;
#pragma unroll
    for (int k = 0; k < NC; ++k) n += total[k];
    const int base = n >> 3, rem = n & 7;
    auto place = [&](int p) {
        if (n < (int)kXcdPlacementTiles) return p;          // the kernel takes the list in order
        const int k = p & 7;
        return k * base + (k < rem ? k : rem) + (p >> 3);
    };
    int pos[NC];
    int start = 0;
#pragma unroll
    for (int k = 0; k < NC; ++k) {
        pos[k] = start + before[k] + scan[k] - cnt[k];
        start += total[k];
    }
    for (int i = lo; i < hi; ++i) {
        const TileDesc td = slots[i];
        if (td.rows <= 0) continue;
        const int c = cls(td);
        int p = 0;
#pragma unroll
        for (int k = 0; k < NC; ++k)
            if (c == k) p = pos[k]++;
        tiles[place(p)] = td;
    }
    if (tid == 0) header[1] = n;
}

// Routing and work list in one launch for decode-sized batches (at most kSmallPairs routed pairs and
// kSmallExperts experts): with a handful of tokens the two kernels above are all latency, and so is
// the launch between them.  One workgroup; thread p owns pair p.  The group of an expert starts at
// the number of pairs with a smaller id, a pair's place inside it is the number of earlier pairs with
// the same id (both counted from a copy of the ids in LDS), which is the same stable order as
// route_kernel's.  Tiles are written straight into the final list: tiles of experts with a rank
// above 32 first, then the others, in expert order (order_tiles_kernel's order for 32-row tiles,
// the only tile height such a batch gets).
constexpr int kSmallPairs = 256, kSmallExperts = 256;
__global__ __launch_bounds__(kSmallPairs) void route_small_kernel(const RouteArgs a, TileDesc* __restrict__ list,
                                                                  const milo_w3lr_expert* __restrict__ experts) {
    __shared__ int32_t s_id[kSmallPairs];
    __shared__ int32_t s_cnt[kSmallExperts], s_start[kSmallExperts], s_tile0[kSmallExperts];
    __shared__ int32_t s_bad, s_total;
    const int tid = threadIdx.x;
    if (tid == 0) s_bad = 0;
    int id = -1;
    if (tid < a.P) {
        id = a.ids[tid];
        if (id < 0 || id >= a.E) id = -1;
    }
    s_id[tid] = id;
    __syncthreads();
    if (tid < a.P && id < 0) s_bad = 1;
    // expert e = tid: its pair count, the pairs before its group, and the tiles before its own in the list
    if (tid < a.E) {
        int cnt = 0, less = 0;
        for (int p = 0; p < a.P; ++p) {
            const int v = s_id[p];
            cnt += v == tid;
            less += v >= 0 && v < tid;
        }
        s_cnt[tid] = cnt;
        s_start[tid] = less;
    }
    __syncthreads();
    if (tid < a.E) {
        const milo_w3lr_expert& me = experts[tid];
        const bool low = me.w1.r <= 32 && me.w3.r <= 32 && me.w2.r <= 32;
        int before = 0, high_tiles = 0;
        for (int e = 0; e < a.E; ++e) {
            const int nt = (s_cnt[e] + a.bm - 1) / a.bm;
            if (nt == 0) continue;
            const milo_w3lr_expert& ex = experts[e];
            const bool elow = ex.w1.r <= 32 && ex.w3.r <= 32 && ex.w2.r <= 32;
            high_tiles += elow ? 0 : nt;
            if (elow == low && e < tid) before += nt;
        }
        s_tile0[tid] = low ? high_tiles + before : before;
        const int nt = (s_cnt[tid] + a.bm - 1) / a.bm;
        for (int i = 0; i < nt; ++i) {
            TileDesc td;
            td.expert = tid;
            td.row0 = s_start[tid] + i * a.bm;
            td.rows = s_cnt[tid] - i * a.bm < a.bm ? s_cnt[tid] - i * a.bm : a.bm;
            td.pad = 0;
            list[s_tile0[tid] + i] = td;
        }
        if (tid == 0) {
            int total = 0;
            for (int e = 0; e < a.E; ++e) total += (s_cnt[e] + a.bm - 1) / a.bm;
            s_total = total;
        }
    }
    if (tid < a.P && id >= 0) {
        int before = 0;
        for (int p = 0; p < tid; ++p) before += s_id[p] == id;
        const int pos = s_start[id] + before;
        a.sorted[pos] = tid;
        a.sorted_token[pos] = tid / a.topk;
    }
    for (int i = tid; i < a.n_flags; i += kSmallPairs) a.flags[i] = 0u;
    __syncthreads();
    if (tid == 0) {
        a.header[0] = s_bad ? MILO_ERR_ROUTING : MILO_OK;
        a.header[1] = s_total;
        a.header[3] = 0;
    }
}

// y[t, h..h+3] = fp16( sum_j O[t*topk + j, h..h+3] ), slots in order, invalid ids skipped.  BF: rows
// and result are bfloat16.
template <bool BF>
__global__ __launch_bounds__(256) void combine_kernel(const f16* __restrict__ O, int splits,
                                                      int64_t split_stride,
                                                      const int32_t* __restrict__ ids, int E,
                                                      int topk, int64_t T, int64_t H,
                                                      f16* __restrict__ Y) {
    const int64_t t = blockIdx.y;
    const int64_t h = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (h >= H) return;
    // rows are added slot by slot, split by split; eight loads are in flight at a time
    f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
    const int total = topk * splits;
    for (int base = 0; base < total; base += 8) {
        u32x2 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int q = base + i;
            const int j = q / splits, s = q - j * splits;
            bool ok = q < total;
            if (ok) {
                const int id = ids[t * topk + j];
                ok = id >= 0 && id < E;
            }
            v[i] = u32x2{0u, 0u};
            if (ok) v[i] = *reinterpret_cast<const u32x2*>(O + s * split_stride + (t * topk + j) * H + h);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (BF) {       // a bfloat16 is the upper half of the binary32 with the same value
                sum[0] += __builtin_bit_cast(float, v[i].x << 16);
                sum[1] += __builtin_bit_cast(float, v[i].x & 0xffff0000u);
                sum[2] += __builtin_bit_cast(float, v[i].y << 16);
                sum[3] += __builtin_bit_cast(float, v[i].y & 0xffff0000u);
            } else {
                const f16x4 f = __builtin_bit_cast(f16x4, v[i]);
#pragma unroll
                for (int e = 0; e < 4; ++e) sum[e] += (float)f[e];
            }
        }
    }
    u32x2 ob;
    if (BF) {
        ob = u32x2{pack_bf16(sum[0], sum[1]), pack_bf16(sum[2], sum[3])};
    } else {
        f16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (f16)sum[e];
        ob = __builtin_bit_cast(u32x2, o);
    }
    *reinterpret_cast<u32x2*>(Y + t * H + h) = ob;
}

struct MoeLayout {
    int bm;
    int max_tiles;
    int64_t ldt;
    int parts_up, parts_down;   // parts of T = X V^T for the gate/up and the down projection
    int splits_down;            // K splits of the down projection
    size_t off_header, off_flags, off_sorted, off_token, off_slots, off_tiles, off_t1, off_t3, off_tp1, off_tp3, off_h, off_o, total;
    int64_t max_tiles32;
};

static bool moe_layout(int64_t T, int64_t H, int64_t F, int E, int topk, int r_max, MoeLayout* L) {
    if (T <= 0 || E <= 0 || topk <= 0 || r_max < 0) return false;
    if (!weight_shape_ok(F, H) || !weight_shape_ok(H, F)) return false;
    if (H % 4 != 0) return false;
    const int64_t P = T * topk;
    if (P > (int64_t)0x3fffffff || E > 65536) return false;
    if (((uint64_t)r_max + 256) * (uint64_t)(H > F ? H : F) * 2 >= 0xFFFFFFF0ull) return false;
    // activations are addressed with 32-bit offsets inside the kernels
    if ((uint64_t)T * H * 2 >= 0x80000000ull || (uint64_t)P * F * 2 >= 0x80000000ull) return false;
    const int64_t avg = P / E;
    // Tile height: an expert whose rows do not fit one tile streams its weights once more, a
    // taller tile costs more activation copies and a shallower pipeline; measured on the Mixtral
    // shape the crossovers lie near 26 and 56 rows per expert.
    L->bm = avg >= 56 ? 128 : (avg >= 26 ? 64 : 32);
    // tuning override, read once per process so that the workspace query and the call agree
    static const int bm_override = [] {
        const char* e = getenv("MILO_MOE_BM");
        const int v = e ? atoi(e) : 0;
        return (v == 32 || v == 64 || v == 128) ? v : 0;
    }();
    if (bm_override) L->bm = bm_override;
    const int64_t max_tiles32 = (P + 31) / 32 + E;      // bound for the smallest tile height
    const int64_t max_tiles = (P + L->bm - 1) / L->bm + E;
    if (max_tiles > 65535) return false;
    L->max_tiles = (int)max_tiles;
    L->ldt = ((int64_t)r_max + 15) / 16 * 16;
    L->parts_up = r_max > 0 ? tiled_t_parts(H) : 0;
    L->parts_down = r_max > 0 ? tiled_t_parts(F) : 0;
    const int parts = L->parts_up > L->parts_down ? L->parts_up : L->parts_down;
    if ((uint64_t)(parts > 0 ? parts : 1) * (uint64_t)P * (uint64_t)L->ldt * 4 >= 0xFFFFFFF0ull) return false;
    // the down projection has few column tiles (hidden / 256): split K when they do not fill the chip
    // (counted in full tiles: the partly filled last tile of an expert is cheap)
    int64_t est_tiles = (P + L->bm - 1) / L->bm;
    int split_cap = 64;
    if (L->bm == 32) {
        // Decode-sized batches: nearly every tile is an expert's only, partly filled one, and it costs a
        // full pass over the expert's weight whatever its rows, so the tiles to count are the experts
        // that receive anything: E (1 - (1 - 1/E)^P) for evenly spread pairs.  Measured on the Mixtral
        // shape (16, 4 and 1 tokens), splits beyond eight lose more to short workgroups than they gain.
        const double used = (double)E * (1.0 - pow(1.0 - 1.0 / (double)E, (double)P));
        if ((int64_t)(used + 0.5) > est_tiles) est_tiles = (int64_t)(used + 0.5);
        split_cap = 8;
    }
    L->splits_down = tiled_k_splits(est_tiles * ((H + 255) / 256), F, 0);
    if (L->splits_down > split_cap) L->splits_down = split_cap;
    static const int splits_override = [] {
        const char* e = getenv("MILO_MOE_SPLITS");
        const int v = e ? atoi(e) : 0;
        return (v >= 1 && v <= 16) ? v : 0;
    }();
    if (splits_override) L->splits_down = splits_override;
    size_t off = 0;
    L->off_header = off; off = align_up(off + 64, 256);
    L->max_tiles32 = max_tiles32;
    L->off_flags = off;  off = align_up(off + 2 * (size_t)max_tiles32 * 16, 256);   // gate/up launch, down launch
    L->off_sorted = off; off = align_up(off + (size_t)P * 4, 256);
    L->off_token = off;  off = align_up(off + (size_t)P * 4, 256);
    L->off_slots = off;  off = align_up(off + (size_t)max_tiles32 * sizeof(TileDesc), 256);
    L->off_tiles = off;  off = align_up(off + (size_t)max_tiles32 * sizeof(TileDesc), 256);
    L->off_t1 = off;     off = align_up(off + (size_t)P * L->ldt * 2, 256);
    L->off_t3 = off;     off = align_up(off + (size_t)P * L->ldt * 2, 256);
    L->off_tp1 = off;    off = align_up(off + (size_t)parts * P * L->ldt * 4, 256);
    L->off_tp3 = off;    off = align_up(off + (size_t)L->parts_up * P * L->ldt * 4, 256);
    L->off_h = off;      off = align_up(off + (size_t)P * F * 2, 256);
    L->off_o = off;      off = align_up(off + (size_t)L->splits_down * P * H * 2, 256);
    L->total = off;
    return true;
}

static int check_weight(const milo_w3lr_weight& w, int64_t N, int64_t K) {
    if (!w.q3) return MILO_ERR_NULL;
    if (w.r < 0 || w.r > N || w.r > K) return MILO_ERR_RANK;
    if (w.r > 0 && (!w.U || !w.V)) return MILO_ERR_RANK;
    if (w.flags & ~(MILO_W3_SYMMETRIC | MILO_LR_INT3)) return MILO_ERR_SHAPE;
    if (w.r > 0 && (w.flags & MILO_LR_INT3)) {
        if (w.r > MILO_LR3_MAX_RANK) return MILO_ERR_RANK;
        if ((N % kGroup) != 0) return MILO_ERR_SHAPE;
    }
    if (!aligned16(w.q3) || !aligned16(w.U) || !aligned16(w.V))
        return MILO_ERR_ALIGN;
    return MILO_OK;
}

}  // namespace milo

using namespace milo;

extern "C" int milo_moe_w3lr_check_experts(const milo_w3lr_expert* experts, int E, int64_t H,
                                           int64_t F, int* r_max_out) {
    return milo_moe_w3lr_check_experts_flags(experts, E, H, F, 0u, r_max_out);
}

extern "C" int milo_moe_w3lr_check_experts_flags(const milo_w3lr_expert* experts, int E, int64_t H,
                                                 int64_t F, unsigned flags, int* r_max_out) {
    if (!experts) return MILO_ERR_NULL;
    if (flags & ~MILO_ACT_BF16) return MILO_ERR_SHAPE;
    if (E <= 0 || !weight_shape_ok(F, H) || !weight_shape_ok(H, F)) return MILO_ERR_SHAPE;
    int r_max = 0;
    for (int e = 0; e < E; ++e) {
        const milo_w3lr_weight* ws[3] = {&experts[e].w1, &experts[e].w3, &experts[e].w2};
        for (int i = 0; i < 3; ++i) {
            const int64_t N = (i < 2) ? F : H, K = (i < 2) ? H : F;
            const int st = check_weight(*ws[i], N, K);
            if (st != MILO_OK) return st;
            // the bf16 kernels read U and V as bf16 arrays: no INT3 compensators there
            if ((flags & MILO_ACT_BF16) && ws[i]->r > 0 && (ws[i]->flags & MILO_LR_INT3)) return MILO_ERR_SHAPE;
            if (ws[i]->r > r_max) r_max = ws[i]->r;
        }
        // gate and up projection share a launch: their compensators are both INT3 or both fp16
        if (experts[e].w1.r > 0 && experts[e].w3.r > 0 &&
            ((experts[e].w1.flags ^ experts[e].w3.flags) & MILO_LR_INT3))
            return MILO_ERR_SHAPE;
    }
    if (r_max_out) *r_max_out = r_max;
    return MILO_OK;
}

extern "C" size_t milo_moe_w3lr_workspace(int64_t T, int64_t H, int64_t F, int E, int topk,
                                          int r_max) {
    MoeLayout L;
    if (!moe_layout(T, H, F, E, topk, r_max, &L)) return 0;
    return L.total;
}

extern "C" int milo_moe_w3lr_forward(const milo_half* X, int64_t T, int64_t H, int64_t F,
                                     const milo_w3lr_expert* experts, int E, int r_max,
                                     const int32_t* topk_ids, const float* topk_weights, int topk,
                                     milo_half* Y, void* workspace, size_t workspace_bytes,
                                     void* stream_) {
    return milo_moe_w3lr_forward_flags(X, T, H, F, experts, E, r_max, topk_ids, topk_weights, topk, 0u, Y, workspace,
                                       workspace_bytes, stream_);
}

extern "C" int milo_moe_w3lr_forward_flags(const milo_half* X, int64_t T, int64_t H, int64_t F,
                                           const milo_w3lr_expert* experts, int E, int r_max,
                                           const int32_t* topk_ids, const float* topk_weights, int topk,
                                           unsigned call_flags, milo_half* Y, void* workspace, size_t workspace_bytes,
                                           void* stream_) {
    if (!X || !experts || !topk_ids || !topk_weights || !Y) return MILO_ERR_NULL;
    if (call_flags & ~MILO_ACT_BF16) return MILO_ERR_SHAPE;
    const int bf = (call_flags & MILO_ACT_BF16) ? 1 : 0;
    MoeLayout L;
    if (!moe_layout(T, H, F, E, topk, r_max, &L)) return MILO_ERR_SHAPE;
    if (r_max > H || r_max > F) return MILO_ERR_RANK;
    if (!workspace || workspace_bytes < L.total) return MILO_ERR_WORKSPACE;
    if (!aligned16(X) || !aligned16(Y) || !aligned16(workspace) || !aligned16(experts) ||
        !aligned16(topk_ids) || !aligned16(topk_weights))
        return MILO_ERR_ALIGN;
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = reinterpret_cast<char*>(workspace);
    int32_t* header = reinterpret_cast<int32_t*>(ws + L.off_header);
    int32_t* sorted = reinterpret_cast<int32_t*>(ws + L.off_sorted);
    int32_t* sorted_token = reinterpret_cast<int32_t*>(ws + L.off_token);
    TileDesc* slots = reinterpret_cast<TileDesc*>(ws + L.off_slots);
    TileDesc* tiles = reinterpret_cast<TileDesc*>(ws + L.off_tiles);
    f16* T1 = reinterpret_cast<f16*>(ws + L.off_t1);
    f16* T3 = reinterpret_cast<f16*>(ws + L.off_t3);
    float* Tp1 = reinterpret_cast<float*>(ws + L.off_tp1);
    float* Tp3 = reinterpret_cast<float*>(ws + L.off_tp3);
    f16* Hbuf = reinterpret_cast<f16*>(ws + L.off_h);
    f16* O = reinterpret_cast<f16*>(ws + L.off_o);
    const int P = (int)(T * topk);

    RouteArgs ra;
    ra.ids = topk_ids; ra.P = P; ra.E = E; ra.bm = L.bm;
    ra.topk = topk; ra.sorted = sorted; ra.sorted_token = sorted_token; ra.tiles = slots; ra.header = header;
    uint32_t* flags = reinterpret_cast<uint32_t*>(ws + L.off_flags);
    ra.flags = flags; ra.n_flags = (int32_t)(2 * 4 * L.max_tiles32);
    ra.max_tiles = L.max_tiles;
    int st;
    if (P <= kSmallPairs && E <= kSmallExperts && L.bm == 32) {
        route_small_kernel<<<dim3(1), dim3(kSmallPairs), 0, stream>>>(ra, tiles, experts);
        st = launch_status();
        if (st != MILO_OK) return st;
    } else {
        route_kernel<<<dim3((unsigned)E), dim3(kRouteThreads), 0, stream>>>(ra);
        st = launch_status();
        if (st != MILO_OK) return st;
        order_tiles_kernel<<<dim3(1), dim3(kRouteThreads), 0, stream>>>(slots, L.max_tiles, L.bm, tiles, header, experts);
        st = launch_status();
        if (st != MILO_OK) return st;
    }

    RowSpace rs;
    rs.tiles = tiles; rs.n_tiles = header + 1; rs.experts = experts;
    rs.M = P;
    const int mb = L.bm / 32;
    // with few rows per expert nearly every expert is a single tile: its weights are read once
    const int once = L.bm < 64 ? 1 : 0;

    // gate / up projection
    rs.which[0] = 0; rs.which[1] = 1;
    rs.x_rows = sorted_token;
    {
        TiledArgs ga;
        ga.rs = rs; ga.X = reinterpret_cast<const f16*>(X); ga.ldx = H; ga.x_bytes = (uint64_t)T * H * 2;
        ga.N = F; ga.K = H;
        ga.T[0] = T1; ga.T[1] = T3; ga.ldt = L.ldt; ga.t_bytes = (uint64_t)P * L.ldt * 2;
        ga.Tp[0] = Tp1; ga.Tp[1] = Tp3; ga.tp_bytes = (uint64_t)L.parts_up * P * L.ldt * 4;
        ga.t_part_stride = (int64_t)P * L.ldt; ga.t_parts = L.parts_up; ga.v_tiles = L.parts_up; ga.ksplit = 1;
        ga.out_split_stride = 0; ga.flags = flags; ga.self_clean = 0; ga.weights_once = once;
        ga.t_dist = 0; ga.lr_splits = 1; ga.lr_step = 0; ga.act_bf16 = bf;
        ga.flags_status = reinterpret_cast<uint32_t*>(header + 3);
        ga.lr3_rank = bf ? 0 : (r_max < MILO_LR3_MAX_RANK ? r_max : MILO_LR3_MAX_RANK);    // (any weight's compensator may be INT3)
        ga.out = Hbuf; ga.ldo = F; ga.out_rows = nullptr; ga.out_scale = nullptr;
        st = launch_tiled(ga, 2, mb, EPI_SWIGLU, L.max_tiles, stream);
        if (st != MILO_OK) return st;
    }
    // down projection (T2 reuses the T1 buffer: T1 is dead once the gate/up kernel has run)
    rs.which[0] = 2; rs.which[1] = 2;
    rs.x_rows = nullptr;
    {
        TiledArgs da;
        da.rs = rs; da.X = Hbuf; da.ldx = F; da.x_bytes = (uint64_t)P * F * 2;
        da.N = H; da.K = F;
        da.T[0] = T1; da.T[1] = T1; da.ldt = L.ldt; da.t_bytes = (uint64_t)P * L.ldt * 2;
        da.Tp[0] = Tp1; da.Tp[1] = Tp1; da.tp_bytes = (uint64_t)L.parts_down * P * L.ldt * 4;
        da.t_part_stride = (int64_t)P * L.ldt; da.t_parts = L.parts_down; da.v_tiles = L.parts_down;
        da.ksplit = L.splits_down; da.out_split_stride = (int64_t)P * H; da.flags = flags + 4 * L.max_tiles32;
        da.self_clean = 0; da.weights_once = once;
        da.t_dist = 0; da.lr_splits = 1; da.lr_step = 0; da.act_bf16 = bf;
        da.flags_status = reinterpret_cast<uint32_t*>(header + 3);
        da.lr3_rank = bf ? 0 : (r_max < MILO_LR3_MAX_RANK ? r_max : MILO_LR3_MAX_RANK);
        da.out = O; da.ldo = H; da.out_rows = sorted; da.out_scale = topk_weights;
        st = launch_tiled(da, 1, mb, EPI_SCALE_SCATTER, L.max_tiles, stream);
        if (st != MILO_OK) return st;
    }
    {
        const unsigned gx = (unsigned)((H / 4 + 255) / 256);
        if (T > 65535) {
            // grid.y limit: split the token range
            for (int64_t t0 = 0; t0 < T; t0 += 65535) {
                const int64_t nt = (T - t0) < 65535 ? (T - t0) : 65535;
                auto kern = bf ? combine_kernel<true> : combine_kernel<false>;
                kern<<<dim3(gx, (unsigned)nt), dim3(256), 0, stream>>>(
                    O + t0 * topk * H, L.splits_down, (int64_t)P * H, topk_ids + t0 * topk, E, topk, nt, H,
                    reinterpret_cast<f16*>(Y) + t0 * H);
            }
        } else {
            auto kern = bf ? combine_kernel<true> : combine_kernel<false>;
            kern<<<dim3(gx, (unsigned)T), dim3(256), 0, stream>>>(
                O, L.splits_down, (int64_t)P * H, topk_ids, E, topk, T, H, reinterpret_cast<f16*>(Y));
        }
        st = launch_status();
    }
    return st;
}

extern "C" int milo_moe_w3lr_routing_status(const void* workspace, void* stream) {
    if (!workspace) return MILO_ERR_NULL;
    int32_t header[4] = {0, 0, 0, 0};
    if (hipMemcpyAsync(header, workspace, sizeof(header), hipMemcpyDeviceToHost,
                       (hipStream_t)stream) != hipSuccess)
        return MILO_ERR_HIP;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return MILO_ERR_HIP;
    if (header[3] != 0) return MILO_ERR_WAIT;       // a wait inside a kernel gave up
    return header[0] == MILO_OK ? MILO_OK : MILO_ERR_ROUTING;
}
