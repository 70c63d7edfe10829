// Argument blocks and host-side launchers of the GEMM kernels (internal to the library).
#pragma once

#include "milo_device.h"

namespace milo {

// Same bytes as the public milo_w3lr_weight.
struct WeightDev {
    const void* q3;
    const f16* U;       // fp16 [N x r], or with MILO_LR_INT3 the packed U^T blob [pad16(r) x N]
    const f16* V;       // fp16 [r x K], or with MILO_LR_INT3 the packed V blob [pad16(r) x K]
    int32_t r;
    uint32_t flags;     // MILO_W3_SYMMETRIC | MILO_LR_INT3
};
static_assert(sizeof(WeightDev) == sizeof(milo_w3lr_weight), "weight descriptor layout");
static_assert(sizeof(milo_w3lr_expert) == 3 * sizeof(WeightDev), "expert descriptor layout");

// One M-tile of a grouped problem: rows [row0, row0 + rows) of the expert-sorted row space.
struct TileDesc {
    int32_t expert;
    int32_t row0;
    int32_t rows;
    int32_t pad;
};

// Row-space conventions of the tiled kernel.
//   Ungrouped (tiles == nullptr): tile y covers rows [y*BM, min(M, (y+1)*BM)), weights = w[].
//   Grouped: tile y = tiles[y] if y < *n_tiles (else the workgroup exits); the weights are
//   experts[tile.expert].{w1,w3,w2}[which[a]].
//   Input row of tile row R:  x_rows ? x_rows[R] : R.
struct RowSpace {
    const TileDesc* tiles;
    const int32_t* n_tiles;
    const milo_w3lr_expert* experts;
    int which[2];
    WeightDev w[2];
    int64_t M;
    const int32_t* x_rows;
};

struct TiledArgs {
    RowSpace rs;
    const f16* X;       // input rows, leading dimension ldx
    int64_t ldx;
    uint64_t x_bytes;   // size of the X buffer in bytes (< 2 GiB: it is addressed with 32-bit offsets)
    int64_t N, K;       // weight shape (out x in)
    // T = X V^T per weight stream, [rows x ldt] fp16, zero beyond the rank.  It is formed during the
    // launch by v_tiles extra workgroups per M-tile: workgroup p multiplies its share of K into the fp32
    // partial Tp[.] + p * t_part_stride, and whichever column finishes last adds the partials in
    // column order, writes T and raises the tile's flag; the other workgroups read T after that.
    f16* T[2];
    int64_t ldt;
    uint64_t t_bytes;   // size of each T buffer in bytes
    float* Tp[2];       // partials, [t_parts][rows x ldt] fp32
    uint64_t tp_bytes;  // size of each partial buffer in bytes (all parts)
    int64_t t_part_stride;   // elements between consecutive parts
    int t_parts;        // 0 when no weight has a compensator
    int v_tiles;        // workgroups per M-tile that form T: t_parts (they belong to split 0)
    int ksplit;         // K splits; split z multiplies its share of the chunks
    int m_tiles;        // upper bound of the number of M-tiles (set by launch_tiled)
    int lr3_rank;       // largest rank an INT3 compensator of this launch may have (0: none can occur)
    int weights_once;   // non-zero: every weight is read by one M-tile only (non-temporal loads)
    uint32_t* flags;    // per M-tile t: [4t] parts done, [4t+1] T ready, [4t+2] readers done; zero at launch
    int self_clean;     // non-zero: the last reader of a tile's T clears its words (else the caller does before the next launch)
    int act_bf16;       // non-zero: activations, compensators and outputs are bfloat16 (MILO_ACT_BF16)
    int t_dist;         // non-zero: every part of T adds a share of the rows once all parts are written, and the
                        // tile's flag counts the parts that are done (large ranks; the single GEMM only)
    int lr_splits;      // K splits that apply the low-rank term, each to lr_step ranks (1: the first split does all)
    int lr_step;        // ranks per such split, a multiple of 64
    uint32_t* flags_status;  // set non-zero if a wait ever gave up
    // EPI 0: fp16 [rows x ldo], or with ksplit > 1 fp32 partial sums, split z at out + z * out_split_stride
    // EPI 1: fp16 [rows x ldo];  EPI 2: fp16 [.. x ldo], split z at out + z * out_split_stride
    void* out;
    int64_t ldo;
    int64_t out_split_stride;   // elements
    const int32_t* out_rows;   // EPI 2: output row of tile row R (nullptr: R)
    const float* out_scale;    // EPI 2: factor per output row (nullptr: 1)
};

// From this many M-tiles on, the tiled kernel gives each XCD a fixed contiguous share of the tile
// list (and the MoE work list is dealt accordingly).
constexpr uint32_t kXcdPlacementTiles = 128;

enum { EPI_STORE = 0, EPI_SWIGLU = 1, EPI_SCALE_SCATTER = 2 };

// Launchers.  mb = tile rows / 32 (1, 2 or 4); m_tiles = grid extent over tiles.
int launch_tiled(const TiledArgs& a, int nw, int mb, int epi, int m_tiles, hipStream_t stream);
// Parts of T and K splits the launchers use for a K of nchunks 128-column chunks.
int tiled_t_parts(int64_t K);
// Which of the two GEMM kernels milo_w3lr_gemm takes for a problem (true: the weight-streaming decode kernel).
bool gemm_takes_decode(int64_t M, int64_t N, int64_t K, int r);

constexpr int kDecDoneBytes = 8192;  // sign-off words: up to 2048 resident workgroups
constexpr int kDecMaxWorkers = 32;  // workgroups forming T = X V^T in the decode kernel

struct DecodeArgs {
    const f16* X;       // [M x K], M <= 16
    int M;
    int64_t N, K;
    WeightDev w;
    f16* Y;             // [M x N]
    // filled in by launch_decode from the workspace
    uint32_t* ctrl;     // [0] T workers done, [3] a wait gave up; zero between launches
    uint32_t* done;     // one sign-off word per streaming workgroup; zero between launches
    f16* T;             // [kh][16 x ldt] fp16: X V^T per K part, zero beyond the rank
    int64_t ldt;
    int rblocks;        // ceil(r / 16)
    int nt;             // number of T workers (the first nt workgroups)
    int kh;             // K parts of T (2048 columns each)
    uint32_t spin_limit;    // polls after which a wait inside the kernel gives up
    // sizes and counts worked out on the host, so that a wave's first memory requests do not wait for
    // arithmetic (divisions, 64-bit products) or for further loads of launch parameters
    uint32_t units;         // N * K / 64: 16 bytes each in plane A, 12 in plane B
    uint32_t nb;            // N / 16 row blocks
    uint32_t nmain;         // streaming workgroups of the launch
    uint32_t turns;         // row-block groups per streaming workgroup
    uint32_t chunks_per_wave;   // ceil(ceil(K / 256) / 16)
    uint32_t rot_mask;      // largest power of two not above 16 * chunks_per_wave, minus one
    uint32_t x_bytes, t_bytes, u_bytes;     // extents of X, T and (fp16) U
};
size_t decode_workspace_bytes(int r, int64_t K);
int launch_decode(DecodeArgs a, void* workspace, hipStream_t stream);

}  // namespace milo
