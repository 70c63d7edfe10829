// Weight-streaming kernel for the compensated W3A16 linear at M <= 16 (decode): ONE launch that
// streams the packed weight once from HBM, forms T = X V^T cooperatively and adds T U^T.
//
// Weight stream.  A workgroup of sixteen waves owns 16*R output features over the whole K.  K is
// cut into chunks of 256 columns; wave w takes chunks w, w + 16, ... for all R 16-row blocks.  For
// a chunk a lane loads one unit per 16-row block (24 bytes of codes, fp16 scale and zero-point)
// with fully coalesced 16- and 12-byte buffer loads and no branches (lanes without data read out
// of range and get zeros), converts it in registers and feeds it as the A operand of
// v_mfma_f32_16x16x32_f16 (lane quad q = group 4c+q, eight steps of eight codes).
// The activations of a chunk, X[0..15][256c .. 256c+255], are the B operand of every block.  A wave
// copies them into its own 8-KB LDS slot with up to eight coalesced 1-KB buffer-to-LDS loads (two
// full 512-byte row pieces each, no registers involved); the 16-byte segment that sits at slot
// position p of row j is segment p ^ j of the row, which makes the later per-lane ds_read_b128 of
// the B fragments conflict free although the 16 lanes of a quad read 16 rows.  A slot is written
// and read by one wave only, so the main loop takes no barrier; the waves' partial sums are added
// in a fixed order at the very end.
//
// Why sixteen waves.  A CU accepts vector memory requests only as fast as earlier ones return, and
// a wave cannot convert anything while it is queueing requests.  Timestamps inside an eight-wave
// version (two chunks per wave, everything requested up front) showed the first wave of every SIMD
// queueing for 3 us and converting for 3.5 us, the second one queueing for 5.3 us and converting
// after that: half of the conversion ran after the last byte had arrived.  With sixteen waves of
// half the work each, a wave is through with its requests after a quarter of the stream and
// converts while the later waves of its SIMD still queue.
//
// Low-rank term.  The first `nt` workgroups do no streaming: each computes whole blocks of 16
// ranks of T = X V^T over a part of K (the parts are never added up across workgroups), writes
// them as fp16 and is counted.  The streaming workgroups only need T in their epilogue, where
// they add T U^T with a few more MFMAs.  Wave 0 of a streaming workgroup, whose requests are
// accepted first and which is therefore done long before the others, fetches the U rows and,
// once all workers have been counted, T into LDS.  The workers never wait for anything, they have
// the lowest workgroup ids, and the grid never exceeds what the device keeps resident, so that
// wait always ends.  Data that crosses workgroups is written and read with device-coherent
// accesses, and worker 0 restores the control words to zero for the next launch.
#include <stdlib.h>

#include <type_traits>

#include "milo_host.h"
#include "milo_kernels.h"

namespace milo {

constexpr int kDecWaves = 16;                               // waves of a workgroup
constexpr int kDecThreads = 64 * kDecWaves;
constexpr int kDecTWaves = 8;                               // waves of a T worker that take a chunk each
constexpr int kDecSlotBytes = 16 * 512;                     // one chunk of X: 16 rows x 256 k
constexpr int kDecLdsBytes = kDecWaves * kDecSlotBytes;     // 128 KB

__device__ __forceinline__ void buf_store16_coherent(BufRsrc r, uint32_t off, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, 17);
}
__device__ __forceinline__ void buf_store8_coherent(BufRsrc r, uint32_t off, u32x2 v) {
    __builtin_amdgcn_raw_buffer_store_b64(v, r, off, 0, 17);
}
typedef __attribute__((address_space(3))) void* LdsPtr;

// Compile-time loop: f(std::integral_constant<int, I>) for I in [B, E).
template <int B, int E, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (B < E) {
        f(std::integral_constant<int, B>{});
        static_for<B + 1, E>(f);
    }
}

// Staging of one chunk of X (16 rows x 256 columns, the B operand of every row block) in an
// 8-KB LDS slot: copy i moves rows 2i, 2i+1 with one coalesced 1-KB buffer-to-LDS load, lane l ->
// row 2i + l/32, slot position p = l%32, which receives segment p ^ row of the row's 32 segments of
// 8 columns.  Only the first XC copies are issued, XC = ceil(M / 2) rounded up to a power of two:
// rows beyond them keep whatever the slot held, which only reaches output columns (tokens) >= M,
// and those are never stored.  Rows >= M inside the copies lie past the end of X and read as zero.
struct XCopy {
    uint32_t xseg, xrow;
    __device__ __forceinline__ XCopy(int lane, uint32_t K) {
        const uint32_t crow = (uint32_t)lane >> 5, cp = (uint32_t)lane & 31u;
        xseg = (cp ^ crow) << 4;
        xrow = crow * 2u * K;
    }
    // kc = first column of the chunk; a chunk that reaches beyond K (the last one when K is not a
    // multiple of 256, or one past the end) must not wrap into the next row: only the first `lim`
    // bytes of its 512-byte row pieces exist.  lim is a multiple of 128, so whether a lane's segment
    // exists depends on its 128-byte quarter only, which the xor with 2i changes for i >= 4.
    // `base` is added to every offset (the first row of a block of V rows).
    template <int XC>
    __device__ __forceinline__ void issue(BufRsrc xb, unsigned char* slot, uint32_t kc, uint32_t K, bool valid,
                                          uint32_t base = 0u) const {
        const uint32_t lim = (!valid || kc >= K) ? 0u : (K - kc >= 256u ? 512u : 2u * (K - kc));
        const bool ok_lo = (xseg & 0x180u) < lim;
        const bool ok_hi = ((xseg & 0x180u) ^ 0x80u) < lim;
#pragma unroll
        for (int i = 0; i < XC; ++i) {
            // (the constant goes through an opaque scalar so that the per-lane offsets are formed
            // here, four cheap operations per copy, instead of living in registers across the loop)
            uint32_t flip = 32u * i, uni = __builtin_amdgcn_readfirstlane(4u * i * K + 2u * kc + base);
            asm volatile("" : "+s"(flip), "+s"(uni));
            const uint32_t off = ((xseg ^ flip) + xrow) + uni;
            const uint32_t o = (i < 4 ? ok_lo : ok_hi) ? off : kOobOffset;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xb, (LdsPtr)(slot + i * 1024), 16, o, 0, 0, 0);
        }
        asm volatile("" ::: "memory");
    }
};

// B fragments of a staged chunk: step t, lane (j16, q) = X[j16][8 (8q + t) .. + 7] of the chunk.
__device__ __forceinline__ void read_bfrags(const unsigned char* slot, int j16, int q, f16x8 (&bfrag)[8]) {
#pragma unroll
    for (int t = 0; t < 8; ++t)
        bfrag[t] = __builtin_bit_cast(
            f16x8, *reinterpret_cast<const u32x4*>(slot + j16 * 512 + (((8 * q + t) ^ j16) << 4)));
}

// T worker.  Work item (jb, h) = rank block jb (16 ranks) over K part h (kDecTWaves chunks of 256
// columns, one per wave): T_h[m][j] = sum over the part of X[m][k] V[j][k].  The parts are NOT
// added up: the streaming workgroups multiply every T_h with U, which gives the same sum without
// a reduction across workgroups.  Both operands are staged like the activations of the main
// path (coalesced 1-KB buffer-to-LDS copies into a wave-private slot, xor-swizzled), and all
// copies of an item are requested at once.  The upper half of the workgroup's waves has no work
// here and only takes part in the barriers.
// Q: V is the INT3 blob of milo_pack_lr3, [16 rblocks x K] in the layout of a weight: a lane loads
// the unit of rank 16 jb + lane % 16, group 4c + lane / 16, exactly as a streaming wave does for a
// row block, and converts it with the zero-point-free conversion (the quantizer is symmetric).
// BF: activations, V and T are bf16 (MILO_ACT_BF16).
template <int XC, bool Q, bool BF>
__device__ __forceinline__ void decode_t_worker(const DecodeArgs& a, unsigned char* smem) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const bool active = wave < kDecTWaves;
    const int j16 = lane & 15, q = lane >> 4;
    const int M = a.M, r = a.w.r;
    const uint32_t K = (uint32_t)a.K;
    const BufRsrc xb = make_rsrc(a.X, (uint64_t)M * K * 2u);
    const BufRsrc vb = make_rsrc(a.w.V, (uint64_t)r * K * 2u);      // < 4 GiB (checked on the host)
    const BufRsrc tb = make_rsrc(a.T, (uint64_t)a.kh * 16u * (uint64_t)a.ldt * 2u);
    unsigned char* const xs = smem + (wave & (kDecTWaves - 1)) * 2 * kDecSlotBytes;     // X chunk, then V chunk
    unsigned char* const vs = xs + kDecSlotBytes;
    f32x4* const red = reinterpret_cast<f32x4*>(smem);              // [wave][64 lanes], after a barrier
    const XCopy xc(lane, K);

    for (int item = blockIdx.x; item < a.rblocks * a.kh; item += a.nt) {
        const int jb = item / a.kh, h = item - jb * a.kh;
        f32x4 tacc = {0.0f, 0.0f, 0.0f, 0.0f};
        if (active) {
            const uint32_t c = (uint32_t)(h * kDecTWaves + wave), kc = c * 256u;
            xc.issue<XC>(xb, xs, kc, K, true);
            if (Q) {
                const uint32_t G = K / kGroup;
                const W3Buf vq = make_w3buf(a.w.V, a.ldt, a.K);
                const RawUnit u = load_unit_buf(vq, 4u * c + q < G ? ((uint32_t)jb * G + 4u * c) * 16u + lane : (1u << 27));
                wait_vmem();
                f16x8 bfrag[8];
                read_bfrags(xs, j16, q, bfrag);
                dequant_unit_steps<true>(u, [&](int t, f16x8 frag) { tacc = mfma16(frag, bfrag[t], tacc); });
            } else {
                // rows >= r lie past the end of V and read as zero
                xc.issue<8>(vb, vs, kc, K, true, (uint32_t)(16 * jb) * K * 2u);
                wait_vmem();
                f16x8 bfrag[8], afrag[8];
                read_bfrags(xs, j16, q, bfrag);
                read_bfrags(vs, j16, q, afrag);
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    tacc = BF ? mfma16_bf16(__builtin_bit_cast(bf16x8, afrag[t]), __builtin_bit_cast(bf16x8, bfrag[t]), tacc)
                              : mfma16(afrag[t], bfrag[t], tacc);
            }
        }
        __syncthreads();                                    // every wave has read its slots
        if (active) red[wave * 64 + lane] = tacc;
        __syncthreads();
        if (wave == 0) {
            f32x4 part[kDecTWaves];
#pragma unroll
            for (int p = 0; p < kDecTWaves; ++p) part[p] = red[p * 64 + lane];
            __builtin_amdgcn_sched_barrier(0);
            f32x4 sum = part[0];
#pragma unroll
            for (int p = 1; p < kDecTWaves; ++p)
#pragma unroll
                for (int x = 0; x < 4; ++x) sum[x] += part[p][x];
            // element v of lane l = rank 16*jb + 4*(l/16) + v, token l%16
            u32x2 ob;
            if (BF) {
                ob = u32x2{pack_bf16(sum[0], sum[1]), pack_bf16(sum[2], sum[3])};
            } else {
                f16x4 o;
#pragma unroll
                for (int x = 0; x < 4; ++x) o[x] = (f16)sum[x];
                ob = __builtin_bit_cast(u32x2, o);
            }
            buf_store8_coherent(tb, (uint32_t)(((h * 16 + j16) * a.ldt + 16 * jb + 4 * q) * 2), ob);
        }
        __syncthreads();                                    // red is read before the slots are refilled
    }
    // all T stores of this workgroup are complete before it is counted
    wait_vmem();
    __syncthreads();
    if (tid == 0) atomicAdd(a.ctrl + 0, 1u);
}

// Bounded wait until every T worker has been counted; a wait that gives up sets an error word.
__device__ __forceinline__ void decode_wait_t(const DecodeArgs& a) {
    for (uint32_t spins = 0;
         __hip_atomic_load(a.ctrl + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (uint32_t)a.nt; ++spins) {
        __builtin_amdgcn_s_sleep(1);
        if (spins > a.spin_limit) {
            atomicOr(a.ctrl + 3, 1u);
            break;
        }
    }
}

// LR: 0 = no low-rank term, 1 = rank a multiple of 8 and at most 128 (U and T fragments come
// through LDS), 2 = any other rank (plain loads in the epilogue).
constexpr int kDecKS = 4;                                       // k-steps of 32 ranks, LR == 1
constexpr int kDecULds = kDecLdsBytes;                          // U fragments [R][kDecKS][64] x 16 B
constexpr int kDecTLds = kDecULds + 4 * kDecKS * 1024;          // T fragments [kDecTFrags][64] x 16 B
constexpr int kDecTFrags = 16;                                  // (K parts) x (k-steps used) at most, LR == 1
constexpr int kDecLdsTotal = kDecTLds + kDecTFrags * 1024;      // 160 KB, all a workgroup can have

// One turn of a streaming wave: R row blocks x the wave's chunks of K (chunks wave, wave + 16, ...,
// rotated per workgroup so that the workgroups, which all read the same X, do not walk the same
// L2 channels in step).
//
// The first chunk is requested up front: its activations, then its R units.  While unit (j, b) is
// converted, unit (j + 1, b) is requested into the registers it frees, and the activations of
// chunk j + 1 right after those of chunk j have been read into registers (one slot per wave).
// Vector memory operations complete in order, so "unit (j, b) and the activations of chunk j have
// arrived" is a fixed count of younger operations (the build script checks that the compiler adds
// no memory operation of its own and keeps the order):
//   request order   X0 W00 .. W0(R-1) | X1 W10 | W11 | ... | X2 W20 | ...
//   unit (j, 0):    2 (R - 1)              (the other units of chunk j)
//   unit (j, b>0):  2 (R - 1) + XC         (the rest of chunk j, X(j+1), the first b units of chunk j + 1)
//   last chunk:     2 (R - 1 - b)          (nothing is requested any more)
// For K up to 4096 a wave has a single chunk and everything is requested up front.
template <int R, int XC, bool SYM, bool BF>
struct DecodeStream {
    const W3Buf& wb;
    BufRsrc xb;
    XCopy xc;
    unsigned char* slot;        // the wave's slot
    uint32_t K, G, NB, C, span, first, lane, q, j16;

    __device__ __forceinline__ uint32_t chunk_of(uint32_t j) const {
        uint32_t idx = first + kDecWaves * j;
        if (idx >= span) idx -= span;
        return idx;
    }
    __device__ __forceinline__ void issue_x(uint32_t j) const {
        xc.issue<XC>(xb, slot, chunk_of(j) * 256u, K, true);
    }
    __device__ __forceinline__ void issue_w(uint32_t j, uint32_t rb, RawUnit& u) const {
        const uint32_t c = chunk_of(j);
        // (an index of 2^27 is past the end of every weight the host accepts, and 16 * 2^27 does not wrap)
        const bool ok = 4u * c + q < G && rb < NB;
        u = load_unit_buf_once(wb, ok ? (rb * G + 4u * c) * 16u + lane : (1u << 27));
        asm volatile("" ::: "memory");      // the loads keep this order (the waits count them)
    }

    template <bool LAST>
    __device__ __forceinline__ void chunk(uint32_t j, uint32_t rb0, RawUnit (&u)[R], f32x4 (&acc)[R]) const {
        f16x8 bfrag[8];
        static_for<0, R>([&](auto b_c) {
            constexpr int b = decltype(b_c)::value;
            __builtin_amdgcn_sched_barrier(0);      // nothing of this unit moves above its wait
            MILO_WAIT_VMEM(LAST ? 2 * (R - 1 - b) : (b == 0 ? 2 * (R - 1) : 2 * (R - 1) + XC));
            __builtin_amdgcn_sched_barrier(0);
            if (b == 0) {
                read_bfrags(slot, (int)j16, (int)q, bfrag);
                if (!LAST) {
                    // the slot is free once its fragments are in registers
                    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                    issue_x(j + 1);
                }
            }
            pin_unit_params(u[b]);          // nothing is computed from this unit before the wait
            if (BF)
                dequant_unit_steps_bf16(u[b], [&](int t, bf16x8 frag) {
                    acc[b] = mfma16_bf16(frag, __builtin_bit_cast(bf16x8, bfrag[t]), acc[b]);
                });
            else
                dequant_unit_steps<SYM>(u[b], [&](int t, f16x8 frag) { acc[b] = mfma16(frag, bfrag[t], acc[b]); });
            if (!LAST) {
                __builtin_amdgcn_sched_barrier(0);
                issue_w(j + 1, rb0 + b, u[b]);
            }
        });
    }

    __device__ __forceinline__ void run(uint32_t rb0, f32x4 (&acc)[R]) const {
        RawUnit u[R];
        issue_x(0);
#pragma unroll
        for (int b = 0; b < R; ++b) issue_w(0, rb0 + b, u[b]);
        for (uint32_t j = 0; j + 1 < C; ++j) chunk<false>(j, rb0, u, acc);
        chunk<true>(C - 1, rb0, u, acc);
    }
};


// Scatters the dequantized unit of one rank (64 consecutive output features, w[P] = features 2P and
// 2P + 1 of the group) into the U fragments of the R row blocks that start O16 blocks into the
// group: feature 16 (O16 + b) + jj of rank j goes to fragment (b, j / 32), lane (jj, (j % 32) / 8),
// element j % 8.  `frag0` points at that element of block 0's fragment for jj = 0.
template <int R, int O16>
__device__ __forceinline__ void scatter_u_rank(const uint32_t (&w)[32], unsigned char* frag0) {
#pragma unroll
    for (int b = 0; b < R; ++b)
#pragma unroll
        for (int jj = 0; jj < 16; ++jj) {
            const int n = 16 * (O16 + b) + jj;
            const uint32_t v = w[n >> 1];
            *reinterpret_cast<unsigned short*>(frag0 + b * (kDecKS * 1024) + jj * 16) =
                (unsigned short)((n & 1) ? (v >> 16) : v);
        }
}

// SYM: the weight blob is symmetric (zero-point-free conversion).  Q (with LR == 1): the compensator
// is the pair of INT3 blobs of milo_pack_lr3.
template <int R, int LR, int XC, bool SYM, bool Q, bool BF>
__global__ __launch_bounds__(kDecThreads) void w3lr_decode_kernel(const void* q3_, const f16* X_, uint32_t units_, uint32_t K_,
                                                                  uint32_t nb_, int M_, int nt_, uint32_t nmain_, uint32_t cpw_,
                                                                  uint32_t rot_mask_, uint32_t x_bytes_, const DecodeArgs a_) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // What a streaming wave needs for its first requests comes as leading scalar arguments, which the
    // hardware places in registers when it starts the wave (the build asks for that with
    // -amdgpu-kernarg-preload-count); everything else is read from the argument block when it is
    // needed.  The values are the same as the block's.
    DecodeArgs a = a_;
    a.w.q3 = q3_; a.X = X_; a.units = units_; a.K = (int64_t)K_; a.nb = nb_; a.M = M_; a.nt = nt_; a.nmain = nmain_;
    a.chunks_per_wave = cpw_; a.rot_mask = rot_mask_; a.x_bytes = x_bytes_;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nworkers = LR > 0 ? a.nt : 0;
    if (LR > 0 && (int)blockIdx.x < nworkers) {
        decode_t_worker<XC, Q, BF>(a, smem);
    } else {
        const int j16 = lane & 15, q = lane >> 4;
        const int M = a.M;
        const uint32_t K = (uint32_t)a.K;                   // < 2^27 (checked on the host)
        const uint32_t G = K / kGroup;
        const uint32_t NB = a.nb;                           // 16-row blocks
        const int r = a.w.r;
        W3Buf wb;
        wb.a = make_rsrc(a.w.q3, (uint64_t)(a.units * 16u));                // (units <= 2^26)
        wb.b = make_rsrc(reinterpret_cast<const char*>(a.w.q3) + (uint64_t)a.units * 16u, (uint64_t)(a.units * 12u));
        const uint32_t nmain = a.nmain;
        const BufRsrc tb = make_rsrc(a.T, (uint64_t)a.t_bytes);
        const int ksu = (r + 31) >> 5;                  // k-steps of 32 ranks in use
        // (T fragments in LDS: K part h, k-step i -> h * ksu + i)
        bool t_ready = false;

        const int wave_s = __builtin_amdgcn_readfirstlane(wave);        // known to be uniform
        DecodeStream<R, XC, SYM, BF> st{wb,
                               make_rsrc(a.X, (uint64_t)a.x_bytes),
                               XCopy(lane, K),
                               smem + wave_s * kDecSlotBytes,
                               K, G, NB, 0u, 0u, 0u, (uint32_t)lane, (uint32_t)q, (uint32_t)j16};
        st.C = a.chunks_per_wave;
        st.span = st.C * kDecWaves;
        // (rotation by a masked product instead of a remainder: no division before the first request)
        st.first = (uint32_t)wave_s + ((blockIdx.x * 5u) & a.rot_mask);
        if (st.first >= st.span) st.first -= st.span;

        // (every streaming workgroup has at least one turn: the number of turns is first looked at after it)
        uint32_t turn = 0, blk = blockIdx.x - nworkers;
        do {
            const uint32_t rb0 = blk * R;
            f32x4 acc[R];
#pragma unroll
            for (int b = 0; b < R; ++b) acc[b] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            f32x4* const red = reinterpret_cast<f32x4*>(smem);          // wave w, block b at 512 w + 64 b
            u32x4* const ulds = reinterpret_cast<u32x4*>(smem + kDecULds);
            u32x4* const tbuf = reinterpret_cast<u32x4*>(smem + kDecTLds);

            if (rb0 < NB) st.run(rb0, acc);
            // each wave leaves its partial sums in its own slot, which it has finished reading
#pragma unroll
            for (int b = 0; b < R; ++b) red[wave * (kDecSlotBytes / 16) + b * 64 + lane] = acc[b];
            if (LR > 0 && wave == 0) {
                // Everything the epilogue needs besides the partial sums, fetched by the wave that
                // is done first, while the others still stream; its requests go ahead of theirs.
                // U rows of the R row blocks as MFMA A fragments (k-step i, lane (j16, q) =
                // U[n][32i + 8q ..]), then, once every T worker has been counted, T as B
                // fragments with device-coherent reads: the workers wrote it during this launch.
                __builtin_amdgcn_s_setprio(3);
                if (LR == 1 && Q) {
                    // INT3 U: the blob holds U^T [ldt x N] with groups of 64 along N, and this
                    // workgroup's 16 R rows lie inside one group.  Lane l takes rank l (then l +
                    // 64): one unit, converted, and scattered into the fragment layout the
                    // epilogue reads.  Ranks past the compensator's read as zero units, which
                    // also clears the rest of the last k-step.
                    const W3Buf uq = make_w3buf(a.w.U, a.ldt, a.N);
                    const uint32_t GN = (uint32_t)(a.N >> 6), g = rb0 >> 2, o16 = rb0 & 3u;
                    for (uint32_t j = (uint32_t)lane; j < 32u * (uint32_t)ksu; j += 64u) {
                        const bool ok = j < (uint32_t)a.ldt && rb0 < NB;
                        const RawUnit u = load_unit_buf(uq, ok ? ((j >> 4) * GN + g) * 16u + (j & 15u) : (1u << 27));
                        uint32_t w[32];
                        dequant_unit<true>(u, w);
                        unsigned char* const frag0 =
                            smem + kDecULds + (((j >> 5) * 64u + ((j & 31u) >> 3) * 16u) * 16u + (j & 7u) * 2u);
                        if (R == 4) scatter_u_rank<R, 0>(w, frag0);
                        else if (R == 2) { if (o16 == 0) scatter_u_rank<R, 0>(w, frag0); else scatter_u_rank<R, 2>(w, frag0); }
                        else {
                            if (o16 == 0) scatter_u_rank<R, 0>(w, frag0);
                            else if (o16 == 1) scatter_u_rank<R, 1>(w, frag0);
                            else if (o16 == 2) scatter_u_rank<R, 2>(w, frag0);
                            else scatter_u_rank<R, 3>(w, frag0);
                        }
                    }
                } else if (LR == 1) {
                    const BufRsrc ub = make_rsrc(a.w.U, (uint64_t)a.u_bytes);
#pragma unroll 1
                    for (int b = 0; b < R; ++b) {
                        const uint32_t nrow = (rb0 + b) * 16u + j16;
#pragma unroll 1
                        for (int i = 0; i < ksu; ++i) {
                            const uint32_t k0 = 32u * i + 8u * q;
                            const uint32_t off =
                                (rb0 + b < NB && k0 < (uint32_t)r) ? (nrow * r + k0) * 2u : kOobOffset;
                            unsigned char* const dst = smem + kDecULds + (b * kDecKS + i) * 1024;
                            __builtin_amdgcn_raw_ptr_buffer_load_lds(ub, (LdsPtr)dst, 16, off, 0, 0, 0);
                        }
                    }
                }
                if (!t_ready) {
                    decode_wait_t(a);
                    if (LR == 1) {
                        int f = 0;
                        uint32_t ldt = (uint32_t)a.ldt;         // (offsets formed here, not kept from the top)
                        asm volatile("" : "+s"(ldt));
#pragma unroll 1
                        for (int h = 0; h < a.kh; ++h) {
#pragma unroll 1
                            for (int i = 0; i < ksu; ++i, ++f) {
                                const uint32_t k0 = 32u * i + 8u * q;
                                const uint32_t off = (k0 < ldt) ? ((h * 16u + j16) * ldt + k0) * 2u : kOobOffset;
                                unsigned char* const dst = smem + kDecTLds + f * 1024;
                                __builtin_amdgcn_raw_ptr_buffer_load_lds(tb, (LdsPtr)dst, 16, off, 0, 0, 17);
                            }
                        }
                    }
                    t_ready = true;
                }
                wait_vmem();
                __builtin_amdgcn_s_setprio(0);
                // this workgroup needs the control words and (LR == 1) T in memory no more
                if (LR == 1 && turn == 0 && lane == 0)
                    __hip_atomic_store(a.done + (blockIdx.x - nworkers), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();                                       // partial sums, U and T are in LDS
            if (wave < R) {
                // wave b finishes row block b: sum of the waves' partials in wave order
                const int b = wave;
                // (all partials are requested before the first addition: one LDS round trip, not sixteen)
                f32x4 part[kDecWaves];
#pragma unroll
                for (int pw = 0; pw < kDecWaves; ++pw) part[pw] = red[pw * (kDecSlotBytes / 16) + b * 64 + lane];
                __builtin_amdgcn_sched_barrier(0);
                f32x4 sum = part[0];
#pragma unroll
                for (int pw = 1; pw < kDecWaves; ++pw)
#pragma unroll
                    for (int e = 0; e < 4; ++e) sum[e] += part[pw][e];
                const uint32_t nb = (rb0 + b) * 16u;
                if (LR == 1) {
                    int f = 0;
#pragma unroll 1
                    for (int h = 0; h < a.kh; ++h) {
#pragma unroll 1
                        for (int i = 0; i < ksu; ++i, ++f)
                            sum = BF ? mfma16_bf16(__builtin_bit_cast(bf16x8, ulds[(b * kDecKS + i) * 64 + lane]),
                                                   __builtin_bit_cast(bf16x8, tbuf[f * 64 + lane]), sum)
                                     : mfma16(__builtin_bit_cast(f16x8, ulds[(b * kDecKS + i) * 64 + lane]),
                                              __builtin_bit_cast(f16x8, tbuf[f * 64 + lane]), sum);
                    }
                } else if (LR == 2) {
                    const int64_t nrow = (int64_t)nb + j16;
                    for (int ks = 0; ks < r; ks += 32) {
                        const int k0 = ks + 8 * q;
                        f16x8 av = zero_f16x8();
                        if (nrow < a.N) av = load_row8(a.w.U + nrow * r, k0, r, (r & 7) == 0);
                        for (int h = 0; h < a.kh; ++h) {
                            const f16x8 bv = __builtin_bit_cast(
                                f16x8, buf_load16_coherent(tb, k0 < a.ldt ? (uint32_t)(((h * 16 + j16) * a.ldt + k0) * 2)
                                                                          : kOobOffset));
                            sum = BF ? mfma16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv), sum)
                                     : mfma16(av, bv, sum);
                        }
                    }
                }
                // D[v]: feature nb + 4q + v, token j16.  (The output address is formed here, from
                // scalars the compiler cannot move: formed at the top of the kernel it would sit in
                // registers through the whole stream, or in scratch memory, a round trip to memory
                // right before the store.)
                uint32_t n_out = (uint32_t)a.N, m_out = (uint32_t)M;
                asm volatile("" : "+s"(n_out), "+s"(m_out));
                const uint32_t n = nb + 4u * q;
                if ((uint32_t)j16 < m_out && n < n_out) {
                    u32x2 ob;
                    if (BF) {
                        ob = u32x2{pack_bf16(sum[0], sum[1]), pack_bf16(sum[2], sum[3])};
                    } else {
                        f16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) o[e] = (f16)sum[e];
                        ob = __builtin_bit_cast(u32x2, o);
                    }
                    *reinterpret_cast<u32x2*>(a.Y + ((uint64_t)j16 * n_out + n)) = ob;
                }
            }
            if (turn + 1 < a.turns) __syncthreads();      // slots, U and the partial sums are reused
            blk += nmain;
        } while (++turn < a.turns);
    }

    // LR == 2: the streaming workgroups read T from memory in their epilogue, so they sign off last.
    if (LR == 2 && (int)blockIdx.x >= nworkers) {
        __syncthreads();
        if (tid == 0)
            __hip_atomic_store(a.done + (blockIdx.x - nworkers), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // Worker 0 stays until every streaming workgroup has signed off (which each does only after
    // it has seen all workers counted), then restores the control words for the next launch.
    // With LR == 1 the sign-offs come in the middle of the streaming work, so this wait ends
    // before the kernel would have ended anyway.  No returning atomic on a shared word is
    // involved: hundreds of those on one address serialize for several microseconds.
    if (LR > 0 && blockIdx.x == 0 && wave == 0) {
        const uint32_t nmain = a.nmain;
        bool all = false;
        for (uint32_t spins = 0; !all; ++spins) {
            all = true;
            for (uint32_t base = 0; base < nmain; base += 64) {
                const uint32_t idx = base + (uint32_t)lane;
                const uint32_t v =
                    idx < nmain ? __hip_atomic_load(a.done + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 1u;
                all = all && (__builtin_amdgcn_ballot_w64(v != 0u) == ~0ull);
            }
            if (!all) {
                __builtin_amdgcn_s_sleep(8);
                if (spins > (a.spin_limit >> 2)) {
                    atomicOr(a.ctrl + 3, 2u);
                    break;
                }
            }
        }
        if (all) {
            for (uint32_t base = 0; base < nmain; base += 64)
                if (base + (uint32_t)lane < nmain)
                    __hip_atomic_store(a.done + base + lane, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (lane == 0) __hip_atomic_store(a.ctrl + 0, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Workgroups the device keeps resident at once (one 128-KB-LDS workgroup per CU), cached per
// device; also raises the kernels' dynamic LDS limit once.
typedef void (*DecodeKernel)(const void*, const f16*, uint32_t, uint32_t, uint32_t, int, int, uint32_t, uint32_t, uint32_t, uint32_t,
                             const DecodeArgs);
// Variants: R x LR x XC for plain weights with an fp16 compensator (the generic path LR == 2 is not
// specialised by XC); with an INT3 compensator R x XC (LR == 1); with the symmetric conversion the
// shape that matters for speed, R == 4 with LR 0 or 1 (other shapes take the plain conversion, which
// gives the same bits).
template <int R, int LR, bool SYM, bool Q>
static DecodeKernel decode_variant_xc(int xc) {
    if constexpr (LR == 2) {
        return w3lr_decode_kernel<R, LR, 8, false, false, false>;
    } else {
        if (xc == 1) return w3lr_decode_kernel<R, LR, 1, SYM, Q, false>;
        if (xc == 2) return w3lr_decode_kernel<R, LR, 2, SYM, Q, false>;
        if (xc == 4) return w3lr_decode_kernel<R, LR, 4, SYM, Q, false>;
        return w3lr_decode_kernel<R, LR, 8, SYM, Q, false>;
    }
}
template <int LR, bool SYM, bool Q>
static DecodeKernel decode_variant_r(int R, int xc) {
    if (R == 4) return decode_variant_xc<4, LR, SYM, Q>(xc);
    if constexpr (SYM) {
        return nullptr;
    } else {
        if (R == 2) return decode_variant_xc<2, LR, SYM, Q>(xc);
        return decode_variant_xc<1, LR, SYM, Q>(xc);
    }
}
// bf16 activations: R x LR with all eight activation copies (no specialisation by M)
template <int LR>
static DecodeKernel decode_variant_bf(int R) {
    if (R == 4) return w3lr_decode_kernel<4, LR, 8, false, false, true>;
    if (R == 2) return w3lr_decode_kernel<2, LR, 8, false, false, true>;
    return w3lr_decode_kernel<1, LR, 8, false, false, true>;
}
static DecodeKernel decode_variant(int R, int lr, int xc, bool sym, bool q, bool bf = false) {
    if (bf) return q ? nullptr : lr == 0 ? decode_variant_bf<0>(R) : lr == 1 ? decode_variant_bf<1>(R) : decode_variant_bf<2>(R);
    if (q) return lr == 1 ? decode_variant_r<1, false, true>(R, xc) : nullptr;
    if (sym && R == 4 && lr < 2) return lr == 0 ? decode_variant_r<0, true, false>(R, xc) : decode_variant_r<1, true, false>(R, xc);
    if (lr == 0) return decode_variant_r<0, false, false>(R, xc);
    if (lr == 1) return decode_variant_r<1, false, false>(R, xc);
    return decode_variant_r<2, false, false>(R, xc);
}
static int decode_capacity() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return 0;
        for (int R = 1; R <= 4; R *= 2)
            for (int lr = 0; lr < 3; ++lr)
                for (int xc = 1; xc <= 8; xc *= 2)
                    for (int v = 0; v < 4; ++v) {       // plain, symmetric, INT3 compensator, bf16
                        const DecodeKernel k = decode_variant(R, lr, xc, v == 1, v == 2, v == 3);
                        if (k && hipFuncSetAttribute(reinterpret_cast<const void*>(k),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize,
                                                     kDecLdsTotal) != hipSuccess)
                            return 0;
                    }
        cached[dev] = cus;
    }
    return cached[dev];
}

// K parts of the T workers: kDecTWaves chunks of 256 columns each.
static int decode_k_parts(int64_t K) { return (int)((K + 256 * kDecTWaves - 1) / (256 * kDecTWaves)); }

size_t decode_workspace_bytes(int r, int64_t K) {
    if (r <= 0) return 256;
    const size_t rblocks = ((size_t)r + 15) / 16;
    // control words | sign-off words of the streaming workgroups | T fp16 [K parts][16 x ldt]
    return 256 + kDecDoneBytes + align_up((size_t)decode_k_parts(K) * 16 * rblocks * 16 * 2, 256);
}

// Row blocks per workgroup (16 R rows).  Every workgroup stages all of X once per turn and streams
// R row blocks; a CU takes in activations (from L2) roughly five times as fast as weights (from
// HBM), and the launch takes as long as its busiest CU: `turns` rounds of that.  The estimate picks
// R = 4 for the wide up projections, R = 1 for small weights, and for a long-K down projection whose
// R = 1 grid would exceed the resident workgroups by a few (a second round for a handful of
// blocks) the next R, which fits in one round.
static int decode_rows_per_workgroup(int64_t N, int64_t K, int slots) {
    const double x_bytes = 32.0 * (double)K, blk_bytes = 7.0 * (double)K;       // 16 rows of fp16 / of 3.5 bit
    int best = 1;
    double best_cost = 0.0;
    for (int R = 1; R <= 4; R *= 2) {
        const int64_t blocks = (N + 16 * R - 1) / (16 * R);
        const int64_t turns = (blocks + slots - 1) / slots;
        const double cost = (double)turns * (x_bytes / 130.0 + R * blk_bytes / 25.0);
        if (R == 1 || cost < best_cost) {
            best = R;
            best_cost = cost;
        }
    }
    return best;
}

int launch_decode(DecodeArgs a, void* workspace, hipStream_t stream) {
    const int cap = decode_capacity();
    if (cap <= 0) return MILO_ERR_HIP;
    const int r = a.w.r;
    a.rblocks = (r + 15) / 16;
    a.ldt = (int64_t)a.rblocks * 16;
    // V (padded to whole rank blocks) is addressed with 32-bit byte offsets
    if ((uint64_t)a.ldt * (uint64_t)a.K * 2u >= 0xFFFFFFF0ull) return MILO_ERR_SHAPE;
    char* ws = reinterpret_cast<char*>(workspace);
    a.ctrl = reinterpret_cast<uint32_t*>(ws);
    a.done = reinterpret_cast<uint32_t*>(ws + 256);
    a.T = reinterpret_cast<f16*>(ws + 256 + kDecDoneBytes);
    a.kh = decode_k_parts(a.K);
    a.spin_limit = 1u << 24;
    // T workers: one per block of 16 ranks and K part, at most kDecMaxWorkers and never more than
    // a quarter of the resident workgroups (a worker then takes several items in turn)
    int nt = a.rblocks * a.kh;
    if (nt > kDecMaxWorkers) nt = kDecMaxWorkers;
    if (nt > cap / 4) nt = cap / 4 > 0 ? cap / 4 : 1;
    a.nt = nt;
    const int workers = r > 0 ? nt : 0;
    if (cap <= workers || (size_t)cap * 4 > kDecDoneBytes) return MILO_ERR_HIP;
    int R = decode_rows_per_workgroup(a.N, a.K, cap - workers);
    static const int r_override = [] {                          // tuning override, read once per process
        const char* e = getenv("MILO_DEC_R");
        const int v = e ? atoi(e) : 0;
        return (v == 1 || v == 2 || v == 4) ? v : 0;
    }();
    if (r_override) R = r_override;
    const int rows = 16 * R;
    const int64_t blocks = (a.N + rows - 1) / rows;
    const int grid = (int)(blocks < cap - workers ? blocks : cap - workers) + workers;
    const bool int3 = (a.w.flags & MILO_LR_INT3) != 0;
    const bool lds_path = ((r & 7) == 0 || int3) && r <= 32 * kDecKS && a.kh * ((r + 31) / 32) <= kDecTFrags &&
                          (uint64_t)a.N * (uint64_t)r * 2u < 0xFFFFFFF0ull;
    const int lr = r == 0 ? 0 : lds_path ? 1 : 2;
    const int xc = a.M <= 2 ? 1 : a.M <= 4 ? 2 : a.M <= 8 ? 4 : 8;    // activation copies per chunk: rows 2i, 2i+1
    const bool q = r > 0 && (a.w.flags & MILO_LR_INT3) != 0;
    // an INT3 compensator only runs on the staged path: its T fragments must fit the workgroup's LDS
    if (q && lr != 1) return MILO_ERR_SHAPE;
    const bool bf = (a.w.flags & MILO_ACT_BF16) != 0;
    if (bf && q) return MILO_ERR_SHAPE;
    const DecodeKernel kernel = decode_variant(R, lr, xc, (a.w.flags & MILO_W3_SYMMETRIC) != 0, q, bf);
    if (!kernel) return MILO_ERR_HIP;
    const uint32_t nchunks = (uint32_t)((a.K + 255) / 256);
    a.units = (uint32_t)(a.N * (a.K / kGroup));
    a.nb = (uint32_t)(a.N >> 4);
    a.nmain = (uint32_t)(grid - workers);
    a.turns = (uint32_t)((blocks + a.nmain - 1) / a.nmain);
    a.chunks_per_wave = (nchunks + kDecWaves - 1) / kDecWaves;
    uint32_t pow2 = kDecWaves;
    while (pow2 * 2u <= a.chunks_per_wave * kDecWaves) pow2 *= 2u;
    a.rot_mask = pow2 - 1u;
    a.x_bytes = (uint32_t)((uint64_t)a.M * (uint64_t)a.K * 2u);            // (< 2^32: checked by the caller)
    a.t_bytes = (uint32_t)((uint64_t)a.kh * 16u * (uint64_t)a.ldt * 2u);
    a.u_bytes = (uint32_t)((uint64_t)a.N * (uint64_t)(r > 0 ? r : 0) * 2u);   // (fp16 U; < 2^32 on the staged path)
    kernel<<<dim3((unsigned)grid), dim3(kDecThreads), lr == 1 ? kDecLdsTotal : kDecLdsBytes, stream>>>(
        a.w.q3, a.X, a.units, (uint32_t)a.K, a.nb, a.M, a.nt, a.nmain, a.chunks_per_wave, a.rot_mask, a.x_bytes, a);
    return launch_status();
}

}  // namespace milo
