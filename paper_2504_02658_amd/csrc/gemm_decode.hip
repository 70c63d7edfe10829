// Weight-streaming kernel for the compensated W3A16 linear at M <= 16 (decode): ONE launch that
// streams the packed weight once from HBM, forms T = X V^T cooperatively and adds T U^T.
//
// Weight stream.  A workgroup of eight waves owns 16*R output features over the whole K.  K is
// walked in pieces of 16 chunks of 256; wave w takes chunks w and w+8 of the piece for all R
// 16-row blocks, so for K = 4096 every load of the launch is issued in the first few hundred
// cycles.  For a chunk a
// lane loads one unit per 16-row block (24 bytes of codes, fp16 scale and zero-point) with fully
// coalesced 16- and 12-byte buffer loads and no branches (lanes without data read out of range
// and get zeros), converts it in registers and feeds it as the A operand of
// v_mfma_f32_16x16x32_f16 (lane quad q = group 4c+q, eight steps of eight codes).
// The activations of a chunk, X[0..15][256c .. 256c+255], are the B operand of every block.  The
// workgroup stages a whole piece of X (16 rows x 4096 columns, 128 KB) in LDS once: a wave
// copies each of its chunks with eight coalesced 1-KB buffer-to-LDS loads (two full 512-byte row pieces
// each, no registers involved); the
// 16-byte segment that sits at slot position p of row j is segment p ^ j of the row, which makes
// the later per-lane ds_read_b128 of the B fragments conflict free although the 16 lanes of a
// quad read 16 rows.  A slot is written and read by one wave only, so the main loop takes no
// barrier; the waves' partial sums are added in a fixed order at the very end.
//
// Low-rank term.  The first `nt` workgroups do no streaming: each computes whole blocks of 16
// ranks of T = X V^T over all of K (so no sum crosses workgroups), writes them as fp16 and is
// counted.  The streaming workgroups only need T in their epilogue, where they add T U^T with a
// few more MFMAs once all workers have been counted.  The workers never wait for anything, they
// have the lowest workgroup ids, and the grid never exceeds what the device keeps resident, so the
// epilogue's wait always ends.  Data that crosses workgroups is written and read with
// device-coherent accesses, and the last workgroup to leave restores the control words to zero
// for the next launch.
#include <stdlib.h>

#include <type_traits>

#include "milo_host.h"
#include "milo_kernels.h"

namespace milo {

constexpr int kDecWaves = 8;
constexpr int kDecThreads = 64 * kDecWaves;
constexpr int kDecPiece = 16;                               // chunks of 256 k staged at a time
constexpr int kDecSlotBytes = 16 * 512;                     // one chunk of X: 16 rows x 256 k
constexpr int kDecLdsBytes = kDecPiece * kDecSlotBytes;     // 128 KB

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


// T worker.  Work item (jb, h) = rank block jb (16 ranks) over K part h (kDecWaves chunks of 256
// columns, one per wave): T_h[m][j] = sum over the part of X[m][k] V[j][k].  The parts are NOT
// added up: the streaming workgroups multiply every T_h with U, which gives the same sum without
// a reduction across workgroups.  Both operands are staged like the activations of the main
// path (coalesced 1-KB buffer-to-LDS copies into a wave-private slot, xor-swizzled), and all
// copies of an item are requested at once: the streaming workgroups fill the memory system's
// queues within a microsecond of the launch, and a request made later waits behind all of theirs.
__device__ __forceinline__ void decode_t_worker(const DecodeArgs& a, unsigned char* smem) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int j16 = lane & 15, q = lane >> 4;
    const int M = a.M, r = a.w.r;
    const uint32_t K = (uint32_t)a.K;
    const BufRsrc xb = make_rsrc(a.X, (uint64_t)M * K * 2u);
    const BufRsrc vb = make_rsrc(a.w.V, (uint64_t)r * K * 2u);      // < 4 GiB (checked on the host)
    const BufRsrc tb = make_rsrc(a.T, (uint64_t)a.kh * 16u * (uint64_t)a.ldt * 2u);
    unsigned char* const xs = smem + wave * 2 * kDecSlotBytes;      // X chunk, then V chunk
    unsigned char* const vs = xs + kDecSlotBytes;
    f32x4* const red = reinterpret_cast<f32x4*>(smem);              // [wave][64 lanes], after a barrier
    const uint32_t crow = (uint32_t)lane >> 5, cp = (uint32_t)lane & 31u;
    const uint32_t xseg = (cp ^ crow) << 4;
    const uint32_t xrow = crow * 2u * K;

    for (int item = blockIdx.x; item < a.rblocks * a.kh; item += a.nt) {
        const int jb = item / a.kh, h = item - jb * a.kh;
        const uint32_t kc = (uint32_t)(h * kDecWaves + wave) * 256u;
        const uint32_t lim = (kc >= K) ? 0u : (K - kc >= 256u ? 512u : 2u * (K - kc));
        const bool ok_lo = (xseg & 0x180u) < lim;
        const bool ok_hi = ((xseg & 0x180u) ^ 0x80u) < lim;
        // rows >= M lie past the end of X, rows >= r past the end of V: they read as zero
        const uint32_t vbase = (uint32_t)(16 * jb) * K * 2u;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t off = ((xseg ^ (32u * i)) + xrow) + (4u * i * K + 2u * kc);
            const bool ok = i < 4 ? ok_lo : ok_hi;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xb, (LdsPtr)(xs + i * 1024), 16, ok ? off : kOobOffset, 0, 0, 0);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(vb, (LdsPtr)(vs + i * 1024), 16, ok ? off + vbase : kOobOffset, 0,
                                                     0, 0);
        }
        wait_vmem();
        f32x4 tacc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int pos = j16 * 512 + (((8 * q + t) ^ j16) << 4);
            tacc = mfma16(__builtin_bit_cast(f16x8, *reinterpret_cast<const u32x4*>(vs + pos)),
                          __builtin_bit_cast(f16x8, *reinterpret_cast<const u32x4*>(xs + pos)), tacc);
        }
        __syncthreads();                                    // every wave has read its slots
        red[wave * 64 + lane] = tacc;
        __syncthreads();
        if (wave == 0) {
            f32x4 sum = red[lane];
#pragma unroll
            for (int p = 1; p < kDecWaves; ++p) {
                const f32x4 v = red[p * 64 + lane];
#pragma unroll
                for (int x = 0; x < 4; ++x) sum[x] += v[x];
            }
            // element v of lane l = rank 16*jb + 4*(l/16) + v, token l%16
            f16x4 o;
#pragma unroll
            for (int x = 0; x < 4; ++x) o[x] = (f16)sum[x];
            buf_store8_coherent(tb, (uint32_t)(((h * 16 + j16) * a.ldt + 16 * jb + 4 * q) * 2),
                                __builtin_bit_cast(u32x2, o));
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
        if (spins > (1u << 24)) {
            atomicOr(a.ctrl + 3, 1u);
            break;
        }
    }
}

// LR: 0 = no low-rank term, 1 = rank a multiple of 8 and at most 128 (U fragments are copied into
// LDS at the start of the kernel, T comes through LDS), 2 = any other rank (plain loads).
// The wave that fetches T for its workgroup: the first one, whose loads are served first and
// which therefore has time to spare at the end.
constexpr int kDecTWave = 0;
constexpr int kDecKS = 4;                                       // k-steps of 32 ranks, LR == 1
constexpr int kDecULds = kDecLdsBytes;                          // U fragments [R][kDecKS][64] x 16 B
constexpr int kDecTLds = kDecULds + 4 * kDecKS * 1024;          // T fragments [kDecTFrags][64] x 16 B
constexpr int kDecTFrags = 8;                                   // (K parts) x (k-steps used) at most, LR == 1
constexpr int kDecLdsTotal = kDecTLds + kDecTFrags * 1024;      // 152 KB

template <int R, int LR>
__global__ __launch_bounds__(kDecThreads) void w3lr_decode_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int nworkers = LR > 0 ? a.nt : 0;
    if (LR > 0 && (int)blockIdx.x < nworkers) {
        decode_t_worker(a, smem);
    } else {
        constexpr int CPW = kDecPiece / kDecWaves;  // chunks of a piece per wave
        const int j16 = lane & 15, q = lane >> 4;
        const int M = a.M;
        const uint32_t K = (uint32_t)a.K;                   // < 2^27 (checked on the host)
        const uint32_t G = K / kGroup;
        const uint32_t NB = (uint32_t)(a.N >> 4);           // 16-row blocks
        const uint32_t nchunks = (G + 3) / 4;
        const uint32_t npieces = (nchunks + kDecPiece - 1) / kDecPiece;
        const int r = a.w.r;
        const W3Buf wb = make_w3buf(a.w.q3, a.N, a.K);
        const BufRsrc xb = make_rsrc(a.X, (uint64_t)M * K * 2u);
        // Staging: copy i of a chunk moves rows 2i, 2i+1: lane l -> row 2i + l/32, slot position
        // p = l%32, which receives segment p ^ row of the row's 32 segments of 8 columns.
        // Byte offset of that segment = row*2K + 16*(p ^ row) + 2*kc, split into a per-lane part
        // that does not depend on i (the xor with 2i is applied to the segment bits) and a
        // uniform part.  Rows >= M lie past the end of X and read as zero.
        const uint32_t crow = (uint32_t)lane >> 5, cp = (uint32_t)lane & 31u;
        const uint32_t xseg = (cp ^ crow) << 4;
        const uint32_t xrow = crow * 2u * K;
        const uint32_t rot = (blockIdx.x * 5u) & (kDecPiece - 1);
        bool t_fetched = false;     // T is (being) copied into this workgroup's LDS
        // Tells worker 0 that this workgroup needs the control words and T no more.
        auto sign_off = [&]() {
            if (lane == 0)
                __hip_atomic_store(a.done + (blockIdx.x - nworkers), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        };
        const BufRsrc tb = make_rsrc(a.T, (uint64_t)a.kh * 16u * (uint64_t)a.ldt * 2u);
        const int ksu = (r + 31) >> 5;                  // k-steps of 32 ranks in use
        const int nfrag = a.kh * ksu;                   // T fragments: K part h, k-step i -> h * ksu + i
        // Copies T (device-coherent reads: the workers wrote it during this launch) into LDS as
        // MFMA B fragments; only to be called once all workers have been seen done.
        auto fetch_t = [&]() {
            int h = 0, i = 0;
#pragma unroll
            for (int f = 0; f < kDecTFrags; ++f) {
                if (f < nfrag) {
                    const int k0 = 32 * i + 8 * q;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        tb, (LdsPtr)(smem + kDecTLds + f * 1024), 16,
                        (k0 < a.ldt) ? (uint32_t)(((h * 16 + j16) * a.ldt + k0) * 2) : kOobOffset, 0, 0, 17);
                    if (++i == ksu) { i = 0; ++h; }
                }
            }
        };
        unsigned char* const myslot = smem + wave * kDecSlotBytes;      // slot of chunk ci: + 8*ci slots

        for (uint32_t blk = blockIdx.x - nworkers; blk * R < NB; blk += gridDim.x - nworkers) {
            const uint32_t rb0 = blk * R;
            f32x4 acc[R];
#pragma unroll
            for (int b = 0; b < R; ++b) acc[b] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

            if (LR == 1 && wave < R) {
                // U rows of row block `wave` as MFMA A fragments, copied into LDS now so that the
                // epilogue finds them there: k-step i, lane (j16, q) = U[n][32i + 8q ..].
                const BufRsrc ub = make_rsrc(a.w.U, (uint64_t)a.N * (uint64_t)r * 2u);
                const uint32_t nrow = (rb0 + wave) * 16u + j16;
#pragma unroll
                for (int i = 0; i < kDecKS; ++i) {
                    const uint32_t k0 = 32u * i + 8u * q;
                    const uint32_t off = (rb0 + wave < NB && k0 < (uint32_t)r) ? (nrow * r + k0) * 2u : kOobOffset;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        ub, (LdsPtr)(smem + kDecULds + (wave * kDecKS + i) * 1024), 16, off, 0, 0, 0);
                }
                asm volatile("" ::: "memory");
            }

            for (uint32_t p = 0; p < npieces; ++p) {
                // This wave's two chunks of the piece, everything requested up front: for each chunk
                // its activations, which go straight from L2 into the wave's LDS slot, then the
                // weights (one unit per lane and row block: the 64 lanes of the wave read 64
                // consecutive units, lane quad q being group 4c + q).  The chunk order is rotated
                // per workgroup so that the workgroups, which all read the same X, do not walk the
                // same L2 channels in step.  A lane or block without data gets a unit index past
                // the end.
                RawUnit u[CPW][R];
                uint32_t workers_done = 0;
#pragma unroll
                for (int ci = 0; ci < CPW; ++ci) {
                    const uint32_t cw = (wave + kDecWaves * ci + rot) & (kDecPiece - 1);
                    const uint32_t chunk = p * kDecPiece + cw;
                    const uint32_t kc = chunk * 256u;
                    unsigned char* const slot = myslot + kDecWaves * ci * kDecSlotBytes;
                    // A chunk that reaches beyond K (the last one when K is not a multiple of 256, or
                    // one past the end) must not wrap into the next row: only the first `lim` bytes
                    // of its 512-byte row pieces exist.  lim is a multiple of 128, so whether a
                    // lane's segment exists depends on its 128-byte quarter only, which the xor
                    // with 2i changes for i >= 4.
                    const uint32_t lim = (kc >= K) ? 0u : (K - kc >= 256u ? 512u : 2u * (K - kc));
                    const bool ok_lo = (xseg & 0x180u) < lim;
                    const bool ok_hi = ((xseg & 0x180u) ^ 0x80u) < lim;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const uint32_t off = ((xseg ^ (32u * i)) + xrow) + (4u * i * K + 2u * kc);
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(xb, (LdsPtr)(slot + i * 1024), 16,
                                                                 (i < 4 ? ok_lo : ok_hi) ? off : kOobOffset, 0, 0, 0);
                    }
                    asm volatile("" ::: "memory");
                    // (an index >= 2^26 is past the end of every weight the host accepts, and the
                    // sum of the two parts stays below 2^28, so 16 * index does not wrap)
                    const uint32_t lane_u = (4u * chunk + (uint32_t)q < G) ? (uint32_t)lane : (1u << 26);
#pragma unroll
                    for (int b = 0; b < R; ++b) {
                        const uint32_t base = (rb0 + b < NB) ? ((rb0 + b) * G + 4u * chunk) * 16u : (1u << 27);
                        u[ci][b] = load_unit_buf_once(wb, base + lane_u);
                        asm volatile("" ::: "memory");      // the loads keep this order (the waits count them)
                    }
                }
                // Vector memory operations complete in order, so unit (ci, b) and the activations of
                // its chunk have arrived once at most the operations issued after that unit's two
                // loads are outstanding.  The slots are private to the wave, so no barrier is
                // involved, and the first unit is converted while most of the rest is still on its
                // way.  (The counts rely on the compiler adding no memory operation of its own in
                // between; the build script checks that.)
                f16x8 bfrag[8];
                static_for<0, CPW * R>([&](auto su_c) {
                    constexpr int su = decltype(su_c)::value;
                    constexpr int ci = su / R, b = su % R;
                    constexpr int kIssued = CPW * (8 + 2 * R);
                    __builtin_amdgcn_sched_barrier(0);      // nothing of this unit moves above its wait
                    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kIssued - (ci * (8 + 2 * R) + 8 + 2 * (b + 1))) : "memory");
                    __builtin_amdgcn_sched_barrier(0);
                    if (b == 0) {
                        const unsigned char* slot = myslot + kDecWaves * ci * kDecSlotBytes;
#pragma unroll
                        for (int t = 0; t < 8; ++t)
                            bfrag[t] = __builtin_bit_cast(
                                f16x8,
                                *reinterpret_cast<const u32x4*>(slot + j16 * 512 + (((8 * q + t) ^ j16) << 4)));
                    }
                    pin_unit_params(u[ci][b]);  // nothing is computed from this unit before the wait
                    dequant_unit_steps(u[ci][b], [&](int t, f16x8 frag) {
                        acc[b] = mfma16(frag, bfrag[t], acc[b]);
                    });
                    // The wave that will hand T to the others looks for it while it still has
                    // work (reads of data written during the launch cross the whole chip and
                    // take a microsecond each): of the S units it converts, it requests the
                    // count of finished workers after unit P1, looks at it two units later and,
                    // if all are done, starts the copy of T into LDS, which then runs under the
                    // remaining units; otherwise it asks once more.
                    constexpr int S = CPW * R, P1 = S / 2 - 2 >= 0 ? S / 2 - 2 : 0, E1 = P1 + 2, E2 = E1 + 2;
                    if (LR == 1 && wave == kDecTWave && p == npieces - 1 && !t_fetched) {
                        if (su == P1 && E1 < S)
                            workers_done = __hip_atomic_load(a.ctrl + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        if ((su == E1 && E1 < S) || (su == E2 && E2 < S)) {
                            if (__builtin_amdgcn_readfirstlane(workers_done) >= (uint32_t)a.nt) {
                                fetch_t();
                                t_fetched = true;
                                sign_off();
                            } else if (su == E1 && E2 < S) {
                                workers_done =
                                    __hip_atomic_load(a.ctrl + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            }
                        }
                    }
                });
            }

            // ------------------------------------------------------------ reduce + low rank + store
            // Each wave leaves its partial sums in its own first slot, which it has finished reading.
            f32x4* const red = reinterpret_cast<f32x4*>(smem);          // wave w, block b at 512 w + 64 b
            u32x4* const ulds = reinterpret_cast<u32x4*>(smem + kDecULds);
            u32x4* const tbuf = reinterpret_cast<u32x4*>(smem + kDecTLds);
#pragma unroll
            for (int b = 0; b < R; ++b) red[wave * (kDecSlotBytes / 16) + b * 64 + lane] = acc[b];
            if (LR > 0 && wave == kDecTWave) {
                // One wave gets T for the whole workgroup and hands it over through LDS (LR == 1);
                // if the early look above did not find the workers done, it waits for them here.
                if (!t_fetched) {
                    decode_wait_t(a);
                    if (LR == 1) {
                        fetch_t();
                        sign_off();
                    }
                    t_fetched = true;
                }
                wait_vmem();
            }
            __syncthreads();                                       // partial sums and T are in LDS
            if (wave < R) {
                // wave b finishes row block b: sum of the eight waves' partials in wave order
                const int b = wave;
                f32x4 part[kDecWaves];
#pragma unroll
                for (int pw = 0; pw < kDecWaves; ++pw) part[pw] = red[pw * (kDecSlotBytes / 16) + b * 64 + lane];
                f32x4 sum = part[0];
#pragma unroll
                for (int pw = 1; pw < kDecWaves; ++pw)
#pragma unroll
                    for (int e = 0; e < 4; ++e) sum[e] += part[pw][e];
                const uint32_t nb = (rb0 + b) * 16u;
                if (LR == 1) {
                    int i = 0;
#pragma unroll
                    for (int f = 0; f < kDecTFrags; ++f) {
                        if (f < nfrag) {
                            sum = mfma16(__builtin_bit_cast(f16x8, ulds[(b * kDecKS + i) * 64 + lane]),
                                         __builtin_bit_cast(f16x8, tbuf[f * 64 + lane]), sum);
                            if (++i == ksu) i = 0;
                        }
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
                            sum = mfma16(av, bv, sum);
                        }
                    }
                }
                // D[v]: feature nb + 4q + v, token j16
                const int64_t n = (int64_t)nb + 4 * q;
                if (j16 < M && n < a.N) {
                    f16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (f16)sum[e];
                    *reinterpret_cast<f16x4*>(a.Y + (int64_t)j16 * a.N + n) = o;
                }
            }
            if (blk + (gridDim.x - nworkers) < (NB + R - 1) / R * 1u) __syncthreads();   // slots are reused
        }
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
        const uint32_t nmain = gridDim.x - (uint32_t)nworkers;
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
                if (spins > (1u << 22)) {
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

// Workgroups the device keeps resident at once (one 512-thread, 128-KB-LDS workgroup per CU),
// cached per device; also raises the kernels' dynamic LDS limit once.
typedef void (*DecodeKernel)(const DecodeArgs);
template <int LR>
static DecodeKernel decode_variant_lr(int R) {
    if (R == 4) return w3lr_decode_kernel<4, LR>;
    if (R == 2) return w3lr_decode_kernel<2, LR>;
    return w3lr_decode_kernel<1, LR>;
}
static DecodeKernel decode_variant(int R, int lr) {
    if (lr == 0) return decode_variant_lr<0>(R);
    if (lr == 1) return decode_variant_lr<1>(R);
    return decode_variant_lr<2>(R);
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
                if (hipFuncSetAttribute(reinterpret_cast<const void*>(decode_variant(R, lr)),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kDecLdsTotal) != hipSuccess)
                    return 0;
        cached[dev] = cus;
    }
    return cached[dev];
}

// K parts of the T workers: kDecWaves chunks of 256 columns each.
static int decode_k_parts(int64_t K) { return (int)((K + 256 * kDecWaves - 1) / (256 * kDecWaves)); }

size_t decode_workspace_bytes(int r, int64_t K) {
    if (r <= 0) return 256;
    const size_t rblocks = ((size_t)r + 15) / 16;
    // control words | sign-off words of the streaming workgroups | T fp16 [K parts][16 x ldt]
    return 256 + kDecDoneBytes + align_up((size_t)decode_k_parts(K) * 16 * rblocks * 16 * 2, 256);
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
    // T workers: one per block of 16 ranks and K part, at most kDecMaxWorkers and never more than
    // a quarter of the resident workgroups (a worker then takes several items in turn)
    int nt = a.rblocks * a.kh;
    if (nt > kDecMaxWorkers) nt = kDecMaxWorkers;
    if (nt > cap / 4) nt = cap / 4 > 0 ? cap / 4 : 1;
    a.nt = nt;
    const int workers = r > 0 ? nt : 0;
    if (cap <= workers || (size_t)cap * 4 > kDecDoneBytes) return MILO_ERR_HIP;
    // Rows per workgroup (16*R): as many as still leave about one workgroup per CU, because every
    // workgroup stages all of X once.
    int R = 4;
    const int64_t want = (int64_t)(cap - workers) * 3 / 4;
    while (R > 1 && (a.N + 16 * R - 1) / (16 * R) < want) R >>= 1;
    if (const char* e = getenv("MILO_DEC_R")) {                 // tuning override
        const int v = atoi(e);
        if (v == 1 || v == 2 || v == 4) R = v;
    }
    const int rows = 16 * R;
    const int64_t blocks = (a.N + rows - 1) / rows;
    const int grid = (int)(blocks < cap - workers ? blocks : cap - workers) + workers;
    const bool lds_path = (r & 7) == 0 && r <= 32 * kDecKS && a.kh * ((r + 31) / 32) <= kDecTFrags &&
                          (uint64_t)a.N * (uint64_t)r * 2u < 0xFFFFFFF0ull;
    const int lr = r == 0 ? 0 : lds_path ? 1 : 2;
    decode_variant(R, lr)<<<dim3((unsigned)grid), dim3(kDecThreads), lr == 1 ? kDecLdsTotal : kDecLdsBytes, stream>>>(a);
    return launch_status();
}

}  // namespace milo
