// Weight-streaming kernel for the compensated W3A16 linear at M <= 16 (decode): ONE launch that
// streams the packed weight once from HBM, forms T = X V^T cooperatively and adds T U^T.
//
// Weight stream.  A workgroup of eight waves owns 16*R output features over the whole K.  K is
// walked in pieces of 16 chunks of 256; wave w takes chunks w and w+8 of the piece for all R
// 16-row blocks, so for K = 4096 every load of the launch is issued in the first few hundred
// cycles.  For a chunk a
// lane loads one unit per 16-row block (24 bytes of codes, one scale, one zero-point) with fully
// coalesced 16- and 8-byte buffer loads and no branches (lanes without data read out of range
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
// Low-rank term.  The first `nt` workgroups do no streaming: each computes one K-slice of
// T = X V^T (fp32 partial in the workspace); whichever of them finishes last adds the partials in
// slice order (so the result does not depend on which one that was), writes T as fp16 and
// raises a flag.  The streaming workgroups only need T in their epilogue, where they add T U^T
// with a few more MFMAs.  The workers never wait for anything, they have the lowest workgroup
// ids, and the grid never exceeds what the device keeps resident, so the epilogue's wait always
// ends.  Data that crosses workgroups is written and read with device-coherent accesses, and
// the last workgroup to leave restores the control words to zero for the next launch.
#include <stdlib.h>

#include "milo_host.h"
#include "milo_kernels.h"

namespace milo {

constexpr int kDecWaves = 8;
constexpr int kDecThreads = 64 * kDecWaves;
constexpr int kDecPiece = 16;                               // chunks of 256 k staged at a time
constexpr int kDecSlotBytes = 16 * 512;                     // one chunk of X: 16 rows x 256 k
constexpr int kDecLdsBytes = kDecPiece * kDecSlotBytes;     // 128 KB
constexpr int kDecRankPass = 128;       // ranks a T worker handles per pass (8 MFMA blocks)

__device__ __forceinline__ void buf_store16_coherent(BufRsrc r, uint32_t off, u32x4 v) {
    __builtin_amdgcn_raw_buffer_store_b128(v, r, off, 0, 17);
}
__device__ __forceinline__ void buf_store8_coherent(BufRsrc r, uint32_t off, u32x2 v) {
    __builtin_amdgcn_raw_buffer_store_b64(v, r, off, 0, 17);
}
typedef __attribute__((address_space(3))) void* LdsPtr;


// One K-slice of T = X V^T, then (last arriver only) the sum over slices.
__device__ __forceinline__ void decode_t_worker(const DecodeArgs& a, unsigned char* smem) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int j16 = lane & 15, q = lane >> 4;
    const int M = a.M, r = a.w.r;
    const int64_t K = a.K;
    const BufRsrc xb = make_rsrc(a.X, (uint64_t)M * (uint64_t)K * 2u);
    const BufRsrc vb = make_rsrc(a.w.V, (uint64_t)r * (uint64_t)K * 2u);
    const BufRsrc pb = make_rsrc(a.t_partial, (uint64_t)a.nt * a.rblocks * 64 * 16);
    const BufRsrc tb = make_rsrc(a.T, (uint64_t)16 * a.ldt * 2u);
    const int64_t k_lo = (int64_t)blockIdx.x * a.slice;
    const int64_t k_hi = (k_lo + a.slice < K) ? k_lo + a.slice : K;
    f32x4* red = reinterpret_cast<f32x4*>(smem);            // [wave][8 blocks][64 lanes] = 128 KB

    for (int jp = 0; jp < r; jp += kDecRankPass) {
        f32x4 tacc[8];
#pragma unroll
        for (int jb = 0; jb < 8; ++jb) tacc[jb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        const int nblk = (r - jp + 15) / 16 < 8 ? (r - jp + 15) / 16 : 8;
        // wave w takes the 32-wide k-steps w, w+16, ... of the slice
        for (int64_t k0 = k_lo + 32 * wave; k0 < k_hi; k0 += 32 * kDecWaves) {
            const int64_t k = k0 + 8 * q;
            const f16x8 xv = __builtin_bit_cast(
                f16x8, buf_load16(xb, j16 < M ? (uint32_t)(((int64_t)j16 * K + k) * 2) : kOobOffset));
            f16x8 vv[8];
#pragma unroll
            for (int jb = 0; jb < 8; ++jb) {
                // rows >= r lie past the end of V and read as zero
                const int64_t row = jp + 16 * jb + j16;
                vv[jb] = __builtin_bit_cast(
                    f16x8, buf_load16(vb, jb < nblk ? (uint32_t)((row * K + k) * 2) : kOobOffset));
            }
#pragma unroll
            for (int jb = 0; jb < 8; ++jb)
                if (jb < nblk) tacc[jb] = mfma16(vv[jb], xv, tacc[jb]);
        }
        __syncthreads();
#pragma unroll
        for (int jb = 0; jb < 8; ++jb)
            if (jb < nblk) red[(wave * 8 + jb) * 64 + lane] = tacc[jb];
        __syncthreads();
        // partial[slice][rank block][lane] keeps the MFMA D layout:
        // element v of lane l = rank 16*jb + 4*(l/16) + v, token l%16.
        const uint32_t pbase = (uint32_t)(((int64_t)blockIdx.x * a.rblocks + jp / 16) * 64 * 16);
        for (int e = tid; e < nblk * 64; e += kDecThreads) {
            f32x4 sum = red[e];
#pragma unroll
            for (int p = 1; p < kDecWaves; ++p) {
                const f32x4 v = red[p * 8 * 64 + e];
#pragma unroll
                for (int x = 0; x < 4; ++x) sum[x] += v[x];
            }
            buf_store16_coherent(pb, pbase + (uint32_t)e * 16u, __builtin_bit_cast(u32x4, sum));
        }
    }
    // all partial stores of this workgroup are complete before it is counted
    wait_vmem();
    __syncthreads();
    int last = 0;
    if (tid == 0) last = (atomicAdd(a.ctrl + 0, 1u) == (uint32_t)a.nt - 1u) ? 1 : 0;
    if (!__syncthreads_or(last)) return;

    // Last slice to arrive: add the partials in slice order and write T as fp16 [16 x ldt].
    // All loads of a batch of entries are issued together, then summed through LDS.
    const int entries = a.rblocks * 64;
    const int per_batch = (kDecLdsBytes / 16) / a.nt;        // entries whose nt partials fit in LDS
    for (int e0 = 0; e0 < entries; e0 += per_batch) {
        const int ne = (entries - e0) < per_batch ? (entries - e0) : per_batch;
        __syncthreads();
        for (int i = tid; i < ne * a.nt; i += kDecThreads) {
            const int s = i / ne, e = i - s * ne;
            red[i] = __builtin_bit_cast(
                f32x4, buf_load16_coherent(pb, (uint32_t)((((int64_t)s * a.rblocks) * 64 + e0 + e) * 16)));
        }
        __syncthreads();
        for (int e = tid; e < ne; e += kDecThreads) {
            f32x4 sum = red[e];
            for (int s = 1; s < a.nt; ++s) {
                const f32x4 v = red[s * ne + e];
#pragma unroll
                for (int x = 0; x < 4; ++x) sum[x] += v[x];
            }
            const int jb = (e0 + e) >> 6, l = (e0 + e) & 63;
            f16x4 o;
#pragma unroll
            for (int x = 0; x < 4; ++x) o[x] = (f16)sum[x];
            buf_store8_coherent(tb, (uint32_t)(((l & 15) * a.ldt + 16 * jb + 4 * (l >> 4)) * 2),
                                __builtin_bit_cast(u32x2, o));
        }
    }
    wait_vmem();
    __syncthreads();
    if (tid == 0) __hip_atomic_store(a.ctrl + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int R>
__global__ __launch_bounds__(kDecThreads) void w3lr_decode_kernel(const DecodeArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int j16 = lane & 15, q = lane >> 4;
    const int M = a.M;
    const int64_t N = a.N, K = a.K;
    const int G = (int)(K / kGroup);
    const int nchunks = (G + 3) / 4;
    const int npieces = (nchunks + kDecPiece - 1) / kDecPiece;
    const int r = a.w.r;
    const int nworkers = r > 0 ? a.nt : 0;
    constexpr int ROWS = 16 * R;                // output features per workgroup
    constexpr int CPW = kDecPiece / kDecWaves;  // chunks of a piece per wave

    if ((int)blockIdx.x < nworkers) {
        decode_t_worker(a, smem);
    } else {
        const W3Buf wb = make_w3buf(a.w.q3, a.w.scales, a.w.zeros, N, K);
        const BufRsrc xb = make_rsrc(a.X, (uint64_t)M * (uint64_t)K * 2u);
        // Staging: copy i of a chunk moves rows 2i, 2i+1: lane l -> row 2i + l/32, slot position
        // p = l%32, which receives segment p ^ row of the row's 32 segments of 8 columns.
        const int crow = lane >> 5, cp = lane & 31;
        const int rot = (int)(blockIdx.x * 5u) & (kDecPiece - 1);
        bool t_seen = false;        // this workgroup has already waited for T

        for (int64_t blk = (int64_t)blockIdx.x - nworkers; blk * ROWS < N;
             blk += (int64_t)gridDim.x - nworkers) {
            const int64_t n0 = blk * ROWS;
            uint32_t ubase[R];
#pragma unroll
            for (int b = 0; b < R; ++b) {
                const int64_t n = n0 + 16 * b + j16;
                ubase[b] = (n < N) ? (uint32_t)unit_index(n, 0, G) : kOobUnit;
            }
            f32x4 acc[R];
#pragma unroll
            for (int b = 0; b < R; ++b) acc[b] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

            for (int p = 0; p < npieces; ++p) {
                // This wave's two chunks of the piece.  For each: its activations go straight from L2
                // into the wave's LDS slot (buffer-to-LDS copies, no registers), then its weights
                // are loaded; lane quad q takes group 4c + q of chunk c.  The chunk order is rotated
                // per workgroup so that the workgroups, which all read the same X, do not walk the
                // same L2 channels in step.
                RawUnit u[CPW][R];
#pragma unroll
                for (int ci = 0; ci < CPW; ++ci) {
                    const int cw = (wave + kDecWaves * ci + rot) & (kDecPiece - 1);   // chunk within the piece
                    const int64_t kc = ((int64_t)p * kDecPiece + cw) * 256;
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int row = 2 * i + crow;
                        const int seg = cp ^ row;
                        const bool in = row < M && kc + seg * 8 < K;
                        const uint32_t off = in ? (uint32_t)(((int64_t)row * K + kc + seg * 8) * 2) : kOobOffset;
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(
                            xb, (LdsPtr)(smem + (wave + kDecWaves * ci) * kDecSlotBytes + i * 1024), 16, off, 0, 0,
                            0);
                    }
                    asm volatile("" ::: "memory");
                    const int g = 4 * (p * kDecPiece + cw) + q;
#pragma unroll
                    for (int b = 0; b < R; ++b)
                        u[ci][b] = load_unit_buf(wb, (g < G && ubase[b] != kOobUnit) ? ubase[b] + (uint32_t)g * 16u
                                                                                      : kOobUnit);
                    asm volatile("" ::: "memory");
                }
#pragma unroll
                for (int ci = 0; ci < CPW; ++ci) {
                    // Vector memory operations complete in order: once at most the operations issued
                    // after this chunk's copies are outstanding (its R*4 weight loads and everything
                    // of the later chunks), the copies have landed in LDS.  The slot is private to
                    // the wave, so no barrier is involved.  (The count relies on the compiler adding
                    // no memory operation of its own in between; the build script checks that.)
                    if (ci == 0)
                        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(R * 4 + (CPW - 1) * (8 + R * 4)) : "memory");
                    else
                        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(R * 4) : "memory");
                    const unsigned char* slot = smem + (wave + kDecWaves * ci) * kDecSlotBytes;
                    f16x8 bfrag[8];
#pragma unroll
                    for (int t = 0; t < 8; ++t)
                        bfrag[t] = __builtin_bit_cast(
                            f16x8,
                            *reinterpret_cast<const u32x4*>(slot + j16 * 512 + (((8 * q + t) ^ j16) << 4)));
#pragma unroll
                    for (int b = 0; b < R; ++b)
                        dequant_unit_steps(u[ci][b], [&](int t, f16x8 frag) {
                            acc[b] = mfma16(frag, bfrag[t], acc[b]);
                        });
                }
            }

            // ------------------------------------------------------------ reduce + low rank + store
            __syncthreads();                                       // everyone is done with the slots
            f32x4* red = reinterpret_cast<f32x4*>(smem);          // [wave][block][lane], <= 32 KB
            u32x4* tbuf = reinterpret_cast<u32x4*>(smem + 64 * 1024);   // T fragments [k-step][lane]
            constexpr int KS = 4;                   // k-steps of 32 kept as fragments (r <= 128)
            const bool fast = r > 0 && (r & 7) == 0 && r <= 32 * KS;
#pragma unroll
            for (int b = 0; b < R; ++b) red[(wave * R + b) * 64 + lane] = acc[b];
            __syncthreads();
            f32x4 sum = {0.0f, 0.0f, 0.0f, 0.0f};
            f16x8 uf[KS];
            if (wave == kDecWaves - 1 && r > 0) {
                // One wave fetches T for the whole workgroup: T is written by the worker workgroups
                // during this launch, so it is read with device-coherent loads, after its flag has
                // been seen up, and handed to the others through LDS.
                if (!t_seen) {
                    for (uint32_t spins = 0;
                         __hip_atomic_load(a.ctrl + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u; ++spins) {
                        __builtin_amdgcn_s_sleep(1);
                        if (spins > (1u << 24)) { atomicOr(a.ctrl + 3, 1u); break; }
                    }
                }
                if (fast) {
                    const BufRsrc tb = make_rsrc(a.T, (uint64_t)16 * a.ldt * 2u);
#pragma unroll
                    for (int i = 0; i < KS; ++i) {
                        const int k0 = 32 * i + 8 * q;
                        tbuf[i * 64 + lane] =
                            buf_load16_coherent(tb, (k0 < a.ldt) ? (uint32_t)((j16 * a.ldt + k0) * 2) : kOobOffset);
                    }
                }
            }
            t_seen = true;
            if (wave < R) {
                // wave b finishes row block b: sum of the eight waves' partials in wave order, with
                // the U rows of the block requested first so that their latency overlaps the sum
                const int b = wave;
                const int64_t nrow = n0 + 16 * b + j16;
                if (fast) {
                    const BufRsrc ub = make_rsrc(a.w.U, (uint64_t)N * (uint64_t)r * 2u);
#pragma unroll
                    for (int i = 0; i < KS; ++i) {
                        const int k0 = 32 * i + 8 * q;
                        uf[i] = __builtin_bit_cast(
                            f16x8, buf_load16(ub, (nrow < N && k0 < r) ? (uint32_t)((nrow * r + k0) * 2) : kOobOffset));
                    }
                }
                f32x4 part[kDecWaves];
#pragma unroll
                for (int pw = 0; pw < kDecWaves; ++pw) part[pw] = red[(pw * R + b) * 64 + lane];
                sum = part[0];
#pragma unroll
                for (int pw = 1; pw < kDecWaves; ++pw)
#pragma unroll
                    for (int e = 0; e < 4; ++e) sum[e] += part[pw][e];
            }
            __syncthreads();                                       // T fragments are in LDS
            if (wave < R) {
                const int b = wave;
                const int64_t nb = n0 + 16 * b;
                const int64_t nrow = nb + j16;
                if (fast) {
#pragma unroll
                    for (int i = 0; i < KS; ++i)
                        if (32 * i < r) sum = mfma16(uf[i], __builtin_bit_cast(f16x8, tbuf[i * 64 + lane]), sum);
                } else if (r > 0) {
                    const BufRsrc tb = make_rsrc(a.T, (uint64_t)16 * a.ldt * 2u);
                    for (int ks = 0; ks < r; ks += 32) {
                        const int k0 = ks + 8 * q;
                        f16x8 av = zero_f16x8();
                        if (nrow < N) av = load_row8(a.w.U + nrow * r, k0, r, (r & 7) == 0);
                        const f16x8 bv = __builtin_bit_cast(
                            f16x8,
                            buf_load16_coherent(tb, k0 < a.ldt ? (uint32_t)((j16 * a.ldt + k0) * 2) : kOobOffset));
                        sum = mfma16(av, bv, sum);
                    }
                }
                // D[v]: feature nb + 4q + v, token j16
                const int64_t n = nb + 4 * q;
                if (j16 < M && n < N) {
                    f16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (f16)sum[e];
                    *reinterpret_cast<f16x4*>(a.Y + (int64_t)j16 * N + n) = o;
                }
            }
            __syncthreads();        // smem is reused by the next block of this workgroup
        }
    }

    // Leave: the last workgroup restores the control words for the next launch.  Every streaming
    // workgroup has read T before it gets here, and every worker has written its share.
    if (r > 0) {
        __syncthreads();
        if (tid == 0) {
            const uint32_t old = atomicAdd(a.ctrl + 2, 1u);
            if (old == gridDim.x - 1u) {
                __hip_atomic_store(a.ctrl + 0, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(a.ctrl + 1, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(a.ctrl + 2, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// Workgroups the device keeps resident at once (one 512-thread, 128-KB-LDS workgroup per CU),
// cached per device; also raises the kernels' dynamic LDS limit once.
typedef void (*DecodeKernel)(const DecodeArgs);
static DecodeKernel decode_variant(int R) {
    if (R == 4) return w3lr_decode_kernel<4>;
    if (R == 2) return w3lr_decode_kernel<2>;
    return w3lr_decode_kernel<1>;
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
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(decode_variant(R)),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kDecLdsBytes) != hipSuccess)
                return 0;
        cached[dev] = cus;
    }
    return cached[dev];
}

size_t decode_workspace_bytes(int r) {
    if (r <= 0) return 256;
    const size_t rblocks = ((size_t)r + 15) / 16;
    // control words | T fp16 [16 x ldt] | partials [kDecMaxSlices][rblocks][64] f32x4
    return 256 + align_up(16 * rblocks * 16 * 2, 256) + (size_t)kDecMaxSlices * rblocks * 64 * 16;
}

int launch_decode(DecodeArgs a, void* workspace, hipStream_t stream) {
    const int cap = decode_capacity();
    if (cap <= 0) return MILO_ERR_HIP;
    const int r = a.w.r;
    a.rblocks = (r + 15) / 16;
    a.ldt = (int64_t)a.rblocks * 16;
    char* ws = reinterpret_cast<char*>(workspace);
    a.ctrl = reinterpret_cast<uint32_t*>(ws);
    a.T = reinterpret_cast<f16*>(ws + 256);
    a.t_partial = reinterpret_cast<f32x4*>(ws + 256 + align_up((size_t)16 * a.rblocks * 16 * 2, 256));
    // K-slices of T: about 512 columns each (one 32-wide step per wave of a worker), at most
    // kDecMaxSlices and never more than a quarter of the resident workgroups
    int nt = (int)((a.K + 511) / 512);
    if (nt > kDecMaxSlices) nt = kDecMaxSlices;
    if (nt > cap / 4) nt = cap / 4 > 0 ? cap / 4 : 1;
    int64_t slice = (a.K + nt - 1) / nt;
    slice = (slice + 63) / 64 * 64;
    nt = (int)((a.K + slice - 1) / slice);
    a.nt = nt;
    a.slice = (int)slice;
    const int workers = r > 0 ? nt : 0;
    if (cap <= workers) return MILO_ERR_HIP;
    // Rows per workgroup (16*R): as many as still leave about one workgroup per CU, because every
    // workgroup stages all of X once.
    int R = 4;
    const int64_t want = (int64_t)(cap - workers) * 3 / 4;
    while (R > 1 && (a.N + 16 * R - 1) / (16 * R) < want) R >>= 1;
    if (const char* e = getenv("MILO_DEC_R")) R = atoi(e);      // tuning override
    const int rows = 16 * R;
    const int64_t blocks = (a.N + rows - 1) / rows;
    const int grid = (int)(blocks < cap - workers ? blocks : cap - workers) + workers;
    decode_variant(R)<<<dim3((unsigned)grid), dim3(kDecThreads), kDecLdsBytes, stream>>>(a);
    return launch_status();
}

}  // namespace milo
