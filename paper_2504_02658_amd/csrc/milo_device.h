// Device-side building blocks shared by the gfx950 kernels: vector types, the MFMA
// wrappers, the packed-unit addressing and the in-register 3-bit -> fp16 conversion.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/milo.h"

namespace milo {

typedef _Float16 f16;
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kGroup = 64;          // weights per quantization group (one unit)
constexpr int kWave = 64;

// ---------------------------------------------------------------------------------------------
// Packed weight view.  Unit u = ((n/16) * G + g) * 16 + n%16 with G = K/64 groups per row;
// plane A holds 16 bytes per unit (code words 0..3), plane B (right behind it) 12 bytes per unit:
// code words 4, 5 and one word with the fp16 scale (low half) and zero-point (high half).
struct W3View {
    const u32x4* planeA;
    const uint32_t* planeB;         // three words per unit
    int G;                          // groups per row
};

__host__ __device__ inline W3View make_view(const void* q3, int64_t N, int64_t K) {
    W3View v;
    v.planeA = reinterpret_cast<const u32x4*>(q3);
    v.planeB = reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(q3) + (N * K) / 4);
    v.G = static_cast<int>(K / kGroup);
    return v;
}

__host__ __device__ inline int64_t unit_index(int64_t n, int64_t g, int64_t G) {
    return ((n >> 4) * G + g) * 16 + (n & 15);
}

// Raw data of one unit as a lane holds it in registers.
struct RawUnit {
    u32x4 a;        // words 0..3
    u32x2 b;        // words 4, 5
    uint32_t sz;    // fp16 scale (low half) and zero-point (high half)
};
__device__ __forceinline__ f16 f16_bits(uint32_t v) { return __builtin_bit_cast(f16, (unsigned short)v); }

__device__ __forceinline__ RawUnit zero_unit() {
    RawUnit r;
    r.a = u32x4{0u, 0u, 0u, 0u};
    r.b = u32x2{0u, 0u};
    r.sz = 0u;
    return r;
}

__device__ __forceinline__ RawUnit load_unit(const W3View& w, int64_t u) {
    RawUnit r;
    r.a = w.planeA[u];
    r.b = u32x2{w.planeB[3 * u], w.planeB[3 * u + 1]};
    r.sz = w.planeB[3 * u + 2];
    return r;
}

// ---------------------------------------------------------------------------------------------
// Raw buffer access.  A buffer descriptor carries the byte size of the array, and a load whose
// offset falls outside returns zero without any branch: kernels mark a lane as "no data" by
// giving it an out-of-range offset instead of diverging.  Offsets are 32-bit, so every array
// addressed this way must be smaller than 4 GiB (checked on the host).
typedef __amdgpu_buffer_rsrc_t BufRsrc;
constexpr uint32_t kOobOffset = 0xFFFFFFF0u;

__device__ __forceinline__ BufRsrc make_rsrc(const void* p, uint64_t bytes) {
    const uint32_t n = bytes > 0xFFFFFFF0ull ? 0xFFFFFFF0u : (uint32_t)bytes;
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, n, 0x00020000);
}
__device__ __forceinline__ u32x4 buf_load16(BufRsrc r, uint32_t off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
}
// Device-coherent variant (sc0 sc1): for data another workgroup wrote during this launch.
__device__ __forceinline__ u32x4 buf_load16_coherent(BufRsrc r, uint32_t off) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 17);
}
__device__ __forceinline__ u32x2 buf_load8(BufRsrc r, uint32_t off) {
    return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
}
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
__device__ __forceinline__ u32x3 buf_load12(BufRsrc r, uint32_t off) {
    return __builtin_amdgcn_raw_buffer_load_b96(r, off, 0, 0);
}

// All vector memory operations issued so far by this wave (loads, stores and buffer-to-LDS copies)
// have completed; nothing may be moved across.
__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// A hand-counted wait: at most N of this wave's vector memory operations are still outstanding
// (they complete in order).  Built with MILO_FULL_WAITS every such wait is for everything, which
// assumes nothing about what else is in flight: the build script makes a second library that way,
// and a GPU test compares the two bit for bit.
#ifdef MILO_FULL_WAITS
#define MILO_WAIT_VMEM(N) asm volatile("s_waitcnt vmcnt(0)" ::: "memory")
#else
#define MILO_WAIT_VMEM(N) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory")
#endif

// The two planes of a packed weight as buffers.
struct W3Buf {
    BufRsrc a, b;
};
__device__ __forceinline__ W3Buf make_w3buf(const void* q3, int64_t N, int64_t K) {
    const uint64_t units = (uint64_t)N * (uint64_t)(K / kGroup);
    W3Buf w;
    w.a = make_rsrc(q3, units * 16);
    w.b = make_rsrc(reinterpret_cast<const char*>(q3) + units * 16, units * 12);
    return w;
}
// Unit u with two loads (16 and 12 bytes), or an all-zero unit (which dequantizes to zeros) when
// u lies past the end of the weight, e.g. kOobUnit.
constexpr uint32_t kOobUnit = 0x0FFFFFFFu;
__device__ __forceinline__ RawUnit load_unit_buf(const W3Buf& w, uint32_t u) {
    RawUnit r;
    r.a = buf_load16(w.a, u * 16u);
    const u32x3 t = buf_load12(w.b, u * 12u);
    r.b = u32x2{t.x, t.y};
    r.sz = t.z;
    return r;
}
// The same with the non-temporal hint, for weights a kernel reads exactly once: measurably faster
// for the decode kernel, whose whole traffic is such reads.
__device__ __forceinline__ RawUnit load_unit_buf_once(const W3Buf& w, uint32_t u) {
    RawUnit r;
    r.a = __builtin_amdgcn_raw_buffer_load_b128(w.a, u * 16u, 0, 2);
    const u32x3 t = __builtin_amdgcn_raw_buffer_load_b96(w.b, u * 12u, 0, 2);
    r.b = u32x2{t.x, t.y};
    r.sz = t.z;
    return r;
}

// Pins a loaded unit at this point of the program: nothing computed from it can be scheduled
// earlier.  Without it the compiler converts the scale and zero-point of the NEXT chunk right
// after issuing their loads and puts the wait for them in the middle of the current chunk.
__device__ __forceinline__ void pin_unit(RawUnit& u) {
    asm volatile("" : "+v"(u.a.x), "+v"(u.a.y), "+v"(u.a.z), "+v"(u.a.w), "+v"(u.b.x), "+v"(u.b.y), "+v"(u.sz));
}
// The same for the scale and the zero-point alone (the values whose conversion the compiler likes
// to start early); the code words stay untouched, which keeps them in the registers they were
// loaded into.
__device__ __forceinline__ void pin_unit_params(RawUnit& u) {
    asm volatile("" : "+v"(u.sz));
}

// ---------------------------------------------------------------------------------------------
// (a & mask) | orv in one VALU op (v_and_or_b32).  On gfx9-family encodings a VOP3 instruction
// cannot carry a 32-bit literal, so with literal operands the compiler emits and + or; hiding
// the constants behind an empty asm puts them in registers once and lets the and-or pattern
// match, while the instruction itself stays visible to the scheduler.
__device__ __forceinline__ uint32_t in_sgpr(uint32_t v) {
    asm("" : "+s"(v));
    return v;
}
__device__ __forceinline__ uint32_t in_vgpr(uint32_t v) {
    asm("" : "+v"(v));
    return v;
}
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t orv) {
    return (a & mask) | orv;
}

// 3-bit -> fp16 conversion of one unit (Section 3.3 of the paper, "MiLo Dequant", reworked for
// this layout and for packed fp16 arithmetic).  A 3-bit field e sitting at mantissa bit b of an
// fp16 whose exponent says 2^(10-b) reads as 2^(10-b) + e, so OR-ing the right exponent pattern
// over the masked field converts the integer without any int->float instruction, two codes per
// 32-bit register: fields at b = 0, 3, 6 need no shift (patterns 0x6400 = 1024, 0x5800 = 128,
// 0x4C00 = 16).  With zr = the zero-point rounded to an integer (clamped to -8..15), the value
//      w = s * ((h - (2^(10-b) + zr)) + (zr - z))  =  s * (e - z)
// is formed by one packed subtraction, which is exact (small integers), and one packed fma with
// the per-unit constants s and c = (zr - z) * s; for integer zero-points c is 0 and the only
// rounding is the final one, for real-valued ones c adds an error below 2^-12 s.
// Output: w[P] = packed fp16 (W_dq[2P], W_dq[2P+1]) for the unit's 32 code pairs.
__device__ __forceinline__ uint32_t pack2(f16 v) {
    f16x2 p = {v, v};
    return __builtin_bit_cast(uint32_t, p);
}
__device__ __forceinline__ f16x8 unit_frag(const uint32_t (&w)[32], int t);

// The conversion is written in groups of five independent operations of one kind (five field
// extractions, five subtractions, five fmas) pinned with scheduling barriers: a dependent packed
// op can only issue about three slots after its producer, and left alone the compiler serialises
// extract -> subtract -> fma per pair through one temporary, which halves the VALU rate.
// `on_step(t, frag)` is called as soon as the eight codes 8t .. 8t+7 (the A operand of MFMA step
// t, t = 0..7 in order) are ready, so the caller's MFMAs interleave with the rest of the unit.
struct UnitConsts {
    uint32_t A0, A3, A6, S2, C2;
};
// SYM: the unit comes from the symmetric quantizer (Section 3.2.3, Eq. symm_int3; the "symmetric"
// kernel of Section 3.3): its zero-point is 4 by construction, so the biased zero-points are
// compile-time constants and the correction term is zero; only the scale is read from the unit.
template <bool SYM = false>
__device__ __forceinline__ UnitConsts unit_consts(const RawUnit& ru) {
    UnitConsts c;
    c.S2 = pack2(f16_bits(ru.sz));
    if (SYM) {
        c.A0 = 0x64046404u;     // 1024 + 4
        c.A3 = 0x58205820u;     // 128 + 4
        c.A6 = 0x4D004D00u;     // 16 + 4
        c.C2 = 0u;
        return c;
    }
    const float s = (float)f16_bits(ru.sz);
    const float z = (float)f16_bits(ru.sz >> 16);
    const float zr = __builtin_fminf(__builtin_fmaxf(__builtin_rintf(z), -8.0f), 15.0f);
    c.A0 = pack2((f16)(1024.0f + zr));
    c.A3 = pack2((f16)(128.0f + zr));
    c.A6 = pack2((f16)(16.0f + zr));
    c.C2 = pack2((f16)((zr - z) * s));
    return c;
}
__device__ __forceinline__ uint32_t pk_sub(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(f16x2, a) - __builtin_bit_cast(f16x2, b));
}
__device__ __forceinline__ uint32_t pk_fma(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_bit_cast(
        uint32_t, __builtin_elementwise_fma(__builtin_bit_cast(f16x2, a), __builtin_bit_cast(f16x2, b),
                                            __builtin_bit_cast(f16x2, c)));
}

template <bool SYM = false, typename OnStep>
__device__ __forceinline__ void dequant_unit_steps(const RawUnit& ru, OnStep&& on_step) {
    const UnitConsts c = unit_consts<SYM>(ru);
    const uint32_t B0 = in_vgpr(0x64006400u), B3 = in_vgpr(0x58005800u), B6 = in_vgpr(0x4C004C00u);
    const uint32_t M0 = in_sgpr(0x00070007u), M3 = in_sgpr(0x00380038u), M6 = in_sgpr(0x01C001C0u);
    const uint32_t d[6] = {ru.a.x, ru.a.y, ru.a.z, ru.a.w, ru.b.x, ru.b.y};
    uint32_t w[32];
    int next = 0;
#pragma unroll
    for (int j = 0; j < 6; ++j) {
        const uint32_t sh = d[j] >> 9;
        uint32_t h[5];
        h[0] = and_or(d[j], M0, B0);
        h[1] = and_or(d[j], M3, B3);
        h[2] = and_or(d[j], M6, B6);
        h[3] = and_or(sh, M0, B0);
        h[4] = and_or(sh, M3, B3);
        __builtin_amdgcn_sched_barrier(0);
        h[0] = pk_sub(h[0], c.A0);
        h[1] = pk_sub(h[1], c.A3);
        h[2] = pk_sub(h[2], c.A6);
        h[3] = pk_sub(h[3], c.A0);
        h[4] = pk_sub(h[4], c.A3);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 5; ++i) w[5 * j + i] = pk_fma(h[i], c.S2, c.C2);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 7; ++t) {
            if (t == next && 4 * t + 3 <= 5 * j + 4) {
                on_step(t, unit_frag(w, t));
                ++next;
            }
        }
    }
    // Pairs 30 and 31 are spread over the spare bits 15 / 31 of three words each; shifting the
    // words by 9, 8 and 7 lines the three bits up at mantissa bits 6, 7, 8.
    const uint32_t S6 = in_sgpr(0x00400040u), S7 = in_sgpr(0x00800080u), S8 = in_sgpr(0x01000100u);
    uint32_t t0 = and_or(d[0] >> 9, S6, B6);
    uint32_t t1 = and_or(d[3] >> 9, S6, B6);
    const uint32_t x0 = d[1] >> 8, x1 = d[4] >> 8, y0 = d[2] >> 7, y1 = d[5] >> 7;
    __builtin_amdgcn_sched_barrier(0);
    t0 = and_or(x0, S7, t0);
    t1 = and_or(x1, S7, t1);
    __builtin_amdgcn_sched_barrier(0);
    t0 = and_or(y0, S8, t0);
    t1 = and_or(y1, S8, t1);
    __builtin_amdgcn_sched_barrier(0);
    t0 = pk_sub(t0, c.A6);
    t1 = pk_sub(t1, c.A6);
    __builtin_amdgcn_sched_barrier(0);
    w[30] = pk_fma(t0, c.S2, c.C2);
    w[31] = pk_fma(t1, c.S2, c.C2);
    __builtin_amdgcn_sched_barrier(0);
    on_step(7, unit_frag(w, 7));
}

// Two units converted in lock step (ten independent operations per group): the tiled kernel
// feeds two weight streams from one set of B fragments.  on_step(t, frag0, frag1), t = 0..7.
template <bool SYM = false, typename OnStep>
__device__ __forceinline__ void dequant_units2_steps(const RawUnit& r0, const RawUnit& r1, OnStep&& on_step) {
    const UnitConsts c0 = unit_consts<SYM>(r0), c1 = unit_consts<SYM>(r1);
    const uint32_t B0 = in_vgpr(0x64006400u), B3 = in_vgpr(0x58005800u), B6 = in_vgpr(0x4C004C00u);
    const uint32_t M0 = in_sgpr(0x00070007u), M3 = in_sgpr(0x00380038u), M6 = in_sgpr(0x01C001C0u);
    const uint32_t S6 = in_sgpr(0x00400040u), S7 = in_sgpr(0x00800080u), S8 = in_sgpr(0x01000100u);
    const uint32_t d0[6] = {r0.a.x, r0.a.y, r0.a.z, r0.a.w, r0.b.x, r0.b.y};
    const uint32_t d1[6] = {r1.a.x, r1.a.y, r1.a.z, r1.a.w, r1.b.x, r1.b.y};
    uint32_t w0[32], w1[32];
    int next = 0;
#pragma unroll
    for (int j = 0; j < 6; ++j) {
        const uint32_t s0 = d0[j] >> 9, s1 = d1[j] >> 9;
        uint32_t h0[5], h1[5];
        h0[0] = and_or(d0[j], M0, B0);
        h1[0] = and_or(d1[j], M0, B0);
        h0[1] = and_or(d0[j], M3, B3);
        h1[1] = and_or(d1[j], M3, B3);
        h0[2] = and_or(d0[j], M6, B6);
        h1[2] = and_or(d1[j], M6, B6);
        h0[3] = and_or(s0, M0, B0);
        h1[3] = and_or(s1, M0, B0);
        h0[4] = and_or(s0, M3, B3);
        h1[4] = and_or(s1, M3, B3);
        h0[0] = pk_sub(h0[0], c0.A0);
        h1[0] = pk_sub(h1[0], c1.A0);
        h0[1] = pk_sub(h0[1], c0.A3);
        h1[1] = pk_sub(h1[1], c1.A3);
        h0[2] = pk_sub(h0[2], c0.A6);
        h1[2] = pk_sub(h1[2], c1.A6);
        h0[3] = pk_sub(h0[3], c0.A0);
        h1[3] = pk_sub(h1[3], c1.A0);
        h0[4] = pk_sub(h0[4], c0.A3);
        h1[4] = pk_sub(h1[4], c1.A3);
#pragma unroll
        for (int i = 0; i < 5; ++i) {
            w0[5 * j + i] = pk_fma(h0[i], c0.S2, c0.C2);
            w1[5 * j + i] = pk_fma(h1[i], c1.S2, c1.C2);
        }
#pragma unroll
        for (int t = 0; t < 7; ++t) {
            if (t == next && 4 * t + 3 <= 5 * j + 4) {
                on_step(t, unit_frag(w0, t), unit_frag(w1, t));
                ++next;
            }
        }
    }
    uint32_t p0 = and_or(d0[0] >> 9, S6, B6), q0 = and_or(d0[3] >> 9, S6, B6);
    uint32_t p1 = and_or(d1[0] >> 9, S6, B6), q1 = and_or(d1[3] >> 9, S6, B6);
    p0 = and_or(d0[1] >> 8, S7, p0);
    q0 = and_or(d0[4] >> 8, S7, q0);
    p1 = and_or(d1[1] >> 8, S7, p1);
    q1 = and_or(d1[4] >> 8, S7, q1);
    p0 = and_or(d0[2] >> 7, S8, p0);
    q0 = and_or(d0[5] >> 7, S8, q0);
    p1 = and_or(d1[2] >> 7, S8, p1);
    q1 = and_or(d1[5] >> 7, S8, q1);
    w0[30] = pk_fma(pk_sub(p0, c0.A6), c0.S2, c0.C2);
    w0[31] = pk_fma(pk_sub(q0, c0.A6), c0.S2, c0.C2);
    w1[30] = pk_fma(pk_sub(p1, c1.A6), c1.S2, c1.C2);
    w1[31] = pk_fma(pk_sub(q1, c1.A6), c1.S2, c1.C2);
    on_step(7, unit_frag(w0, 7), unit_frag(w1, 7));
}

// ---------------------------------------------------------------------------------------------
// bf16 variant of the conversion (activations, compensator and output in bf16; Section 3.3 names
// FP16 only, this is the same idea on the other 16-bit format).  bf16 has seven mantissa bits, so a
// 3-bit field reads as an integer in place only at bit 0 (exponent pattern 0x4300: 128 + e) and at
// bit 3 (0x4180: 16 + e); the fields at bits 6, 9 and 12 are shifted down first.  bf16 has no packed
// arithmetic here, and its eight significant bits could not hold s * (e - z) anyway: a bf16 is the
// upper half of a binary32, so each value is widened with a shift or a mask, w = fma(B + e, s,
// -(B + z) s) is formed in binary32 (the product is exact, the constant is exact for integer
// zero-points), and two results are rounded to a bf16 pair with one conversion: one rounding per
// weight, as in the fp16 path.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// (B + e_lo, B + e_hi) as a bf16 pair in `h`  ->  bf16 pair of s * (e - z); c = -(B + z) * s
__device__ __forceinline__ uint32_t bf16_pair(uint32_t h, float s, float c) {
    const float lo = __builtin_bit_cast(float, h << 16), hi = __builtin_bit_cast(float, h & 0xffff0000u);
    return pack_bf16(__builtin_fmaf(lo, s, c), __builtin_fmaf(hi, s, c));
}
template <typename OnStep>
__device__ __forceinline__ void dequant_unit_steps_bf16(const RawUnit& ru, OnStep&& on_step) {
    const float s = (float)f16_bits(ru.sz);
    const float z = (float)f16_bits(ru.sz >> 16);
    const float c0 = -(128.0f + z) * s, c3 = -(16.0f + z) * s;
    const uint32_t B0 = in_vgpr(0x43004300u), B3 = in_vgpr(0x41804180u);
    const uint32_t M0 = in_sgpr(0x00070007u), M3 = in_sgpr(0x00380038u);
    const uint32_t d[6] = {ru.a.x, ru.a.y, ru.a.z, ru.a.w, ru.b.x, ru.b.y};
    uint32_t w[32];
    int next = 0;
#pragma unroll
    for (int j = 0; j < 6; ++j) {
        const uint32_t s6 = d[j] >> 6, s12 = d[j] >> 12;
        w[5 * j + 0] = bf16_pair(and_or(d[j], M0, B0), s, c0);
        w[5 * j + 1] = bf16_pair(and_or(d[j], M3, B3), s, c3);
        w[5 * j + 2] = bf16_pair(and_or(s6, M0, B0), s, c0);
        w[5 * j + 3] = bf16_pair(and_or(s6, M3, B3), s, c3);
        w[5 * j + 4] = bf16_pair(and_or(s12, M0, B0), s, c0);
#pragma unroll
        for (int t = 0; t < 7; ++t) {
            if (t == next && 4 * t + 3 <= 5 * j + 4) {
                const u32x4 v = {w[4 * t + 0], w[4 * t + 1], w[4 * t + 2], w[4 * t + 3]};
                on_step(t, __builtin_bit_cast(bf16x8, v));
                ++next;
            }
        }
    }
    // pairs 30 and 31: bits 15 / 31 of words 0..2 and 3..5 carry bits 0, 1, 2
    const uint32_t S0 = in_sgpr(0x00010001u), S1 = in_sgpr(0x00020002u), S2 = in_sgpr(0x00040004u);
    uint32_t t0 = and_or(d[0] >> 15, S0, B0), t1 = and_or(d[3] >> 15, S0, B0);
    t0 = and_or(d[1] >> 14, S1, t0);
    t1 = and_or(d[4] >> 14, S1, t1);
    t0 = and_or(d[2] >> 13, S2, t0);
    t1 = and_or(d[5] >> 13, S2, t1);
    w[30] = bf16_pair(t0, s, c0);
    w[31] = bf16_pair(t1, s, c0);
    const u32x4 v = {w[28], w[29], w[30], w[31]};
    on_step(7, __builtin_bit_cast(bf16x8, v));
}
// Two units in lock step (the tiled kernel's two weight streams).  on_step(t, frag0, frag1).
template <typename OnStep>
__device__ __forceinline__ void dequant_units2_steps_bf16(const RawUnit& r0, const RawUnit& r1, OnStep&& on_step) {
    const float s0 = (float)f16_bits(r0.sz), z0 = (float)f16_bits(r0.sz >> 16);
    const float s1 = (float)f16_bits(r1.sz), z1 = (float)f16_bits(r1.sz >> 16);
    const float c00 = -(128.0f + z0) * s0, c03 = -(16.0f + z0) * s0;
    const float c10 = -(128.0f + z1) * s1, c13 = -(16.0f + z1) * s1;
    const uint32_t B0 = in_vgpr(0x43004300u), B3 = in_vgpr(0x41804180u);
    const uint32_t M0 = in_sgpr(0x00070007u), M3 = in_sgpr(0x00380038u);
    const uint32_t d0[6] = {r0.a.x, r0.a.y, r0.a.z, r0.a.w, r0.b.x, r0.b.y};
    const uint32_t d1[6] = {r1.a.x, r1.a.y, r1.a.z, r1.a.w, r1.b.x, r1.b.y};
    uint32_t w0[32], w1[32];
    int next = 0;
#pragma unroll
    for (int j = 0; j < 6; ++j) {
        const uint32_t a6 = d0[j] >> 6, a12 = d0[j] >> 12, b6 = d1[j] >> 6, b12 = d1[j] >> 12;
        w0[5 * j + 0] = bf16_pair(and_or(d0[j], M0, B0), s0, c00);
        w1[5 * j + 0] = bf16_pair(and_or(d1[j], M0, B0), s1, c10);
        w0[5 * j + 1] = bf16_pair(and_or(d0[j], M3, B3), s0, c03);
        w1[5 * j + 1] = bf16_pair(and_or(d1[j], M3, B3), s1, c13);
        w0[5 * j + 2] = bf16_pair(and_or(a6, M0, B0), s0, c00);
        w1[5 * j + 2] = bf16_pair(and_or(b6, M0, B0), s1, c10);
        w0[5 * j + 3] = bf16_pair(and_or(a6, M3, B3), s0, c03);
        w1[5 * j + 3] = bf16_pair(and_or(b6, M3, B3), s1, c13);
        w0[5 * j + 4] = bf16_pair(and_or(a12, M0, B0), s0, c00);
        w1[5 * j + 4] = bf16_pair(and_or(b12, M0, B0), s1, c10);
#pragma unroll
        for (int t = 0; t < 7; ++t) {
            if (t == next && 4 * t + 3 <= 5 * j + 4) {
                const u32x4 v0 = {w0[4 * t + 0], w0[4 * t + 1], w0[4 * t + 2], w0[4 * t + 3]};
                const u32x4 v1 = {w1[4 * t + 0], w1[4 * t + 1], w1[4 * t + 2], w1[4 * t + 3]};
                on_step(t, __builtin_bit_cast(bf16x8, v0), __builtin_bit_cast(bf16x8, v1));
                ++next;
            }
        }
    }
    const uint32_t S0 = in_sgpr(0x00010001u), S1 = in_sgpr(0x00020002u), S2 = in_sgpr(0x00040004u);
    uint32_t p0 = and_or(d0[0] >> 15, S0, B0), q0 = and_or(d0[3] >> 15, S0, B0);
    uint32_t p1 = and_or(d1[0] >> 15, S0, B0), q1 = and_or(d1[3] >> 15, S0, B0);
    p0 = and_or(d0[1] >> 14, S1, p0);
    q0 = and_or(d0[4] >> 14, S1, q0);
    p1 = and_or(d1[1] >> 14, S1, p1);
    q1 = and_or(d1[4] >> 14, S1, q1);
    p0 = and_or(d0[2] >> 13, S2, p0);
    q0 = and_or(d0[5] >> 13, S2, q0);
    p1 = and_or(d1[2] >> 13, S2, p1);
    q1 = and_or(d1[5] >> 13, S2, q1);
    w0[30] = bf16_pair(p0, s0, c00);
    w0[31] = bf16_pair(q0, s0, c00);
    w1[30] = bf16_pair(p1, s1, c10);
    w1[31] = bf16_pair(q1, s1, c10);
    const u32x4 v0 = {w0[28], w0[29], w0[30], w0[31]};
    const u32x4 v1 = {w1[28], w1[29], w1[30], w1[31]};
    on_step(7, __builtin_bit_cast(bf16x8, v0), __builtin_bit_cast(bf16x8, v1));
}
__device__ __forceinline__ f32x4 mfma16_bf16(bf16x8 a, bf16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma32_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// All 32 pairs of a unit at once (for the dense dequantization kernel).
template <bool SYM = false>
__device__ __forceinline__ void dequant_unit(const RawUnit& ru, uint32_t (&w)[32]) {
    dequant_unit_steps<SYM>(ru, [&](int t, f16x8 frag) {
        const u32x4 v = __builtin_bit_cast(u32x4, frag);
        w[4 * t + 0] = v.x;
        w[4 * t + 1] = v.y;
        w[4 * t + 2] = v.z;
        w[4 * t + 3] = v.w;
    });
}

// The A operand of MFMA step t (t = 0..7) of a dequantized unit: codes 8t .. 8t+7.
__device__ __forceinline__ f16x8 unit_frag(const uint32_t (&w)[32], int t) {
    u32x4 v = {w[4 * t + 0], w[4 * t + 1], w[4 * t + 2], w[4 * t + 3]};
    return __builtin_bit_cast(f16x8, v);
}

// ---------------------------------------------------------------------------------------------
// MFMA wrappers (gfx950).  Operand layouts, lane l of the wave:
//   16x16x32: A lane holds row l%16, k = 8*(l/16) .. +7 ; B lane holds column l%16, same k ;
//             D[v] (v = 0..3) is row 4*(l/16) + v, column l%16.
//   32x32x16: A lane holds row l%32, k = 8*(l/32) .. +7 ; B lane holds column l%32, same k ;
//             D[v] (v = 0..15) is row 8*(v/4) + 4*(l/32) + v%4, column l%32.
__device__ __forceinline__ f32x4 mfma16(f16x8 a, f16x8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma32(f16x8 a, f16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f16x8 zero_f16x8() {
    u32x4 v = {0u, 0u, 0u, 0u};
    return __builtin_bit_cast(f16x8, v);
}

__device__ __forceinline__ f16x8 load_f16x8(const f16* p) {
    return __builtin_bit_cast(f16x8, *reinterpret_cast<const u32x4*>(p));
}

// 8 consecutive fp16 of a row of length `len` starting at column k0 (k0 % 8 == 0): one 16-byte
// load when the row stride keeps it aligned and the slice is inside, element-wise otherwise.
__device__ __forceinline__ f16x8 load_row8(const f16* row, int k0, int len, bool aligned16) {
    if (k0 + 8 <= len && aligned16) return load_f16x8(row + k0);
    f16x8 r = zero_f16x8();
#pragma unroll
    for (int v = 0; v < 8; ++v)
        if (k0 + v < len) r[v] = row[k0 + v];
    return r;
}

}  // namespace milo
