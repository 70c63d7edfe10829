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
// plane A holds 16 bytes per unit, plane B (right behind it) 8 bytes per unit.
struct W3View {
    const u32x4* planeA;
    const u32x2* planeB;
    const f16* scales;
    const f16* zeros;
    int G;                          // groups per row
};

__host__ __device__ inline W3View make_view(const void* q3, const void* scales, const void* zeros,
                                            int64_t N, int64_t K) {
    W3View v;
    v.planeA = reinterpret_cast<const u32x4*>(q3);
    v.planeB = reinterpret_cast<const u32x2*>(reinterpret_cast<const char*>(q3) + (N * K) / 4);
    v.scales = reinterpret_cast<const f16*>(scales);
    v.zeros = reinterpret_cast<const f16*>(zeros);
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
    f16 s, z;
};

__device__ __forceinline__ RawUnit zero_unit() {
    RawUnit r;
    r.a = u32x4{0u, 0u, 0u, 0u};
    r.b = u32x2{0u, 0u};
    r.s = (f16)0.0f;
    r.z = (f16)0.0f;
    return r;
}

// STREAM = true marks the loads non-temporal: the decode kernel reads every weight byte exactly
// once, so keeping it out of the caches' replacement order protects the activations.
template <bool STREAM>
__device__ __forceinline__ RawUnit load_unit(const W3View& w, int64_t u) {
    RawUnit r;
    if (STREAM) {
        r.a = __builtin_nontemporal_load(w.planeA + u);
        r.b = __builtin_nontemporal_load(w.planeB + u);
        r.s = __builtin_nontemporal_load(w.scales + u);
        r.z = __builtin_nontemporal_load(w.zeros + u);
    } else {
        r.a = w.planeA[u];
        r.b = w.planeB[u];
        r.s = w.scales[u];
        r.z = w.zeros[u];
    }
    return r;
}

// ---------------------------------------------------------------------------------------------
// (a & mask) | orv in one VALU op.  The mask sits in an SGPR: on gfx9-family encodings a VOP3
// instruction cannot carry a 32-bit literal, and without this the compiler emits and + or.
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t orv) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(orv));
    return r;
}

// Two fp16 values h (low, high half of a register) -> two fp16 values S*h + C, evaluated as an
// fp32 fused multiply-add with one rounding to fp16 (compiles to v_fma_mixlo/mixhi_f16).
__device__ __forceinline__ uint32_t scale_pair(uint32_t h, float S, float C) {
    f16x2 v = __builtin_bit_cast(f16x2, h);
    f16x2 r;
    r.x = (f16)__builtin_fmaf((float)v.x, S, C);
    r.y = (f16)__builtin_fmaf((float)v.y, S, C);
    return __builtin_bit_cast(uint32_t, r);
}

// 3-bit -> fp16 conversion of one unit (Section 3.3 of the paper, "MiLo Dequant", reworked for
// this layout): a 3-bit field sitting at mantissa bit b of an fp16 whose exponent field says
// 2^10 reads as 1024 + 2^b * e, so OR-ing 0x6400 over the masked field converts the integer
// without any int->float instruction, two codes per 32-bit register.  Fields at b = 0, 3, 6
// are usable without a shift.  The bias and the field's 2^b factor are then removed together
// with the zero-point and the scale by one fp32 fma per element:
//      w = (s / 2^b) * h - (1024 / 2^b + z) * s  =  s * (e - z)
// which is exact up to the single final rounding to fp16 for any real-valued z.
// Output: w[P] = packed fp16 (W_dq[2P], W_dq[2P+1]) for the unit's 32 code pairs.
__device__ __forceinline__ void dequant_unit(const RawUnit& ru, uint32_t (&w)[32]) {
    const float s = (float)ru.s;
    const float z = (float)ru.z;
    const float S1 = s, S8 = s * 0.125f, S64 = s * 0.015625f;
    const float C1 = -(1024.0f + z) * s;
    const float C8 = -(128.0f + z) * s;
    const float C64 = -(16.0f + z) * s;
    const uint32_t kBias = 0x64006400u;
    const uint32_t d[6] = {ru.a.x, ru.a.y, ru.a.z, ru.a.w, ru.b.x, ru.b.y};
    uint32_t sh[6];
#pragma unroll
    for (int j = 0; j < 6; ++j) {
        sh[j] = d[j] >> 9;
        w[5 * j + 0] = scale_pair(and_or(d[j], 0x00070007u, kBias), S1, C1);
        w[5 * j + 1] = scale_pair(and_or(d[j], 0x00380038u, kBias), S8, C8);
        w[5 * j + 2] = scale_pair(and_or(d[j], 0x01C001C0u, kBias), S64, C64);
        w[5 * j + 3] = scale_pair(and_or(sh[j], 0x00070007u, kBias), S1, C1);
        w[5 * j + 4] = scale_pair(and_or(sh[j], 0x00380038u, kBias), S8, C8);
    }
    // Pairs 30 and 31 are spread over the spare bits 15 / 31 of three words each; shifting the
    // words by 9, 8 and 7 lines the three bits up at mantissa bits 6, 7, 8 (a 2^6 field).
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        uint32_t t = and_or(sh[3 * p], 0x00400040u, kBias);
        t = and_or(d[3 * p + 1] >> 8, 0x00800080u, t);
        t = and_or(d[3 * p + 2] >> 7, 0x01000100u, t);
        w[30 + p] = scale_pair(t, S64, C64);
    }
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
