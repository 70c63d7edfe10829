// Shared by the two quantizers (pack.hip, compress.hip): 16 lanes hold the 64 codes of one unit, four
// each, and write them in the zero-waste 3-bit layout (Section 3.3).
#pragma once
#include "milo_device.h"

namespace milo {

// 16 lanes cooperate on one unit (64 weights, one float4 each); a wave packs four units that
// are consecutive groups of one row, so every load instruction of a wave reads 1 KB of that row.
constexpr int kPackThreads = 256;
constexpr int kUnitsPerBlock = kPackThreads / 16;

__device__ __forceinline__ float shfl_xor16(float v, int m) { return __shfl_xor(v, m, 16); }
__device__ __forceinline__ uint32_t shfl_xor16(uint32_t v, int m) {
    return (uint32_t)__shfl_xor((int)v, m, 16);
}

// Lane l16 of the 16 holds the codes 4*l16 .. 4*l16+3 of unit u in q; lane 0 stores the unit.
__device__ __forceinline__ void store_unit(const uint32_t (&q)[4], int l16, f16 s16, f16 z16, int64_t u,
                                           uint32_t* __restrict__ planeA, uint32_t* __restrict__ planeB) {
    // This lane owns code pairs P0 = 2*l16 (codes 4*l16, 4*l16+1) and P0+1.  Build its share of
    // the six words, then OR the shares of the 16 lanes together.
    uint32_t d[6] = {0u, 0u, 0u, 0u, 0u, 0u};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int P = 2 * l16 + h;
        const uint32_t lo = q[2 * h], hi = q[2 * h + 1];
        if (P < 30) {
            const int j = P / 5, c = P - 5 * j;
            const uint32_t bits = (lo << (3 * c)) | (hi << (16 + 3 * c));
#pragma unroll
            for (int jj = 0; jj < 6; ++jj)
                if (jj == j) d[jj] |= bits;
        } else {
            const int base = (P == 30) ? 0 : 3;
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                const uint32_t bits = (((lo >> i) & 1u) << 15) | (((hi >> i) & 1u) << 31);
#pragma unroll
                for (int jj = 0; jj < 6; ++jj)
                    if (jj == base + i) d[jj] |= bits;
            }
        }
    }
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) {
#pragma unroll
        for (int jj = 0; jj < 6; ++jj) d[jj] |= shfl_xor16(d[jj], m);
    }

    if (l16 == 0) {
        *reinterpret_cast<u32x4*>(planeA + 4 * u) = u32x4{d[0], d[1], d[2], d[3]};
        planeB[3 * u] = d[4];
        planeB[3 * u + 1] = d[5];
        planeB[3 * u + 2] = (uint32_t)__builtin_bit_cast(unsigned short, s16) |
                            ((uint32_t)__builtin_bit_cast(unsigned short, z16) << 16);
    }
}

}  // namespace milo
