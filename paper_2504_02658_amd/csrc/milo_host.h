// Host-side helpers shared by the entry points: argument checks and launch error handling.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/milo.h"

namespace milo {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Compute units of the current device (256 if the query fails); cached per device.
inline int device_cus() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
        cached[dev] = cus;
    }
    return cached[dev];
}

// K splits for a tiled GEMM whose grid would have `tiles` workgroups, next to `others` workgroups
// of the same launch that do not split (the ones forming X V^T): as many as fit on the chip at once
// at two workgroups per CU, as long as a split keeps at least eight 128-column chunks.
inline int tiled_k_splits(int64_t tiles, int64_t K, int64_t others) {
    const int64_t nchunks = (K / 64 + 1) / 2;
    int64_t room = 2 * (int64_t)device_cus() - others;
    if (room < (int64_t)device_cus()) room = device_cus();
    int64_t s = tiles > 0 ? room / tiles : 1;
    if (s > nchunks / 8) s = nchunks / 8;
    if (s > 16) s = 16;
    if (s < 1) s = 1;
    return (int)s;
}

// K % 64 == 0, N % 16 == 0, both positive, and N*K small enough for 64-bit byte arithmetic
// and 32-bit group counts per row.
inline bool weight_shape_ok(int64_t N, int64_t K) {
    if (N <= 0 || K <= 0) return false;
    if ((K % 64) != 0 || (N % 16) != 0) return false;
    if (K > (int64_t(1) << 30) || N > (int64_t(1) << 30)) return false;
    if (N > (int64_t(1) << 56) / K) return false;
    // units, and the bytes of 16 rows of activations, are addressed with 32-bit offsets; the
    // kernels mark "no data" with unit indices from 2^26 up
    if (N * (K / 64) > (int64_t(1) << 26) || K > (int64_t(1) << 26)) return false;
    return true;
}

inline int launch_status() {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? MILO_OK : MILO_ERR_HIP;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace milo
