// milo_w3lr_gemm_static: the compensated linear for callers that cannot allocate or bring a
// workspace.  It runs the kernels of milo_w3lr_gemm on a scratch array that lives in the library's
// device image.
#include "milo_host.h"
#include "milo_kernels.h"

using namespace milo;

namespace milo {
constexpr size_t kStaticScratchBytes = (size_t)MILO_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

__global__ void scratch_clear_kernel(u32x4* p, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
        p[i] = u32x4{0u, 0u, 0u, 0u};
}
}  // namespace milo

// Device address of `scratch` on the current device, looked up once per device: each device holds
// its own copy of the array at its own address, and the array's name is not an address that host
// code may hand to a kernel or to a memory routine.
static int static_scratch(void** out) {
    static void* ptr[64] = {nullptr};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return MILO_ERR_HIP;
    void* p = __atomic_load_n(&ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(milo::scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return MILO_ERR_HIP;
        }
        __atomic_store_n(&ptr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return MILO_OK;
}

extern "C" int milo_w3lr_gemm_static(const milo_half* X, int64_t M, int64_t N, int64_t K, const void* q3,
                                     const milo_half* U, const milo_half* V, int r, milo_half* Y,
                                     void* stream) {
    if (!X || !q3 || !Y) return MILO_ERR_NULL;
    const size_t need = milo_w3lr_gemm_workspace(M, N, K, r);       // 0 for an invalid shape or rank
    if (need == 0) return (r < 0) ? MILO_ERR_RANK : MILO_ERR_SHAPE;
    if (need > kStaticScratchBytes) return MILO_ERR_WORKSPACE;
    void* ws = nullptr;
    const int st = static_scratch(&ws);
    if (st != MILO_OK) return st;
    // The array keeps what the last call left.  The kernels leave their control words at zero,
    // but a call that failed half-way may not have, and the flag words of another shape lie
    // elsewhere: the control block and the flag / sign-off words behind it are cleared first, by
    // a small fill kernel (not a memset, so that the call can be captured in a HIP graph).
    size_t head = 256 + (gemm_takes_decode(M, N, K, r) ? (size_t)kDecDoneBytes : align_up((size_t)((M + 31) / 32) * 16, 256));
    if (head > need) head = need;
    const size_t n16 = head / 16;
    scratch_clear_kernel<<<dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
        reinterpret_cast<u32x4*>(ws), n16);
    if (launch_status() != MILO_OK) return MILO_ERR_HIP;
    return milo_w3lr_gemm(X, M, N, K, q3, U, V, r, Y, ws, kStaticScratchBytes, stream);
}
