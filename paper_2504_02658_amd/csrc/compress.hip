// milo_compress_w3lr: the MiLo compression loop (Algorithm 1) on the device.
//
// One outer iteration is  R = W - U V;  a few half-quadratic updates of the zero-points z for the
// target R with the scales fixed (Section 3.2, Eq. update_We / update_z);  E = W - W_dq;  a truncated
// SVD of E split as U = U^ S^(1/2), V = S^(1/2) V^ (Eq. UV);  the error eps_t (Eq. epsilon).  The host
// reads eps_t after every iteration and applies the stop rule (Eq. stop_condition).
//
// The SVD is the only step that is not a plain transcription: an exact SVD of a 14336 x 4096 matrix
// per iteration is what makes the method slow on the paper's own hardware, and the loop only needs the
// leading r (<= 128) triplets.  They come from a block subspace iteration with l = r + 8 vectors:
//     Y = E Vb^T, Q = orth(Y) (Cholesky QR), B = Q^T E, B B^T = Ub S^2 Ub^T (Jacobi),
//     U = Q Ub_r S_r^(1/2),  V = S_r^(-1/2) Ub_r^T B,  next basis Vb = S^(-1) Ub^T B
// started from a random basis with a few extra rounds in the first outer iteration and warm-started
// from the previous right singular vectors afterwards (E changes little between outer iterations, so
// the outer loop itself is the power iteration).  All matrix products are fp32 on the vector units:
// they are tall-skinny (l <= 136) and read E once or twice; the compressor runs offline.
//
// Compiled with -ffp-contract=off like the quantizer: the half-quadratic update follows its
// formulas one rounding per operation.
#include "milo_device.h"
#include "milo_host.h"
#include "pack_device.h"

namespace milo {

constexpr int kSketchExtra = 8;                                   // l = r + 8 basis vectors
constexpr int kSketchMax = MILO_COMPRESS_MAX_RANK + kSketchExtra;
constexpr int kSmallThreads = 256;

// ------------------------------------------------------------------ per-group parameters (fixed scales)
// s = fp16((max - min) / 7) of W's group (1 for a degenerate group), z0 = -min / s, real-valued.
__global__ __launch_bounds__(kPackThreads) void group_params_kernel(const float* __restrict__ W, int64_t N, int64_t K,
                                                                    float* __restrict__ s, float* __restrict__ z) {
    const int64_t G = K / kGroup;
    const int64_t gu = (int64_t)blockIdx.x * kUnitsPerBlock + (threadIdx.x >> 4);
    const int l16 = threadIdx.x & 15;
    if (gu >= N * G) return;
    const float4 v = *reinterpret_cast<const float4*>(W + gu * kGroup + 4 * l16);
    float mn = fminf(fminf(v.x, v.y), fminf(v.z, v.w));
    float mx = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
#pragma unroll
    for (int m = 1; m < 16; m <<= 1) {
        mn = fminf(mn, shfl_xor16(mn, m));
        mx = fmaxf(mx, shfl_xor16(mx, m));
    }
    if (l16 == 0) {
        float sf = (float)(f16)((mx - mn) / 7.0f);
        if (!(sf > 0.0f && sf <= 65504.0f)) sf = 1.0f;
        s[gu] = sf;
        z[gu] = (-mn) / sf;
    }
}

// ------------------------------------------------------------------ half-quadratic zero-point updates
// 16 lanes per group, the 64 targets stay in registers over all iterations.  RE holds R on entry and
// E = W - s (W_q - z) on exit (codes and z of the last update).
__device__ __forceinline__ float code_of(float r, float sf, float zf) {
    float t = r / sf;
    t = t + zf;
    t = __builtin_rintf(t);
    return fminf(fmaxf(t, 0.0f), 7.0f);
}

__global__ __launch_bounds__(kPackThreads) void hqq_kernel(const float* __restrict__ W, float* __restrict__ RE,
                                                           const float* __restrict__ s, float* __restrict__ z, int64_t units,
                                                           int iters, float pm1, float beta, float kappa) {
    const int64_t gu = (int64_t)blockIdx.x * kUnitsPerBlock + (threadIdx.x >> 4);
    const int l16 = threadIdx.x & 15;
    if (gu >= units) return;
    const int64_t at = gu * kGroup + 4 * l16;
    const float4 r4 = *reinterpret_cast<const float4*>(RE + at);
    const float r[4] = {r4.x, r4.y, r4.z, r4.w};
    const float sf = s[gu];
    const float inv_s = 1.0f / sf;
    float zf = z[gu];
    // |e|^(p-1) through the hardware's exp2 and log2 (about 1 ulp each): the threshold it feeds is a
    // smooth function, no decision hangs on its last bits.  The code itself does: code_of divides.
    for (int it = 0; it < iters; ++it) {
        const float inv_beta = 1.0f / beta;
        float acc = 0.0f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float q = code_of(r[i], sf, zf);
            const float wdq = sf * (q - zf);
            const float e = r[i] - wdq;
            const float ae = fabsf(e);
            const float thr = ae > 0.0f ? __builtin_amdgcn_exp2f(pm1 * __builtin_amdgcn_logf(ae)) * inv_beta : 0.0f;
            const float m = copysignf(fmaxf(ae - thr, 0.0f), e);           // shrink_lp(e)
            acc += q - (r[i] - m) * inv_s;
        }
#pragma unroll
        for (int m = 1; m < 16; m <<= 1) acc += shfl_xor16(acc, m);
        zf = acc * (1.0f / 64.0f);
        beta *= kappa;
    }
    const float4 w4 = *reinterpret_cast<const float4*>(W + at);
    const float w[4] = {w4.x, w4.y, w4.z, w4.w};
    float e[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) e[i] = w[i] - sf * (code_of(r[i], sf, zf) - zf);
    *reinterpret_cast<float4*>(RE + at) = float4{e[0], e[1], e[2], e[3]};
    if (l16 == 0) z[gu] = zf;
}

// Codes of the target R with the fixed scales and z rounded to fp16, packed (Section 3.3).
__global__ __launch_bounds__(kPackThreads) void pack_given_kernel(const float* __restrict__ R, const float* __restrict__ s,
                                                                  const float* __restrict__ z, int64_t N, int64_t K,
                                                                  uint32_t* __restrict__ planeA, uint32_t* __restrict__ planeB) {
    const int64_t G = K / kGroup;
    const int64_t gu = (int64_t)blockIdx.x * kUnitsPerBlock + (threadIdx.x >> 4);
    const int l16 = threadIdx.x & 15;
    if (gu >= N * G) return;
    const int64_t n = gu / G, g = gu - n * G;
    const float4 r4 = *reinterpret_cast<const float4*>(R + gu * kGroup + 4 * l16);
    const float r[4] = {r4.x, r4.y, r4.z, r4.w};
    const float sf = s[gu];
    const f16 z16 = (f16)fminf(fmaxf(z[gu], -65504.0f), 65504.0f);
    const float zf = (float)z16;
    uint32_t q[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) q[i] = (uint32_t)code_of(r[i], sf, zf);
    store_unit(q, l16, (f16)sf, z16, unit_index(n, g, G), planeA, planeB);
}

// ------------------------------------------------------------------ In - U V: the new target, or its norm
// One workgroup per 64 x 64 tile, a thread owns 4 x 4 of it.  MODE 0 writes Out = In - U V, MODE 1
// writes the tile's sum of squares of In - U V (fp64) to partial[tile].
template <int MODE>
__global__ __launch_bounds__(256) void resid_kernel(const float* __restrict__ In, const float* __restrict__ U,
                                                    const float* __restrict__ V, int r, int64_t N, int64_t K,
                                                    float* __restrict__ Out, double* __restrict__ partial) {
    __shared__ float Us[16][68];      // [rank][row]
    __shared__ float Vs[16][68];      // [rank][column]
    __shared__ double red[256];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int64_t i0 = (int64_t)blockIdx.y * 64, j0 = (int64_t)blockIdx.x * 64;
    float acc[4][4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) acc[x][y] = 0.0f;
    for (int k0 = 0; k0 < r; k0 += 16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e;
            const int kk = idx & 15, ii = idx >> 4;                   // U is [N x r]: rank fastest
            Us[kk][ii] = (i0 + ii < N && k0 + kk < r) ? U[(i0 + ii) * r + k0 + kk] : 0.0f;
            const int jj = idx & 63, kv = idx >> 6;                   // V is [r x K]: column fastest
            Vs[kv][jj] = (k0 + kv < r) ? V[(int64_t)(k0 + kv) * K + j0 + jj] : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const float4 a = *reinterpret_cast<const float4*>(&Us[kk][4 * ty]);
            const float4 b = *reinterpret_cast<const float4*>(&Vs[kk][4 * tx]);
            const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) acc[x][y] = fmaf(av[x], bv[y], acc[x][y]);
        }
        __syncthreads();
    }
    double sq = 0.0;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int64_t gi = i0 + 4 * ty + x;
        if (gi >= N) continue;
        const int64_t at = gi * K + j0 + 4 * tx;
        const float4 w = *reinterpret_cast<const float4*>(In + at);
        const float4 o = {w.x - acc[x][0], w.y - acc[x][1], w.z - acc[x][2], w.w - acc[x][3]};
        if (MODE == 0) {
            *reinterpret_cast<float4*>(Out + at) = o;
        } else {
            sq += (double)o.x * o.x + (double)o.y * o.y + (double)o.z * o.z + (double)o.w * o.w;
        }
    }
    if (MODE == 1) {
        red[tid] = sq;
        __syncthreads();
        for (int h = 128; h > 0; h >>= 1) {
            if (tid < h) red[tid] += red[tid + h];
            __syncthreads();
        }
        if (tid == 0) partial[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = red[0];
    }
}

__global__ __launch_bounds__(256) void sum_partials_kernel(const double* __restrict__ partial, int64_t count,
                                                           double* __restrict__ out) {
    __shared__ double red[256];
    double a = 0.0;
    for (int64_t i = threadIdx.x; i < count; i += 256) a += partial[i];
    red[threadIdx.x] = a;
    __syncthreads();
    for (int h = 128; h > 0; h >>= 1) {
        if (threadIdx.x < h) red[threadIdx.x] += red[threadIdx.x + h];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = red[0];
}

// ------------------------------------------------------------------ fp32 products of the subspace iteration
// C [M x N] = sum over k < Kd of A(i, k) B(k, j) with A(i, k) = A[i * sai + k * sak] and
// B(k, j) = B[k * sbk + j * sbj]: either operand plain or transposed.  64 x 64 x 16 tiles; blockIdx.z
// takes the k range [z * kchunk, (z + 1) * kchunk) and writes its own copy of C (dense, row length N)
// at C + z * part_stride, summed afterwards in a fixed order.
struct SgemmArgs {
    const float* A;
    int64_t sai, sak;
    const float* B;
    int64_t sbk, sbj;
    float* C;
    int64_t ldc, part_stride;
    int M, N, Kd, kchunk;
};

__global__ __launch_bounds__(256) void sgemm_kernel(SgemmArgs g) {
    __shared__ float As[16][68];      // [k][i]
    __shared__ float Bs[16][68];      // [k][j]
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int i0 = blockIdx.y * 64, j0 = blockIdx.x * 64;
    const int kbeg = blockIdx.z * g.kchunk;
    const int kend = min(g.Kd, kbeg + g.kchunk);
    const bool a_k_fast = g.sak == 1, b_k_fast = g.sbk == 1;     // walk the unit-stride index fastest
    float acc[4][4];
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
        for (int y = 0; y < 4; ++y) acc[x][y] = 0.0f;
    for (int k0 = kbeg; k0 < kend; k0 += 16) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int idx = tid + 256 * e;
            {
                const int kk = a_k_fast ? (idx & 15) : (idx >> 6);
                const int ii = a_k_fast ? (idx >> 4) : (idx & 63);
                const int gi = i0 + ii, gk = k0 + kk;
                As[kk][ii] = (gi < g.M && gk < kend) ? g.A[(int64_t)gi * g.sai + (int64_t)gk * g.sak] : 0.0f;
            }
            {
                const int kk = b_k_fast ? (idx & 15) : (idx >> 6);
                const int jj = b_k_fast ? (idx >> 4) : (idx & 63);
                const int gj = j0 + jj, gk = k0 + kk;
                Bs[kk][jj] = (gj < g.N && gk < kend) ? g.B[(int64_t)gk * g.sbk + (int64_t)gj * g.sbj] : 0.0f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const float4 a = *reinterpret_cast<const float4*>(&As[kk][4 * ty]);
            const float4 b = *reinterpret_cast<const float4*>(&Bs[kk][4 * tx]);
            const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
            for (int x = 0; x < 4; ++x)
#pragma unroll
                for (int y = 0; y < 4; ++y) acc[x][y] = fmaf(av[x], bv[y], acc[x][y]);
        }
        __syncthreads();
    }
    float* C = g.C + (int64_t)blockIdx.z * g.part_stride;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int gi = i0 + 4 * ty + x;
#pragma unroll
        for (int y = 0; y < 4; ++y) {
            const int gj = j0 + 4 * tx + y;
            if (gi < g.M && gj < g.N) C[(int64_t)gi * g.ldc + gj] = acc[x][y];
        }
    }
}

__global__ __launch_bounds__(256) void sum_parts_kernel(const float* __restrict__ parts, int S, int64_t part_stride,
                                                        int M, int N, float* __restrict__ C, int64_t ldc) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)M * N) return;
    float a = 0.0f;
    for (int z = 0; z < S; ++z) a += parts[(int64_t)z * part_stride + e];
    C[(e / N) * ldc + (e % N)] = a;
}

// Uniform numbers in (-1, 1) from a counter hash: the starting basis of the subspace iteration.
__global__ __launch_bounds__(256) void random_basis_kernel(float* __restrict__ out, int64_t count, uint32_t seed) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    uint32_t h = (uint32_t)i * 0x9E3779B1u + seed;
    h ^= (uint32_t)(i >> 32) * 0x85EBCA77u;
    h ^= h >> 16; h *= 0x7FEB352Du;
    h ^= h >> 15; h *= 0x846CA68Bu;
    h ^= h >> 16;
    out[i] = ((float)(h >> 8) + 0.5f) * (1.0f / 8388608.0f) - 1.0f;
}

// ------------------------------------------------------------------ small dense factorizations (one workgroup)
// Gm [l x l] symmetric positive definite (a Gram matrix Y^T Y) = L L^T.  Writes Rinv = L^-T (upper
// triangular, dense) so that Q = Y Rinv has orthonormal columns.  A pivot that is not safely positive
// (a rank-deficient sketch) is replaced by a small multiple of the mean diagonal: the result stays
// finite and the directions concerned carry no weight in the later steps.
__global__ __launch_bounds__(kSmallThreads) void cholesky_inverse_kernel(const float* __restrict__ Gm, int l,
                                                                         float* __restrict__ Rinv) {
    extern __shared__ float lds[];
    const int ld = l + 1;
    float* A = lds;                    // lower triangle: L;  strictly upper triangle, row j: column j of L^-1
    float* dinv = lds + l * ld;        // 1 / L_jj
    float* misc = dinv + l;
    const int tid = threadIdx.x;
    for (int e = tid; e < l * l; e += kSmallThreads) A[(e / l) * ld + e % l] = Gm[e];
    __syncthreads();
    if (tid == 0) {
        float tr = 0.0f;
        for (int i = 0; i < l; ++i) tr += A[i * ld + i];
        misc[0] = fmaxf(tr / (float)l, 1e-30f) * 1e-10f;
    }
    __syncthreads();
    const float floor_pivot = misc[0];
    for (int j = 0; j < l; ++j) {
        if (tid == 0) {
            const float d = sqrtf(fmaxf(A[j * ld + j], floor_pivot));
            A[j * ld + j] = d;
            dinv[j] = 1.0f / d;
        }
        __syncthreads();
        const float dj = dinv[j];
        for (int i = j + 1 + tid; i < l; i += kSmallThreads) A[i * ld + j] *= dj;
        __syncthreads();
        const int w = l - j - 1;
        for (int e = tid; e < w * w; e += kSmallThreads) {
            const int i = j + 1 + e / w, k = j + 1 + e % w;
            if (k <= i) A[i * ld + k] -= A[i * ld + j] * A[k * ld + j];
        }
        __syncthreads();
    }
    // column j of L^-1 by forward substitution, one thread per column; x_i (i > j) is kept at A[j][i]
    for (int j = tid; j < l; j += kSmallThreads) {
        for (int i = j + 1; i < l; ++i) {
            float a = A[i * ld + j] * dinv[j];
            for (int k = j + 1; k < i; ++k) a += A[i * ld + k] * A[j * ld + k];
            A[j * ld + i] = -a * dinv[i];
        }
    }
    __syncthreads();
    // Rinv[k][j] = (L^-1)[j][k] for j >= k
    for (int e = tid; e < l * l; e += kSmallThreads) {
        const int k = e / l, j = e % l;
        Rinv[e] = j > k ? A[k * ld + j] : (j == k ? dinv[k] : 0.0f);
    }
}

// Gm [l x l] symmetric (B B^T) = Ub diag(lambda) Ub^T by cyclic Jacobi rotations, l / 2 disjoint
// pairs per step in round-robin order, at most `sweeps` sweeps (fewer when a sweep finds nothing to
// rotate, which a warm-started basis reaches quickly).  With sigma = sqrt(lambda) sorted descending it writes
//   Mx [l x r] = Ub_r sigma_r^(1/2),  Vm [r x l] = sigma_r^(-1/2) Ub_r^T,  Wm [l x l] = sigma^-1 Ub^T
// (rows of Vm and Wm whose sigma is negligible are zero) and sigma itself.
__global__ __launch_bounds__(kSmallThreads) void jacobi_factors_kernel(const float* __restrict__ Gm, int l, int r, int sweeps,
                                                                       float* __restrict__ Mx, float* __restrict__ Vm,
                                                                       float* __restrict__ Wm, float* __restrict__ sigma) {
    extern __shared__ float lds[];
    const int ld = l + 1;
    float* A = lds;                        // [l][ld]
    float* E = lds + l * ld;               // eigenvectors in columns
    __shared__ float cs[kSketchMax / 2 + 1][2];
    __shared__ int pq[kSketchMax / 2 + 1][2];
    __shared__ float lam[kSketchMax];
    __shared__ int place[kSketchMax];
    const int tid = threadIdx.x;
    for (int e = tid; e < l * l; e += kSmallThreads) {
        const int i = e / l, j = e % l;
        A[i * ld + j] = 0.5f * (Gm[e] + Gm[j * l + i]);
        E[i * ld + j] = i == j ? 1.0f : 0.0f;
    }
    __syncthreads();
    const int n = (l + 1) & ~1;            // players of the round-robin; player l (if l is odd) sits out
    const int half = n / 2;
    __shared__ int rotated;
    for (int sweep = 0; sweep < sweeps; ++sweep) {
        if (tid == 0) rotated = 0;
        __syncthreads();
        for (int step = 0; step < n - 1; ++step) {
            if (tid < half) {
                const int a = tid == 0 ? 0 : 1 + (tid - 1 + step) % (n - 1);
                const int bq = n - 1 - tid;
                const int b = 1 + (bq - 1 + step) % (n - 1);
                int p = min(a, b), q = max(a, b);
                float c = 1.0f, s = 0.0f;
                if (q < l) {
                    const float apq = A[p * ld + q];
                    const float app = A[p * ld + p], aqq = A[q * ld + q];
                    if (fabsf(apq) > 1e-30f && fabsf(apq) > 6e-8f * sqrtf(fabsf(app * aqq))) {
                        rotated = 1;
                        const float tau = (aqq - app) / (2.0f * apq);
                        const float t = copysignf(1.0f, tau) / (fabsf(tau) + sqrtf(1.0f + tau * tau));
                        c = 1.0f / sqrtf(1.0f + t * t);
                        s = t * c;
                    }
                } else {
                    q = -1;
                }
                cs[tid][0] = c; cs[tid][1] = s;
                pq[tid][0] = p; pq[tid][1] = q;
            }
            __syncthreads();
            // columns: A <- A J, E <- E J
            for (int e = tid; e < half * l; e += kSmallThreads) {
                const int m = e / l, i = e % l;
                const int p = pq[m][0], q = pq[m][1];
                if (q < 0) continue;
                const float c = cs[m][0], s = cs[m][1];
                const float ap = A[i * ld + p], aq = A[i * ld + q];
                A[i * ld + p] = c * ap - s * aq;
                A[i * ld + q] = s * ap + c * aq;
                const float ep = E[i * ld + p], eq = E[i * ld + q];
                E[i * ld + p] = c * ep - s * eq;
                E[i * ld + q] = s * ep + c * eq;
            }
            __syncthreads();
            // rows: A <- J^T A
            for (int e = tid; e < half * l; e += kSmallThreads) {
                const int m = e / l, j = e % l;
                const int p = pq[m][0], q = pq[m][1];
                if (q < 0) continue;
                const float c = cs[m][0], s = cs[m][1];
                const float ap = A[p * ld + j], aq = A[q * ld + j];
                A[p * ld + j] = c * ap - s * aq;
                A[q * ld + j] = s * ap + c * aq;
            }
            __syncthreads();
        }
        if (rotated == 0) break;       // a whole sweep without a rotation: diagonal to working precision
        __syncthreads();
    }
    // order: place[i] = position of eigenvalue i in descending order
    for (int i = tid; i < l; i += kSmallThreads) lam[i] = A[i * ld + i];
    __syncthreads();
    for (int i = tid; i < l; i += kSmallThreads) {
        int pos = 0;
        for (int j = 0; j < l; ++j) pos += (lam[j] > lam[i] || (lam[j] == lam[i] && j < i)) ? 1 : 0;
        place[i] = pos;
    }
    __syncthreads();
    __shared__ float top;
    if (tid == 0) {
        float t = 0.0f;
        for (int i = 0; i < l; ++i) t = fmaxf(t, lam[i]);
        top = sqrtf(fmaxf(t, 0.0f));
    }
    __syncthreads();
    for (int e = tid; e < l * l; e += kSmallThreads) {
        const int i = e / l, c = e % l;          // eigenvector c (unsorted), component i
        const int k = place[c];
        const float sg = sqrtf(fmaxf(lam[c], 0.0f));
        const bool live = sg > 1e-7f * top && sg > 0.0f;
        const float u = E[i * ld + c];
        Wm[k * l + i] = live ? u / sg : 0.0f;
        if (k < r) {
            const float h = sqrtf(sg);
            Mx[i * r + k] = u * h;
            Vm[k * l + i] = live ? u / h : 0.0f;
        }
        if (i == 0) sigma[k] = sg;
    }
}

// ------------------------------------------------------------------ host side
struct CompressLayout {
    int l;                         // width of the sketch
    size_t RE, s, z, Vb, Bm, Y, Q, Gm, Rinv, Mx, Vm, Wm, sigma, parts, partial, eps2, total;
    int64_t parts_floats;
};

static int sgemm_splits(int M, int N, int Kd) {
    const int64_t tiles = (int64_t)((M + 63) / 64) * ((N + 63) / 64);
    if (tiles >= 256) return 1;
    int64_t s = (512 + tiles - 1) / tiles;
    if (s > Kd / 256) s = Kd / 256;
    if (s > 64) s = 64;
    return s < 1 ? 1 : (int)s;
}

static CompressLayout compress_layout(int64_t N, int64_t K, int r) {
    CompressLayout L{};
    int64_t l = (int64_t)r + kSketchExtra;
    if (l > N) l = N;
    if (l > K) l = K;
    if (r == 0) l = 0;
    L.l = (int)l;
    const int64_t G = K / kGroup;
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes, 256); return o; };
    L.RE = take((size_t)N * K * 4);
    L.s = take((size_t)N * G * 4);
    L.z = take((size_t)N * G * 4);
    L.Vb = take((size_t)l * K * 4);
    L.Bm = take((size_t)l * K * 4);
    L.Y = take((size_t)N * l * 4);
    L.Q = take((size_t)N * l * 4);
    L.Gm = take((size_t)l * l * 4);
    L.Rinv = take((size_t)l * l * 4);
    L.Mx = take((size_t)l * (r > 0 ? r : 1) * 4);
    L.Vm = take((size_t)l * (r > 0 ? r : 1) * 4);
    L.Wm = take((size_t)l * l * 4);
    L.sigma = take((size_t)(l > 0 ? l : 1) * 4);
    int64_t pf = 1;
    if (l > 0) {
        auto need = [&](int M_, int N_, int Kd_) {
            const int S = sgemm_splits(M_, N_, Kd_);
            if (S > 1 && (int64_t)S * M_ * N_ > pf) pf = (int64_t)S * M_ * N_;
        };
        need((int)N, (int)l, (int)K);        // Y = E Vb^T
        need((int)l, (int)K, (int)N);        // B = Q^T E
        need((int)l, (int)l, (int)N);        // Y^T Y
        need((int)l, (int)l, (int)K);        // B B^T
        need((int)N, (int)l, (int)l);
        need((int)N, (int)(r > 0 ? r : 1), (int)l);
        need((int)l, (int)K, (int)l);
    }
    L.parts_floats = pf;
    L.parts = take((size_t)pf * 4);
    L.partial = take((size_t)((N + 63) / 64) * (K / 64) * 8);
    L.eps2 = take(8);
    L.total = at;
    return L;
}

static bool compress_shape_ok(int64_t N, int64_t K) {
    return weight_shape_ok(N, K) && N < (int64_t(1) << 24) && K < (int64_t(1) << 24);
}

// C = A B through the strided kernel, split over the reduction when the output has few tiles.
static void sgemm(const float* A, int64_t sai, int64_t sak, const float* B, int64_t sbk, int64_t sbj, float* C, int64_t ldc,
                  int M, int N, int Kd, float* parts, hipStream_t st) {
    const int S = sgemm_splits(M, N, Kd);
    SgemmArgs g{A, sai, sak, B, sbk, sbj, C, ldc, 0, M, N, Kd, Kd};
    const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64), (unsigned)S);
    if (S == 1) {
        sgemm_kernel<<<grid, dim3(256), 0, st>>>(g);
        return;
    }
    g.kchunk = ((Kd + S - 1) / S + 15) / 16 * 16;
    g.C = parts;
    g.ldc = N;
    g.part_stride = (int64_t)M * N;
    sgemm_kernel<<<grid, dim3(256), 0, st>>>(g);
    const int64_t count = (int64_t)M * N;
    sum_parts_kernel<<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st>>>(parts, S, g.part_stride, M, N, C, ldc);
}

// Sliding-mean stop rule of Eq. stop_condition on the errors so far (the mean of the last three, or of
// as many as there are, against the same mean one iteration earlier).
static bool stop_rule(const double* eps, int count, double tol) {
    if (count < 2) return false;
    auto mean = [&](int lo, int hi) {      // [lo, hi)
        double a = 0.0;
        for (int i = lo; i < hi; ++i) a += eps[i];
        return a / (double)(hi - lo);
    };
    const double cur = mean(count >= 3 ? count - 3 : 0, count);
    const double prev = count >= 4 ? mean(count - 4, count - 1) : mean(0, count - 1);
    return (prev - cur) / prev < tol;
}

}  // namespace milo

using namespace milo;

extern "C" size_t milo_compress_w3lr_workspace(int64_t N, int64_t K, int r) {
    if (!compress_shape_ok(N, K) || r < 0 || r > MILO_COMPRESS_MAX_RANK || r > N || r > K) return 0;
    return compress_layout(N, K, r).total;
}

extern "C" int milo_compress_w3lr(const float* W, int64_t N, int64_t K, const milo_compress_params* prm, void* q3, float* U,
                                  float* V, double* eps, int* iters_run, void* workspace, size_t workspace_bytes,
                                  void* stream) {
    if (!W || !prm || !q3 || !workspace || !eps || !iters_run) return MILO_ERR_NULL;
    const int r = prm->rank;
    if (r < 0 || r > MILO_COMPRESS_MAX_RANK || r > N || r > K) return MILO_ERR_RANK;
    if (r > 0 && (!U || !V)) return MILO_ERR_NULL;
    if (!compress_shape_ok(N, K)) return MILO_ERR_SHAPE;
    if (prm->iters < 1 || prm->hqq_iters < 0 || prm->power_iters < 0 || prm->refine_iters < 0 || !(prm->p > 0.0f && prm->p < 1.0f) ||
        !(prm->beta > 0.0f) || !(prm->kappa > 0.0f))
        return MILO_ERR_SHAPE;
    if (!aligned16(W) || !aligned16(q3) || !aligned16(workspace) || (r > 0 && (!aligned16(U) || !aligned16(V))))
        return MILO_ERR_ALIGN;
    const CompressLayout L = compress_layout(N, K, r);
    if (workspace_bytes < L.total) return MILO_ERR_WORKSPACE;

    hipStream_t st = (hipStream_t)stream;
    char* ws = reinterpret_cast<char*>(workspace);
    float* RE = reinterpret_cast<float*>(ws + L.RE);
    float* s = reinterpret_cast<float*>(ws + L.s);
    float* z = reinterpret_cast<float*>(ws + L.z);
    float* Vb = reinterpret_cast<float*>(ws + L.Vb);
    float* Bm = reinterpret_cast<float*>(ws + L.Bm);
    float* Y = reinterpret_cast<float*>(ws + L.Y);
    float* Q = reinterpret_cast<float*>(ws + L.Q);
    float* Gm = reinterpret_cast<float*>(ws + L.Gm);
    float* Rinv = reinterpret_cast<float*>(ws + L.Rinv);
    float* Mx = reinterpret_cast<float*>(ws + L.Mx);
    float* Vm = reinterpret_cast<float*>(ws + L.Vm);
    float* Wm = reinterpret_cast<float*>(ws + L.Wm);
    float* sigma = reinterpret_cast<float*>(ws + L.sigma);
    float* parts = reinterpret_cast<float*>(ws + L.parts);
    double* partial = reinterpret_cast<double*>(ws + L.partial);
    double* eps2 = reinterpret_cast<double*>(ws + L.eps2);

    const int l = L.l;
    const int64_t units = N * (K / kGroup);
    const unsigned unit_blocks = (unsigned)((units + kUnitsPerBlock - 1) / kUnitsPerBlock);
    const dim3 tiles((unsigned)(K / 64), (unsigned)((N + 63) / 64));
    const int64_t ntiles = (int64_t)tiles.x * tiles.y;
    const size_t small_lds = ((size_t)2 * l * (l + 1) + 2 * l + 16) * sizeof(float);
    if (l > 0) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(&cholesky_inverse_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)small_lds) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void*>(&jacobi_factors_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)small_lds) != hipSuccess)
            return MILO_ERR_HIP;
    }

    group_params_kernel<<<dim3(unit_blocks), dim3(kPackThreads), 0, st>>>(W, N, K, s, z);
    if (l > 0) {
        const int64_t count = (int64_t)l * K;
        random_basis_kernel<<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st>>>(Vb, count, prm->seed);
    }
    *iters_run = 0;
    for (int t = 0; t < prm->iters; ++t) {
        // R = W - U V (the first target is W itself)
        resid_kernel<0><<<tiles, dim3(256), 0, st>>>(W, U, V, t == 0 ? 0 : r, N, K, RE, nullptr);
        hqq_kernel<<<dim3(unit_blocks), dim3(kPackThreads), 0, st>>>(W, RE, s, z, units, prm->hqq_iters, prm->p - 1.0f,
                                                                    prm->beta, prm->kappa);
        if (r > 0) {
            const int rounds = 1 + (t == 0 ? prm->power_iters : prm->refine_iters);
            for (int it = 0; it < rounds; ++it) {
                sgemm(RE, K, 1, Vb, 1, K, Y, l, (int)N, l, (int)K, parts, st);              // Y = E Vb^T
                sgemm(Y, 1, l, Y, l, 1, Gm, l, l, l, (int)N, parts, st);                     // Y^T Y
                cholesky_inverse_kernel<<<dim3(1), dim3(kSmallThreads), small_lds, st>>>(Gm, l, Rinv);
                sgemm(Y, l, 1, Rinv, l, 1, Q, l, (int)N, l, l, parts, st);                   // Q = Y R^-1
                sgemm(Q, 1, l, RE, K, 1, Bm, K, l, (int)K, (int)N, parts, st);               // B = Q^T E
                sgemm(Bm, K, 1, Bm, 1, K, Gm, l, l, l, (int)K, parts, st);                   // B B^T
                jacobi_factors_kernel<<<dim3(1), dim3(kSmallThreads), small_lds, st>>>(Gm, l, r, 12, Mx, Vm, Wm, sigma);
                sgemm(Wm, l, 1, Bm, K, 1, Vb, K, l, (int)K, l, parts, st);                   // next basis
            }
            sgemm(Q, l, 1, Mx, r, 1, U, r, (int)N, r, l, parts, st);                         // U = Q Ub_r S_r^(1/2)
            sgemm(Vm, l, 1, Bm, K, 1, V, K, r, (int)K, l, parts, st);                        // V = S_r^(-1/2) Ub_r^T B
        }
        resid_kernel<1><<<tiles, dim3(256), 0, st>>>(RE, U, V, r, N, K, nullptr, partial);
        sum_partials_kernel<<<dim3(1), dim3(256), 0, st>>>(partial, ntiles, eps2);
        double e2 = 0.0;
        if (hipMemcpyAsync(&e2, eps2, sizeof(double), hipMemcpyDeviceToHost, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)
            return MILO_ERR_HIP;
        eps[t] = sqrt(e2);
        *iters_run = t + 1;
        if (!(eps[t] == eps[t])) break;                                   // not a number: nothing more to gain
        if (prm->tol >= 0.0f && stop_rule(eps, t + 1, (double)prm->tol)) break;
    }
    // the stored format: target W - U V, fixed scales, z rounded to fp16
    resid_kernel<0><<<tiles, dim3(256), 0, st>>>(W, U, V, r, N, K, RE, nullptr);
    uint32_t* planeA = reinterpret_cast<uint32_t*>(q3);
    uint32_t* planeB = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(q3) + (N * K) / 4);
    pack_given_kernel<<<dim3(unit_blocks), dim3(kPackThreads), 0, st>>>(RE, s, z, N, K, planeA, planeB);
    return launch_status();
}
