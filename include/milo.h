/*
 * milo.h — C ABI of the MI355X-native W3A16 + low-rank expert linear
 * (inference hot path of MiLo, arXiv 2504.02658).
 *
 * What the library computes (paper Section 3.1.2, compensated weight
 * W~ = Q^-1(W_q) + U V, and Section 3.2, Eq. wq / wdq):
 *
 *      Y = X * dequant(Q3)^T + (X * V^T) * U^T
 *
 *   X  [M x K]  fp16 activations, row-major
 *   W  [N x K]  weight (out x in); the Q3 blob holds its 3-bit codes q in 0..7 and
 *               one fp16 scale s and one fp16 zero-point z per group of 64
 *               consecutive k of a row:  W_dq[n,k] = s[n,g] * (q[n,k] - z[n,g])
 *   U  [N x r], V [r x K]  fp16 low-rank compensator of rank r (r may be 0)
 *   Y  [M x N]  fp16, row-major; accumulation is fp32, one rounding at the end.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller unless the
 *     argument comment says "host".  The library never frees or keeps a pointer
 *     and allocates nothing: scratch memory comes in through `workspace`.
 *   - fp16 values are IEEE binary16 bit patterns (`milo_half` = uint16_t).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All calls only enqueue work on that stream and return without waiting.
 *   - Every call returns a milo_status (0 = OK).  Argument errors are detected
 *     on the host before anything is launched; the library never aborts.
 *   - Shapes: K % 64 == 0, N % 16 == 0, M >= 1, group size must be 64
 *     (the only group size of the paper's kernel, appendix "Correctness Test").
 *   - Pointers must be 16-byte aligned; inputs and outputs must not alias.
 *
 * Packed format ("Q3 blob": exactly 3 bits per weight for the codes, Section 3.3 "Zero bit
 * waste 3-bit weights packing", plus the two fp16 parameters of every group of 64, i.e. 28 bytes
 * per group = 3.5 bits per weight in total; the concrete layout is this library's own):
 *   - unit(n, g) = the 64 codes of row n, group g, with its scale and zero-point; units are ordered
 *         u = ((n / 16) * (K / 64) + g) * 16 + n % 16
 *   - the codes of a unit are six little-endian 32-bit words d0..d5; plane A (first N*K/4 bytes of
 *     the blob) stores d0..d3 of unit u at byte 16u, plane B (the next 3*N*K/16 bytes) stores at
 *     byte 12u the three words d4, d5, p, where p = scale bits | zero-point bits << 16 (both
 *     IEEE binary16)
 *   - the unit's codes form pairs P = (q[2P], q[2P+1]) = (lo, hi); for P < 30,
 *     word j = P / 5, slot c = P % 5: lo in bits 3c..3c+2, hi in bits
 *     16+3c..16+3c+2; bits 15 and 31 of words 0,1,2 carry bits 0,1,2 of pair 30
 *     (lo in bit 15, hi in bit 31), those of words 3,4,5 carry pair 31.
 *   A kernel lane fetches a whole unit with one 16-byte and one 12-byte load.
 */
#ifndef MILO_H
#define MILO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t milo_half;

enum milo_status {
    MILO_OK = 0,
    MILO_ERR_NULL = 1,       /* a required pointer is NULL                                  */
    MILO_ERR_SHAPE = 2,      /* K % 64, N % 16, M < 1, a size overflows (N*K/64 > 2^26, K > 2^26, an
                                array the kernels address with 32-bit offsets), bad top-k / E */
    MILO_ERR_GROUP = 3,      /* group_size != 64                                            */
    MILO_ERR_RANK = 4,       /* r < 0, r > min(N, K), or r > 0 with U or V NULL             */
    MILO_ERR_WORKSPACE = 5,  /* workspace NULL or smaller than the *_workspace() size       */
    MILO_ERR_ROUTING = 6,    /* an expert id outside 0..E-1 was met (reported after the run)*/
    MILO_ERR_ALIGN = 7,      /* a pointer is not 16-byte aligned                            */
    MILO_ERR_WAIT = 8,       /* a bounded wait inside a kernel gave up (see milo_workspace_status) */
    MILO_ERR_HIP = 100       /* a HIP runtime call failed (launch error, no device, ...)    */
};

/* Static text for a status code; never NULL. */
const char* milo_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
int milo_version(void);

/* Bytes of the Q3 blob of an [N x K] weight: exactly N*K*7/16 (0 if the shape is invalid). */
size_t milo_w3_packed_bytes(int64_t N, int64_t K);

/*
 * Quantize and pack (Section 3.2 Eq. wq with U = V = 0, round-to-nearest; Section 3.3).
 * Per group: s = fp16((max - min) / 7), z = round(-min / s), q = clamp(round(w / s + z), 0, 7),
 * all in binary32 with round-half-even and no fused multiply-add; a group whose fp16 scale is
 * zero or not finite stores s = 1, z = fp16(-min), q = 0.
 *   W       [N x K] fp32 row-major (device, read only)
 *   q3      out, milo_w3_packed_bytes(N, K) bytes (codes, scales and zero-points)
 * Errors: NULL, SHAPE, GROUP, ALIGN, HIP.
 */
int milo_pack_w3(const float* W, int64_t N, int64_t K, int group_size, void* q3, void* stream);

/*
 * The same with the symmetric INT3 quantizer (Section 3.2.3, Eq. symm_int3: q = round(7 w / (2 s))
 * + 4 with s the largest magnitude of the group).  The blob has the same layout and is used by the
 * same GEMM entry points: its scale word holds the step d = fp16(2 s / 7) and its zero word 4, so
 * that dequantization is d * (q - 4).  Codes are computed with the stored step, q = clamp(round(w /
 * d) + 4, 0, 7), in binary32 with round-half-even; the clamp is needed because w = +s maps to 8.
 * A group whose fp16 step is zero or not finite stores d = 1, q = 4 (dequantizes to 0).
 * Arguments and errors as milo_pack_w3.
 */
int milo_pack_w3_sym(const float* W, int64_t N, int64_t K, int group_size, void* q3, void* stream);

/*
 * Test aid: the parts of a Q3 blob.  codes[n*K + k] = q[n,k] as bytes; scales and zeros
 * [N x K/64] fp16 row-major.  Each output may be NULL (not all three).
 */
int milo_unpack_w3(const void* q3, int64_t N, int64_t K, uint8_t* codes, milo_half* scales,
                   milo_half* zeros, void* stream);

/*
 * Dequantize a packed weight to dense fp16 (Eq. wdq), W_dq [N x K] row-major, with the same
 * in-register conversion the GEMM kernels use.  Used to build the residual W - W_dq that the
 * compensator is fitted to, and by the tests.
 */
int milo_dequant_w3(const void* q3, int64_t N, int64_t K, milo_half* W_dq, void* stream);

/*
 * Prepare a freshly allocated workspace (for milo_w3lr_gemm or milo_moe_w3lr_forward): zero-fills
 * all `workspace_bytes` with a small fill kernel on `stream` (the kernels synchronise through
 * counters and flags in it that must start at zero).  Call it once after allocating the workspace
 * and again after a call on it returned an error or milo_workspace_status reported MILO_ERR_WAIT;
 * the kernels leave their counters and flags cleared when they finish, so successive calls need no
 * further preparation and no memset (which makes them safe to capture in a HIP graph and replay).
 * Errors: NULL, WORKSPACE (fewer than 256 bytes), ALIGN, HIP.
 */
int milo_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/*
 * Waits for `stream`, then reports whether a kernel that used this workspace (of milo_w3lr_gemm or
 * of milo_moe_w3lr_forward) gave up a wait.  The kernels hand T = X V^T from the workgroups that form
 * it to the ones that use it inside one launch; the consumers' wait is bounded (about a second), and
 * one that runs out sets a word in the control block and goes on with whatever T holds, so the
 * output of that call is not to be used.  This needs the whole launch to make progress together: the
 * launches are sized for an otherwise idle device, and the producers have the lowest workgroup ids,
 * which the hardware dispatches first; a device kept busy by other streams' kernels can break that.
 * MILO_ERR_WAIT: discard the outputs written since the last MILO_OK and call milo_workspace_init
 * before the next use (a GEMM workspace keeps the word until then; the MoE call clears its own at
 * the start of every forward, so there the status refers to the last forward).
 * Errors: NULL, ALIGN, WAIT, HIP.
 */
int milo_workspace_status(const void* workspace, void* stream);

/*
 * One compensated W3A16 linear:  Y = X dequant(Q3)^T + (X V^T) U^T.
 *   X [M x K] fp16;  q3 as written by milo_pack_w3 (its zero-points may be any finite fp16,
 *   integer or not);  U [N x r], V [r x K] fp16 row-major, ignored when r == 0;  Y [M x N] fp16.
 *   workspace: at least milo_w3lr_gemm_workspace(M, N, K, r) bytes of device memory, prepared
 *   once with milo_workspace_init; beyond the control block its contents are scratch.  Calls that
 *   share a workspace must be ordered on one stream (concurrent calls would race on it).
 * M <= 16 takes the weight-streaming decode kernel (a single launch that also forms X V^T),
 * larger M the tiled MFMA kernel (which also forms X V^T inside the launch; when the problem has
 * too few tiles to fill the device it splits K over workgroups and a second small kernel adds the
 * fp32 partial sums in a fixed order, so the result is rounded once and two runs agree bit for bit).
 * The workspace size depends on the device the call is made on (the K split follows its number of
 * compute units): query it with that device current.
 * Errors: NULL, SHAPE, RANK, WORKSPACE, ALIGN, HIP.
 */
size_t milo_w3lr_gemm_workspace(int64_t M, int64_t N, int64_t K, int r);
int milo_w3lr_gemm(const milo_half* X, int64_t M, int64_t N, int64_t K,
                   const void* q3, const milo_half* U, const milo_half* V, int r,
                   milo_half* Y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same with weight flags (see above): `U` and `V` are fp16 arrays, or with MILO_LR_INT3 the two
 * blobs of milo_pack_lr3.  milo_w3lr_gemm is this call with flags = 0.
 * Errors: as milo_w3lr_gemm; RANK also for MILO_LR_INT3 with r > MILO_LR3_MAX_RANK, SHAPE for
 * MILO_LR_INT3 with N % 64 != 0 or unknown flag bits.
 */
int milo_w3lr_gemm_flags(const milo_half* X, int64_t M, int64_t N, int64_t K,
                         const void* q3, const void* U, const void* V, int r, unsigned flags,
                         milo_half* Y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * INT3 compensator (Section 3.2.3, Eq. symm_int3; Algorithm 1's output step "Quantize U, V").
 * Both factors are quantized with the symmetric INT3 quantizer of milo_pack_w3_sym in groups of 64
 * along their long dimension: U [N x r] along N (64 consecutive output features of one rank share a
 * step), V [r x K] along K.  The blobs have the Q3 layout described at the top of this file, of the
 * matrices U^T [rp x N] and V [rp x K] with rp = r rounded up to a multiple of 16 (the added rows are
 * zero): 3.5 bits per element of the compensator instead of 16.  The kernels dequantize them like
 * weights (one fp16 rounding per element) while they form X V^T and add T U^T.
 *   U [N x r], V [r x K]  fp32 row-major (device, read only)
 *   u3, v3                out, *u_bytes and *v_bytes of milo_lr3_packed_bytes(N, K, r, ..)
 * Errors: NULL, SHAPE (also N % 64 != 0), RANK (r < 1 or r > MILO_LR3_MAX_RANK), ALIGN, HIP.
 */
int milo_lr3_packed_bytes(int64_t N, int64_t K, int r, size_t* u_bytes, size_t* v_bytes);
int milo_pack_lr3(const float* U, const float* V, int64_t N, int64_t K, int r,
                  void* u3, void* v3, void* stream);

/*
 * The MiLo compression loop (Algorithm 1) for one weight: alternates a quantization step and a
 * compensation step until the error stops improving, and writes the Q3 blob and the compensator.
 *   quantization step (Section 3.2, Eq. update_We, Eq. update_z): target R = W - U V, scales fixed to
 *       the round-to-nearest scales of W (fp16((max - min) / 7) per group of 64, as milo_pack_w3),
 *       `hqq_iters` half-quadratic updates of the real-valued zero-points with the l_p shrinkage
 *       operator (norm `p` < 1, penalty `beta` growing by the factor `kappa` per update);
 *   compensation step (Eq. UV): rank-r truncated SVD of E = W - W_dq, U = U^ S^(1/2), V = S^(1/2) V^.
 *       The leading triplets come from a block subspace iteration with r + 8 vectors, warm-started
 *       from the previous iteration's right singular vectors: one round per iteration plus
 *       `power_iters` extra rounds in the first iteration (which starts from a basis seeded by `seed`)
 *       and `refine_iters` extra rounds in every later one.  Close to, not equal to, the exact
 *       truncation: with the defaults of the Python binding (2 and 0) eps_t ends within about one
 *       percent of the exact SVD's on small matrices and closer on large ones; more rounds close the gap;
 *   error eps_t = ||W - W_dq - U V||_F (Eq. epsilon), copied to the host after every iteration; the
 *       loop ends after `iters` iterations or when (mean of the last three errors so far) has
 *       improved by less than the fraction `tol` over the same mean one iteration earlier
 *       (Eq. stop_condition; a negative tol disables the rule).
 * Output: q3 = codes of W - U V with those scales and the zero-points rounded to fp16 (any finite
 * fp16, not integers), in the layout of milo_pack_w3; U [N x r], V [r x K] fp32 row-major (round them
 * to fp16, or pass them to milo_pack_lr3 for Algorithm 1's last line "Quantize U, V").
 *   W [N x K]      fp32 row-major (device, read only)
 *   params         host pointer
 *   q3             out, device, milo_w3_packed_bytes(N, K) bytes
 *   U, V           out, device; may be NULL when rank == 0
 *   eps            out, HOST array of at least params->iters doubles: eps_t of the iterations run
 *   iters_run      out, HOST: how many iterations ran
 *   workspace      device, at least milo_compress_w3lr_workspace(N, K, rank) bytes (about 1.1 N K floats),
 *                  scratch; no preparation needed
 * The call synchronizes `stream` once per iteration (the stop rule runs on the host), so it cannot be
 * captured in a graph; it is an offline tool, not part of the inference path.
 * Errors: NULL, SHAPE (also bad parameter values), RANK (rank < 0, > MILO_COMPRESS_MAX_RANK or
 * > min(N, K)), WORKSPACE, ALIGN, HIP.
 */
#define MILO_COMPRESS_MAX_RANK 128
typedef struct milo_compress_params {
    int32_t rank;            /* r */
    int32_t iters;           /* outer iterations at most, >= 1 (the paper stops at 20 at the latest) */
    int32_t hqq_iters;       /* zero-point updates per outer iteration, >= 0 */
    int32_t power_iters;     /* extra subspace rounds in the first outer iteration, >= 0 */
    int32_t refine_iters;    /* extra subspace rounds in every later outer iteration, >= 0 */
    float p;                 /* 0 < p < 1 */
    float beta;              /* > 0 */
    float kappa;             /* > 0 */
    float tol;               /* stop threshold; negative: run all `iters` iterations */
    uint32_t seed;
} milo_compress_params;
size_t milo_compress_w3lr_workspace(int64_t N, int64_t K, int rank);
int milo_compress_w3lr(const float* W, int64_t N, int64_t K, const milo_compress_params* params,
                       void* q3, float* U, float* V, double* eps, int* iters_run,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * milo_w3lr_gemm for callers that cannot allocate and cannot bring a workspace: code that runs
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * result and errors as milo_w3lr_gemm, bit for bit, without `workspace`: the scratch memory is a
 * fixed array of MILO_STATIC_SCRATCH_BYTES inside the library's device image (every GPU the library
 * runs on holds its copy until the process ends).  The call allocates nothing; a problem whose
 * milo_w3lr_gemm_workspace(M, N, K, r) exceeds MILO_STATIC_SCRATCH_BYTES is refused with
 * MILO_ERR_WORKSPACE (all decode shapes fit; large M with a K split may not).  The control words
 * of the array are cleared by a small fill kernel at the start of every call (no memset, so the call
 * can be captured), then the kernels of milo_w3lr_gemm run on it.  All calls on one GPU share that
 * GPU's array: calls that overlap in time on one GPU (different streams) race; order them.  The
 * array's device address is looked up on the first call on a device (make that call outside a
 * graph capture).  milo_workspace_status does not apply; a wait that gave up inside this call is
 * not reported.
 */
#define MILO_STATIC_SCRATCH_BYTES (4u << 20)
int milo_w3lr_gemm_static(const milo_half* X, int64_t M, int64_t N, int64_t K,
                          const void* q3, const milo_half* U, const milo_half* V, int r,
                          milo_half* Y, void* stream);

/*
 * Weight flags (the `flags` argument of milo_w3lr_gemm_flags and the `flags` field of milo_w3lr_weight).
 *   MILO_W3_SYMMETRIC  the Q3 blob was written by milo_pack_w3_sym, so every zero-point is 4: the
 *                      kernels may use the conversion without zero-point arithmetic (Section 3.3,
 *                      the symmetric kernel).  The result is the same bit for bit with or without
 *                      the flag; setting it on a blob that is not symmetric gives wrong results.
 *   MILO_LR_INT3       U and V are not fp16 arrays but the INT3 blobs written by milo_pack_lr3
 *                      (Section 3.2.3, "Quantized low-rank mixture compensators"; the last step of
 *                      Algorithm 1).  Needs r <= MILO_LR3_MAX_RANK and N % 64 == 0.
 *   MILO_ACT_BF16      (a call flag: milo_w3lr_gemm_flags, milo_moe_w3lr_forward_flags; not stored in a
 *                      weight) X, U, V and Y are bfloat16 instead of fp16: the weights are dequantized
 *                      to bf16 (one rounding each, computed in binary32) and multiplied on the bf16
 *                      matrix cores, accumulation stays fp32.  Cannot be combined with MILO_LR_INT3.
 */
#define MILO_W3_SYMMETRIC 1u
#define MILO_LR_INT3 2u
#define MILO_ACT_BF16 4u
#define MILO_LR3_MAX_RANK 128

/* One packed weight with its compensator (all device pointers). */
typedef struct milo_w3lr_weight {
    const void* q3;
    const void* U;           /* fp16 [N x r], or the U blob of milo_pack_lr3; NULL when r == 0 */
    const void* V;           /* fp16 [r x K], or the V blob of milo_pack_lr3; NULL when r == 0 */
    int32_t r;
    uint32_t flags;          /* MILO_W3_SYMMETRIC | MILO_LR_INT3, else 0 */
} milo_w3lr_weight;

/* A SwiGLU expert: w1, w3 are [F x H] (gate, up), w2 is [H x F] (down). */
typedef struct milo_w3lr_expert {
    milo_w3lr_weight w1, w3, w2;
} milo_w3lr_expert;

/*
 * Host-side validation of an expert table before it is copied to the device.
 *   experts  HOST array of E entries;  r_max_out (host, may be NULL) receives the largest rank.
 * Errors: NULL, SHAPE, RANK, ALIGN.
 */
int milo_moe_w3lr_check_experts(const milo_w3lr_expert* experts, int E, int64_t H, int64_t F,
                                int* r_max_out);
/* The same for a table that will be used with call flags (MILO_ACT_BF16: the compensators are bf16
 * arrays, and no weight may carry MILO_LR_INT3).  Errors: as above; SHAPE also for unknown flags. */
int milo_moe_w3lr_check_experts_flags(const milo_w3lr_expert* experts, int E, int64_t H, int64_t F,
                                      unsigned flags, int* r_max_out);

/*
 * Top-k routed MoE feed-forward layer over compensated W3A16 experts:
 *     y_t = sum_j gates[t,j] * lin_w2^e( SiLU(lin_w1^e(x_t)) * lin_w3^e(x_t) ),   e = ids[t,j]
 * with SiLU(a) = a / (1 + exp(-a)) and every lin the compensated linear above.  Tokens are
 * grouped per expert inside the call; the router (gate GEMM, softmax, top-k) is the caller's.
 * Always-on shared experts are passed as extra routing columns with weight 1.
 *   X            [T x H] fp16
 *   experts      DEVICE array of E entries (a byte copy of a host table that passed
 *                milo_moe_w3lr_check_experts);  r_max = largest rank in the table
 *   topk_ids     [T x topk] int32, the ids of one token must be distinct
 *   topk_weights [T x topk] fp32
 *   Y            [T x H] fp16
 *   workspace    at least milo_moe_w3lr_workspace(T, H, F, E, topk, r_max) bytes
 * An id outside 0..E-1 contributes nothing and raises a flag that
 * milo_moe_w3lr_routing_status() reports; an expert with no tokens is legal.
 * Each routed pair's weighted expert output is kept as fp16 (per K split of the down projection,
 * when that is split); the combine adds a token's slots (and splits) in a fixed order in fp32 and
 * rounds once, so two runs give bit-identical results.
 * Errors: NULL, SHAPE, RANK, WORKSPACE, ALIGN, HIP.
 */
size_t milo_moe_w3lr_workspace(int64_t T, int64_t H, int64_t F, int E, int topk, int r_max);
int milo_moe_w3lr_forward(const milo_half* X, int64_t T, int64_t H, int64_t F,
                          const milo_w3lr_expert* experts, int E, int r_max,
                          const int32_t* topk_ids, const float* topk_weights, int topk,
                          milo_half* Y, void* workspace, size_t workspace_bytes, void* stream);
/*
 * The same with call flags: 0, or MILO_ACT_BF16 for bfloat16 X, Y and compensators (the intermediate
 * SwiGLU output and the per-pair expert outputs are bfloat16 too).  The expert table must have passed
 * milo_moe_w3lr_check_experts_flags with the same flags.  milo_moe_w3lr_forward is this call with flags 0.
 * Errors: as milo_moe_w3lr_forward; SHAPE also for unknown flags.
 */
int milo_moe_w3lr_forward_flags(const milo_half* X, int64_t T, int64_t H, int64_t F,
                                const milo_w3lr_expert* experts, int E, int r_max,
                                const int32_t* topk_ids, const float* topk_weights, int topk,
                                unsigned flags, milo_half* Y, void* workspace, size_t workspace_bytes,
                                void* stream);

/*
 * Waits for `stream` and returns MILO_ERR_ROUTING if the last milo_moe_w3lr_forward that used
 * this workspace met an expert id out of range, MILO_ERR_WAIT if a wait inside it gave up (see
 * milo_workspace_status), MILO_OK otherwise.
 */
int milo_moe_w3lr_routing_status(const void* workspace, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MILO_H */
