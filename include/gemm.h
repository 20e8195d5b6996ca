/*
 * libgemm -- dense GEMM with a fused epilogue for AMD Instinct MI355X (gfx950).
 *
 *     C = act( alpha * op(A) * op(B) + beta * C + bias )
 *
 * This is the operation whose hand-optimised kernels the paper studies in its GEMM case
 * study (Section 5.4, Table 1: matrix-core use, tiling, vectorised access, padding or
 * swizzled shared-memory layouts, thread-block swizzle, double buffering).  The paper
 * never writes the formula; the plain BLAS statement above is what every call computes.
 *
 * Storage is ROW-MAJOR with explicit leading dimensions (in elements):
 *   transA = GEMM_OP_N : A is M x K, op(A)(i,k) = A[i*lda + k], lda >= K
 *   transA = GEMM_OP_T : A is stored K x M, op(A)(i,k) = A[k*lda + i], lda >= M
 *   transB = GEMM_OP_N : B is K x N, op(B)(k,j) = B[k*ldb + j], ldb >= N
 *   transB = GEMM_OP_T : B is stored N x K ("column-major B"), op(B)(k,j) = B[j*ldb + k], ldb >= K
 *   C is M x N, C(i,j) = C[i*ldc + j], ldc >= N.
 * Products are accumulated in fp32 (bf16 x bf16 and fp16 x fp16 products are exact), the
 * epilogue runs in fp32, and the result is rounded once, to nearest-even, into the type of C.
 * IEEE special values behave as in that arithmetic: subnormal inputs are multiplied (not flushed
 * to zero), fp32 results below the normal range stay subnormal, a result beyond the largest
 * finite value of the type of C becomes an infinity, Inf times zero is a NaN.
 *
 * All matrix and bias pointers are DEVICE pointers owned by the caller; the library never
 * allocates, frees or retains them.  gemm_run is asynchronous: it enqueues work on the given
 * HIP stream and returns without synchronising, in every case.  The one thing it may do besides
 * launching kernels is grow the handle's split-K workspace with hipMalloc (see gemm_create and
 * gemm_reserve_workspace); it never frees device memory.  Nothing here throws, aborts or prints.
 */
#ifndef LIBGEMM_GEMM_H
#define LIBGEMM_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gemm_handle_s* gemm_handle_t;

typedef enum {
    GEMM_OK = 0,
    GEMM_ERR_INVALID_ARG = 1,   /* null handle/pointer, negative size, small ld, unknown enum value */
    GEMM_ERR_UNSUPPORTED = 2,   /* a valid request outside what is built (see gemm_run) */
    GEMM_ERR_ALLOC = 3,         /* workspace allocation failed */
    GEMM_ERR_HIP = 4,           /* a HIP call or kernel launch failed */
    GEMM_ERR_SCRATCH_LIMIT = 5  /* gemm_run_noalloc only: the plan needs more than GEMM_NOALLOC_SCRATCH_BYTES */
} gemm_status_t;

typedef enum { GEMM_OP_N = 0, GEMM_OP_T = 1 } gemm_op_t;

/* Element types: IEEE binary32, IEEE binary16, bfloat16 (upper half of a binary32). */
typedef enum { GEMM_F32 = 0, GEMM_F16 = 1, GEMM_BF16 = 2 } gemm_dtype_t;

/* Activations of the fused epilogue (activation kernels are one of the benchmark families of
 * Section 5.2 of the paper; fused here so that C is written once):
 *   GEMM_ACT_GELU_ERF   the exact GELU, x * Phi(x) = x/2 * (1 + erf(x / sqrt 2))
 *   GEMM_ACT_RELU       max(x, 0); a NaN stays a NaN
 *   GEMM_ACT_SILU       x * sigmoid(x) = x / (1 + exp(-x))
 *   GEMM_ACT_GELU_TANH  x/2 * (1 + tanh(sqrt(2/pi) * (x + 0.044715 x^3))) */
typedef enum {
    GEMM_ACT_NONE = 0, GEMM_ACT_GELU_ERF = 1, GEMM_ACT_RELU = 2, GEMM_ACT_SILU = 3, GEMM_ACT_GELU_TANH = 4
} gemm_act_t;

/*
 * Fused epilogue.  A NULL pointer passed to gemm_run means
 * { out_dtype = dtype of A and B, bias = NULL, act = GEMM_ACT_NONE }.
 */
typedef struct {
    gemm_dtype_t out_dtype;   /* type of C, both when read (beta != 0) and when written:
                                 the type of A and B, or GEMM_F32 */
    const void*  bias;        /* device pointer to N elements added to every row, or NULL */
    gemm_dtype_t bias_dtype;  /* type of bias; ignored when bias is NULL */
    gemm_act_t   act;         /* applied last, to alpha*op(A)*op(B) + beta*C + bias */
} gemm_epilogue_t;

/*
 * Creates a handle on the current HIP device.  The handle owns only a split-K workspace
 * (allocated on first need, grown on demand, freed by gemm_destroy).  Calls that use the handle
 * must be made with the same device current; otherwise they return GEMM_ERR_INVALID_ARG.
 *
 * Workspace rule.  A call whose plan splits K needs fp32 scratch for the partial results.  When
 * the handle's buffer is too small, gemm_run allocates a larger one (hipMalloc, at least twice the
 * old size, at least 32 MiB) and goes on; the old buffer is neither freed nor waited for, because
 * work enqueued earlier may still be using it: it is kept by the handle until
 * gemm_reserve_workspace or gemm_destroy.  A caller that cannot have hipMalloc inside gemm_run (a
 * stream capture, a latency-critical loop) sizes the workspace once with gemm_reserve_workspace;
 * calls that fit it allocate nothing.
 * Errors: GEMM_ERR_INVALID_ARG if out is NULL; GEMM_ERR_HIP if no device is usable.
 */
gemm_status_t gemm_create(gemm_handle_t* out);

/*
 * Makes the handle's workspace at least `bytes` large and frees every buffer that an earlier growth
 * set aside.  This is the one call besides gemm_destroy that frees device memory, and it may block:
 * the caller must have synchronised every stream that used the handle.  The skinny family needs
 * split_k * M * N * 4 bytes; the macro-tile family needs, for a split last round, (tiles in that
 * round) * split_k * (tile rows * tile columns) * 4, and for k slices split_k * M * N * 4;
 * 256 MiB covers every shape of the bench.  bytes == 0 only frees the set-aside buffers.
 * Errors: GEMM_ERR_INVALID_ARG for a null handle or another current device; GEMM_ERR_ALLOC if the
 * allocation failed (the old workspace stays); GEMM_ERR_HIP if freeing failed.
 */
gemm_status_t gemm_reserve_workspace(gemm_handle_t h, size_t bytes);

/* Size in bytes of the handle's current workspace (0 before the first split-K call or reservation).
 * Errors: GEMM_ERR_INVALID_ARG for null arguments. */
gemm_status_t gemm_workspace_size(gemm_handle_t h, size_t* bytes);

/*
 * Enqueues C = act(alpha*op(A)*op(B) + beta*C + bias) on `stream` (a hipStream_t passed as
 * void*; NULL is the default stream).
 *
 *   M, N, K         sizes, >= 0.  M == 0 or N == 0: nothing is launched.  K == 0: the product is
 *                   an empty sum, C = act(beta*C + bias).
 *   dtype           type of A and B.
 *   alpha, beta     host scalars.  beta == 0 makes C write-only: its old contents, NaN and Inf
 *                   included, do not reach the result.
 *   A, B            device pointers, read only; may be NULL only if the operand is empty.
 *   C               device pointer, M x N, written (and read iff beta != 0).  Must not overlap A,
 *                   B or bias.
 *   epilogue        see gemm_epilogue_t; may be NULL.
 *
 * Any shape, leading dimension and alignment is accepted for all three types.  The fast
 * matrix-core kernels need 16-byte aligned A and B, leading dimensions that are multiples of
 * 8 elements and a contiguous dimension that is a multiple of 8 (bf16/fp16); other calls run
 * a slower general kernel with the same result contract.
 *
 * Errors (C is untouched in every error case detected before launch):
 *   GEMM_ERR_INVALID_ARG  null handle; negative size; ld smaller than the stored row; a null
 *                         matrix pointer for a non-empty operand; an enum value out of range; a
 *                         current device other than the handle's.
 *   GEMM_ERR_UNSUPPORTED  out_dtype neither the input type nor GEMM_F32.
 *   GEMM_ERR_ALLOC        the split-K workspace could not be grown (hipMalloc failed, or it has
 *                         been grown 48 times without a gemm_reserve_workspace in between).
 *   GEMM_ERR_HIP          a launch failed (the HIP error is consumed).
 *
 * A handle must not be used from two streams at once (they would share the workspace);
 * distinct handles may run concurrently.  The same call on the same data always yields the
 * same bits (no floating-point atomics; fixed split-K summation order).
 */
gemm_status_t gemm_run(gemm_handle_t h, int64_t M, int64_t N, int64_t K,
                       gemm_op_t transA, gemm_op_t transB, gemm_dtype_t dtype,
                       float alpha, const void* A, int64_t lda,
                       const void* B, int64_t ldb,
                       float beta, void* C, int64_t ldc,
                       const gemm_epilogue_t* epilogue, void* stream);

/*
 * gemm_run for callers that cannot allocate device memory at all: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * bits in C as gemm_run; the one difference is where split-K partial results go: into a buffer of
 * GEMM_NOALLOC_SCRATCH_BYTES that is part of the library's device image (each GPU the library runs
 * on holds its copy from load until the process ends) instead of the handle's workspace.  The
 * call never invokes hipMalloc, hipFree or any allocating routine.
 *
 * A call whose plan needs more scratch than that returns GEMM_ERR_SCRATCH_LIMIT before anything
 * is launched, C untouched (the need per plan is stated at gemm_reserve_workspace: 32 rows on a
 * 16384 x 16384 weight in four k slices take 8 MiB; a plan that does not split K takes none).
 * Every call on one GPU shares that GPU's buffer, whatever the handle or stream: calls that may
 * overlap in time on one GPU race on it and must be ordered by the caller (one stream, or events).
 * The buffer keeps the last call's contents; the kernels write every partial result before the
 * reduction reads it, so nothing needs clearing between calls.
 * Errors otherwise as gemm_run (GEMM_ERR_ALLOC cannot occur).
 */
#define GEMM_NOALLOC_SCRATCH_BYTES (32u << 20)
gemm_status_t gemm_run_noalloc(gemm_handle_t h, int64_t M, int64_t N, int64_t K,
                               gemm_op_t transA, gemm_op_t transB, gemm_dtype_t dtype,
                               float alpha, const void* A, int64_t lda,
                               const void* B, int64_t ldb,
                               float beta, void* C, int64_t ldc,
                               const gemm_epilogue_t* epilogue, void* stream);

/*
 * The same product for `batch` independent problems of one shape, whose matrices lie at constant
 * distances in memory (the shape of the per-head products of attention, which the paper names as
 * the reason GEMM matters, Section 5.4):
 *
 *     C_b = act( alpha * op(A_b) * op(B_b) + beta * C_b + bias ),   b = 0 .. batch-1,
 *     A_b = A + b*strideA,  B_b = B + b*strideB,  C_b = C + b*strideC   (strides in elements)
 *
 * Every other argument means what it means in gemm_run and applies to each matrix; bias is shared
 * by the whole batch.  strideA or strideB may be 0 (one operand shared by all products);
 * strideC must be at least (M-1)*ldc + N so that no two results overlap.  batch == 0 does
 * nothing.  The fast kernels additionally need strideA and strideB to be multiples of 16 bytes;
 * other strides run the general kernel.  One launch covers up to 65535 matrices; a longer batch
 * is enqueued as consecutive launches.
 *
 * Errors: as gemm_run, and GEMM_ERR_INVALID_ARG for a negative batch or stride or an
 * overlapping strideC.
 */
gemm_status_t gemm_run_batched(gemm_handle_t h, int64_t batch, int64_t M, int64_t N, int64_t K,
                               gemm_op_t transA, gemm_op_t transB, gemm_dtype_t dtype,
                               float alpha, const void* A, int64_t lda, int64_t strideA,
                               const void* B, int64_t ldb, int64_t strideB,
                               float beta, void* C, int64_t ldc, int64_t strideC,
                               const gemm_epilogue_t* epilogue, void* stream);

/* Frees the workspace, the buffers set aside by earlier growth, and the handle.  The caller must have synchronised the streams that used
 * it.  NULL is accepted.  Errors: GEMM_ERR_HIP if freeing device memory failed. */
gemm_status_t gemm_destroy(gemm_handle_t h);

/* A static, never-NULL description of a status code. */
const char* gemm_status_string(gemm_status_t s);

/* ---- kernel choice: inspection and override (the paper's "tiling" strategy, Table 1, is a
 * tunable here; the bench harness sweeps it and records the evidence) ---- */

typedef enum {
    GEMM_KERNEL_AUTO = 0,      /* let the library choose (default) */
    GEMM_KERNEL_GENERAL = 1,   /* one thread per output element, any shape/alignment */
    GEMM_KERNEL_MFMA_TILE = 2, /* LDS-staged macro-tile kernel on MFMA */
    GEMM_KERNEL_SKINNY = 3     /* streaming kernels with split-K for few rows of C.  bf16 / fp16, M <= 64: variant 0
                                  for a row-major B (K x N), variant 1 for B stored N x K (an A stored K x M is first
                                  gathered into a row-major copy in the workspace).  fp32, M <= 8, A row-major:
                                  variants 2 and 3, the same two layouts on the vector ALUs.  B stored N x K, bf16 /
                                  fp16, A row-major, has two one-launch forms besides variant 1: variant 4 on the vector
                                  ALUs (M <= 8; automatic up to 4 rows) and variant 5, variant 1 with 16 columns per
                                  workgroup (M <= 16; automatic for 5 to 16 rows on weights of 128 MiB at most).  The
                                  layout and type of the call decide among them; variant -1 takes the automatic one, a
                                  variant forced against the call is GEMM_ERR_UNSUPPORTED */
} gemm_kernel_t;

typedef struct {
    gemm_kernel_t kernel;   /* which family */
    int32_t variant;        /* tile variant index within the family; -1 = automatic */
    int32_t split_k;        /* number of K slices; 0 = automatic, 1 = none.  Skinny family: every
                             * column group is cut into that many slices.  Macro-tile family, the
                             * tiles on the 16x16x32 MFMA (256x256, 256x128, 128x256, 128x128): only
                             * the tiles of the last, partly filled round of workgroups (all tiles when
                             * there are fewer tiles than compute units) are cut, each into that many
                             * shares of the k range (at most one share per 32-element slab).
                             * Every other tile variant: the whole product is cut into that many
                             * ranges of K (whole 32-element slabs; fewer if K has not enough of
                             * them), computed side by side into fp32 partial results and added by a
                             * second kernel; this needs N to be a multiple of 8.  Batched calls, and
                             * calls that miss that condition, return GEMM_ERR_UNSUPPORTED.  Slices
                             * are added in a fixed order: results do not vary from run to run. */
} gemm_plan_t;

/* Forces the plan used by later gemm_run calls on this handle; a NULL plan restores automatic
 * choice.  A forced plan that cannot run a given call (alignment, shape) makes that call return
 * GEMM_ERR_UNSUPPORTED.  Errors: GEMM_ERR_INVALID_ARG for a null handle or out-of-range fields. */
gemm_status_t gemm_set_plan(gemm_handle_t h, const gemm_plan_t* plan);

/* Reports the plan the most recent successful gemm_run on this handle used.  (An automatic plan may
 * run a C with a thin last strip of columns or rows as two products, the whole tiles and the strip;
 * the plan of the whole tiles is the one reported.)
 * Errors: GEMM_ERR_INVALID_ARG for null arguments. */
gemm_status_t gemm_get_last_plan(gemm_handle_t h, gemm_plan_t* out);

/* The plan an automatic call of this shape would take on a device with `compute_units` compute
 * units, for operands on 16-byte boundaries, matrices of a batch packed back to back, no epilogue
 * terms.  Host arithmetic only: no device is touched and no handle is needed, so the choice can be
 * inspected (and is tested) without a GPU.  For a call made as two products (see
 * gemm_get_last_plan) it is the plan of the whole tiles.
 * Errors: GEMM_ERR_INVALID_ARG for a null `out`, sizes below 1, leading dimensions too small or an
 * unknown enum; GEMM_ERR_UNSUPPORTED for an out_dtype that is neither dtype nor GEMM_F32. */
gemm_status_t gemm_plan_query(int32_t compute_units, int64_t batch, int64_t M, int64_t N, int64_t K,
                              gemm_op_t transA, gemm_op_t transB, gemm_dtype_t dtype, gemm_dtype_t out_dtype,
                              int64_t lda, int64_t ldb, int64_t ldc, gemm_plan_t* out);

/*
 * The roofline rule of the paper (Section 4.3) that the automatic choice starts from.  A call is
 * placed by its arithmetic intensity, 2*M*N*K*batch flop over the bytes of one pass over every
 * operand (A, B, C written, C read if `reads_c`, the bias if `has_bias`), against two ridge points of
 * the MI355X roofline at 8 TB/s: 19.7 flop/byte, where the fp32 vector ALUs (157.3 TFLOP/s) meet the
 * memory roof, and the ridge of the matrix cores for the operand type (bf16, fp16: 2.5 PFLOP/s ->
 * 312.5; fp32: 157.3 TFLOP/s -> 19.7).  Left of the first: memory-bound, the streaming kernels are
 * candidates and bytes per second is the objective; right of the second: compute-bound, matrix-core
 * tiles only; in between: middle zone, both families compete and measured thresholds decide.
 * Host arithmetic only.  `intensity` may be NULL.
 * Errors: GEMM_ERR_INVALID_ARG for a null `cls`, sizes below 1 or an unknown enum.
 */
typedef enum { GEMM_MEMORY_BOUND = 0, GEMM_MIDDLE_ZONE = 1, GEMM_COMPUTE_BOUND = 2 } gemm_roofline_t;
gemm_status_t gemm_roofline_class(int64_t batch, int64_t M, int64_t N, int64_t K, gemm_dtype_t dtype, gemm_dtype_t out_dtype,
                                  int32_t reads_c, int32_t has_bias, gemm_dtype_t bias_dtype, gemm_roofline_t* cls,
                                  double* intensity);

/* Name of a tile variant of a family (static storage), or NULL if the index is out of range.
 * Lets a harness enumerate variants: loop until NULL. */
const char* gemm_variant_name(gemm_kernel_t kernel, int32_t variant);

#ifdef __cplusplus
}
#endif
#endif /* LIBGEMM_GEMM_H */
