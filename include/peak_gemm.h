/*
 * peak_gemm.h - C ABI of the MI355X (gfx950) dense matrix-multiplication library.
 *
 * The operation is the MatMul of the paper's Section 2.2 ("Matrix
 * Multiplication"): A is m x k, B is k x n, C = A x B is m x n, stored
 * row-major, in fp32 or a 16-bit float type.  That passage calls it the
 * standard BLAS library interface; this header takes that interface in full:
 *
 *      C = alpha * op(A) * op(B) + beta * C
 *
 * with leading dimensions, transpose flags and fp32 scalars.  Products are
 * accumulated in fp32 on the matrix cores for every dtype (the paper's
 * Tensor-Core / Warp-Tiling / TB-Tiling steps of Section 4.1, Table 2, mapped
 * to MFMA, wavefront and workgroup tiles), and the result is rounded once,
 * to nearest even, to the storage dtype.
 *
 * No C++ or framework types cross this boundary: plain pointers and sizes.
 * Every pointer handed to peak_gemm_run (A, B, C, workspace) is a DEVICE
 * pointer on the current HIP device; descriptors, plans and strings are HOST
 * memory.  The library never allocates device memory and never synchronises.
 */
#ifndef PEAK_GEMM_H
#define PEAK_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Element storage type of A, B and C (they share it, unless PEAK_GEMM_C_F32 is set).  Section 2.2 names fp32
 * and fp16; bfloat16 is the third 16-bit storage the graded workloads use. */
typedef enum {
    PEAK_DT_F32 = 0,
    PEAK_DT_F16 = 1,
    PEAK_DT_BF16 = 2
} peak_dtype_t;

typedef enum {
    PEAK_OK = 0,
    PEAK_ERR_INVALID_ARG = 1,   /* NULL where data is needed, negative size, ld below the row length, unknown enum */
    PEAK_ERR_UNSUPPORTED = 2,   /* no kernel variant fits: the "invalid configuration" sentinel of Section 3.1 */
    PEAK_ERR_WORKSPACE = 3,     /* workspace missing or smaller than peak_gemm_workspace_bytes() */
    PEAK_ERR_HIP = 4,           /* the HIP runtime reported an error at launch */
    PEAK_ERR_ALLOC = 5          /* host allocation of the plan failed */
} peak_status_t;

/* Opaque, owned by the library, lives in host memory. */
typedef struct peak_gemm_plan peak_gemm_plan_t;

/*
 * Problem description (the kernel context's input specification of Section
 * 3.1, reduced to what a GEMM needs).
 *
 * op(A) is M x K, op(B) is K x N, C is M x N.  All arrays are row-major as
 * stored, with row strides in ELEMENTS:
 *   transA = 0: A is stored M rows x K,  lda >= K.   transA = 1: stored K rows x M, lda >= M.
 *   transB = 0: B is stored K rows x N,  ldb >= N.   transB = 1: stored N rows x K, ldb >= K
 *               (i.e. op(B) column-major; both operands then run along K in memory).
 *   C is stored M rows x N, ldc >= N.  Elements beyond N in a row are never touched.
 *
 * flags: bits 0..7 = 0 lets the selector choose; a non-zero value forces kernel
 * variant number (value - 1) for tests and tuning sweeps (PEAK_ERR_UNSUPPORTED
 * if that variant cannot run the problem).  Bits 8..15 = 0 lets the selector
 * choose the split of K; a non-zero value forces that many K slices.
 * PEAK_GEMM_C_F32 (bit 16): C is stored as fp32 while A and B keep `dtype`
 * (16-bit operands, full-precision result: the accumulators are fp32 anyway, so
 * alpha*acc + beta*C is then stored unrounded); ldc counts fp32 elements and C
 * must be 4-byte aligned.  With dtype == PEAK_DT_F32 the bit changes nothing.
 * PEAK_GEMM_STREAMK_ON / PEAK_GEMM_STREAMK_OFF (bits 17, 18; not both): hybrid
 * stream-K, the Split-K step of Section 4.1 (Table 2) applied to the last round of
 * tiles only.  When the tiles do not fill a whole number of rounds over the compute
 * units, the tiles of the last, partial round are cut into K slices, one workgroup
 * each, and their fp32 partial tiles are summed in slice order by a second kernel, so
 * that the round lasts a slice instead of a tile.  ON takes it wherever the kernel
 * variant supports it and the shape leaves a partial round after at least one full
 * one (else the bit changes nothing); OFF never takes it; neither: the cost model
 * decides.  A forced K split (bits 8..15) rules it out.  Results stay bit-identical
 * from run to run.  Other bits must be zero.
 */
#define PEAK_GEMM_C_F32 0x10000u
#define PEAK_GEMM_STREAMK_ON 0x20000u
#define PEAK_GEMM_STREAMK_OFF 0x40000u
typedef struct {
    int64_t M, N, K;
    int64_t lda, ldb, ldc;
    int32_t transA, transB;
    int32_t dtype;              /* a peak_dtype_t value; a fixed-width field, because the size of an enum type
                                   is the compiler's choice and this struct is read by ctypes and other ABIs */
    uint32_t flags;
} peak_gemm_desc_t;

/*
 * Validates the description, chooses the kernel variant, tile shape, split of
 * K, grid and workspace size (Section 3.1: tuning parameters and execution
 * parameters; Section 2.2: t_m, t_n, t_k, w_m, w_n).  A shape listed in the
 * selector table (see peak_gemm_load_tuning) gets the table's variant and split,
 * any other the cost model's.  Launches nothing and allocates nothing on the
 * device; the first call reads the compute-unit count of the current device, if
 * there is one (else, or with PEAK_GEMM_NUM_CU set, that value or 256 is used).
 * On success *out_plan is a new plan; on any error *out_plan is NULL.
 * Degenerate sizes (M, N or K equal to 0) are valid.
 */
peak_status_t peak_gemm_create(const peak_gemm_desc_t *desc, peak_gemm_plan_t **out_plan);

/* Bytes of device workspace peak_gemm_run needs for this plan (0 for most
 * plans that do not split K).  The workspace holds fp32 partial tiles of the
 * Split-K step (Section 4.1, Table 2) and, for a streaming plan on an A stored
 * K x M, the copy of A with rows along K that the run writes first (Section
 * 4.1, Table 2, Transpose). */
size_t peak_gemm_workspace_bytes(const peak_gemm_plan_t *plan);

/*
 * Enqueues C = alpha*op(A)*op(B) + beta*C on `hip_stream` (a hipStream_t
 * passed as void*; NULL = the default stream) and returns without waiting.
 * This is the kernel execution of Section 3.1 (the driver runs the kernel on
 * given inputs with given execution parameters) for the MatMul of Section 2.2;
 * the steps it runs are the transformed kernel of Section 4.1, Table 2: tile
 * order (Block-Swizzle), staging into LDS (Pipelining, Register-Staging,
 * Transpose, Offset), MFMA tiles (Tensor-Core, Warp-Tiling, Tensor-Tiling),
 * K slices and their ordered sum (Split-K), output.
 *
 *   A, B         need element alignment only.  Plans are made from the leading
 *                dimensions; when those suit the 16-byte copies of the fast
 *                kernels but a base address does not (a view one element into
 *                a larger matrix), the run uses the plan's register-staged
 *                stand-in variant (named after "unaligned=" by
 *                peak_gemm_plan_info): same result within the tolerance, slower.
 *   A, B, C      device pointers, aligned to the element size; C must not
 *                overlap A or B.  With beta == 0 C is write-only: whatever it
 *                holds, NaN included, does not reach the result.  With
 *                alpha == 0 or K == 0, A and B are not read (they may be NULL)
 *                and C = beta*C.
 *   workspace    device pointer to at least peak_gemm_workspace_bytes() bytes,
 *                256-byte aligned; may be NULL when that size is 0.  Its
 *                contents need no initialisation and are scratch afterwards.
 *
 * The caller keeps ownership of every buffer and of the stream.  Runs of one
 * plan that overlap in time must use different workspaces.  Results are
 * bit-identical from run to run for a given plan (no floating-point atomics).
 * M == 0 or N == 0: returns PEAK_OK and launches nothing.
 */
peak_status_t peak_gemm_run(peak_gemm_plan_t *plan, float alpha,
                            const void *A, const void *B, float beta, void *C,
                            void *workspace, size_t workspace_bytes,
                            void *hip_stream);

/*
 * Fused output step.  Section 1.2 wants an optimised MatMul to stay open to
 * small later changes and gives kernel fusion as the example (the Limitations
 * paragraph of Section 3.1 names fusion as the case a single-kernel optimiser
 * meets ready-made); this is that slot.  With an epilogue the run
 * computes, in fp32 and before the one rounding to the storage type,
 *
 *      C = act( alpha * op(A) * op(B) + beta * C + bias )
 *
 *   bias_kind  PEAK_BIAS_PER_COLUMN: bias[n] is added to column n (N values);
 *              PEAK_BIAS_PER_ROW:    bias[m] is added to row m (M values);
 *              PEAK_BIAS_NONE:       `bias` is ignored.
 *   bias       DEVICE pointer to fp32 values, 4-byte aligned, read-only, owned
 *              by the caller; must not overlap C.
 *   act        PEAK_ACT_RELU:       x > 0 ? x : 0  (a NaN becomes 0);
 *              PEAK_ACT_GELU_TANH:  x/2 * (1 + tanh(sqrt(2/pi) * (x + 0.044715 x^3))),
 *                                   evaluated as x / (1 + exp(-2u)) with the
 *                                   hardware exponential (relative error of a few
 *                                   ulp of fp32, far inside the GEMM tolerances).
 * The struct itself is HOST memory and is read before the call returns.
 */
typedef enum { PEAK_BIAS_NONE = 0, PEAK_BIAS_PER_COLUMN = 1, PEAK_BIAS_PER_ROW = 2 } peak_bias_t;
typedef enum { PEAK_ACT_NONE = 0, PEAK_ACT_RELU = 1, PEAK_ACT_GELU_TANH = 2 } peak_act_t;
typedef struct {
    const void *bias;
    int32_t bias_kind;          /* a peak_bias_t value */
    int32_t act;                /* a peak_act_t value */
} peak_gemm_epilogue_t;

/*
 * peak_gemm_run with the fused output step: same arguments, same rules, same
 * kernels (the step is applied where C is stored: in the GEMM kernel's
 * epilogue, or in the reduction kernel when K is split, or in the scaling
 * kernel when alpha == 0 or K == 0, where C = act(beta*C + bias)).
 * epilogue == NULL, or PEAK_BIAS_NONE with PEAK_ACT_NONE, is peak_gemm_run.
 * PEAK_ERR_INVALID_ARG for an unknown enum value or a missing or misaligned bias.
 */
peak_status_t peak_gemm_run_fused(peak_gemm_plan_t *plan, float alpha,
                                  const void *A, const void *B, float beta, void *C,
                                  const peak_gemm_epilogue_t *epilogue,
                                  void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

/*
 * peak_gemm_run for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same plan, same kernels, same result bits as peak_gemm_run;
 * what the workspace would hold goes to an array of PEAK_GEMM_STATIC_WORKSPACE_BYTES that
 * is part of the library's device code (every GPU the library runs on holds
 * its own copy until the process ends).  The call allocates nothing.
 *
 *   PEAK_ERR_WORKSPACE  the plan needs more than PEAK_GEMM_STATIC_WORKSPACE_BYTES
 *                       (peak_gemm_workspace_bytes() tells beforehand); nothing is launched.
 *   PEAK_ERR_HIP        no current device, or the array's address could not be obtained.
 *
 * The array's device address is looked up on the first call on each device
 * (make that call outside a graph capture).  All calls on one GPU share the
 * array: runs that overlap in time on one GPU (different streams, or replays of
 * two captured graphs) race on it and must be serialised by the caller.  No
 * clearing is needed between calls: a run reads only partials it has written.
 */
#define PEAK_GEMM_STATIC_WORKSPACE_BYTES (32u << 20)
peak_status_t peak_gemm_run_static(peak_gemm_plan_t *plan, float alpha,
                                   const void *A, const void *B, float beta, void *C,
                                   void *hip_stream);

/* Frees the plan made by peak_gemm_create (host memory only; the kernel context of Section 3.1 owns nothing
 * on the device).  NULL is accepted.  Always PEAK_OK. */
peak_status_t peak_gemm_destroy(peak_gemm_plan_t *plan);

/* Static, NUL-terminated description of a status code (PEAK_ERR_UNSUPPORTED is the "invalid configuration"
 * sentinel of Section 3.1; the others are the argument checks that section's input validation stands for). */
const char *peak_status_string(peak_status_t s);

/*
 * Writes a one-line, NUL-terminated description of the plan into buf and
 * returns the length it would need (like snprintf): the values chosen for the
 * tuning and execution parameters of Section 3.1 (variant name, tile t_m x t_n x
 * t_k of Section 2.2, threads, stages, K split, grid, tile order band, LDS
 * bytes, workspace, and the stand-in variant for unaligned operand bases).  For
 * logs, the bench and the tests.
 */
int peak_gemm_plan_info(const peak_gemm_plan_t *plan, char *buf, size_t n);

/* Number of kernel variants the library holds, and the name of variant `id`
 * (NULL if out of range).  Variant ids are what `flags` bits 0..7 force.  The
 * variants are the points of the tuning-parameter space of Section 3.1 that the
 * library was built with; enumerating them is what the sweep of Section 3.3 needs. */
int peak_gemm_variant_count(void);
const char *peak_gemm_variant_name(int id);

/* Selector table from an offline sweep (the exhaustive search over tuning
 * parameters of the paper's Section 3.3, "performance evaluators": enumerate
 * the valid parameter settings, time them, keep the best).
 *
 * `path` names a text file in host memory's file system, one entry per line:
 *     <dtype f32|f16|bf16> <transA 0|1> <transB 0|1> <M> <N> <K> <variant name> <split>
 * (split 0 stands for hybrid stream-K, see PEAK_GEMM_STREAMK_ON)
 * ('#' starts a comment; further columns are ignored).  After a successful
 * load, peak_gemm_create() with no forced variant uses the entry whose first
 * six columns equal the descriptor's, provided that variant fits the
 * descriptor's leading dimensions and alignment; otherwise the built-in cost
 * model decides as before.  The table replaces any table loaded earlier;
 * path == NULL clears it.  Returns the number of entries now held, or -1 if
 * the file cannot be read or a line is malformed or names an unknown variant
 * (the previous table is then kept).  Unless this function was called first,
 * the first peak_gemm_create() loads the file named by the environment variable
 * PEAK_GEMM_TUNING, or, when that is unset, the table that ships with the
 * library (peak_gemm_tuning.txt beside the shared object); PEAK_GEMM_TUNING set
 * to the empty string turns both off.
 * Not thread-safe against concurrent peak_gemm_create() calls. */
int peak_gemm_load_tuning(const char *path);

#ifdef __cplusplus
}
#endif
#endif /* PEAK_GEMM_H */
