/*
 * CPU oracle for C = alpha * op(A) * op(B) + beta * C_in.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is
 * checked against; the library itself never calls it.  It shares no code,
 * header, table or helper with the GPU path.
 *
 * What it computes is the matrix product as the paper defines it (Section
 * 2.2, "Matrix Multiplication": A is m x k, B is k x n, C = A x B is m x n,
 * row-major storage, one dot product of a row of A with a column of B per
 * output element), widened to the BLAS form with alpha, beta, leading
 * dimensions and transpose flags that the same passage refers to as the
 * standard library interface.  Element storage may be fp32, IEEE half or
 * bfloat16; every product and sum is carried in fp64 (the product of two
 * such values is exact in fp64), summed over k in ascending order, and the
 * result is kept in fp64 - it is never rounded back to the storage type.
 *
 *   A(i,k) = transA ? a[k*lda + i] : a[i*lda + k]
 *   B(k,j) = transB ? b[j*ldb + k] : b[k*ldb + j]
 *   ref[i*N + j] = alpha * sum_k A(i,k)*B(k,j) + (beta == 0 ? 0 : beta * c_in[i*ldc + j])
 *
 * As in BLAS, beta == 0 means C_in is not read (a NaN there does not reach
 * the result) and alpha == 0 means A and B are not read.
 *
 * Two loop orders are provided and must give bit-identical results, since
 * each adds the products of one (i,j) in ascending k:
 *   order 0: for i, for j, for k          (the definition, written out)
 *   order 1: for i, for k, for j          (same sums, walks B along rows;
 *                                          used when B is stored k-major so
 *                                          that large cases finish)
 * Rows are shared out over threads; nothing else is blocked or reordered.
 *
 * Pins (tests/test_oracle_*.py): exact int64 brute force on small integer
 * matrices, identity and permutation operands, closed-form products,
 * (AB)^T = B^T A^T, transpose-flag equivalence, linearity in alpha/beta,
 * numpy's fp64 product, and the element decoders against numpy/torch for
 * all 65536 bit patterns.
 *
 * oracle_bias_act is the fused output step some callers ask for (kernel fusion
 * is the example Section 1.2 gives of the small changes an optimised MatMul has
 * to stay open to): ref <- act(ref + bias), in fp64, applied
 * to the finished alpha*op(A)*op(B) + beta*C_in.  Pins: hand cases where the
 * order of bias and activation matters, row- against column-bias on a
 * non-square zero product, row subsets, torch's fp64 tanh-form GELU, the
 * identity gelu(x) - gelu(-x) = x.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { OR_F32 = 0, OR_F16 = 1, OR_BF16 = 2 };

/* IEEE binary16 -> double, decoded field by field. */
double oracle_decode_f16(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int ex = (h >> 10) & 0x1F;
    int man = h & 0x3FF;
    double v;
    if (ex == 0) {
        v = (double)man * (1.0 / 16777216.0);            /* man * 2^-24 (subnormal or zero) */
    } else if (ex == 31) {
        if (man == 0) {
            v = 1.0 / 0.0;
        } else {
            v = 0.0 / 0.0;
            return v;                                     /* NaN: sign is irrelevant */
        }
    } else {
        v = ldexp(1.0 + (double)man * (1.0 / 1024.0), ex - 15);
    }
    return sign ? -v : v;
}

/* bfloat16 is the upper half of an fp32 word. */
double oracle_decode_bf16(uint16_t h)
{
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

static double load_elem(const void *p, int64_t idx, int dtype)
{
    switch (dtype) {
    case OR_F32:  return (double)((const float *)p)[idx];
    case OR_F16:  return oracle_decode_f16(((const uint16_t *)p)[idx]);
    default:      return oracle_decode_bf16(((const uint16_t *)p)[idx]);
    }
}

typedef struct {
    int dtype, cdtype, transA, transB, order;
    int64_t M, N, K, lda, ldb, ldc;
    double alpha, beta;
    const void *A, *B, *Cin;
    const int64_t *rows;     /* NULL: all rows 0..M-1; else nrows logical row indices */
    int64_t nrows;
    double *ref;             /* nrows x N, row r of ref <-> logical row rows[r] */
    int tid, nthreads;
} job_t;

static void *worker(void *arg)
{
    const job_t *jb = (const job_t *)arg;
    const int64_t N = jb->N, K = jb->K;
    double *acc = NULL;
    double *arow = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
    if (jb->order == 1) acc = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));

    for (int64_t r = jb->tid; r < jb->nrows; r += jb->nthreads) {
        const int64_t i = jb->rows ? jb->rows[r] : r;
        double *out = jb->ref + r * N;
        if (jb->alpha == 0.0) {
            /* BLAS convention: with alpha == 0 the operands are not referenced */
            for (int64_t j = 0; j < N; ++j) out[j] = 0.0;
            goto scale;
        }
        /* decode row i of op(A) once */
        for (int64_t k = 0; k < K; ++k)
            arow[k] = load_elem(jb->A, jb->transA ? k * jb->lda + i : i * jb->lda + k, jb->dtype);

        if (jb->order == 0) {
            for (int64_t j = 0; j < N; ++j) {
                double s = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    double b = load_elem(jb->B, jb->transB ? j * jb->ldb + k : k * jb->ldb + j, jb->dtype);
                    s += arow[k] * b;
                }
                out[j] = s;
            }
        } else {
            for (int64_t j = 0; j < N; ++j) acc[j] = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const double a = arow[k];
                for (int64_t j = 0; j < N; ++j) {
                    double b = load_elem(jb->B, jb->transB ? j * jb->ldb + k : k * jb->ldb + j, jb->dtype);
                    acc[j] += a * b;
                }
            }
            for (int64_t j = 0; j < N; ++j) out[j] = acc[j];
        }
scale:
        for (int64_t j = 0; j < N; ++j) {
            double v = jb->alpha == 0.0 ? 0.0 : jb->alpha * out[j];
            if (jb->beta != 0.0)
                v += jb->beta * load_elem(jb->Cin, i * jb->ldc + j, jb->cdtype);
            out[j] = v;
        }
    }
    free(arow);
    free(acc);
    return NULL;
}

/*
 * Returns 0 on success, 1 on bad arguments.
 * order: 0 = i,j,k   1 = i,k,j   -1 = pick (1 when B is stored k-major, i.e. transB == 0).
 * rows/nrows: optional subset of logical rows of C to compute (rows == NULL: all M rows,
 * nrows is then ignored).  ref must hold (rows ? nrows : M) * N doubles.
 * alpha and beta are the fp32 scalars of the interface, widened by the caller.
 * cdtype is the storage type of C_in, which may differ from that of A and B
 * (16-bit operands with an fp32 C); ldc counts elements of that type.
 */
int oracle_gemm_c(int dtype, int cdtype, int transA, int transB,
                  int64_t M, int64_t N, int64_t K,
                  double alpha, const void *A, int64_t lda,
                  const void *B, int64_t ldb,
                  double beta, const void *Cin, int64_t ldc,
                  const int64_t *rows, int64_t nrows,
                  double *ref, int order, int nthreads)
{
    if (dtype < 0 || dtype > 2 || cdtype < 0 || cdtype > 2 || M < 0 || N < 0 || K < 0 || !ref) return 1;
    if (lda < (transA ? M : K) || ldb < (transB ? K : N)) return 1;
    if (beta != 0.0 && (!Cin || ldc < N)) return 1;
    if (K > 0 && M > 0 && N > 0 && alpha != 0.0 && (!A || !B)) return 1;
    if (rows) {
        for (int64_t r = 0; r < nrows; ++r)
            if (rows[r] < 0 || rows[r] >= M) return 1;
    } else {
        nrows = M;
    }
    if (order < 0) order = transB ? 0 : 1;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 256) nthreads = 256;
    if ((int64_t)nthreads > nrows) nthreads = nrows > 0 ? (int)nrows : 1;

    job_t jobs[256];
    pthread_t th[256];
    for (int t = 0; t < nthreads; ++t) {
        job_t *jb = &jobs[t];
        jb->dtype = dtype; jb->cdtype = cdtype; jb->transA = transA; jb->transB = transB; jb->order = order;
        jb->M = M; jb->N = N; jb->K = K; jb->lda = lda; jb->ldb = ldb; jb->ldc = ldc;
        jb->alpha = alpha; jb->beta = beta; jb->A = A; jb->B = B; jb->Cin = Cin;
        jb->rows = rows; jb->nrows = nrows; jb->ref = ref; jb->tid = t; jb->nthreads = nthreads;
    }
    if (nthreads == 1) {
        worker(&jobs[0]);
        return 0;
    }
    for (int t = 0; t < nthreads; ++t) pthread_create(&th[t], NULL, worker, &jobs[t]);
    for (int t = 0; t < nthreads; ++t) pthread_join(th[t], NULL);
    return 0;
}


/* A, B and C_in share one storage type. */
int oracle_gemm(int dtype, int transA, int transB,
                int64_t M, int64_t N, int64_t K,
                double alpha, const void *A, int64_t lda,
                const void *B, int64_t ldb,
                double beta, const void *Cin, int64_t ldc,
                const int64_t *rows, int64_t nrows,
                double *ref, int order, int nthreads)
{
    return oracle_gemm_c(dtype, dtype, transA, transB, M, N, K, alpha, A, lda, B, ldb, beta, Cin, ldc,
                         rows, nrows, ref, order, nthreads);
}

enum { OR_BIAS_NONE = 0, OR_BIAS_PER_COLUMN = 1, OR_BIAS_PER_ROW = 2 };
enum { OR_ACT_NONE = 0, OR_ACT_RELU = 1, OR_ACT_GELU_TANH = 2 };

/*
 * ref(i,j) <- act(ref(i,j) + b(i,j)) for the rows oracle_gemm produced.
 *   bias_kind  PER_COLUMN: b(i,j) = bias[j] (N fp32 values, one per column of C)
 *              PER_ROW:    b(i,j) = bias[i] (M fp32 values, i the logical row of C)
 *   act        RELU:       x > 0 ? x : 0
 *              GELU_TANH:  x/2 * (1 + tanh( sqrt(2/pi) * (x + 0.044715 x^3) ))
 *                          (the tanh form of Hendrycks and Gimpel's GELU)
 * rows/nrows as in oracle_gemm.  Returns 0 on success, 1 on bad arguments.
 */
int oracle_bias_act(int64_t M, int64_t N, const int64_t *rows, int64_t nrows, double *ref,
                    int bias_kind, const float *bias, int act)
{
    if (M < 0 || N < 0 || !ref) return 1;
    if (bias_kind < 0 || bias_kind > 2 || act < 0 || act > 2) return 1;
    if (bias_kind != OR_BIAS_NONE && !bias) return 1;
    if (!rows) nrows = M;
    const double c = sqrt(2.0 / acos(-1.0));
    for (int64_t r = 0; r < nrows; ++r) {
        const int64_t i = rows ? rows[r] : r;
        if (i < 0 || i >= M) return 1;
        for (int64_t j = 0; j < N; ++j) {
            double x = ref[r * N + j];
            if (bias_kind == OR_BIAS_PER_COLUMN) x += (double)bias[j];
            if (bias_kind == OR_BIAS_PER_ROW) x += (double)bias[i];
            if (act == OR_ACT_RELU) x = x > 0.0 ? x : 0.0;
            if (act == OR_ACT_GELU_TANH) x = 0.5 * x * (1.0 + tanh(c * (x + 0.044715 * x * x * x)));
            ref[r * N + j] = x;
        }
    }
    return 0;
}
