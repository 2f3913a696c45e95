/* Driver for the sanitizer test of the CPU oracle: oracle/oracle_gemm.c built with
 * AddressSanitizer and UndefinedBehaviorSanitizer and called over small problems of
 * every storage type, layout, padding, row subset, loop order and thread count, with the
 * operands in exactly sized heap blocks so that any access beyond what the arguments
 * describe is caught.  Checks integer results against a plain triple loop.  Exit 0 = clean. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_gemm_c(int dtype, int cdtype, int transA, int transB, int64_t M, int64_t N, int64_t K, double alpha, const void *A,
                  int64_t lda, const void *B, int64_t ldb, double beta, const void *Cin, int64_t ldc, const int64_t *rows,
                  int64_t nrows, double *ref, int order, int nthreads);
int oracle_bias_act(int64_t M, int64_t N, const int64_t *rows, int64_t nrows, double *ref, int bias_kind, const float *bias, int act);
double oracle_decode_f16(uint16_t h);
double oracle_decode_bf16(uint16_t h);

static unsigned rng = 2024;
static int small_int(void) { rng = rng * 1664525u + 1013904223u; return (int)((rng >> 10) % 7) - 3; }

/* encode a small integer in the storage type: 0 fp32, 1 f16, 2 bf16 */
static void put(void *base, int dtype, int64_t idx, int v)
{
    if (dtype == 0) { ((float *)base)[idx] = (float)v; return; }
    float f = (float)v;
    uint32_t b;
    memcpy(&b, &f, 4);
    if (dtype == 2) { ((uint16_t *)base)[idx] = (uint16_t)(b >> 16); return; }
    /* f16 of a small integer: sign, exponent rebias, 10 mantissa bits (exact for |v| < 2048) */
    uint16_t h = 0;
    if (v != 0) {
        const uint32_t sign = b >> 31, exp = (b >> 23) & 0xFF, man = b & 0x7FFFFF;
        h = (uint16_t)((sign << 15) | ((exp - 127 + 15) << 10) | (man >> 13));
    }
    ((uint16_t *)base)[idx] = h;
}

int main(void)
{
    long cases = 0;
    for (int i = 0; i < 65536; i += 97) { (void)oracle_decode_f16((uint16_t)i); (void)oracle_decode_bf16((uint16_t)i); }
    for (int dtype = 0; dtype < 3; ++dtype)
        for (int ta = 0; ta < 2; ++ta)
            for (int tb = 0; tb < 2; ++tb)
                for (int it = 0; it < 40; ++it) {
                    const int64_t M = 1 + (it * 7) % 9, N = 1 + (it * 5) % 11, K = (it % 8 == 0) ? 0 : 1 + (it * 3) % 13;
                    const int64_t lda = (ta ? M : K) + it % 3 + (K == 0), ldb = (tb ? K : N) + it % 2 + (K == 0), ldc = N + it % 4;
                    const int cdtype = (dtype != 0 && it % 5 == 0) ? 0 : dtype;
                    const int es = dtype == 0 ? 4 : 2, esc = cdtype == 0 ? 4 : 2;
                    const int64_t arows = ta ? K : M, brows = tb ? N : K;
                    void *A = malloc((size_t)(arows * lda * es) + 1), *B = malloc((size_t)(brows * ldb * es) + 1), *C = malloc((size_t)(M * ldc * esc));
                    int *ia = calloc((size_t)(M * K) + 1, sizeof(int)), *ib = calloc((size_t)(K * N) + 1, sizeof(int)), *ic = calloc((size_t)(M * N), sizeof(int));
                    memset(A, 0x7F, (size_t)(arows * lda * es) + 1); memset(B, 0x7F, (size_t)(brows * ldb * es) + 1); memset(C, 0x7F, (size_t)(M * ldc * esc));
                    for (int64_t i = 0; i < M; ++i) for (int64_t k = 0; k < K; ++k) { ia[i * K + k] = small_int(); put(A, dtype, ta ? k * lda + i : i * lda + k, ia[i * K + k]); }
                    for (int64_t k = 0; k < K; ++k) for (int64_t j = 0; j < N; ++j) { ib[k * N + j] = small_int(); put(B, dtype, tb ? j * ldb + k : k * ldb + j, ib[k * N + j]); }
                    for (int64_t i = 0; i < M; ++i) for (int64_t j = 0; j < N; ++j) { ic[i * N + j] = small_int(); put(C, cdtype, i * ldc + j, ic[i * N + j]); }
                    const double alpha = (double)(it % 4 - 1), beta = (double)(it % 3 - 1);
                    int64_t rows[4] = {M - 1, 0, M / 2, M - 1};
                    const int use_rows = it % 3 == 1;
                    const int64_t nr = use_rows ? 4 : M;
                    double *ref = malloc((size_t)(nr * N) * sizeof(double));
                    for (int order = -1; order <= 1; ++order)
                        for (int threads = 1; threads <= 5; threads += 2) {
                            const int rc = oracle_gemm_c(dtype, cdtype, ta, tb, M, N, K, alpha, A, lda, B, ldb, beta, beta != 0.0 ? C : NULL, ldc,
                                                         use_rows ? rows : NULL, use_rows ? 4 : 0, ref, order, threads);
                            if (rc != 0) { fprintf(stderr, "oracle_gemm_c refused a valid call\n"); return 1; }
                            for (int64_t r = 0; r < nr; ++r) {
                                const int64_t i = use_rows ? rows[r] : r;
                                for (int64_t j = 0; j < N; ++j) {
                                    long s = 0;
                                    for (int64_t k = 0; k < K; ++k) s += (long)ia[i * K + k] * ib[k * N + j];
                                    const double want = alpha * (double)s + (beta != 0.0 ? beta * (double)ic[i * N + j] : 0.0);
                                    if (ref[r * N + j] != want) { fprintf(stderr, "wrong value dtype %d ta %d tb %d it %d\n", dtype, ta, tb, it); return 1; }
                                }
                            }
                            ++cases;
                        }
                    float *bias = malloc((size_t)(M > N ? M : N) * sizeof(float));
                    for (int64_t i = 0; i < (M > N ? M : N); ++i) bias[i] = (float)small_int();
                    for (int kind = 0; kind < 3; ++kind)
                        for (int act = 0; act < 3; ++act)
                            if (oracle_bias_act(M, N, use_rows ? rows : NULL, use_rows ? 4 : 0, ref, kind, bias, act) != 0) return 1;
                    /* refusals must come before any access */
                    if (oracle_gemm_c(dtype, cdtype, ta, tb, M, N, K, 1.0, A, (ta ? M : K) - 1, B, ldb, 0.0, NULL, ldc, NULL, 0, ref, -1, 1) == 0 && (ta ? M : K) > 0) return 1;
                    rows[1] = M;
                    if (oracle_gemm_c(dtype, cdtype, ta, tb, M, N, K, 1.0, A, lda, B, ldb, 0.0, NULL, ldc, rows, 4, ref, -1, 1) == 0) return 1;
                    free(bias); free(ref); free(A); free(B); free(C); free(ia); free(ib); free(ic);
                }
    printf("oracle sanitizer run clean: %ld calls checked\n", cases);
    return 0;
}
