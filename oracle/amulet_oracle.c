/*
 * CPU oracle for AMULET's matrix-multiplication-like tasks.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the HIP path, and
 * only the tests, the smoke check and the bench's cpu_baseline leg may call it.
 *
 * What it computes is the triple loop the paper states for its tasks
 * (Fig. 1 "expected revenue", Fig. 2 "net weighted strength", and Query 1-3 of
 * the "Test Queries" figure in Sec. 6.3):
 *
 *     for i < M, j < N, k < K:   R[i][j] += g( A[i][k] * B[k][j], params[j] )
 *
 * with, writing p for the product A[i][k]*B[k][j]:
 *
 *     IDENTITY  g = p                                    (plain matmul, Sec. 6.1)
 *     DISCOUNT  g = p - (p > thres[j]) * p * dis[j]      (Fig. 1 / Query 1)
 *     BOOST     g = p + (p > thres[j]) * (p - thres[j])  (Fig. 2 / Query 2)
 *     COUNT_GT  g = (p > thres[j])                       (Query 3, with the
 *               constant generalised to the thres[j] operand form the same
 *               figure allows)
 *
 * Readings of points the paper leaves open:
 *  - Inputs and outputs are fp32 (the paper's listings use double; the
 *    workloads this build is measured on are fp32).  The product p is ONE
 *    IEEE round-to-nearest fp32 multiply and the comparison p > thres[j] is
 *    done on that fp32 value, strictly (the paper's "gtcmp"): a tie does not
 *    trigger.  Everything after the comparison is carried in double, and the
 *    k-sum is accumulated in double in increasing k.
 *  - "(p > thres) * x" is a mask/select, as the paper's "Mask -" DAG node and
 *    masked SIMD subtract say (Sec. 4.3.1): the term is x when the predicate
 *    holds and absent otherwise.
 *  - The common sub-expression p is evaluated once (the paper's DAG after
 *    CSE), i.e. DISCOUNT's subtracted part is p*dis.
 *  - "+=": the sum is added to what R already holds (the inner kernel adds
 *    its sub-results to C, Fig. "12x16 inner kernel").
 *
 * abs_sum (optional) receives sum_k |g(...)| per output, the denominator of
 * the fp32 parity metric  |R_gpu - R_ref| / sum_k |term|.
 *
 * Built as a small shared library with gcc (-O2 -fopenmp -ffp-contract=off).
 * Threads split the rows i; the arithmetic of one (i,j) output is never split
 * or reordered.
 */
#include <float.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* float expressions must be evaluated in float: the product is rounded once. */
#if !defined(FLT_EVAL_METHOD) || FLT_EVAL_METHOD != 0
#error "oracle needs FLT_EVAL_METHOD == 0 (fp32 products rounded to fp32)"
#endif

enum { ORACLE_IDENTITY = 0, ORACLE_DISCOUNT = 1, ORACLE_BOOST = 2, ORACLE_COUNT_GT = 3 };

/* One term g(p, params[j]) in double; p is the already rounded fp32 product. */
static double oracle_term(int task, float p, const float *params, int64_t N, int64_t j)
{
    const double pd = (double)p;
    switch (task) {
    case ORACLE_IDENTITY:
        return pd;
    case ORACLE_DISCOUNT: {
        const float thres = params[j];
        const double dis = (double)params[N + j];
        if (p > thres)
            return pd - pd * dis;
        return pd;
    }
    case ORACLE_BOOST: {
        const float thres = params[j];
        if (p > thres)
            return pd + (pd - (double)thres);
        return pd;
    }
    case ORACLE_COUNT_GT: {
        const float thres = params[j];
        return (p > thres) ? 1.0 : 0.0;
    }
    default:
        return NAN;
    }
}

/*
 * R[i*ldr+j] = (float)( (double)R[i*ldr+j] + sum_k g(fl32(A[i*lda+k]*B[k*ldb+j]), params[j]) )
 *
 * params: DISCOUNT thres[0..N) then dis[0..N); BOOST and COUNT_GT thres[0..N);
 *         IDENTITY ignores it (may be NULL).
 * abs_sum: NULL, or M*N doubles (row stride N) receiving sum_k |term|.
 * nthreads <= 0 means "all cores OpenMP reports".
 * Returns 0, or -1 for an unknown task; *threads_used (if not NULL) gets the
 * number of threads the row loop ran on.
 */
int oracle_mmlike_f32(int task, int64_t M, int64_t N, int64_t K,
                      const float *A, int64_t lda,
                      const float *B, int64_t ldb,
                      const float *params,
                      float *R, int64_t ldr,
                      double *abs_sum, int nthreads, int *threads_used)
{
    if (task < ORACLE_IDENTITY || task > ORACLE_COUNT_GT)
        return -1;
    int used = 1;
#ifdef _OPENMP
    if (nthreads <= 0)
        nthreads = omp_get_max_threads();
    if ((int64_t)nthreads > M)
        nthreads = M > 0 ? (int)M : 1;
    used = nthreads;
#pragma omp parallel for schedule(static) num_threads(nthreads)
#endif
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            double abs_acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const float p = A[i * lda + k] * B[k * ldb + j]; /* one fp32 RN multiply */
                const double t = oracle_term(task, p, params, N, j);
                acc += t;
                abs_acc += fabs(t);
            }
            R[i * ldr + j] = (float)((double)R[i * ldr + j] + acc);
            if (abs_sum)
                abs_sum[i * N + j] = abs_acc;
        }
    }
    if (threads_used)
        *threads_used = used;
    return 0;
}

/*
 * Natural-join count written as a matrix product (the join-as-matmul
 * translation the paper's introduction cites): with A[i][k] = 1 when tuple i
 * of the left relation carries join key k, and B[k][j] likewise for the right
 * relation, R[i][j] += sum_k A[i][k]*B[k][j] counts the matching keys.
 * Any int8 values are accepted; the sum is formed in int64 and the call
 * returns -2 (leaving that element unwritten) if R_in + sum leaves int32.
 */
int oracle_count_i8(int64_t M, int64_t N, int64_t K,
                    const int8_t *A, int64_t lda,
                    const int8_t *B, int64_t ldb,
                    int32_t *R, int64_t ldr, int nthreads, int *threads_used)
{
    int used = 1;
    int status = 0;
#ifdef _OPENMP
    if (nthreads <= 0)
        nthreads = omp_get_max_threads();
    if ((int64_t)nthreads > M)
        nthreads = M > 0 ? (int)M : 1;
    used = nthreads;
#pragma omp parallel for schedule(static) num_threads(nthreads)
#endif
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            int64_t acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += (int64_t)A[i * lda + k] * (int64_t)B[k * ldb + j];
            acc += (int64_t)R[i * ldr + j];
            if (acc > INT32_MAX || acc < INT32_MIN) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
                status = -2;
            } else {
                R[i * ldr + j] = (int32_t)acc;
            }
        }
    }
    if (threads_used)
        *threads_used = used;
    return status;
}
