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

enum { ORACLE_THRES_COL = 0, ORACLE_THRES_ROW = 1, ORACLE_THRES_CONST = 2, ORACLE_THRES_ELEM = 3 };

/* One term g(p, thres, dis) in double; p is the already rounded fp32 product. */
static double oracle_term(int task, float p, float thres, double dis)
{
    const double pd = (double)p;
    switch (task) {
    case ORACLE_IDENTITY:
        return pd;
    case ORACLE_DISCOUNT:
        if (p > thres)
            return pd - pd * dis;
        return pd;
    case ORACLE_BOOST:
        if (p > thres)
            return pd + (pd - (double)thres);
        return pd;
    case ORACLE_COUNT_GT:
        return (p > thres) ? 1.0 : 0.0;
    default:
        return NAN;
    }
}

/*
 * The general form of the paper's test queries ("Test Queries" figure, Sec. 6.3):
 *
 *   R[i][j] += sum_k g( fl32(a(i,k) * b(k,j)), thres(i,j), dis[j] )
 *
 * a(i,k) is A[i*lda+k], or A[k*lda+i] when transA (the variant that indexes
 * A as [k][i]); b(k,j) is B[k*ldb+j], or B[j*ldb+k] when transB.  The threshold
 * operand takes the four forms the figure lists: thres[j] (COL), thres[i] (ROW),
 * a constant (CONST, thres[0]) and thres[i][j] (ELEM, row pitch ldt).  dis is
 * indexed by j as printed (only the DISCOUNT task reads it).
 */
int oracle_mmlike_f32_general(int task, int thres_form, int transA, int transB,
                              int64_t M, int64_t N, int64_t K,
                              const float *A, int64_t lda,
                              const float *B, int64_t ldb,
                              const float *thres, int64_t ldt, const float *dis,
                              float *R, int64_t ldr,
                              double *abs_sum, int nthreads, int *threads_used)
{
    if (task < ORACLE_IDENTITY || task > ORACLE_COUNT_GT)
        return -1;
    if (thres_form < ORACLE_THRES_COL || thres_form > ORACLE_THRES_ELEM)
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
            float th = 0.0f;
            double d = 0.0;
            if (task != ORACLE_IDENTITY) {
                switch (thres_form) {
                case ORACLE_THRES_COL: th = thres[j]; break;
                case ORACLE_THRES_ROW: th = thres[i]; break;
                case ORACLE_THRES_CONST: th = thres[0]; break;
                default: th = thres[i * ldt + j]; break;
                }
                if (task == ORACLE_DISCOUNT)
                    d = (double)dis[j];
            }
            double acc = 0.0;
            double abs_acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const float a = transA ? A[k * lda + i] : A[i * lda + k];
                const float b = transB ? B[j * ldb + k] : B[k * ldb + j];
                const float p = a * b; /* one fp32 RN multiply */
                const double t = oracle_term(task, p, th, d);
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
 * The row-major, thres[j] form with planar parameters:
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
    return oracle_mmlike_f32_general(task, ORACLE_THRES_COL, 0, 0, M, N, K, A, lda, B, ldb, params, 0,
                                     params ? params + N : NULL, R, ldr, abs_sum, nthreads,
                                     threads_used);
}

/*
 * The same general form in the paper's own element type, double (its listings declare
 * double A[M][K], B[K][N], C[M][N]; Sec. 3, Sec. 4.3.3): inputs, outputs and parameters are
 * fp64, the product p is ONE round-to-nearest fp64 multiply, the comparison is made on that
 * fp64 value, strictly, and everything after it (terms, k-sum, the addition to R) is carried
 * in long double (64-bit significand on x86-64), so the reference is more precise than any
 * fp64 summation order it is compared with.
 */
static long double oracle_term_f64(int task, double p, double thres, double dis)
{
    const long double pd = (long double)p;
    switch (task) {
    case ORACLE_IDENTITY:
        return pd;
    case ORACLE_DISCOUNT:
        if (p > thres)
            return pd - pd * (long double)dis;
        return pd;
    case ORACLE_BOOST:
        if (p > thres)
            return pd + (pd - (long double)thres);
        return pd;
    case ORACLE_COUNT_GT:
        return (p > thres) ? 1.0L : 0.0L;
    default:
        return NAN;
    }
}

int oracle_mmlike_f64_general(int task, int thres_form, int transA, int transB,
                              int64_t M, int64_t N, int64_t K,
                              const double *A, int64_t lda,
                              const double *B, int64_t ldb,
                              const double *thres, int64_t ldt, const double *dis,
                              double *R, int64_t ldr,
                              double *abs_sum, int nthreads, int *threads_used)
{
    if (task < ORACLE_IDENTITY || task > ORACLE_COUNT_GT)
        return -1;
    if (thres_form < ORACLE_THRES_COL || thres_form > ORACLE_THRES_ELEM)
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
            double th = 0.0, d = 0.0;
            if (task != ORACLE_IDENTITY) {
                switch (thres_form) {
                case ORACLE_THRES_COL: th = thres[j]; break;
                case ORACLE_THRES_ROW: th = thres[i]; break;
                case ORACLE_THRES_CONST: th = thres[0]; break;
                default: th = thres[i * ldt + j]; break;
                }
                if (task == ORACLE_DISCOUNT)
                    d = dis[j];
            }
            long double acc = 0.0L, abs_acc = 0.0L;
            for (int64_t k = 0; k < K; ++k) {
                const double a = transA ? A[k * lda + i] : A[i * lda + k];
                const double b = transB ? B[j * ldb + k] : B[k * ldb + j];
                const double p = a * b; /* one fp64 RN multiply */
                const long double t = oracle_term_f64(task, p, th, d);
                acc += t;
                abs_acc += fabsl(t);
            }
            R[i * ldr + j] = (double)((long double)R[i * ldr + j] + acc);
            if (abs_sum)
                abs_sum[i * N + j] = (double)abs_acc;
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
