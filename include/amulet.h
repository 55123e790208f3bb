/*
 * amulet.h - C ABI of the MI355X (gfx950) library for AMULET's
 * matrix-multiplication-like tasks.
 *
 * A matrix-multiplication-like task (paper Sec. 4.2) is the triple loop
 *
 *     for i < M, j < N, k < K:   R[i][j] += g( A[i][k] * B[k][j], params[j] )
 *
 * in which g acts on every single product before the k-reduction, so the task
 * is not a GEMM.  The tasks built here are the ones the paper states and
 * measures (Fig. 1, Fig. 2, "Test Queries" figure of Sec. 6.3, Sec. 6.1), plus
 * the join-count-as-matmul case its introduction cites.
 *
 * Conventions common to every entry point
 *  - Every matrix pointer is a DEVICE pointer owned by the caller.  The
 *    library reads A, B, params and reads+writes R; it never frees, retains
 *    or reallocates them.  R must not overlap A, B or params.
 *  - Matrices are row-major with a leading dimension in ELEMENTS (lda >= K,
 *    ldb >= N, ldr >= N): as in the paper's interface (Sec. 5) the rows of a
 *    matrix may be spaced apart in memory.  Any M, N, K >= 0 is accepted;
 *    edge tiles are handled inside.
 *  - `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *    Compute calls only enqueue work and return; they never synchronise or
 *    allocate (amulet_tune, amulet_mmlike_f32_adaptive and the two probes do
 *    both, and say so below).
 *  - Return value: AMULET_OK (0) or a negative amulet_status_t.  Nothing is
 *    enqueued when an argument error is returned.  M == 0, N == 0 or K == 0 is
 *    a successful no-op (R unchanged).
 *  - The k-sum is formed in an order the library chooses (the paper's loop
 *    is order-free, Sec. 4.1).  Tiles that would leave most of the chip idle
 *    (all of them when M x N gives too few tiles to fill it, else those of a
 *    last round of workgroups that is at most half full) have K split over
 *    several workgroups that add their parts to R atomically: floating-point
 *    results of such tiles may differ in the last bits from run to run
 *    (integer results never do; a COUNT_GT count added in parts to a
 *    fractional R is rounded once per part).  R must be
 *    ordinary device memory (hipMalloc or a framework's device allocator):
 *    the hardware atomics used there are not defined on fine-grained or
 *    host-mapped memory.
 *  - A or B holding NaN or +-inf gives unspecified results, and so does a NaN
 *    in thres; +-inf in thres is supported (thres = +inf never triggers, -inf
 *    always does), and so are zeros of either sign and subnormal values.
 */
#ifndef AMULET_H
#define AMULET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    AMULET_IDENTITY = 0, /* g = p                         plain matmul, Sec. 6.1            */
    AMULET_DISCOUNT = 1, /* g = p - (p > thres[j])*p*dis[j]        Fig. 1 / Query 1         */
    AMULET_BOOST = 2,    /* g = p + (p > thres[j])*(p - thres[j])  Fig. 2 / Query 2         */
    AMULET_COUNT_GT = 3  /* g = (p > thres[j])   Query 3, constant in its thres[j] form     */
} amulet_task_t;

typedef enum {
    AMULET_OK = 0,
    AMULET_ERR_TASK = -1,   /* unknown task                                   */
    AMULET_ERR_DIM = -2,    /* a negative dimension                           */
    AMULET_ERR_NULL = -3,   /* a required pointer is NULL                     */
    AMULET_ERR_LD = -4,     /* a leading dimension is smaller than the row    */
    AMULET_ERR_LAUNCH = -5, /* HIP reported an error at launch                */
    AMULET_ERR_SHAPE = -6,  /* unknown tile-shape id, or one the task lacks   */
    AMULET_ERR_RANGE = -7,  /* a dimension exceeds what the kernels index     */
    AMULET_ERR_WORKSPACE = -8 /* the workspace lent to the call is too small   */
} amulet_status_t;

/*
 * R[i][j] += sum_k g(fl32(A[i][k]*B[k][j]), params[j])        (Fig. 1, Fig. 2, Query 1-3)
 *
 * p is one IEEE round-to-nearest fp32 multiply and "p > thres[j]" is decided
 * on that rounded value, strictly, exactly as a plain fp32 loop would; the
 * predicate acts as a mask (the paper's "Mask -" node, Sec. 4.3.1).  This holds
 * bit for bit for DISCOUNT and COUNT_GT, whose g jumps at p = thres.  BOOST's
 * g = p + max(p - thres, 0) is continuous in p, and the kernels evaluate it
 * with fused multiply-adds on the unrounded product: a term differs from the
 * rounded-product term by at most one rounding of p (2^-24 |p|, twice that for
 * a triggered term), inside the tolerance below but not bit-identical to a
 * loop that rounds p first.  The k-sum
 * is formed in fp32 in an order the library chooses (the paper's loop is
 * order-free, Sec. 4.1): results agree with a double-accumulating loop to
 * within 1e-5 * sum_k |term|.
 *
 *   task    one of amulet_task_t
 *   A       M x K fp32, lda >= K            B   K x N fp32, ldb >= N
 *   params  planar fp32: DISCOUNT thres[0..N) then dis[0..N); BOOST and
 *           COUNT_GT thres[0..N); IDENTITY ignores it (may be NULL)
 *   R       M x N fp32, ldr >= N, accumulated into ("+=", Fig. "12x16 inner kernel")
 *
 * The tile shape is the one amulet_tune() cached for this (task, M, N, K), or
 * a built-in default.  Each dimension must be below 2^31 - 2^16.
 */
int amulet_mmlike_f32(int task, int64_t M, int64_t N, int64_t K,
                      const float *A, int64_t lda,
                      const float *B, int64_t ldb,
                      const float *params,
                      float *R, int64_t ldr,
                      void *stream);

/* Same, with the tile shape given explicitly (0 <= shape < amulet_shape_count(task)):
 * the parameterised form of the loop nest, Sec. 4.4, used by the selector's
 * trials and by tests that exercise every shape. */
int amulet_mmlike_f32_shape(int task, int shape, int64_t M, int64_t N, int64_t K,
                            const float *A, int64_t lda,
                            const float *B, int64_t ldb,
                            const float *params,
                            float *R, int64_t ldr,
                            void *stream);

/* Form of the threshold operand of a predicate task: the four the paper's
 * "Test Queries" figure lists (Sec. 6.3). */
typedef enum {
    AMULET_THRES_COL = 0,   /* thres[j], N values                      */
    AMULET_THRES_ROW = 1,   /* thres[i], M values                      */
    AMULET_THRES_CONST = 2, /* one constant, thres[0]                  */
    AMULET_THRES_ELEM = 3   /* thres[i][j], M x N row-major, pitch ldt */
} amulet_thres_form_t;

/*
 * The general form of the test queries (Sec. 6.3):
 *
 *   R[i][j] += sum_k g( fl32(a(i,k)*b(k,j)), thres(i,j), dis[j] )
 *
 * a(i,k) = A[i*lda+k], or A[k*lda+i] when trans_a != 0 (the variant of
 * Sec. 6.3 that indexes A as [k][i]: A is then K x M, lda >= M); b(k,j) = B[k*ldb+j], or B[j*ldb+k]
 * when trans_b != 0 (B is then N x K, ldb >= K).  `thres` is read in the form
 * `thres_form` names (ldt >= N is used by AMULET_THRES_ELEM only); `dis` is
 * dis[0..N) and is read by AMULET_DISCOUNT only; both are ignored (may be
 * NULL) for AMULET_IDENTITY.  `shape` is a tile-shape id of the task, or -1
 * for the selected/default one (every shape of a task, the matrix-core
 * identity kernel included, takes all four layouts).  Other conventions as for amulet_mmlike_f32, which is
 * this call with thres[j], no transposition, shape -1 and planar params.
 */
int amulet_mmlike_f32_general(int task, int thres_form, int trans_a, int trans_b, int shape,
                              int64_t M, int64_t N, int64_t K,
                              const float *A, int64_t lda,
                              const float *B, int64_t ldb,
                              const float *thres, int64_t ldt,
                              const float *dis,
                              float *R, int64_t ldr,
                              void *stream);

/*
 * The same tasks in the paper's own element type (its listings declare
 * double A[M][K], B[K][N], C[M][N]: Sec. 3, Sec. 4.3.3, Sec. 6.3):
 *
 *   R[i][j] += sum_k g( fl64(A[i*lda+k]*B[k*ldb+j]), thres(i,j), dis[j] )
 *
 * One IEEE fp64 multiply per product, strict fp64 comparison, fp64 accumulation
 * in unspecified order.  Row-major operands only; `thres_form`, `thres`, `ldt`
 * and `dis` as for amulet_mmlike_f32_general; all pointers are device pointers
 * to doubles (8-byte aligned), owned by the caller; pitches in elements.  The
 * vector-ALU tile shape is the one selected for the size (amulet_mmlike_f64_adaptive),
 * else a built-in choice.  Enqueues on `stream` and returns; same error codes as
 * the fp32 calls.
 */
int amulet_mmlike_f64(int task, int thres_form,
                      int64_t M, int64_t N, int64_t K,
                      const double *A, int64_t lda,
                      const double *B, int64_t ldb,
                      const double *thres, int64_t ldt,
                      const double *dis,
                      double *R, int64_t ldr,
                      void *stream);

/*
 * amulet_mmlike_f64 with the transposed operand layouts of Sec. 6.3 (as in
 * amulet_mmlike_f32_general: A stored K x M with lda >= M when trans_a != 0,
 * B stored N x K with ldb >= K when trans_b != 0).
 */
int amulet_mmlike_f64_general(int task, int thres_form, int trans_a, int trans_b,
                              int64_t M, int64_t N, int64_t K,
                              const double *A, int64_t lda,
                              const double *B, int64_t ldb,
                              const double *thres, int64_t ldt,
                              const double *dis,
                              double *R, int64_t ldr,
                              void *stream);

/*
 * fp64 tile shapes (the counterpart of the fp32 shape grid, Sec. 4.4-4.6): shape id =
 * k-axis index * 2 + tile; tile 0 = 16 x 128 (4 waves), 1 = 32 x 128 (8 waves); k axis
 * 0 = a workgroup sums a tile's whole K (split only where the launcher's own rule asks
 * for it), 1, 2 = every tile's K in 2, 4 parts added to R with fp64 atomics (not
 * bit-reproducible; ignored in deterministic mode).  The identity task runs on the
 * matrix cores whatever the shape; to it only the tile index means something: 0 = tiles
 * of 64 x 64, 1 = of 128 x 128 (the built-in choice: 64 x 64 for a problem with fewer
 * 128 x 128 tiles than the chip has compute units).
 *   amulet_f64_shape_count      number of shape ids (6)
 *   amulet_f64_shape_name       static string, "invalid" for a bad id
 *   amulet_selected_shape_f64   shape a plain call uses for (task, M, N, K): the cached
 *                               selection of its size bucket, else the built-in choice;
 *                               AMULET_ERR_TASK for a bad task
 *   amulet_mmlike_f64_shape     amulet_mmlike_f64_general with an explicit shape
 *                               (-1: as selected); AMULET_ERR_SHAPE for an id >= count
 */
int amulet_f64_shape_count(void);
const char *amulet_f64_shape_name(int shape);
int amulet_selected_shape_f64(int task, int64_t M, int64_t N, int64_t K);
int amulet_mmlike_f64_shape(int task, int shape, int thres_form, int trans_a, int trans_b,
                            int64_t M, int64_t N, int64_t K,
                            const double *A, int64_t lda,
                            const double *B, int64_t ldb,
                            const double *thres, int64_t ldt,
                            const double *dis,
                            double *R, int64_t ldr,
                            void *stream);

/*
 * (All adaptive calls: a trial's end is waited for on the host before the next is chosen,
 * which costs the GPU some tens of microseconds of idling per trial; when the first trial
 * shows the whole task to be shorter than 3 ms, no further trial is run and the task goes on
 * with the shape just tried.  The environment variable AMULET_ADAPTIVE_MIN_TASK_MS overrides
 * the 3; 0 switches the rule off.  Candidates whose order is fixed in advance -- the identity
 * task's and the join count's -- are enqueued back to back and waited for once.)
 *
 * In-flight adaptive execution (Sec. 4.4-4.6) in the paper's own element type: as
 * amulet_mmlike_f32_adaptive_general, on the fp64 shape grid.  Trials are disjoint row
 * slabs of the caller's R (the shape a plain call would use first, then the k axis,
 * then the tile axis with an early stop; at most half of the rows), scored by time per
 * row; the rest runs with the fastest slab's shape, which is cached for the size
 * bucket and used by later plain fp64 calls.  The result is the complete task, as if
 * amulet_mmlike_f64_general had been called.  Allocates two events and blocks the
 * host while trials run; tasks too small for three slabs, and the identity task (one
 * matrix-core kernel), run whole without trials.  `chosen_shape`, `n_trials` may be
 * NULL.  Same error codes as amulet_mmlike_f64_general.
 */
int amulet_mmlike_f64_adaptive(int task, int thres_form, int trans_a, int trans_b,
                               int64_t M, int64_t N, int64_t K,
                               const double *A, int64_t lda,
                               const double *B, int64_t ldb,
                               const double *thres, int64_t ldt,
                               const double *dis,
                               double *R, int64_t ldr,
                               void *stream, int *chosen_shape, int *n_trials);

/*
 * Packing (Sec. 3.1 and the "with packing" series of Sec. 6): an operand is copied
 * once into storage whose layout suits the kernels' access order, at the price of
 * memory the caller must agree to spend.  The kernels of this library read the
 * caller's row-major operands in place at full speed with one exception, which
 * is what the packed copy removes: when the row pitch of A in bytes is a multiple
 * of 32 KiB and at least 64 KiB (a long power-of-two K), the rows a workgroup of
 * the vector-ALU kernels reads at one k fall into the same cache sets and memory
 * channel, and those kernels run at 45-95 % of their rate.  The packed copy
 * spaces its rows by amulet_packed_ld(), which never collides.
 *
 *   amulet_pitch_collides   1 if rows `ld` elements of `elem_bytes` (1, 4, 8) apart
 *                           collide in that way, else 0
 *   amulet_packed_ld        pitch, in elements, for a packed copy of rows of `cols`
 *                           elements (>= cols; 0 for invalid arguments)
 *   amulet_pack             dst[r*ld_dst + c] = src[r*ld_src + c] for r < rows,
 *                           c < cols; device pointers, dst and src must not overlap;
 *                           enqueued on `stream`; AMULET_ERR_DIM for an element size
 *                           other than 1, 4, 8 or a negative extent, AMULET_ERR_LD
 *                           for a pitch below cols, AMULET_ERR_NULL
 */
int amulet_pitch_collides(int64_t ld, int elem_bytes);
int64_t amulet_packed_ld(int64_t cols, int elem_bytes);
int amulet_pack(int elem_bytes, int64_t rows, int64_t cols,
                const void *src, int64_t ld_src,
                void *dst, int64_t ld_dst, void *stream);

/*
 * The general calls with packing allowed (the user-granted "auto-packing" of
 * Sec. 3.1).  `workspace` is device memory the caller lends for the duration of
 * the call's work on `stream` (the library never allocates in a compute call);
 * amulet_autopack_workspace_bytes(elem_bytes, M, K) is the size a call may need.
 * When A is row-major, its pitch collides (above), the task runs on the vector
 * ALUs and N >= 128, A is first copied to the workspace with a packed pitch
 * (one more kernel on the same stream) and the task reads the copy; otherwise,
 * or when `workspace` is NULL, the call is the plain general call.  Results are
 * those of the plain call (the same kernels on the same values).
 * AMULET_ERR_WORKSPACE if the call wants to pack and `workspace_bytes` is too
 * small; other errors as for the general calls.
 */
size_t amulet_autopack_workspace_bytes(int elem_bytes, int64_t M, int64_t K);
int amulet_mmlike_f32_autopack(int task, int thres_form, int trans_a, int trans_b,
                               int64_t M, int64_t N, int64_t K,
                               const float *A, int64_t lda,
                               const float *B, int64_t ldb,
                               const float *thres, int64_t ldt,
                               const float *dis,
                               float *R, int64_t ldr,
                               void *workspace, size_t workspace_bytes,
                               void *stream);
int amulet_mmlike_f64_autopack(int task, int thres_form, int trans_a, int trans_b,
                               int64_t M, int64_t N, int64_t K,
                               const double *A, int64_t lda,
                               const double *B, int64_t ldb,
                               const double *thres, int64_t ldt,
                               const double *dis,
                               double *R, int64_t ldr,
                               void *workspace, size_t workspace_bytes,
                               void *stream);

/*
 * Natural-join count as a matrix product (the join-as-matmul translation cited
 * in Sec. 1): R[i][j] += sum_k A[i][k]*B[k][j], int8 operands (any values; the
 * workload is 0/1 indicators), int32 result, exact (wraps modulo 2^32 only if
 * the true sum leaves int32).  A is M x K (lda >= K), B is K x N (ldb >= N),
 * R is M x N int32 (ldr >= N).
 * (Diagnostic: the environment variable AMULET_I8_PHASES="g,s,x,h" -- g slot
 * groups per XCD, s 64-k stages between them, XCD modulus x in 1..8, XCD span h
 * in sixteenths of K -- overrides how the persistent kernel of large problems
 * spreads its workgroups' write-backs in time; it changes timing only, never
 * results.)
 */
int amulet_count_i8(int64_t M, int64_t N, int64_t K,
                    const int8_t *A, int64_t lda,
                    const int8_t *B, int64_t ldb,
                    int32_t *R, int64_t ldr,
                    void *stream);

/* Same, with the kernel shape given explicitly
 * (0 <= shape < amulet_shape_count(AMULET_TASK_COUNT_I8)). */
int amulet_count_i8_shape(int shape, int64_t M, int64_t N, int64_t K,
                          const int8_t *A, int64_t lda,
                          const int8_t *B, int64_t ldb,
                          int32_t *R, int64_t ldr,
                          void *stream);

/*
 * The join count written, not accumulated: R[i][j] = sum_k A[i][k]*B[k][j] (the
 * count itself, as the join-as-matmul translation of Sec. 1 produces it; what R
 * held before is ignored and need not be initialised).  Same operands, result
 * type, exactness and error codes as amulet_count_i8; `shape` as for
 * amulet_count_i8_shape, or -1 for the selected shape.  K == 0 sets R to zero.
 * The kernels do not read R where one workgroup owns a tile (large problems:
 * half of the write-back's memory traffic less); a launch that splits K over
 * workgroups clears R with a fill kernel first and adds.  (The persistent
 * kernel's workgroups run in step in this form unless AMULET_I8_PHASES says
 * otherwise.)  Enqueues and returns; nothing is allocated.
 */
int amulet_count_i8_assign(int shape, int64_t M, int64_t N, int64_t K,
                           const int8_t *A, int64_t lda,
                           const int8_t *B, int64_t ldb,
                           int32_t *R, int64_t ldr,
                           void *stream);

/*
 * The join count with operands stored transposed (the layouts of Sec. 6.3
 * applied to this task): A stored K x M (lda >= M) when trans_a != 0, B stored
 * N x K (ldb >= K) when trans_b != 0.  The matrix-core kernels read row-major
 * operands; a transposed operand is first copied, transposed, into `workspace`
 * (device memory the caller lends for the duration of the call's work on
 * `stream`; amulet_count_i8_workspace_bytes gives the size, 0 when neither
 * flag is set, and then `workspace` may be NULL): one more kernel per such
 * operand on the same stream, 3-4 % of the 8192 x 8192 x 4096 join each.
 * The result is that of amulet_count_i8 on the row-major operands, exact.
 * AMULET_ERR_NULL if a workspace is needed and NULL, AMULET_ERR_WORKSPACE if
 * it is too small; other errors as amulet_count_i8.
 *
 * A larger workspace, of amulet_count_i8_repack_workspace_bytes(M, N, K) bytes
 * and 16-byte aligned, is also the operands' aligned home when they need one
 * (this is the packing of Sec. 3.1 for the join count: the fastest kernel
 * streams whole 16-byte units of rows that start on 16-byte boundaries, 64 k
 * at a time, and a workgroup whose whole tile of A rows and B columns exists
 * in memory loads without guards).  An operand whose base or row pitch is not
 * a multiple of 16 bytes, or whose M resp. N is not a multiple of 256, is
 * copied to an aligned pitch with room for whole tiles around it, and when K
 * is not a multiple of 64 both operands are copied with K padded by zero
 * bytes, which add nothing to a count.  The copies are one kernel per operand
 * on `stream`; operands that need none are read in place.  Same result,
 * exact.  (R is never copied: rows of R that are not 16-byte aligned are
 * written by the slower write-back.)
 */
size_t amulet_count_i8_workspace_bytes(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K);
size_t amulet_count_i8_repack_workspace_bytes(int64_t M, int64_t N, int64_t K);
int amulet_count_i8_general(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K,
                            const int8_t *A, int64_t lda,
                            const int8_t *B, int64_t ldb,
                            int32_t *R, int64_t ldr,
                            void *workspace, size_t workspace_bytes,
                            void *stream);

/*
 * amulet_count_i8 with in-flight adaptive execution (Sec. 4.4): the matrix-core kernels of
 * the join count are tried on disjoint slabs of rows of the caller's R (the shape a plain
 * call would use first, then the others from the widest tile down; about two tiles per
 * compute unit each; only rows of the first half of R), time per row decides, the rest of R
 * runs with the winner, which is cached for the size bucket.  The result is the complete
 * count, bit for bit that of amulet_count_i8.  Allocates two events and blocks the host
 * while trials run; problems too small for two slabs (below about four tiles per compute
 * unit: 8192 x 8192 outputs and less) run whole with the built-in or cached shape.
 * `chosen_shape`, `n_trials` may be NULL.  Same arguments and error codes as amulet_count_i8.
 */
int amulet_count_i8_adaptive(int64_t M, int64_t N, int64_t K,
                             const int8_t *A, int64_t lda,
                             const int8_t *B, int64_t ldb,
                             int32_t *R, int64_t ldr,
                             void *stream, int *chosen_shape, int *n_trials);

/*
 * amulet_count_i8_general for callers that cannot allocate and have no
 * workspace to lend: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments without the workspace, same
 * kernels, same exact result; the copies of transposed, unaligned or ragged
 * operands go into a scratch array of AMULET_STATIC_SCRATCH_BYTES (32 MiB) that
 * is part of the library's device image: every GPU the library runs on holds
 * its own copy from load until the process ends.  The call allocates nothing
 * (no hipMalloc, no hipFree, no allocating library routine); its first call on
 * a device looks the array's device address up once.
 *   - AMULET_ERR_WORKSPACE when the copies the general call could make for
 *     this (M, N, K) -- amulet_count_i8_repack_workspace_bytes(M, N, K), about
 *     M*K + K*N bytes rounded up to whole tiles -- do not fit the array;
 *     nothing is enqueued then.  Other errors as amulet_count_i8_general.
 *   - All calls on one GPU share that GPU's array, and it keeps the last
 *     call's contents (the copies overwrite and zero-pad what they need; no
 *     call relies on it being clear).  Two calls whose work overlaps in time on
 *     one GPU (different streams, or threads) race on it: serialise them, or
 *     use amulet_count_i8_general with a workspace per stream.
 */
#define AMULET_STATIC_SCRATCH_BYTES (32u << 20)
int amulet_count_i8_static(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K,
                           const int8_t *A, int64_t lda,
                           const int8_t *B, int64_t ldb,
                           int32_t *R, int64_t ldr,
                           void *stream);

/*
 * Adaptive execution as the paper runs it (Sec. 4.4-4.6): the task is split
 * into disjoint row slabs; the first slabs are computed with trial tile
 * shapes, walked by the two-stage greedy search (first the k axis of the
 * shape grid: staging depth, then every tile's K in 1, 2, 4, 8 parts, the
 * paper's k_c sequence K, K/2, K/4, ...; then the tile axis upward with an
 * early stop, its n_c walk) and scored by time per row,
 * and the rest of the task runs with the winner, so every trial also
 * contributes its part of R ("these intermediate computations also all
 * contribute to the final result").  At most half of the rows serve as
 * trials; a task too small for two trial slabs runs whole with the default
 * shape.  The winner is cached for the size bucket of (task, M, N, K) as
 * amulet_tune does.
 * Unlike amulet_mmlike_f32 this call synchronises with `stream` after each
 * trial (it reads their timings); the remainder is only enqueued.  It
 * allocates no device memory.  Arguments as amulet_mmlike_f32; chosen_shape
 * and n_trials (either may be NULL) receive the winner's id and the number
 * of trial slabs run.
 */
int amulet_mmlike_f32_adaptive(int task, int64_t M, int64_t N, int64_t K,
                               const float *A, int64_t lda,
                               const float *B, int64_t ldb,
                               const float *params,
                               float *R, int64_t ldr,
                               void *stream, int *chosen_shape, int *n_trials);

/*
 * The same adaptive execution for the general form of the test queries
 * (Sec. 6.3; the paper adapts every kernel it generates): threshold operand
 * form and transposed layouts as in amulet_mmlike_f32_general, the remaining
 * arguments as in amulet_mmlike_f32_adaptive, which is this call with thres[j],
 * no transposition and planar params.  Row slabs of a transposed A are column
 * ranges of its storage, of thres[i] / thres[i][j] the matching rows.
 */
int amulet_mmlike_f32_adaptive_general(int task, int thres_form, int trans_a, int trans_b,
                                       int64_t M, int64_t N, int64_t K,
                                       const float *A, int64_t lda,
                                       const float *B, int64_t ldb,
                                       const float *thres, int64_t ldt,
                                       const float *dis,
                                       float *R, int64_t ldr,
                                       void *stream, int *chosen_shape, int *n_trials);

/*
 * Adaptive shape selection (the stand-in for the paper's adaptive execution,
 * Sec. 4.4-4.6): times the candidate tile shapes of `task` on synthetic
 * operands of this size that the call allocates and frees itself, walks them
 * with the paper's two-stage greedy search, caches the winner for
 * (task, M, N, K) and every size in the same bucket (each of M, N, K rounded
 * up to a multiple of 256) and synchronises `stream`.  The device is first run up to
 * its loaded clocks, a trial is the better of two spans of about 2 ms of
 * back-to-back launches, and the search's winner replaces the built-in default
 * only if it also beats it in a direct rematch by more than 3 %.  Unlike the compute calls this
 * one allocates and blocks; it is meant to run once, outside the hot path.
 * task may be 0..3, or AMULET_TASK_COUNT_I8 for amulet_count_i8.
 * Returns the chosen shape id (>= 0) or a negative status.
 */
#define AMULET_TASK_COUNT_I8 100
int amulet_tune(int task, int64_t M, int64_t N, int64_t K, void *stream);

/* Shape table introspection: number of tile shapes of a task, a printable name
 * for one, and the shape amulet_mmlike_f32 / amulet_count_i8 would use now. */
int amulet_shape_count(int task);
const char *amulet_shape_name(int task, int shape);
int amulet_selected_shape(int task, int64_t M, int64_t N, int64_t K);
/* Forget every cached selection. */
void amulet_clear_selections(void);

/*
 * The paper's two-stage greedy parameter search (Sec. 4.4-4.6), over a grid
 * axis0 x axis1 of candidates (k_c-like and n_c-like): with axis1 fixed at
 * its first value, score every axis0 candidate and keep the lowest; then walk
 * axis1 upward from its first value and stop at the first score that is
 * higher than its predecessor's, keeping the predecessor.  `score` is called
 * on the host as score(i0, i1, ctx) and returns a cost (lower is better).
 * Writes the chosen indices; returns the number of score() calls made, or
 * AMULET_ERR_DIM if an axis is empty, AMULET_ERR_NULL for a NULL argument.
 */
typedef double (*amulet_score_fn)(int i0, int i1, void *ctx);
int amulet_greedy_search(int n0, int n1, amulet_score_fn score, void *ctx, int *best0, int *best1);

/*
 * Register demand of an I_h x I_w inner kernel (Sec. 3 inequality and its
 * extension in Sec. 4.3.2), in SIMD registers of width S_w elements:
 *   I_h*ceil(I_w/S_w) sub-results + 1 for A + ceil(I_w/S_w) for B
 *   + 1 per constant leaf + 1 per [i]-indexed leaf + ceil(I_w/S_w) per
 *   [j]-indexed leaf + 1 per [i][j]-indexed leaf + n_temp temporaries.
 * amulet_choose_kernel_height returns the largest I_h <= I_h_max whose demand
 * fits `budget` registers (0 if none does).  The library sizes its per-lane
 * micro-tiles with the same rule against the VGPR budget.
 */
int amulet_register_demand(int I_h, int I_w, int S_w, int n_const, int n_i, int n_j, int n_ij,
                           int n_temp);
int amulet_choose_kernel_height(int I_h_max, int I_w, int S_w, int n_const, int n_i, int n_j,
                                int n_ij, int n_temp, int budget);

/*
 * Measurement aid for the roofline of the vector-ALU tasks (the instruction
 * sequence of Sec. 4.3.1 with nothing around it): runs a register-only loop
 * of the instruction mix of a task (mix 0: fused multiply-add only, as the
 * identity task; 1: multiply, compare, select, FMA, as the discount task;
 * 2: fma, fma, max, add, as the boost task; 3: multiply, subtract, sign bit
 * of the difference added to an integer count, as the count task) with `waves_per_simd`
 * (1..8) resident waves per SIMD on every compute unit, synchronises `stream`,
 * and writes the sustained products per second.  Allocates a small scratch
 * buffer and blocks, like amulet_tune.  Returns AMULET_OK or a negative status.
 */
int amulet_probe_valu(int mix, int waves_per_simd, double *products_per_second, void *stream);

/*
 * The tile order of the kernels (an MI355X-side analogue of the loop order the
 * paper's tiling fixes, Sec. 3): a launch covers a tiles_m x tiles_n grid of
 * R tiles with amulet_tile_grid() workgroups; workgroup b runs on XCD b % 8,
 * and the grid is cut into 8 rectangular parts, one per XCD, so that the
 * workgroups resident on an XCD share A rows and B columns through its L2;
 * when the tile counts do not divide into such parts, into 8 runs of equal
 * length (to within one tile) of one panel-wise order instead, so that every
 * XCD gets the same number of tiles.
 * amulet_tile_of_workgroup writes the tile (tm, tn) of workgroup `block` and
 * returns 1, or returns 0 when that workgroup is padding (it exits at once),
 * or a negative status for bad arguments.  Host-only helpers; every tile is
 * owned by exactly one workgroup.
 */
int64_t amulet_tile_grid(int64_t tiles_m, int64_t tiles_n);
int amulet_tile_of_workgroup(int64_t block, int64_t tiles_m, int64_t tiles_n, int64_t *tm, int64_t *tn);

/*
 * The same aid for the join count (the matrix product of Sec. 1's join
 * translation): a register-only loop of the int8 matrix-core instruction the
 * kernels use, on four independent accumulators per wave, `waves_per_simd`
 * (1..8) waves per SIMD on every compute unit; writes the sustained int8
 * multiply-adds per second (operations = 2 x that).  Allocates a small
 * scratch buffer and blocks.  Returns AMULET_OK or a negative status.
 */
int amulet_probe_mfma_i8(int waves_per_simd, double *macs_per_second, void *stream);

/* Printable text for a status code (static storage). */
const char *amulet_strerror(int code);

/* HIP's text for the error behind the calling thread's last AMULET_ERR_LAUNCH
 * ("no error" if its last launch succeeded).  Static storage. */
const char *amulet_last_launch_error(void);

/*
 * Reproducible floating-point results.  By default a launch may split K over
 * several workgroups per tile (see the conventions at the top: few tiles, or a
 * nearly empty last round of workgroups), whose parts reach R through float
 * atomics in an order that differs from run to run.  With the deterministic
 * mode on (amulet_set_deterministic(1), or AMULET_DETERMINISTIC=1 in the
 * environment when the library is first used) no fp32 / fp64 launch splits K:
 * every output is summed by one workgroup in a fixed order, and two calls on
 * the same inputs with the same tile shape give the same bits, at the price of
 * the idle compute units the split was there to fill.  The integer join count
 * is exact either way and is not affected.  Process-wide; takes effect for
 * calls made after it returns.
 */
void amulet_set_deterministic(int on);
int amulet_get_deterministic(void);

/*
 * Test seam for the error path (the sum order and tiling of Sec. 3-4 play no
 * part): the next n kernel-launch attempts of this process are refused on the
 * host and reported as a failed launch, so that callers and tests can check
 * that AMULET_ERR_LAUNCH comes back, that nothing is cached for a shape that
 * did not run, and that R is left untouched.  Nothing reaches the device for a
 * refused launch.  n <= 0 switches it off.
 */
void amulet_debug_fail_launches(int n);

/* Library version string (static storage). */
const char *amulet_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AMULET_H */
