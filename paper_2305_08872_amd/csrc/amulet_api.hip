// C ABI of the library: argument checks, tile-shape selection, launches.
// Everything a compute call does on the host is here; it enqueues one kernel
// (or a few for very tall int8 problems) on the caller's stream and returns.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <map>
#include <mutex>
#include <tuple>
#include <vector>

#include "amulet.h"
#include "amulet_internal.h"

namespace amulet {

const ValuShapeDesc kValuShapes[VALU_SHAPE_COUNT] = {
    {4, 1, 4, 8, 0, "valu_16x256_k8"},      {4, 1, 8, 8, 0, "valu_32x256_w8_k8"},
    {8, 1, 8, 8, 0, "valu_64x256_k8"},      {4, 2, 8, 8, 0, "valu_32x512_k8"},
    {4, 1, 4, 16, 0, "valu_16x256_k16"},    {4, 1, 8, 16, 0, "valu_32x256_w8_k16"},
    {8, 1, 8, 16, 0, "valu_64x256_k16"},    {4, 2, 8, 16, 0, "valu_32x512_k16"},
    {4, 1, 4, 16, 2, "valu_16x256_k16_s2"}, {4, 1, 8, 16, 2, "valu_32x256_w8_k16_s2"},
    {8, 1, 8, 16, 2, "valu_64x256_k16_s2"}, {4, 2, 8, 16, 2, "valu_32x512_k16_s2"},
    {4, 1, 4, 16, 4, "valu_16x256_k16_s4"}, {4, 1, 8, 16, 4, "valu_32x256_w8_k16_s4"},
    {8, 1, 8, 16, 4, "valu_64x256_k16_s4"}, {4, 2, 8, 16, 4, "valu_32x512_k16_s4"},
    {4, 1, 4, 16, 8, "valu_16x256_k16_s8"}, {4, 1, 8, 16, 8, "valu_32x256_w8_k16_s8"},
    {8, 1, 8, 16, 8, "valu_64x256_k16_s8"}, {4, 2, 8, 16, 8, "valu_32x512_k16_s8"},
};

static const char *const kCountShapeNames[COUNT_SHAPE_COUNT] = {"count_simple", "mfma_i8_128x128_k64",
                                                                "mfma_i8_256x256_k64", "mfma_i8_128x256_k64",
                                                                "mfma_i8_128x128_w8_k128", "mfma_i8_256x256_w16_k64", "mfma_i8_128x256_dma3",
                                                                "mfma_i8_256x256_w16_dma4", "mfma_i8_256x256_w16_dma4_persistent"};

// ---- selection cache ---------------------------------------------------------
// Keyed by task and by size buckets of 256 (the widest tile edge of any shape): sizes that share
// a bucket triple have the same tile grid up to ragged edges, so a choice timed at 8192^3 also
// serves 8191^3 or 8000 x 8192 x 8100.  Every shape of a task accepts every size, so a cached
// id is always valid for the whole bucket.
typedef std::tuple<int, int64_t, int64_t, int64_t> SelKey;
static std::mutex g_sel_mutex;
static std::map<SelKey, int> g_selected;
static inline int64_t sel_bucket(int64_t n) { return (n + 255) / 256; }
static inline SelKey sel_key(int task, int64_t M, int64_t N, int64_t K)
{
    return SelKey(task, sel_bucket(M), sel_bucket(N), sel_bucket(K));
}

static int n_shapes(int task)
{
    if (task == TASK_IDENTITY) return IDENTITY_SHAPE_COUNT;  // eight vector-ALU shapes and the five matrix-core ones
    if (task > TASK_IDENTITY && task <= TASK_COUNT_GT) return VALU_SHAPE_COUNT;
    if (task == AMULET_TASK_COUNT_I8) return COUNT_SHAPE_COUNT;
    return 0;
}

// Built-in choice when nothing was tuned.  The predicate tasks are bound by
// VALU issue, which needs several resident waves per SIMD to keep both issue
// slots busy, so the small 4x4 micro-tile (about 110 registers) with 16-deep
// staging is the measured best at every size; of its two workgroup sizes the
// 8-wave one (32 x 256) is ahead by 2-9 % once there are two such tiles per
// compute unit (or a long K to split, see below), the 4-wave one (16 x 256) below that.
// Identity task: 64 x 64 tiles instead of 128 x 128?  With fewer large tiles than compute units,
// always (four times the tiles fill the chip without a K split, or with a smaller one).  Up to four
// large tiles per unit, when the small tiles' count leaves clearly less of the last tile per unit
// unused: every unit gets a whole number of tiles, so 576 large tiles on 256 units cost three
// tiles' time for 2.25 tiles' work while 2304 small ones are nine each (3072^3: 460 against 422 us,
// 3072^2 x 1024: 180 / 151, 3584^3: 708-733 / 691, 2560^3: 275 / 270).  Where the counts are as even
// the large tile is 2-6 % ahead (it streams half the bytes per operation: 2048^3 128.5 / 131,
// 2816^3 329 / 340, 4096^3 942 / 990), and with more tiles the rounds no longer line up anyway.
static bool identity_small_tile_wanted(int64_t M, int64_t N, bool f64 = false)
{
    const int64_t units = compute_units();
    const int64_t large = ((M + 127) / 128) * ((N + 127) / 128), small = ((M + 63) / 64) * ((N + 63) / 64);
    // (fp64, whose large tile holds two workgroups to a unit: also with exactly one large tile per
    // unit, 2048^3 258 against 272 us, 2048^2 x 512 71 / 80)
    if (large < units + (f64 ? 1 : 0)) return true;
    if (large >= 4 * units) return false;
    auto unused = [&](int64_t tiles) { const int64_t r = (tiles + units - 1) / units * units; return (double)(r - tiles) / (double)r; };
    return unused(small) + 0.05 < unused(large);
}

static int default_shape(int task, int64_t M, int64_t N, int64_t K)
{
    // Matrix cores.  Fewer 128 x 256 tiles than compute units: the register-staged 128 x 128 tile
    // with 8 waves (twice the workgroups; 2048^2 x 4096: 945 against 787 TOP/s).  Else operands
    // streamed straight into LDS: the 256 x 256 tile (one workgroup per compute unit) when its
    // tiles fill whole rounds of the chip, at least two of them, else 128 x 256, whose partial
    // last round costs half as much (6144^2 x 4096: 2074 against 1748 TOP/s).  Both fall back to
    // the register-staged kernel where the problem is not interior and aligned.
    if (task == AMULET_TASK_COUNT_I8) {
        const int64_t tiles128 = ((M + 127) / 128) * ((N + 255) / 256);
        const int64_t tiles256 = ((M + 255) / 256) * ((N + 255) / 256);
        if (tiles128 <= 256) return 4;   // (at exactly one such tile per unit too: 4096 x 2048 x 4096 46 against 57 us)
        // (from three rounds of 256 x 256 tiles on: the persistent form of that kernel, whose
        // workgroups walk their tiles out of phase; measured, persistent against one tile per
        // workgroup, ms: 768 tiles x K = 8192 0.265 / 0.280, 896 x 4096 0.204 / 0.213, 1024 0.2125 /
        // 0.230, 1152 0.249 / 0.267, 1408 0.296 / 0.320, 1536 0.312 / 0.337; below that the one-tile
        // kernel is ahead: 512 tiles 0.125 / 0.121, 576 0.156 / 0.154, 640 x K = 2048 0.114 / 0.106)
        return tiles256 >= 768 ? 8 : 6;
    }
    // a dense contraction: matrix cores, 128 x 128 tile, operands streamed HBM -> LDS where the
    // problem allows it (operands with 16-byte aligned rows in any layout, at least a stage of K;
    // the register-staged kernel otherwise).  The 256 x 256 tile measures 1-3 % behind even at 8192^3; the selector tries all.
    if (task == TASK_IDENTITY) {
        // Ring of 3 stages (three workgroups per compute unit, 768 at a time) except between one
        // and three rounds of the ring of 4 (512 at a time), where whole rounds matter and the
        // ring of 4 fills its rounds better unless 3 wastes clearly less (1024 tiles: 145 against
        // 132-146 TFLOP/s, 1280: 145.5 against 142, 1536: 143.5 against 146).  With more rounds
        // the workgroups' finishing times spread and the fuller unit wins (2048 tiles: 145 against
        // 141, 4096: 149 against 147, 8192 tiles x K = 512: 134 against 128).
        const int64_t tiles = ((M + 127) / 128) * ((N + 127) / 128);
        // 64 x 64 tiles for problems of few tiles (us, against the ring of 3: 512^3 10.0 / 13.4, 1024^3
        // 20.7 / 30.7, 1792^3 109 / 113, 1536^2 x 4096 148 / 166, 512^2 x 8192 40 / 46) and where their
        // count suits the chip better (identity_small_tile_wanted).
        if (identity_small_tile_wanted(M, N)) return IDENTITY_MFMA_SMALL_SHAPE;
        const int64_t round3 = 3 * (int64_t)compute_units(), round4 = 2 * (int64_t)compute_units();
        if (tiles <= round3 || tiles > 3 * round4) return IDENTITY_MFMA_DMA3_SHAPE;
        auto waste = [&](int64_t slots) { const int64_t r = (tiles + slots - 1) / slots * slots; return (double)(r - tiles) / (double)r; };
        return waste(round3) < waste(round4) - 0.05 ? IDENTITY_MFMA_DMA3_SHAPE : IDENTITY_MFMA_DMA4_SHAPE;
    }
    // ... or, with fewer tiles, when K is long (from 8192 on) and the launcher's K split makes up
    // the number (4096 x 512 x 8192: 31.0 against 29.2 TFLOP/s, 4096 x 512 x 32768: 31.3 against
    // 26.6; at K <= 4096 the 4-wave tile stays ahead, 1536^2 x 4096: 28.5 against 27.2)
    const int64_t tiles32 = ((M + 31) / 32) * ((N + 255) / 256);
    if (tiles32 >= 512) return VALU_TILES + 1;
    if (tiles32 >= 128 && K >= 8192) return VALU_TILES + 1;
    return VALU_TILES + 0;
}

static int lookup_shape(int task, int64_t M, int64_t N, int64_t K)
{
    {
        std::lock_guard<std::mutex> lock(g_sel_mutex);
        auto it = g_selected.find(sel_key(task, M, N, K));
        if (it != g_selected.end()) return it->second;
    }
    return default_shape(task, M, N, K);
}

// text of the last HIP error a launch reported (diagnostics for AMULET_ERR_LAUNCH)
static thread_local hipError_t g_last_hip_error = hipSuccess;

static const int64_t kMaxDim = 2147483647LL - 65536LL;

static int check_common(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                        int64_t ldb, const void *R, int64_t ldr)
{
    if (M < 0 || N < 0 || K < 0) return AMULET_ERR_DIM;
    if (M > kMaxDim || N > kMaxDim || K > kMaxDim) return AMULET_ERR_RANGE;
    if (M == 0 || N == 0 || K == 0) return 1;  // nothing to do
    if (!A || !B || !R) return AMULET_ERR_NULL;
    if (lda < K || ldb < N || ldr < N) return AMULET_ERR_LD;
    return AMULET_OK;
}

static inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// Operands of an fp32 task in the general form of the paper's test queries (Sec. 6.3).
struct MmlikeCall {
    int task, thres_form, trans_a, trans_b;
    int64_t M, N, K;
    const float *A; int64_t lda;
    const float *B; int64_t ldb;
    const float *thres; int64_t ldt;
    const float *dis;
    float *R; int64_t ldr;
};

template <int TASK>
static hipError_t launch_form(int form, int shape, const MmlikeArgs &a, hipStream_t s)
{
    switch (form) {
    case THRES_COL: return launch_mmlike_valu_task<TASK, THRES_COL>(shape, a, s);
    case THRES_ROW: return launch_mmlike_valu_task<TASK, THRES_ROW>(shape, a, s);
    case THRES_CONST: return launch_mmlike_valu_task<TASK, THRES_CONST>(shape, a, s);
    default: return launch_mmlike_valu_task<TASK, THRES_ELEM>(shape, a, s);
    }
}

static int run_mmlike(const MmlikeCall &c, int shape, void *stream)
{
    MmlikeArgs a;
    a.A = c.A; a.B = c.B; a.thres = c.thres; a.dis = c.dis; a.R = c.R;
    a.lda = c.lda; a.ldb = c.ldb; a.ldr = c.ldr; a.ldt = c.ldt;
    a.M = (int)c.M; a.N = (int)c.N; a.K = (int)c.K;
    a.transA = c.trans_a; a.transB = c.trans_b;
    a.vec = (aligned16(c.B) && aligned16(c.R) && c.ldb % 4 == 0 && c.ldr % 4 == 0) ? 1 : 0;
    a.vecA = (aligned16(c.A) && c.lda % 4 == 0) ? 1 : 0;
    a.kchunk = (int)c.K;
    a.tail_base = 0; a.tail_blocks = 0; a.tail_splits = 1; a.block_base = 0;
    a.force_splits = 0;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    switch (c.task) {
    case TASK_IDENTITY:
        e = shape >= IDENTITY_MFMA_SHAPE ? launch_identity_mfma(a, shape - IDENTITY_MFMA_SHAPE, s)
                                         : launch_mmlike_valu_task<TASK_IDENTITY, THRES_COL>(shape, a, s);
        break;
    case TASK_DISCOUNT: e = launch_form<TASK_DISCOUNT>(c.thres_form, shape, a, s); break;
    case TASK_BOOST: e = launch_form<TASK_BOOST>(c.thres_form, shape, a, s); break;
    default: e = launch_form<TASK_COUNT_GT>(c.thres_form, shape, a, s); break;
    }
    g_last_hip_error = e;
    return e == hipSuccess ? AMULET_OK : AMULET_ERR_LAUNCH;
}

// Argument checks of an fp32 call; returns 1 when there is nothing to do.
static int check_mmlike(const MmlikeCall &c)
{
    if (c.task < TASK_IDENTITY || c.task > TASK_COUNT_GT) return AMULET_ERR_TASK;
    if (c.thres_form < THRES_COL || c.thres_form > THRES_ELEM) return AMULET_ERR_TASK;
    if (c.M < 0 || c.N < 0 || c.K < 0) return AMULET_ERR_DIM;
    if (c.M > kMaxDim || c.N > kMaxDim || c.K > kMaxDim) return AMULET_ERR_RANGE;
    if (c.M == 0 || c.N == 0 || c.K == 0) return 1;
    if (!c.A || !c.B || !c.R) return AMULET_ERR_NULL;
    if (c.task != TASK_IDENTITY && !c.thres) return AMULET_ERR_NULL;
    if (c.task == TASK_DISCOUNT && !c.dis) return AMULET_ERR_NULL;
    if (c.lda < (c.trans_a ? c.M : c.K) || c.ldb < (c.trans_b ? c.K : c.N) || c.ldr < c.N)
        return AMULET_ERR_LD;
    if (c.task != TASK_IDENTITY && c.thres_form == THRES_ELEM && c.ldt < c.N) return AMULET_ERR_LD;
    return AMULET_OK;
}

// phases of the persistent join-count kernels (see count_i8_dma_persistent_kernel)
static const int kPersPhases[4] = {8, 2, 2, 16};   // groups, stages between groups, XCD modulus, XCD span (sixteenths)

// m_load / n_load: rows of A / columns of B that exist in memory (0: just M, N)
static int run_count(int shape, int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda,
                     const int8_t *B, int64_t ldb, int32_t *R, int64_t ldr, void *stream,
                     int64_t m_load = 0, int64_t n_load = 0, bool assign = false)
{
    CountArgs a;
    a.assign = assign ? 1 : 0;
    a.A = A; a.B = B; a.R = R;
    a.lda = lda; a.ldb = ldb; a.ldr = ldr;
    a.M = (int)M; a.N = (int)N; a.K = (int)K;
    a.Mload = (int)(m_load > M ? m_load : M);
    a.Nload = (int)(n_load > N ? n_load : N);
    a.vecA = (aligned16(A) && lda % 16 == 0) ? 1 : 0;
    a.vecB = (aligned16(B) && ldb % 16 == 0) ? 1 : 0;
    a.vecR = (aligned16(R) && ldr % 4 == 0) ? 1 : 0;
    a.kchunk = (int)K;
    a.block_base = 0;
    a.pers_groups = kPersPhases[0];
    a.pers_group_stages = kPersPhases[1];
    a.pers_xcds = kPersPhases[2];
    a.pers_xcd_span = kPersPhases[3];
    if (assign) {
        // R = form: all workgroups in step.  A phase makes a workgroup sum its first tile in two passes,
        // the second of which has to read R, and the write-back the phases spread out is stores only
        // here (cfg3 0.1875 ms in step against 0.192-0.1945 over twelve phase arrangements; 8192^2 x 1024
        // 0.085 / 0.093).
        a.pers_groups = 1; a.pers_group_stages = 0; a.pers_xcds = 1; a.pers_xcd_span = 0;
    }
    if (const char *e = getenv("AMULET_I8_PHASES")) {   // diagnostic override, "groups,stages,xcds,span"
        int g = 1, st = 0, x = 1, sp = 0;
        if (sscanf(e, "%d,%d,%d,%d", &g, &st, &x, &sp) == 4 && g >= 1 && g <= 64 && st >= 0 && st <= 64 && x >= 1 && x <= 8 &&
            sp >= 0 && sp <= 16) {
            a.pers_groups = g; a.pers_group_stages = st; a.pers_xcds = x; a.pers_xcd_span = sp;
        }
    }
    hipError_t e = launch_count_i8(shape, a, (hipStream_t)stream);
    g_last_hip_error = e;
    return e == hipSuccess ? AMULET_OK : AMULET_ERR_LAUNCH;
}

// ---- synthetic operands for the selector's trials ----------------------------
__global__ void fill_f32_kernel(float *p, size_t n, float lo, float span, uint32_t salt)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        uint32_t h = (uint32_t)i * 2654435761u + salt;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        p[i] = lo + span * (float)(h >> 8) * (1.0f / 16777216.0f);
    }
}
__global__ void fill_i8_kernel(int8_t *p, size_t n, uint32_t salt)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        uint32_t h = (uint32_t)i * 2654435761u + salt;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        p[i] = (int8_t)((h >> 8) % 20u == 0u);
    }
}

struct TrialCtx {
    int task;
    int64_t M, N, K;
    void *A, *B, *params, *R;
    hipStream_t stream;
    hipEvent_t e0, e1;
    int status;
};

// One launch of `shape` on the trial operands.
static int trial_launch(TrialCtx *c, int shape)
{
    if (c->task == AMULET_TASK_COUNT_I8)
        return run_count(shape, c->M, c->N, c->K, (const int8_t *)c->A, c->K, (const int8_t *)c->B, c->N,
                         (int32_t *)c->R, c->N, c->stream);
    MmlikeCall call = {c->task, THRES_COL, 0, 0, c->M, c->N, c->K, (const float *)c->A, c->K,
                       (const float *)c->B, c->N, (const float *)c->params, 0,
                       (const float *)c->params + c->N, (float *)c->R, c->N};
    return run_mmlike(call, shape, c->stream);
}

// Milliseconds of `n` back-to-back launches of `shape`, or a negative value on failure.
static float trial_span_ms(TrialCtx *c, int shape, int n)
{
    (void)hipEventRecord(c->e0, c->stream);
    for (int i = 0; i < n; ++i)
        if (trial_launch(c, shape) != AMULET_OK) { c->status = AMULET_ERR_LAUNCH; return -1.0f; }
    (void)hipEventRecord(c->e1, c->stream);
    float ms = 0.0f;
    if (hipEventSynchronize(c->e1) != hipSuccess || hipEventElapsedTime(&ms, c->e0, c->e1) != hipSuccess) {
        c->status = AMULET_ERR_LAUNCH;
        return -1.0f;
    }
    return ms;
}

// Time per launch of `shape`: a first launch (warm-up, and the estimate of how many launches
// make a span of about 2 ms: a sub-millisecond launch timed alone is at the mercy of the
// clock governor), then the better of two such spans.
static double time_shape(TrialCtx *c, int shape)
{
    const float first = trial_span_ms(c, shape, 1);
    if (first < 0.0f) return 1e30;
    int n = first > 0.0f ? (int)(2.0f / first) + 1 : 64;
    if (n > 64) n = 64;
    float best = 1e30f;
    for (int rep = 0; rep < 2; ++rep) {
        const float ms = trial_span_ms(c, shape, n);
        if (ms < 0.0f) return 1e30;
        if (ms / n < best) best = ms / n;
    }
    return (double)best;
}

static double valu_trial_score(int i0, int i1, void *ctx)
{
    return time_shape((TrialCtx *)ctx, i0 * VALU_TILES + i1);
}

// ---- in-flight adaptive execution (paper Sec. 4.4-4.6) ---------------------------
// Trials run on disjoint row slabs of the caller's own task, so every trial also
// contributes its part of R; whatever is left runs with the winner.
// Estimated duration of a whole task below which an adaptive call stops after its first trial
// (milliseconds; the environment variable AMULET_ADAPTIVE_MIN_TASK_MS overrides it, 0 = never stop).
static double adaptive_min_task_ms()
{
    if (const char *e = getenv("AMULET_ADAPTIVE_MIN_TASK_MS")) return atof(e);
    return 3.0;
}

// Trials whose order does not depend on each other's outcome (a flat list of candidates) are
// enqueued back to back with an event between them and waited for once: one host round trip
// for all of them instead of one each.
struct BatchedTrials {
    enum { MAX = 9 };
    hipEvent_t ev[MAX + 1];
    int shape[MAX];
    int64_t rows[MAX];
    int n;
    bool ok;
    BatchedTrials() : n(0), ok(true) { for (auto &e : ev) e = nullptr; }
    ~BatchedTrials() { for (auto &e : ev) if (e) (void)hipEventDestroy(e); }
    bool begin(hipStream_t s)
    {
        for (auto &e : ev)
            if (hipEventCreate(&e) != hipSuccess) { e = nullptr; ok = false; return false; }
        return hipEventRecord(ev[0], s) == hipSuccess;
    }
    // call after the trial's work was enqueued
    void mark(int shape_id, int64_t n_rows, hipStream_t s)
    {
        shape[n] = shape_id; rows[n] = n_rows; ++n;
        if (hipEventRecord(ev[n], s) != hipSuccess) ok = false;
    }
    // waits for the last trial; returns the index of the fastest per row, or -1
    int finish()
    {
        if (!ok || n == 0 || hipEventSynchronize(ev[n]) != hipSuccess) return -1;
        int best = -1;
        double best_sc = 1e300;
        for (int i = 0; i < n; ++i) {
            float ms = 0.0f;
            if (hipEventElapsedTime(&ms, ev[i], ev[i + 1]) != hipSuccess) return -1;
            const double sc = (double)ms / (double)rows[i];
            if (sc < best_sc) { best_sc = sc; best = i; }
        }
        return best;
    }
};

struct AdaptiveCtx {
    bool short_task;      // the first trial showed a task too short to be worth more trials
    MmlikeCall call;      // the whole task
    int64_t next_row;     // first row no trial has computed yet
    int64_t budget_rows;  // trials may use rows below this
    hipStream_t stream;
    hipEvent_t e0, e1;
    int status;
    int trials;
    double best_score;    // lowest score of any trial so far, and the shape that reached it
    int best_shape;
    double score_of[VALU_SHAPE_COUNT];   // score of a shape already tried (negative: not yet)
};

static bool is_mfma_shape(int task, int shape) { return task == TASK_IDENTITY && shape >= IDENTITY_MFMA_SHAPE; }

// Rows of one trial slab: enough row tiles for 1280 workgroups, i.e. one and a quarter rounds of
// 4-wave workgroups on 256 compute units, two and a half of 8-wave ones.  (A slab of exactly one
// round measured 20 % below the steady rate, its first and last workgroups running on a
// half-empty chip, and seven such slabs cost an 8192^3 call 12 %; at this size six cost 1-2 %.)
static int64_t trial_rows(const MmlikeCall &c, int shape)
{
    int64_t tile_rows = 128, tile_cols = 128;
    const bool mfma = is_mfma_shape(c.task, shape);
    if (mfma && shape == IDENTITY_MFMA_BIG_SHAPE) tile_rows = tile_cols = 256;
    if (mfma && shape == IDENTITY_MFMA_SMALL_SHAPE) tile_rows = tile_cols = 64;
    int64_t want_tiles = 1280;
    if (!mfma) {
        const ValuShapeDesc &d = kValuShapes[shape];
        tile_rows = (int64_t)d.NW * d.TM;
        tile_cols = 256LL * d.NG;
        // a shape that sums every tile's K in s parts launches s workgroups per tile
        if (d.splits > 1 && c.K >= 128) {
            int64_t sp = d.splits;
            if (sp > c.K / 64) sp = c.K / 64;
            want_tiles /= sp > 1 ? sp : 1;
        }
    } else {
        // (matrix-core tiles: one round of what a compute unit holds: three 128 x 128 tiles of the
        // streamed kernel with a ring of 3 stages, two with a ring of 4, one 256 x 256 tile)
        want_tiles = shape == IDENTITY_MFMA_BIG_SHAPE ? 256 : shape == IDENTITY_MFMA_DMA4_SHAPE ? 512 : 768;
    }
    const int64_t tiles_n = (c.N + tile_cols - 1) / tile_cols;
    int64_t row_tiles = (want_tiles + tiles_n - 1) / tiles_n;
    if (row_tiles < 1) row_tiles = 1;
    return row_tiles * tile_rows;
}

// Runs rows [r0, r0 + rows) of the task with `shape`.
static int run_rows(const MmlikeCall &c, int shape, int64_t r0, int64_t rows, hipStream_t s)
{
    MmlikeCall sub = c;
    sub.M = rows;
    sub.A = c.trans_a ? c.A + r0 : c.A + r0 * c.lda;
    sub.R = c.R + r0 * c.ldr;
    if (c.thres_form == THRES_ROW && c.thres) sub.thres = c.thres + r0;
    if (c.thres_form == THRES_ELEM && c.thres) sub.thres = c.thres + r0 * c.ldt;
    return run_mmlike(sub, shape, s);
}

static double adaptive_trial(AdaptiveCtx *x, int shape)
{
    const int64_t rows = trial_rows(x->call, shape);
    if (x->status != AMULET_OK || x->next_row + rows > x->budget_rows) return 1e300;  // no data left to test on
    if (x->short_task) return 1e300;   // (see below)
    (void)hipEventRecord(x->e0, x->stream);
    const int rc = run_rows(x->call, shape, x->next_row, rows, x->stream);
    (void)hipEventRecord(x->e1, x->stream);
    if (rc != AMULET_OK || hipEventSynchronize(x->e1) != hipSuccess) {
        x->status = AMULET_ERR_LAUNCH;
        return 1e300;
    }
    x->next_row += rows;
    x->trials += 1;
    float ms = 0.0f;
    (void)hipEventElapsedTime(&ms, x->e0, x->e1);
    const double sc = (double)ms / (double)rows;   // the paper's score: execution time per unit of work
    if (sc < x->best_score) { x->best_score = sc; x->best_shape = shape; }
    // Every trial costs a host round trip (its end is waited for before the next is chosen):
    // some tens of microseconds in which the GPU idles.  A task that the first trial shows to
    // be a few milliseconds in all is not worth more of them (16384 x 8192 x 1024 identity,
    // 1.9 ms: three trials cost 13 %); it runs on with the shape just tried.
    if (x->trials == 1 && sc * (double)x->call.M < adaptive_min_task_ms()) x->short_task = true;
    return sc;
}

static double adaptive_valu_score(int i0, int i1, void *ctx)
{
    AdaptiveCtx *x = (AdaptiveCtx *)ctx;
    const int shape = i0 * VALU_TILES + i1;
    if (x->score_of[shape] < 0.0) x->score_of[shape] = adaptive_trial(x, shape);   // a shape is tried once
    return x->score_of[shape];
}

}  // namespace amulet

using namespace amulet;

extern "C" {

int amulet_mmlike_f32_general(int task, int thres_form, int trans_a, int trans_b, int shape,
                              int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                              const float *B, int64_t ldb, const float *thres, int64_t ldt,
                              const float *dis, float *R, int64_t ldr, void *stream)
{
    const MmlikeCall c = {task, thres_form, trans_a ? 1 : 0, trans_b ? 1 : 0, M, N, K, A, lda, B, ldb,
                          thres, ldt, dis, R, ldr};
    const int rc = check_mmlike(c);
    if (rc < 0) return rc;
    if (shape < 0)
        shape = lookup_shape(task, M, N, K);
    else if (shape >= n_shapes(task))
        return AMULET_ERR_SHAPE;
    if (rc == 1) return AMULET_OK;
    return run_mmlike(c, shape, stream);
}

// ---- fp64 ------------------------------------------------------------------------------------
struct F64Call {
    int task, thres_form, trans_a, trans_b;
    int64_t M, N, K;
    const double *A; int64_t lda;
    const double *B; int64_t ldb;
    const double *thres; int64_t ldt;
    const double *dis;
    double *R; int64_t ldr;
};

// < 0: error code; 1: nothing to do; 0: go
static int check_f64(const F64Call &c)
{
    if (c.task < TASK_IDENTITY || c.task > TASK_COUNT_GT) return AMULET_ERR_TASK;
    if (c.thres_form < THRES_COL || c.thres_form > THRES_ELEM) return AMULET_ERR_TASK;
    if (c.M < 0 || c.N < 0 || c.K < 0) return AMULET_ERR_DIM;
    if (c.M > kMaxDim || c.N > kMaxDim || c.K > kMaxDim) return AMULET_ERR_RANGE;
    if (c.M == 0 || c.N == 0 || c.K == 0) return 1;
    if (!c.A || !c.B || !c.R) return AMULET_ERR_NULL;
    if (c.task != TASK_IDENTITY && !c.thres) return AMULET_ERR_NULL;
    if (c.task == TASK_DISCOUNT && !c.dis) return AMULET_ERR_NULL;
    if (c.lda < (c.trans_a ? c.M : c.K) || c.ldb < (c.trans_b ? c.K : c.N) || c.ldr < c.N) return AMULET_ERR_LD;
    if (c.task != TASK_IDENTITY && c.thres_form == THRES_ELEM && c.ldt < c.N) return AMULET_ERR_LD;
    return 0;
}

// The fp64 selections share the cache of the fp32 ones under task ids of their own.
static inline int f64_cache_task(int task) { return 1000 + task; }

// Built-in fp64 choice when nothing was adapted: the 4-wave 16 x 128 tile (measured at 4096^3,
// 8192^2 x 2048, 2048^3, 16 x 128 against 32 x 128 with 8 waves: discount 17.0 / 16.6, 16.5 / 16.5;
// count 22.5 / 21.3; boost 16.0 / 15.5 TFLOP/s), except for boost problems of up to 2048^2 outputs
// (15.9 / 16.4), where a workgroup that brings two waves per SIMD fills a launch of one or two
// rounds better.
static int default_shape_f64(int task, int64_t M, int64_t N)
{
    return task == TASK_BOOST && M * N <= 2048LL * 2048LL && M * N >= 1024LL * 1024LL ? 1 : 0;
}

static int lookup_shape_f64(int task, int64_t M, int64_t N, int64_t K)
{
    // (identity: the matrix-core tile; 64 x 64 with fewer 128 x 128 tiles than compute units)
    if (task == TASK_IDENTITY) return identity_small_tile_wanted(M, N, true) ? 0 : 1;
    {
        std::lock_guard<std::mutex> lock(g_sel_mutex);
        auto it = g_selected.find(sel_key(f64_cache_task(task), M, N, K));
        if (it != g_selected.end()) return it->second;
    }
    return default_shape_f64(task, M, N);
}

// Rows [r0, r0 + rows) of the task with `shape`.
static int run_f64_rows(const F64Call &c, int shape, int64_t r0, int64_t rows, void *stream)
{
    MmlikeArgsF64 a;
    a.A = c.trans_a ? c.A + r0 : c.A + r0 * c.lda;
    a.B = c.B; a.dis = c.dis;
    a.thres = c.thres;
    if (c.thres_form == THRES_ROW && c.thres) a.thres = c.thres + r0;
    if (c.thres_form == THRES_ELEM && c.thres) a.thres = c.thres + r0 * c.ldt;
    a.R = c.R + r0 * c.ldr;
    a.lda = c.lda; a.ldb = c.ldb; a.ldr = c.ldr; a.ldt = c.ldt;
    a.M = (int)rows; a.N = (int)c.N; a.K = (int)c.K;
    a.transA = c.trans_a; a.transB = c.trans_b;
    const bool b16 = aligned16(a.B) && c.ldb % 2 == 0;
    // vec: 16-byte accesses to R, and to the rows of a row-major B
    a.vec = (aligned16(a.R) && c.ldr % 2 == 0 && (a.transB || b16)) ? 1 : 0;
    a.vecBt = b16 ? 1 : 0;
    a.vecA = (aligned16(a.A) && c.lda % 2 == 0) ? 1 : 0;
    a.kchunk = (int)c.K;
    a.tail_base = 0; a.tail_blocks = 0; a.tail_splits = 1; a.block_base = 0;
    const hipError_t e = launch_mmlike_f64(c.task, c.thres_form, shape, a, (hipStream_t)stream);
    g_last_hip_error = e;
    return e == hipSuccess ? AMULET_OK : AMULET_ERR_LAUNCH;
}

int amulet_mmlike_f64_shape(int task, int shape, int thres_form, int trans_a, int trans_b, int64_t M, int64_t N,
                            int64_t K, const double *A, int64_t lda, const double *B, int64_t ldb,
                            const double *thres, int64_t ldt, const double *dis, double *R, int64_t ldr,
                            void *stream)
{
    const F64Call c = {task, thres_form, trans_a ? 1 : 0, trans_b ? 1 : 0, M, N, K, A, lda, B, ldb, thres, ldt, dis, R, ldr};
    const int rc = check_f64(c);
    if (rc < 0) return rc;
    if (shape >= F64_SHAPE_COUNT) return AMULET_ERR_SHAPE;
    if (shape < 0) shape = lookup_shape_f64(task, M, N, K);
    if (rc == 1) return AMULET_OK;
    return run_f64_rows(c, shape, 0, M, stream);
}

int amulet_mmlike_f64_general(int task, int thres_form, int trans_a, int trans_b, int64_t M, int64_t N,
                              int64_t K, const double *A, int64_t lda, const double *B, int64_t ldb,
                              const double *thres, int64_t ldt, const double *dis, double *R, int64_t ldr,
                              void *stream)
{
    return amulet_mmlike_f64_shape(task, -1, thres_form, trans_a, trans_b, M, N, K, A, lda, B, ldb, thres, ldt, dis,
                                   R, ldr, stream);
}

int amulet_f64_shape_count(void) { return F64_SHAPE_COUNT; }

const char *amulet_f64_shape_name(int shape)
{
    static const char *const names[F64_SHAPE_COUNT] = {"valu_f64_16x128_k16", "valu_f64_32x128_w8_k16",
                                                       "valu_f64_16x128_k16_s2", "valu_f64_32x128_w8_k16_s2",
                                                       "valu_f64_16x128_k16_s4", "valu_f64_32x128_w8_k16_s4"};
    return shape >= 0 && shape < F64_SHAPE_COUNT ? names[shape] : "invalid";
}

int amulet_selected_shape_f64(int task, int64_t M, int64_t N, int64_t K)
{
    if (task < TASK_IDENTITY || task > TASK_COUNT_GT) return AMULET_ERR_TASK;
    return lookup_shape_f64(task, M, N, K);
}

// In-flight adaptive execution in fp64 (paper Sec. 4.4-4.6 in the paper's own element type):
// the scheme of amulet_mmlike_f32_adaptive_general on the fp64 shape grid.
struct AdaptiveF64 {
    bool short_task;
    F64Call call;
    int64_t next_row, budget_rows;
    hipStream_t stream;
    hipEvent_t e0, e1;
    int status, trials, best_shape;
    double best_score;
    double score_of[F64_SHAPE_COUNT];
};

// A slab of a round and a quarter of workgroups (1280 of 4 waves, 640 of 8), divided by the
// number of K parts of a split shape, which launches that many workgroups per tile.
static int64_t trial_rows_f64(const F64Call &c, int shape)
{
    const int64_t tile_rows = shape % F64_TILES == 1 ? 32 : 16;
    int64_t want = shape % F64_TILES == 1 ? 640 : 1280;
    const int sp = 1 << (shape / F64_TILES);
    if (sp > 1 && c.K >= 128) want /= sp;
    const int64_t tiles_n = (c.N + 127) / 128;
    int64_t row_tiles = (want + tiles_n - 1) / tiles_n;
    if (row_tiles < 1) row_tiles = 1;
    return row_tiles * tile_rows;
}

static double adaptive_f64_score(int i0, int i1, void *ctx)
{
    AdaptiveF64 *x = (AdaptiveF64 *)ctx;
    const int shape = i0 * F64_TILES + i1;
    if (x->score_of[shape] >= 0.0) return x->score_of[shape];   // a shape is tried once
    const int64_t rows = trial_rows_f64(x->call, shape);
    double sc = 1e300;   // no rows left to test on: infinitely slow, which ends the walk
    if (x->status == AMULET_OK && x->next_row + rows <= x->budget_rows && !x->short_task) {
        (void)hipEventRecord(x->e0, x->stream);
        const int rc = run_f64_rows(x->call, shape, x->next_row, rows, x->stream);
        (void)hipEventRecord(x->e1, x->stream);
        if (rc != AMULET_OK || hipEventSynchronize(x->e1) != hipSuccess) {
            x->status = AMULET_ERR_LAUNCH;
        } else {
            x->next_row += rows;
            x->trials += 1;
            float ms = 0.0f;
            (void)hipEventElapsedTime(&ms, x->e0, x->e1);
            sc = (double)ms / (double)rows;   // the paper's score: execution time per unit of work
            if (sc < x->best_score) { x->best_score = sc; x->best_shape = shape; }
            // (a task of a few milliseconds is not worth more host round trips: see adaptive_trial)
            if (x->trials == 1 && sc * (double)x->call.M < adaptive_min_task_ms()) x->short_task = true;
        }
    }
    x->score_of[shape] = sc;
    return sc;
}

int amulet_mmlike_f64_adaptive(int task, int thres_form, int trans_a, int trans_b, int64_t M, int64_t N, int64_t K,
                               const double *A, int64_t lda, const double *B, int64_t ldb, const double *thres,
                               int64_t ldt, const double *dis, double *R, int64_t ldr, void *stream,
                               int *chosen_shape, int *n_trials)
{
    const F64Call c = {task, thres_form, trans_a ? 1 : 0, trans_b ? 1 : 0, M, N, K, A, lda, B, ldb, thres, ldt, dis, R, ldr};
    const int rc = check_f64(c);
    if (rc < 0) return rc;
    int best = lookup_shape_f64(task, M, N, K);
    if (chosen_shape) *chosen_shape = best;
    if (n_trials) *n_trials = 0;
    if (rc == 1) return AMULET_OK;
    AdaptiveF64 x;
    memset(&x, 0, sizeof(x));
    x.call = c;
    x.stream = (hipStream_t)stream;
    x.budget_rows = M / 2;   // at least half of the task runs with the winner
    x.best_score = 1e300;
    x.best_shape = -1;
    for (double &sc : x.score_of) sc = -1.0;
    // the identity task has one fp64 kernel (matrix cores); a task too small to spare the
    // default shape's slab and two more runs whole with that shape
    const bool can_test = task != TASK_IDENTITY &&
                          trial_rows_f64(c, best) + 2 * trial_rows_f64(c, 0) <= x.budget_rows;
    if (can_test && hipEventCreate(&x.e0) == hipSuccess && hipEventCreate(&x.e1) == hipSuccess) {
        // the shape a plain call would use first, then the paper's order: the k axis, then the
        // tile axis upward with an early stop; the winner is the fastest slab of all
        (void)adaptive_f64_score(best / F64_TILES, best % F64_TILES, &x);
        int b0 = 0, b1 = 0;
        amulet_greedy_search(F64_KAXIS, F64_TILES, adaptive_f64_score, &x, &b0, &b1);
        if (x.best_shape >= 0) best = x.best_shape;
    }
    if (x.e0) (void)hipEventDestroy(x.e0);
    if (x.e1) (void)hipEventDestroy(x.e1);
    if (x.status != AMULET_OK) return x.status;
    int out = AMULET_OK;
    if (x.next_row < M) out = run_f64_rows(c, best, x.next_row, M - x.next_row, stream);
    if (out == AMULET_OK && x.trials > 0) {
        std::lock_guard<std::mutex> lock(g_sel_mutex);
        g_selected[sel_key(f64_cache_task(task), M, N, K)] = best;
    }
    if (chosen_shape) *chosen_shape = best;
    if (n_trials) *n_trials = x.trials;
    return out;
}

int amulet_mmlike_f64(int task, int thres_form, int64_t M, int64_t N, int64_t K, const double *A,
                      int64_t lda, const double *B, int64_t ldb, const double *thres, int64_t ldt,
                      const double *dis, double *R, int64_t ldr, void *stream)
{
    return amulet_mmlike_f64_general(task, thres_form, 0, 0, M, N, K, A, lda, B, ldb, thres, ldt, dis, R, ldr,
                                     stream);
}

int amulet_mmlike_f32_shape(int task, int shape, int64_t M, int64_t N, int64_t K, const float *A,
                            int64_t lda, const float *B, int64_t ldb, const float *params, float *R,
                            int64_t ldr, void *stream)
{
    if (task < TASK_IDENTITY || task > TASK_COUNT_GT) return AMULET_ERR_TASK;
    if (shape < 0 || shape >= n_shapes(task)) return AMULET_ERR_SHAPE;
    return amulet_mmlike_f32_general(task, THRES_COL, 0, 0, shape, M, N, K, A, lda, B, ldb, params, 0,
                                     params ? params + N : nullptr, R, ldr, stream);
}

int amulet_mmlike_f32(int task, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                      const float *B, int64_t ldb, const float *params, float *R, int64_t ldr,
                      void *stream)
{
    return amulet_mmlike_f32_general(task, THRES_COL, 0, 0, -1, M, N, K, A, lda, B, ldb, params, 0,
                                     params ? params + N : nullptr, R, ldr, stream);
}

// ---- packing (paper Sec. 3.1) ---------------------------------------------------------------
// Measured on the vector-ALU kernels (4096 x 4096 outputs, K = 4096 of each row used): A row pitch
// 48, 80, 96 KiB 31.7 TFLOP/s; 64 KiB 30.0; 128 KiB 27.0; 192 KiB 29.4; 256 and 512 KiB 20;
// any of these plus 128 bytes 31.7.  With the whole row used (K = 65536 fp32) 14 against 32.
int amulet_pitch_collides(int64_t ld, int elem_bytes)
{
    if (ld <= 0 || (elem_bytes != 1 && elem_bytes != 4 && elem_bytes != 8)) return 0;
    return pitch_collides(ld, elem_bytes) ? 1 : 0;
}

int64_t amulet_packed_ld(int64_t cols, int elem_bytes)
{
    if (cols <= 0 || (elem_bytes != 1 && elem_bytes != 4 && elem_bytes != 8)) return 0;
    int64_t pitch = (cols * elem_bytes + 127) / 128 * 128;   // whole 128-byte lines
    if (pitch % 4096 == 0) pitch += 128;                      // successive rows start 128 bytes apart in a page
    return pitch / elem_bytes;
}

int amulet_pack(int elem_bytes, int64_t rows, int64_t cols, const void *src, int64_t ld_src, void *dst,
                int64_t ld_dst, void *stream)
{
    if (elem_bytes != 1 && elem_bytes != 4 && elem_bytes != 8) return AMULET_ERR_DIM;
    if (rows < 0 || cols < 0) return AMULET_ERR_DIM;
    if (rows == 0 || cols == 0) return AMULET_OK;
    if (!src || !dst) return AMULET_ERR_NULL;
    if (ld_src < cols || ld_dst < cols) return AMULET_ERR_LD;
    const hipError_t e = launch_pack(elem_bytes, rows, cols, src, ld_src, dst, ld_dst, (hipStream_t)stream);
    g_last_hip_error = e;
    return e == hipSuccess ? AMULET_OK : AMULET_ERR_LAUNCH;
}

// Would a vector-ALU task with these operands run on a packed copy of A?  Only a row-major A is
// read row by row at one k (a transposed A is read along its rows), only the vector-ALU kernels
// read it through the scalar path that suffers, and a copy pays only when A is read many times.
static bool autopack_wanted(bool valu_task, int trans_a, int64_t N, int64_t lda, int elem_bytes)
{
    return valu_task && !trans_a && N >= 128 && amulet_pitch_collides(lda, elem_bytes);
}

size_t amulet_autopack_workspace_bytes(int elem_bytes, int64_t M, int64_t K)
{
    if (M <= 0 || K <= 0) return 0;
    const int64_t ld = amulet_packed_ld(K, elem_bytes);
    return ld > 0 ? (size_t)M * (size_t)ld * (size_t)elem_bytes : 0;
}

int amulet_mmlike_f32_autopack(int task, int thres_form, int trans_a, int trans_b, int64_t M, int64_t N,
                               int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
                               const float *thres, int64_t ldt, const float *dis, float *R, int64_t ldr,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    const MmlikeCall c = {task, thres_form, trans_a ? 1 : 0, trans_b ? 1 : 0, M, N, K, A, lda, B, ldb,
                          thres, ldt, dis, R, ldr};
    const int rc = check_mmlike(c);
    if (rc < 0) return rc;
    if (rc == 1) return AMULET_OK;
    if (workspace && autopack_wanted(task != TASK_IDENTITY, trans_a, N, lda, 4)) {
        if (workspace_bytes < amulet_autopack_workspace_bytes(4, M, K)) return AMULET_ERR_WORKSPACE;
        const int64_t ld = amulet_packed_ld(K, 4);
        const int prc = amulet_pack(4, M, K, A, lda, workspace, ld, stream);
        if (prc != AMULET_OK) return prc;
        A = (const float *)workspace;
        lda = ld;
    }
    return amulet_mmlike_f32_general(task, thres_form, trans_a, trans_b, -1, M, N, K, A, lda, B, ldb, thres,
                                     ldt, dis, R, ldr, stream);
}

int amulet_mmlike_f64_autopack(int task, int thres_form, int trans_a, int trans_b, int64_t M, int64_t N,
                               int64_t K, const double *A, int64_t lda, const double *B, int64_t ldb,
                               const double *thres, int64_t ldt, const double *dis, double *R, int64_t ldr,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    // the plain call validates everything; only what the copy itself relies on is checked before it
    if (workspace && A && M > 0 && N > 0 && K > 0 && M <= kMaxDim && K <= kMaxDim && lda >= K &&
        task > TASK_IDENTITY && task <= TASK_COUNT_GT && autopack_wanted(true, trans_a, N, lda, 8)) {
        if (workspace_bytes < amulet_autopack_workspace_bytes(8, M, K)) return AMULET_ERR_WORKSPACE;
        const int64_t ld = amulet_packed_ld(K, 8);
        const int prc = amulet_pack(8, M, K, A, lda, workspace, ld, stream);
        if (prc != AMULET_OK) return prc;
        A = (const double *)workspace;
        lda = ld;
    }
    return amulet_mmlike_f64_general(task, thres_form, trans_a, trans_b, M, N, K, A, lda, B, ldb, thres, ldt,
                                     dis, R, ldr, stream);
}

int amulet_count_i8(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B,
                    int64_t ldb, int32_t *R, int64_t ldr, void *stream)
{
    const int rc = check_common(M, N, K, A, lda, B, ldb, R, ldr);
    if (rc < 0) return rc;
    if (rc == 1) return AMULET_OK;
    return run_count(lookup_shape(AMULET_TASK_COUNT_I8, M, N, K), M, N, K, A, lda, B, ldb, R, ldr,
                     stream);
}

// In-flight adaptive execution for the join count (paper Sec. 4.4): the candidates here are
// not points of a two-parameter grid but the matrix-core kernels themselves (register-staged and
// streamed, 128- to 256-row tiles, one tile per workgroup or persistent), so the walk is flat:
// the shape a plain call would use first, then the others from the widest tile down, each on a
// slab of rows of the caller's R of about two tiles per compute unit, as long as untested rows
// are left in the first half of R; time per row decides, the rest runs with the winner.
int amulet_count_i8_adaptive(int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda, const int8_t *B,
                             int64_t ldb, int32_t *R, int64_t ldr, void *stream, int *chosen_shape, int *n_trials)
{
    const int rc = check_common(M, N, K, A, lda, B, ldb, R, ldr);
    if (rc < 0) return rc;
    int best = lookup_shape(AMULET_TASK_COUNT_I8, M, N, K);
    if (chosen_shape) *chosen_shape = best;
    if (n_trials) *n_trials = 0;
    if (rc == 1) return AMULET_OK;
    // tile height and width of each matrix-core shape (shape 0, the plain loop, is no candidate)
    static const int tile_rows[COUNT_SHAPE_COUNT] = {0, 128, 256, 128, 128, 256, 128, 256, 256};
    static const int tile_cols[COUNT_SHAPE_COUNT] = {0, 128, 256, 256, 128, 256, 256, 256, 256};
    auto slab_rows = [&](int shape) {
        const int64_t tiles_n = (N + tile_cols[shape] - 1) / tile_cols[shape];
        int64_t row_tiles = (2 * (int64_t)compute_units() + tiles_n - 1) / tiles_n;
        if (row_tiles < 1) row_tiles = 1;
        return row_tiles * tile_rows[shape];
    };
    int order[COUNT_SHAPE_COUNT], n_order = 0;
    order[n_order++] = best;
    for (int sidx = COUNT_SHAPE_COUNT - 1; sidx >= 1; --sidx)
        if (sidx != best) order[n_order++] = sidx;
    const int64_t budget = M / 2;
    int64_t next_row = 0;
    int trials = 0, status = AMULET_OK;
    // a task too small to spare the default shape's slab and one more runs whole with that shape,
    // and so does one of a few milliseconds (estimated at 2.2 POP/s plus the read-modify-write of
    // R at 5 TB/s): each slab is a launch with a last round of its own
    const double est_ms = (2.0 * (double)M * (double)N * (double)K / 2.2e15 + 8.0 * (double)M * (double)N / 5.0e12) * 1e3;
    const bool can_test = best >= 1 && slab_rows(best) + slab_rows(order[1]) <= budget && est_ms >= adaptive_min_task_ms();
    if (can_test) {
        // the candidates' order is fixed: enqueued back to back, one wait for all (BatchedTrials)
        BatchedTrials bt;
        if (bt.begin((hipStream_t)stream)) {
            for (int i = 0; i < n_order && status == AMULET_OK; ++i) {
                const int shape = order[i];
                const int64_t rows = slab_rows(shape);
                if (next_row + rows > budget) continue;   // no rows left for this one: a narrower tile may still fit
                if (run_count(shape, rows, N, K, A + next_row * lda, lda, B, ldb, R + next_row * ldr, ldr, stream) !=
                    AMULET_OK) {
                    status = AMULET_ERR_LAUNCH;
                    break;
                }
                bt.mark(shape, rows, (hipStream_t)stream);
                next_row += rows;
                trials += 1;
            }
            if (status == AMULET_OK && trials > 0) {
                const int w = bt.finish();
                if (w < 0) status = AMULET_ERR_LAUNCH;
                else best = bt.shape[w];
            }
        }
    }
    if (status != AMULET_OK) return status;
    int out = AMULET_OK;
    if (next_row < M)
        out = run_count(best, M - next_row, N, K, A + next_row * lda, lda, B, ldb, R + next_row * ldr, ldr, stream);
    if (out == AMULET_OK && trials > 1) {
        std::lock_guard<std::mutex> lock(g_sel_mutex);
        g_selected[sel_key(AMULET_TASK_COUNT_I8, M, N, K)] = best;
    }
    if (chosen_shape) *chosen_shape = best;
    if (n_trials) *n_trials = trials;
    return out;
}

// Row pitch of a transposed copy in the workspace: whole 128-byte lines (so the streamed kernel
// takes it), never a multiple of 4 KiB.
static int64_t i8_copy_ld(int64_t cols) { return amulet_packed_ld(cols, 1); }

size_t amulet_count_i8_workspace_bytes(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    size_t n = 0;
    if (trans_a) n += (size_t)M * (size_t)i8_copy_ld(K);
    if (trans_b) n += (size_t)K * (size_t)i8_copy_ld(N);
    return n;
}

// Extents of the copies in a repacking workspace: K in whole 64s (zero filled), and room for
// whole 256 x 256 tiles around M and N (never initialised: what is computed from it belongs to
// outputs that do not exist and is not written).
static int64_t i8_tile_up(int64_t n) { return (n + 255) / 256 * 256; }

size_t amulet_count_i8_repack_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    const int64_t Kp = (K + 63) / 64 * 64;
    return (size_t)i8_tile_up(M) * (size_t)i8_copy_ld(Kp) + (size_t)Kp * (size_t)i8_copy_ld(i8_tile_up(N));
}

int amulet_count_i8_general(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K, const int8_t *A,
                            int64_t lda, const int8_t *B, int64_t ldb, int32_t *R, int64_t ldr,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    if (M < 0 || N < 0 || K < 0) return AMULET_ERR_DIM;
    if (M > kMaxDim || N > kMaxDim || K > kMaxDim) return AMULET_ERR_RANGE;
    if (M == 0 || N == 0 || K == 0) return AMULET_OK;
    if (!A || !B || !R) return AMULET_ERR_NULL;
    if (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N) || ldr < N) return AMULET_ERR_LD;
    if (trans_a || trans_b) {
        if (!workspace) return AMULET_ERR_NULL;
        if (workspace_bytes < amulet_count_i8_workspace_bytes(trans_a, trans_b, M, N, K)) return AMULET_ERR_WORKSPACE;
    }
    int8_t *w = (int8_t *)workspace;
    hipStream_t s = (hipStream_t)stream;
    // With room for both operands the workspace also serves as their aligned home: an operand
    // whose rows are not 16-byte aligned, or whose extent is not whole tiles, is copied to a
    // pitch that is aligned, with room for whole tiles around it, and when K is not a multiple
    // of 64 both are copied with K padded by zeros (which add nothing to a count).  Every
    // workgroup then loads without guards, and the streamed kernel takes the whole-tile part.
    const int64_t Kp = (K + 63) / 64 * 64;
    const bool repack = workspace && ((uintptr_t)workspace & 15u) == 0 &&
                        workspace_bytes >= amulet_count_i8_repack_workspace_bytes(M, N, K);
    auto rows_aligned = [](const void *p, int64_t ld) { return ((uintptr_t)p & 15u) == 0 && ld % 16 == 0; };
    const bool pad_k = repack && Kp != K;
    const int64_t Kc = pad_k ? Kp : K;               // k extent of the copies
    int64_t m_load = M, n_load = N;
    hipError_t e = hipSuccess;
    if (trans_a) {   // stored K x M: the copy is M x K
        const int64_t ld = i8_copy_ld(Kc);
        e = launch_transpose_i8(K, M, A, lda, w, ld, s);
        if (e == hipSuccess && pad_k) e = launch_zero_block_i8(w, ld, 0, M, K, Kp - K, s);
        A = w; lda = ld;
        if (repack) m_load = i8_tile_up(M);
        w += (repack ? i8_tile_up(M) : M) * ld;
    } else if (repack && (pad_k || !rows_aligned(A, lda) || M % 256 != 0)) {
        const int64_t ld = i8_copy_ld(Kc);
        e = launch_pack_pad_i8(M, K, A, lda, w, ld, M, (Kc + 15) / 16 * 16, s);
        A = w; lda = ld;
        m_load = i8_tile_up(M);
        w += i8_tile_up(M) * ld;
    }
    if (e != hipSuccess) { g_last_hip_error = e; return AMULET_ERR_LAUNCH; }
    if (trans_b) {   // stored N x K: the copy is K x N
        const int64_t ld = repack ? i8_copy_ld(i8_tile_up(N)) : i8_copy_ld(N);
        e = launch_transpose_i8(N, K, B, ldb, w, ld, s);
        if (e == hipSuccess && pad_k) e = launch_zero_block_i8(w, ld, K, Kp - K, 0, N, s);
        B = w; ldb = ld;
        if (repack) n_load = i8_tile_up(N);
    } else if (repack && (pad_k || !rows_aligned(B, ldb) || N % 256 != 0)) {
        const int64_t ld = i8_copy_ld(i8_tile_up(N));
        e = launch_pack_pad_i8(K, N, B, ldb, w, ld, Kc, (N + 15) / 16 * 16, s);
        B = w; ldb = ld;
        n_load = i8_tile_up(N);
    }
    if (e != hipSuccess) { g_last_hip_error = e; return AMULET_ERR_LAUNCH; }
    return run_count(lookup_shape(AMULET_TASK_COUNT_I8, M, N, K), M, N, Kc, A, lda, B, ldb, R, ldr, stream,
                     m_load, n_load);
}

// ---- the join count for callers that cannot allocate --------------------------------------
// The workspace of amulet_count_i8_general, as a file-scope device array: one copy per GPU the
// library is loaded on, held until the process ends.  In host code the array's name is only a
// stand-in for the symbol; the device address is asked for once per device
// (hipGetSymbolAddress, with that device current) and kept, and only that pointer is ever
// handed to a kernel.
static __device__ __align__(256) unsigned char scratch[AMULET_STATIC_SCRATCH_BYTES];
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[16];   // per device, NULL until asked

static int scratch_of_current_device(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= 16)) e = hipErrorInvalidDevice;
    if (e == hipSuccess) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void *p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e == hipSuccess && !p) e = hipErrorInvalidSymbol;
            if (e == hipSuccess) g_scratch_ptr[dev] = p;
        }
        *out = g_scratch_ptr[dev];
    }
    if (e != hipSuccess) {
        g_last_hip_error = e;
        return AMULET_ERR_LAUNCH;
    }
    return AMULET_OK;
}

int amulet_count_i8_static(int trans_a, int trans_b, int64_t M, int64_t N, int64_t K, const int8_t *A,
                           int64_t lda, const int8_t *B, int64_t ldb, int32_t *R, int64_t ldr, void *stream)
{
    if (M < 0 || N < 0 || K < 0) return AMULET_ERR_DIM;
    if (M > kMaxDim || N > kMaxDim || K > kMaxDim) return AMULET_ERR_RANGE;
    if (M == 0 || N == 0 || K == 0) return AMULET_OK;
    // the repacking workspace is the larger of the two sizes the general call knows, so a
    // problem that fits it may take any of that call's paths
    const size_t need = amulet_count_i8_repack_workspace_bytes(M, N, K);
    if (need > (size_t)AMULET_STATIC_SCRATCH_BYTES ||
        amulet_count_i8_workspace_bytes(trans_a, trans_b, M, N, K) > (size_t)AMULET_STATIC_SCRATCH_BYTES)
        return AMULET_ERR_WORKSPACE;
    void *ws = nullptr;
    const int rc = scratch_of_current_device(&ws);
    if (rc != AMULET_OK) return rc;
    return amulet_count_i8_general(trans_a, trans_b, M, N, K, A, lda, B, ldb, R, ldr, ws,
                                   (size_t)AMULET_STATIC_SCRATCH_BYTES, stream);
}

int amulet_count_i8_shape(int shape, int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda,
                          const int8_t *B, int64_t ldb, int32_t *R, int64_t ldr, void *stream)
{
    if (shape < 0 || shape >= COUNT_SHAPE_COUNT) return AMULET_ERR_SHAPE;
    const int rc = check_common(M, N, K, A, lda, B, ldb, R, ldr);
    if (rc < 0) return rc;
    if (rc == 1) return AMULET_OK;
    return run_count(shape, M, N, K, A, lda, B, ldb, R, ldr, stream);
}

int amulet_count_i8_assign(int shape, int64_t M, int64_t N, int64_t K, const int8_t *A, int64_t lda,
                           const int8_t *B, int64_t ldb, int32_t *R, int64_t ldr, void *stream)
{
    if (shape >= COUNT_SHAPE_COUNT) return AMULET_ERR_SHAPE;
    const int rc = check_common(M, N, K, A, lda, B, ldb, R, ldr);
    if (rc < 0) return rc;
    if (M == 0 || N == 0) return AMULET_OK;
    if (!R) return AMULET_ERR_NULL;
    if (ldr < N) return AMULET_ERR_LD;
    if (K == 0) {   // an empty sum: R = 0
        CountArgs z;
        z.R = R; z.ldr = ldr; z.M = (int)M; z.N = (int)N;
        const hipError_t e = launch_zero_r_i32(z, (hipStream_t)stream);
        g_last_hip_error = e;
        return e == hipSuccess ? AMULET_OK : AMULET_ERR_LAUNCH;
    }
    if (shape < 0) {
        shape = lookup_shape(AMULET_TASK_COUNT_I8, M, N, K);
        // (without the read of R the persistent kernel's edge over two 128 x 256 tiles per unit starts
        // later: 768 tiles of 256 x 256 94 against 88 us, 1024 tiles level, 1536 tiles 272 / 277)
        if (shape == 8 && ((M + 255) / 256) * ((N + 255) / 256) < 1024) shape = 6;
    }
    return run_count(shape, M, N, K, A, lda, B, ldb, R, ldr, stream, 0, 0, true);
}

int amulet_greedy_search(int n0, int n1, amulet_score_fn score, void *ctx, int *best0, int *best1)
{
    if (!score || !best0 || !best1) return AMULET_ERR_NULL;
    if (n0 <= 0 || n1 <= 0) return AMULET_ERR_DIM;
    int calls = 0;
    // stage 1: axis 1 at its first value, every axis-0 candidate, keep the lowest score
    int b0 = 0;
    double s_best = 0.0;
    for (int i = 0; i < n0; ++i) {
        const double sc = score(i, 0, ctx);
        ++calls;
        if (i == 0 || sc < s_best) { s_best = sc; b0 = i; }
    }
    // stage 2: walk axis 1 upward; the first score above its predecessor ends the walk
    int b1 = 0;
    double prev = s_best;
    for (int j = 1; j < n1; ++j) {
        const double sc = score(b0, j, ctx);
        ++calls;
        if (sc > prev) break;
        prev = sc;
        b1 = j;
    }
    *best0 = b0;
    *best1 = b1;
    return calls;
}

int amulet_mmlike_f32_adaptive_general(int task, int thres_form, int trans_a, int trans_b, int64_t M, int64_t N,
                                       int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
                                       const float *thres, int64_t ldt, const float *dis, float *R, int64_t ldr,
                                       void *stream, int *chosen_shape, int *n_trials)
{
    const MmlikeCall c = {task, thres_form, trans_a ? 1 : 0, trans_b ? 1 : 0, M, N, K, A, lda, B, ldb,
                          thres, ldt, dis, R, ldr};
    const int rc = check_mmlike(c);
    if (rc < 0) return rc;
    if (chosen_shape) *chosen_shape = lookup_shape(task, M, N, K);
    if (n_trials) *n_trials = 0;
    if (rc == 1) return AMULET_OK;

    AdaptiveCtx x;
    memset(&x, 0, sizeof(x));
    x.call = c;
    x.stream = (hipStream_t)stream;
    x.budget_rows = M / 2;   // at least half of the task runs with the winner
    x.best_score = 1e300;
    x.best_shape = -1;
    for (double &sc : x.score_of) sc = -1.0;
    int best = lookup_shape(task, M, N, K);
    // too small to spare the default shape's slab and two more: run it whole with that shape
    const bool can_test = trial_rows(c, best) + 2 * trial_rows(c, VALU_TILES + 0) <= x.budget_rows;
    if (can_test && hipEventCreate(&x.e0) == hipSuccess && hipEventCreate(&x.e1) == hipSuccess) {
        if (task == TASK_IDENTITY) {
            // the dense contraction runs on the matrix cores: its two tiles are the candidates
            // (a vector-ALU slab runs at a sixth of their rate: one such trial on the caller's
            // rows cost 20 % of an 8192^3 call, and none ever won)
            // (the streamed shapes fall back to the register-staged kernel where they cannot stream)
            // Three candidates whose order is fixed: enqueued back to back, one wait for all.
            const int first = best >= IDENTITY_MFMA_SHAPE ? best : IDENTITY_MFMA_DMA3_SHAPE;
            const int cand[3] = {first, first == IDENTITY_MFMA_DMA4_SHAPE ? IDENTITY_MFMA_DMA3_SHAPE : IDENTITY_MFMA_DMA4_SHAPE,
                                 IDENTITY_MFMA_BIG_SHAPE};
            // (Not for a task of a few milliseconds, estimated at 140 TFLOP/s: each slab is a launch
            // with a last round of its own, which cost 16384 x 8192 x 1024, 1.9 ms, 13 %.)
            const bool worth_it = 2.0 * (double)M * (double)N * (double)K / 1.4e11 >= adaptive_min_task_ms();
            BatchedTrials bt;
            if (worth_it && bt.begin(x.stream)) {
                for (int i = 0; i < 3 && x.status == AMULET_OK; ++i) {
                    const int64_t rows = trial_rows(c, cand[i]);
                    if (x.next_row + rows > x.budget_rows) continue;
                    if (run_rows(c, cand[i], x.next_row, rows, x.stream) != AMULET_OK) { x.status = AMULET_ERR_LAUNCH; break; }
                    bt.mark(cand[i], rows, x.stream);
                    x.next_row += rows;
                    x.trials += 1;
                }
                if (x.status == AMULET_OK && x.trials > 0) {
                    const int w = bt.finish();
                    if (w < 0) x.status = AMULET_ERR_LAUNCH;
                    else x.best_shape = bt.shape[w];
                }
            }
        } else {
            // The shape a plain call would use is tried first, so that the walk can only replace
            // it by something that measured faster on this very task.  Then the paper's order:
            // the k axis (Sec. 4.5), then the tile axis upward with an early stop (Sec. 4.6); a
            // candidate for which no untested rows are left scores as infinitely slow, which
            // ends the walk.  The winner is the fastest slab of all.
            if (best >= 0 && best < VALU_SHAPE_COUNT) x.score_of[best] = adaptive_trial(&x, best);
            int b0 = 0, b1 = 0;
            amulet_greedy_search(VALU_KAXIS, VALU_TILES, adaptive_valu_score, &x, &b0, &b1);
        }
        if (x.best_shape >= 0) best = x.best_shape;
    }
    if (x.e0) (void)hipEventDestroy(x.e0);
    if (x.e1) (void)hipEventDestroy(x.e1);
    if (x.status != AMULET_OK) return x.status;
    int out = AMULET_OK;
    if (x.next_row < M) out = run_rows(c, best, x.next_row, M - x.next_row, x.stream);
    if (out == AMULET_OK && x.trials > 0) {
        std::lock_guard<std::mutex> lock(g_sel_mutex);
        g_selected[sel_key(task, M, N, K)] = best;
    }
    if (chosen_shape) *chosen_shape = best;
    if (n_trials) *n_trials = x.trials;
    return out;
}

int amulet_mmlike_f32_adaptive(int task, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                               const float *B, int64_t ldb, const float *params, float *R, int64_t ldr,
                               void *stream, int *chosen_shape, int *n_trials)
{
    return amulet_mmlike_f32_adaptive_general(task, THRES_COL, 0, 0, M, N, K, A, lda, B, ldb, params, 0,
                                              params ? params + N : nullptr, R, ldr, stream, chosen_shape, n_trials);
}

int amulet_tune(int task, int64_t M, int64_t N, int64_t K, void *stream)
{
    const int ns = n_shapes(task);
    if (ns == 0) return AMULET_ERR_TASK;
    if (M < 0 || N < 0 || K < 0) return AMULET_ERR_DIM;
    if (M > kMaxDim || N > kMaxDim || K > kMaxDim) return AMULET_ERR_RANGE;
    if (M == 0 || N == 0 || K == 0) return default_shape(task, M, N, K);

    // Trials run on a row slab of the task when the whole task would take long
    // (the paper tests parameters on a small part of the input, Sec. 4.4).
    int64_t Mt = M;
    const double cap = 68719476736.0;  // 2^36 products per trial
    if ((double)M * (double)N * (double)K > cap) {
        Mt = (int64_t)(cap / ((double)N * (double)K));
        if (Mt < 2048) Mt = 2048;
        if (Mt > M) Mt = M;
    }
    const bool i8 = task == AMULET_TASK_COUNT_I8;
    const size_t es = i8 ? 1 : 4;
    TrialCtx c;
    memset(&c, 0, sizeof(c));
    c.task = task; c.M = Mt; c.N = N; c.K = K; c.stream = (hipStream_t)stream;
    int result = AMULET_ERR_LAUNCH;
    bool ok = hipMalloc(&c.A, (size_t)Mt * K * es) == hipSuccess &&
              hipMalloc(&c.B, (size_t)K * N * es) == hipSuccess &&
              hipMalloc(&c.R, (size_t)Mt * N * 4) == hipSuccess &&
              hipMalloc(&c.params, (size_t)2 * N * 4) == hipSuccess &&
              hipEventCreate(&c.e0) == hipSuccess && hipEventCreate(&c.e1) == hipSuccess;
    if (ok) {
        if (i8) {
            hipLaunchKernelGGL(fill_i8_kernel, dim3(1024), dim3(256), 0, c.stream, (int8_t *)c.A,
                               (size_t)Mt * K, 17u);
            hipLaunchKernelGGL(fill_i8_kernel, dim3(1024), dim3(256), 0, c.stream, (int8_t *)c.B,
                               (size_t)K * N, 29u);
        } else {
            hipLaunchKernelGGL(fill_f32_kernel, dim3(1024), dim3(256), 0, c.stream, (float *)c.A,
                               (size_t)Mt * K, 0.0f, 1.0f, 17u);
            hipLaunchKernelGGL(fill_f32_kernel, dim3(1024), dim3(256), 0, c.stream, (float *)c.B,
                               (size_t)K * N, 0.0f, 1.0f, 29u);
        }
        hipLaunchKernelGGL(fill_f32_kernel, dim3(64), dim3(256), 0, c.stream, (float *)c.params,
                           (size_t)N, 0.25f, 0.0f, 1u);
        hipLaunchKernelGGL(fill_f32_kernel, dim3(64), dim3(256), 0, c.stream, (float *)c.params + N,
                           (size_t)N, 0.1f, 0.0f, 1u);
        hipLaunchKernelGGL(fill_f32_kernel, dim3(1024), dim3(256), 0, c.stream, (float *)c.R,
                           (size_t)Mt * N, 0.0f, 0.0f, 1u);
        // Bring the device to its loaded clocks first: launches right after idle run up to 10 %
        // faster than the same ones a few milliseconds later, which would favour whichever
        // candidate is tried first.
        // (30 ms of the default shape; 150 ms for the matrix-core tasks, whose clocks keep
        // settling for longer: the persistent join-count kernel measures 0.245 ms cold and 0.223
        // warm, which decided a tune against it)
        const int dflt = default_shape(task, M, N, K);
        const float warm_ms = (i8 || task == TASK_IDENTITY) ? 150.0f : 30.0f;
        float spent = 0.0f;
        for (int i = 0; i < 4096 && spent < warm_ms; ++i) {
            const float ms = trial_span_ms(&c, dflt, 1);
            if (ms < 0.0f) break;
            spent += ms > 0.02f ? ms : 0.02f;
        }
        int chosen;
        if (i8) {
            // shape 0 is the plain per-output loop kept for checking; only the matrix-core
            // shapes are candidates
            chosen = 1;
            double best = 0.0;
            for (int sidx = 1; sidx < COUNT_SHAPE_COUNT; ++sidx) {
                const double t = time_shape(&c, sidx);
                if (sidx == 1 || t < best) { best = t; chosen = sidx; }
            }
        } else {
            int b0 = 0, b1 = 0;
            // identity on the vector ALU has the two staging depths only; the predicate tasks walk
            // the whole k axis (staging depth, then K in 1, 2, 4, 8 parts per tile)
            amulet_greedy_search(task == TASK_IDENTITY ? VALU_DEPTHS : VALU_KAXIS, VALU_TILES, valu_trial_score, &c, &b0, &b1);
            chosen = b0 * VALU_TILES + b1;
            if (task == TASK_IDENTITY) {
                double best = time_shape(&c, chosen);
                for (int sidx = IDENTITY_MFMA_SHAPE; sidx < IDENTITY_SHAPE_COUNT; ++sidx) {
                    const double t = time_shape(&c, sidx);
                    if (t < best) { best = t; chosen = sidx; }
                }
            }
        }
        // the search's winner replaces the built-in default only if it also wins a direct rematch,
        // by more than the 3 % that two timings of one shape can differ by
        if (c.status == AMULET_OK && chosen != dflt && time_shape(&c, chosen) >= 0.97 * time_shape(&c, dflt))
            chosen = dflt;
        (void)hipStreamSynchronize(c.stream);
        if (c.status == AMULET_OK) {
            std::lock_guard<std::mutex> lock(g_sel_mutex);
            g_selected[sel_key(task, M, N, K)] = chosen;
            result = chosen;
        }
    }
    if (c.e0) (void)hipEventDestroy(c.e0);
    if (c.e1) (void)hipEventDestroy(c.e1);
    (void)hipFree(c.A); (void)hipFree(c.B); (void)hipFree(c.R); (void)hipFree(c.params);
    return result;
}

int64_t amulet_tile_grid(int64_t tiles_m, int64_t tiles_n)
{
    if (tiles_m <= 0 || tiles_n <= 0) return 0;
    return xcd_grid(tiles_m, tiles_n);
}

int amulet_tile_of_workgroup(int64_t block, int64_t tiles_m, int64_t tiles_n, int64_t *tm, int64_t *tn)
{
    if (!tm || !tn) return AMULET_ERR_NULL;
    if (tiles_m <= 0 || tiles_n <= 0 || tiles_m > kMaxDim || tiles_n > kMaxDim || block < 0 ||
        block >= xcd_grid(tiles_m, tiles_n) || block > 0x7fffffffLL)
        return AMULET_ERR_DIM;
    int m = 0, n = 0;
    const bool real = xcd_tile((int)block, (int)tiles_m, (int)tiles_n, m, n);
    *tm = m;
    *tn = n;
    return real ? 1 : 0;
}

int amulet_shape_count(int task) { return n_shapes(task); }

const char *amulet_shape_name(int task, int shape)
{
    if (shape < 0 || shape >= n_shapes(task)) return "invalid";
    if (task == AMULET_TASK_COUNT_I8) return kCountShapeNames[shape];
    if (is_mfma_shape(task, shape)) {
        static const char *const names[5] = {"mfma_f32_128x128_k16", "mfma_f32_256x256_w16_k16", "mfma_f32_128x128_dma3",
                                             "mfma_f32_128x128_dma4", "mfma_f32_64x64_dma4"};
        return names[shape - IDENTITY_MFMA_SHAPE];
    }
    return kValuShapes[shape].name;
}

int amulet_selected_shape(int task, int64_t M, int64_t N, int64_t K)
{
    if (n_shapes(task) == 0) return AMULET_ERR_TASK;
    return lookup_shape(task, M, N, K);
}

void amulet_clear_selections(void)
{
    std::lock_guard<std::mutex> lock(g_sel_mutex);
    g_selected.clear();
}

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

int amulet_register_demand(int I_h, int I_w, int S_w, int n_const, int n_i, int n_j, int n_ij,
                           int n_temp)
{
    if (I_h <= 0 || I_w <= 0 || S_w <= 0 || n_const < 0 || n_i < 0 || n_j < 0 || n_ij < 0 || n_temp < 0)
        return AMULET_ERR_DIM;
    const int w = ceil_div(I_w, S_w);
    return I_h * w + 1 + w + n_const + n_i + n_j * w + n_ij + n_temp;
}

int amulet_choose_kernel_height(int I_h_max, int I_w, int S_w, int n_const, int n_i, int n_j, int n_ij,
                                int n_temp, int budget)
{
    for (int h = I_h_max; h >= 1; --h) {
        const int need = amulet_register_demand(h, I_w, S_w, n_const, n_i, n_j, n_ij, n_temp);
        if (need < 0) return need;
        if (need <= budget) return h;
    }
    return 0;
}

const char *amulet_strerror(int code)
{
    switch (code) {
    case AMULET_OK: return "success";
    case AMULET_ERR_TASK: return "unknown task";
    case AMULET_ERR_DIM: return "negative or empty dimension";
    case AMULET_ERR_NULL: return "required pointer is NULL";
    case AMULET_ERR_LD: return "leading dimension smaller than the row length";
    case AMULET_ERR_LAUNCH: return "HIP reported an error at launch";
    case AMULET_ERR_SHAPE: return "unknown tile shape";
    case AMULET_ERR_RANGE: return "dimension too large for the kernels' 32-bit indexing";
    case AMULET_ERR_WORKSPACE: return "workspace too small for the packed copy";
    default: return "unknown status code";
    }
}

const char *amulet_last_launch_error(void) { return hipGetErrorString(g_last_hip_error); }

void amulet_set_deterministic(int on) { g_deterministic.store(on ? 1 : 0, std::memory_order_relaxed); }

int amulet_get_deterministic(void) { return k_split_allowed() ? 0 : 1; }

void amulet_debug_fail_launches(int n) { g_forced_launch_failures.store(n > 0 ? n : 0, std::memory_order_relaxed); }

const char *amulet_version(void) { return "amulet-gfx950 0.1"; }

}  // extern "C"
