// fp32 VALU tile kernels for the matrix-multiplication-like tasks whose g acts
// on each product before the k-sum (paper Fig. 1, Fig. 2, Query 1-3): these
// cannot run on the matrix cores, so the inner kernel is a per-lane register
// micro-tile on the vector ALU, the CDNA form of the paper's register-blocked
// inner kernel (Sec. 3, Fig. "12x16 inner kernel"; Sec. 4.3.3 for the version
// with g inside the kk loop).
//
// Mapping (one workgroup = NW waves, one R tile of NW*TM rows x 256*NG columns):
//   * a lane owns 4*NG columns: column groups g*256 + lane*4 .. +3.  thres[j]
//     and the per-column factor derived from dis[j] live in registers for the
//     whole K loop (the paper reloads them every kk and budgets registers for
//     them, Sec. 4.3.2).
//   * a wave owns TM rows, the same for all its lanes, so A[i][k] is wave
//     uniform: it is fetched through the scalar data cache into SGPRs and used
//     directly as the scalar operand of the multiply.  A never touches LDS or
//     vector registers.
//   * the BK x (256*NG) tile of B is staged global -> registers -> LDS, double
//     buffered, one barrier per tile; a lane reads its own 16-byte column groups
//     back with conflict-free ds_read_b128.
//   * the k-sum is two-level: a partial accumulator over FLUSH_K products,
//     folded into the main accumulator after that many, which keeps fp32
//     round-off of long same-sign sums (K = 8192 retail data) far inside the
//     1e-5 budget.
//   * the K remainder is computed by a k-by-k tail loop, never by zero padding:
//     g(0) is not 0 in general (BOOST with thres < 0, COUNT_GT with thres < 0).
//
// Per product the discount task costs 4 VALU lane-operations (multiply rounded
// to fp32, compare, select of the factor, fused multiply-add), the paper's
// sequence "mul, gtcmp, mul, masksub, add" (Sec. 4.3.1) minus one.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "amulet_internal.h"

#ifndef AMULET_MMLIKE_VALU_IMPL_H
#define AMULET_MMLIKE_VALU_IMPL_H

namespace amulet {

// k-extent of one partial sum of the two-level fp32 accumulation
constexpr int FLUSH_K = 64;

typedef float f4 __attribute__((ext_vector_type(4)));
// the same four floats at any float address: still one 16-byte access (global accesses take
// any address on this target), used where rows are not 16-byte aligned
typedef f4 f4_any __attribute__((aligned(4)));
typedef const __attribute__((address_space(4))) float *sptr_f;      // read through the scalar cache

template <int TASK> struct AccT { typedef float type; };
template <> struct AccT<TASK_COUNT_GT> { typedef int type; };

// Four products of one A value with a lane's group of four B values, folded
// into the (partial) accumulators.  The multiply is a separately rounded fp32
// operation wherever a comparison depends on it.  The four compares are issued
// back to back before the four selects, so each select is at least three
// instructions behind the compare whose mask it reads (the distance gfx950
// wants between a VALU write of a lane mask and its VALU read).
template <int TASK>
__device__ __forceinline__ void fold4(float a, f4 b, const float *th, const float *q,
                                      typename AccT<TASK>::type *acc)
{
    if constexpr (TASK == TASK_IDENTITY) {
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = __builtin_fmaf(a, b[c], acc[c]);
    } else if constexpr (TASK == TASK_DISCOUNT) {
        float p[4], s[4];
        bool m[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) p[c] = a * b[c];          // one RN multiply (contraction is off)
#pragma unroll
        for (int c = 0; c < 4; ++c) m[c] = p[c] > th[c];
#pragma unroll
        for (int c = 0; c < 4; ++c) s[c] = m[c] ? q[c] : 1.0f;  // q = 1 - dis[j]
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] = __builtin_fmaf(p[c], s[c], acc[c]);
    } else if constexpr (TASK == TASK_BOOST) {
        // p + (p > th)(p - th) = p + max(p - th, 0) is continuous in p, so the
        // unrounded product inside the fused operations is within tolerance.
        // One product at a time, fenced: fma, fma, max, add.  Three of the four read a scalar
        // register or an inline constant, and long runs of such instructions issue slower than
        // the same instructions interleaved with the all-vector add (register-only loops: 9.1-9.7
        // clocks per 64 products in groups of four, 8.4 one at a time; the kernel 30.3 -> 32.3
        // TFLOP/s at 8192^3).  Left alone the scheduler builds pairs and runs of ten.
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float d = __builtin_fmaf(a, b[c], -th[c]);
            acc[c] = __builtin_fmaf(a, b[c], acc[c]);
            d = __builtin_fmaxf(d, 0.0f);
            acc[c] += d;
            __builtin_amdgcn_sched_barrier(0);
        }
    } else {
        // The count needs no lane mask: p > th exactly when th - p is negative (a difference of
        // two floats is zero only when they are equal, subnormal results included, and x - x is
        // +0), so the sign bit of the rounded difference is the predicate bit.  The one
        // exception, -0 - (+0) = -0, is excluded by the caller: it never passes a threshold of -0.  multiply,
        // subtract, shift, add: four plain vector instructions, against multiply, compare,
        // select, add, where the compare and the select pass a lane mask through the scalar
        // registers (a register-only loop of such a pair takes about as long as four plain
        // instructions).  Measured: +5 % with A through LDS, +12-14 % with A in scalar registers,
        // which the masks used to crowd out.
        float p[4], d[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) p[c] = a * b[c];          // one RN multiply (contraction is off)
#pragma unroll
        for (int c = 0; c < 4; ++c) d[c] = th[c] - p[c];
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] += (int)(__builtin_bit_cast(unsigned, d[c]) >> 31);
    }
}

// ALDS: the workgroup's rows of A go through LDS too (vector loads a whole tile ahead, then
// broadcast reads), instead of through the scalar cache chunk by chunk.  Slightly more
// registers and LDS traffic; used when the row pitch of A collides (amulet_pitch_collides):
// the scalar path fetches each 128-byte line of A in eight pieces, and when the lines of a
// workgroup's 32 rows all fall into the same L2 sets they are evicted between the pieces.
// PIPE (discount task, 4 x 4 micro-tile): a chunk runs as one software pipeline instead of k by k
// (see the chunk loop); the launcher says when.
template <int TASK, int TF, int TRANS, int TM, int NG, int NW, int BK, int KA, bool ALDS, bool PIPE = false, bool BPRE = false>
__global__ void __launch_bounds__(64 * NW)
mmlike_valu_kernel(const MmlikeArgs args)
{
    static_assert(!BPRE || (!ALDS && TM == 4 && NG == 1), "B values a chunk ahead: scalar-path A, 4 x 4 micro-tile");
    static_assert(!PIPE || (TASK == TASK_DISCOUNT && TM == 4 && NG == 1), "chunk pipeline: discount task, 4 x 4 micro-tile");
    static_assert(!ALDS || (TRANS == 0 && TM == 4 && NG == 1), "A through LDS: row-major operands, 4 x 4 micro-tile");
    typedef typename AccT<TASK>::type acc_t;
    static_assert(KA == 4 && TM % 4 == 0, "a transposed A is fetched as 4 rows x 4 k blocks");
    constexpr int BN = 256 * NG;           // tile columns
    constexpr int NT = 64 * NW;            // threads
    constexpr int F4_PER_ROW = BN / 4;     // float4 slots in one LDS row
    constexpr int LOADS = (BK * F4_PER_ROW) / NT;  // float4 slots staged per thread per tile
    static_assert((BK * F4_PER_ROW) % NT == 0, "B tile must split evenly over the threads");
    static_assert(BK % KA == 0 && (KA == 2 || KA == 4), "A is fetched KA k at a time");
    typedef float av_raw __attribute__((ext_vector_type(KA)));
    typedef av_raw av_t __attribute__((aligned(4)));
    typedef const __attribute__((address_space(4))) av_t *sptr_av;

    __shared__ __attribute__((aligned(16))) float Bs[2][BK][BN];
    constexpr int A_ROWS = NW * TM, A_PITCH = BK + 4;       // rows of the workgroup; padded row of the LDS A tile
    constexpr int A_F4 = A_ROWS * BK / 4;                   // float4 slots of one A tile (<= NT)
    static_assert(A_F4 <= NT, "one staging slot per thread at most");
    __shared__ __attribute__((aligned(16))) float Asl[ALDS ? 2 : 1][ALDS ? A_ROWS : 1][ALDS ? A_PITCH : 4];

    const int M = args.M, N = args.N;
    int K = args.K;
    const bool VEC = args.vec != 0;   // B and R rows are 16-byte aligned: float4 global accesses
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // XCD-aware tile order (xcd_tile in amulet_internal.h): each XCD walks its own rectangular
    // part of the tile grid, so its resident workgroups share A rows and B columns through its L2
    const int tiles_m = (M + NW * TM - 1) / (NW * TM);
    const int tiles_n = (N + BN - 1) / BN;
    int tm, tn;
    // place in the tile order, and which k range of it (see launch_one)
    int block = (int)blockIdx.x + args.block_base, ksplit_idx = (int)blockIdx.y;
    const bool tail_part = args.tail_splits > 1 && block >= args.tail_base;
    if (tail_part) {
        const int rel = block - args.tail_base;
        block = args.tail_base + rel % args.tail_blocks;
        ksplit_idx = rel / args.tail_blocks;
    }
    if (!xcd_tile(block, tiles_m, tiles_n, tm, tn)) return;   // padding: the whole workgroup leaves
    const int row0 = tm * (NW * TM) + wave * TM;
    const int col0 = tn * BN;

    const float *__restrict__ Bg = args.B;
    sptr_f As = (sptr_f)args.A;

    // Wave-uniform row offsets, clamped so edge waves read valid rows.  a(i,k) lives at
    // A[i*lda + k], or at A[k*lda + i] when A is stored transposed (the [k][i]-indexed
    // variant of paper Sec. 6.3): element offset = arow[r] + k * kstride.
    // TRANS (bit 0: A transposed, bit 1: B transposed) is a compile-time choice: each layout's
    // addressing state would otherwise cost the others scalar registers in the hot loop (one
    // kernel serving both transposed operands at run time spilled 30 of them).
    constexpr bool transA = (TRANS & 1) != 0, transB = (TRANS & 2) != 0;
    const int64_t kstride = transA ? args.lda : 1;
    // Split K (every tile when gridDim.y > 1, chosen by the host for problems with too few tiles
    // to fill the chip; else the tail blocks): this workgroup sums k in [kb, kb + kchunk) only
    // and adds its part to R atomically.
    const bool ksplit = gridDim.y > 1 || tail_part;
    if (ksplit) {
        const int kb = ksplit_idx * args.kchunk;
        As += (int64_t)kb * kstride;
        Bg += transB ? (int64_t)kb : (int64_t)kb * args.ldb;
        K = (K - kb < args.kchunk) ? K - kb : args.kchunk;
    }
    const bool rows_full = row0 + TM <= M;
    auto rowc = [&](int r) { const int row = row0 + r; return row < M ? row : M - 1; };
    // Row-major A: one 64-bit offset per row.  Transposed A: the wave's rows are neighbours in
    // memory, so the first row's index and the count of rows that exist say it all (row r of
    // the micro-tile reads row min(r, last valid) of them); eight scalar registers fewer.
    int64_t arow[transA ? 1 : TM];
    const int arow0 = row0 < M ? row0 : M - 1;
    const int last_valid = (M - arow0 < TM ? M - arow0 : TM) - 1;
    auto trow = [&](int r) { return arow0 + (r < last_valid ? r : last_valid); };   // transposed A: row index
    if constexpr (!transA) {
#pragma unroll
        for (int r = 0; r < TM; ++r) arow[r] = (int64_t)rowc(r) * args.lda;
    } else {
        arow[0] = 0;
    }

    // Parameters held in registers for the whole K loop: the discount factor 1 - dis[j] per
    // column, and the threshold in the operand form TF (paper Sec. 6.3): thres[j] per column,
    // thres[i] per row (wave-uniform, scalar), one constant, or thres[i][j] per output (read
    // once per tile, not once per product as a CPU kernel must).
    // The count task reads its predicate from the sign of th - p (see fold4), which takes a
    // threshold of -0 for a negative number when p is +0: thresholds are held as th + 0, which
    // turns -0 into +0 and changes nothing else.
    auto held = [](float t) { return TASK == TASK_COUNT_GT ? t + 0.0f : t; };
    float q[NG * 4];
    float th_col[TF == THRES_COL ? NG * 4 : 1];
    float th_row[TF == THRES_ROW ? TM : 1];
    float th_el[TF == THRES_ELEM ? TM : 1][TF == THRES_ELEM ? NG * 4 : 1];
    float th_const = __builtin_inff();
    if constexpr (TASK != TASK_IDENTITY) {
        if constexpr (TF == THRES_CONST) th_const = held(((sptr_f)args.thres)[0]);
        if constexpr (TF == THRES_ROW) {
#pragma unroll
            for (int r = 0; r < TM; ++r) th_row[r] = held(((sptr_f)args.thres)[rowc(r)]);
        }
        // Wave-uniform thresholds are held in vector registers all the same: a compare whose
        // threshold operand is a scalar register measured 25 % slower in this loop (4096^3
        // discount: 23.7 against 31.5 TFLOP/s with identical instruction counts), so the
        // uniform value is copied into a vector register once, before the K loop.
        if constexpr (TF == THRES_CONST) asm volatile("" : "+v"(th_const));
        if constexpr (TF == THRES_ROW) {
#pragma unroll
            for (int r = 0; r < TM; ++r) asm volatile("" : "+v"(th_row[r]));
        }
    }
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int col = col0 + g * 256 + lane * 4 + c;
            q[g * 4 + c] = 1.0f;
            if constexpr (TF == THRES_COL) th_col[g * 4 + c] = __builtin_inff();
            if (TASK != TASK_IDENTITY && col < N) {
                if constexpr (TF == THRES_COL) th_col[g * 4 + c] = held(args.thres[col]);
                if (TASK == TASK_DISCOUNT) q[g * 4 + c] = 1.0f - args.dis[col];
            }
            if constexpr (TF == THRES_ELEM && TASK != TASK_IDENTITY) {
#pragma unroll
                for (int r = 0; r < TM; ++r)
                    th_el[r][g * 4 + c] = (col < N) ? held(args.thres[(int64_t)rowc(r) * args.ldt + col])
                                                    : __builtin_inff();
            }
        }
    // the four thresholds facing row r, column group g
    auto thres4 = [&](int r, int g, float *t4) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if constexpr (TF == THRES_COL) t4[c] = th_col[g * 4 + c];
            else if constexpr (TF == THRES_ROW) t4[c] = th_row[r];
            else if constexpr (TF == THRES_CONST) t4[c] = th_const;
            else t4[c] = th_el[r][g * 4 + c];
        }
    };

    acc_t part[TM][NG * 4];
    float mainacc[TM][NG * 4];
#pragma unroll
    for (int r = 0; r < TM; ++r)
#pragma unroll
        for (int c = 0; c < NG * 4; ++c) {
            part[r][c] = 0;
            mainacc[r][c] = 0.0f;
        }

    // ---- B tile staging: global -> registers -> LDS -------------------------
    // Thread t stages float4 slot (row t / F4_PER_ROW + it * ROWS_PER_PASS, column group
    // t % F4_PER_ROW) of every tile.  Interior tiles (all columns inside N, rows 16-byte
    // aligned, BK full rows) take the branch-free path.
    constexpr int ROWS_PER_PASS = NT / F4_PER_ROW;
    static_assert(NT % F4_PER_ROW == 0 && LOADS * ROWS_PER_PASS == BK, "slot mapping");
    const int srow = threadIdx.x / F4_PER_ROW;
    const int scol = col0 + (threadIdx.x % F4_PER_ROW) * 4;
    const bool fast_cols = VEC && (col0 + BN <= N);
    const float *bsrc = Bg + (int64_t)srow * args.ldb + scol;   // advanced by BK rows per tile
    const int64_t pass_stride = (int64_t)ROWS_PER_PASS * args.ldb;
    const int64_t tile_stride = (int64_t)BK * args.ldb;
    f4 stage[LOADS];
    // B stored transposed (b(k,j) at B[j*ldb + k], the [j][k]-indexed variant of Sec. 6.3): a thread
    // owns one column of the tile and KPT consecutive k of it, read as float4 along k and
    // scattered into the same [k][n] LDS tile (neighbouring lanes hit neighbouring banks).
    constexpr int TPC = NT / BN;          // threads per column
    constexpr int KPT = BK / TPC;         // k per thread
    static_assert(NT % BN == 0 && BK % TPC == 0 && KPT == 4 * LOADS, "transposed-B slot mapping");
    const int tcol = threadIdx.x % BN;
    const int tk = (threadIdx.x / BN) * KPT;
    const float *btsrc = Bg + (int64_t)(col0 + tcol < N ? col0 + tcol : N - 1) * args.ldb + tk;
    // A tile staging (ALDS): thread t < A_F4 stages float4 slot (row t / (BK / 4), k quad t % (BK / 4))
    const int a_sr = threadIdx.x / (BK / 4), a_sq = (threadIdx.x % (BK / 4)) * 4;
    const float *asrc = nullptr;
    f4 a_stage = {0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (ALDS) {
        const int wg_row0 = tm * A_ROWS;
        const int arow_c = wg_row0 + a_sr < M ? wg_row0 + a_sr : M - 1;   // rows past M are never written back
        asrc = args.A + (ksplit ? (int64_t)ksplit_idx * args.kchunk : 0) + (int64_t)arow_c * args.lda + a_sq;
    }
    auto load_tile = [&](int krows) {
        if constexpr (ALDS) {
            if (threadIdx.x < A_F4) {
                if (krows == BK) {
                    a_stage = args.vecA ? *(const f4 *)asrc : (f4)*(const f4_any *)asrc;
                } else {
                    a_stage = f4{0.0f, 0.0f, 0.0f, 0.0f};
                    if (a_sq + 0 < krows) a_stage.x = asrc[0];
                    if (a_sq + 1 < krows) a_stage.y = asrc[1];
                    if (a_sq + 2 < krows) a_stage.z = asrc[2];
                    if (a_sq + 3 < krows) a_stage.w = asrc[3];
                }
                asrc += BK;
            }
        }
        if (transB) {
            const bool colok = col0 + tcol < N;
#pragma unroll
            for (int it = 0; it < LOADS; ++it) {
                f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                const int kk = tk + 4 * it;
                if (colok) {
                    const float *src = btsrc + 4 * it;
                    if (kk + 3 < krows) {
                        v = *(const f4_any *)src;
                    } else {
                        if (kk + 0 < krows) v.x = src[0];
                        if (kk + 1 < krows) v.y = src[1];
                        if (kk + 2 < krows) v.z = src[2];
                        if (kk + 3 < krows) v.w = src[3];
                    }
                }
                stage[it] = v;
            }
            btsrc += BK;
        } else if (fast_cols && krows == BK) {
#pragma unroll
            for (int it = 0; it < LOADS; ++it)
                stage[it] = *(const f4 *)(bsrc + it * pass_stride);
            bsrc += tile_stride;
        } else {
#pragma unroll
            for (int it = 0; it < LOADS; ++it) {
                f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (srow + it * ROWS_PER_PASS < krows) {
                    const float *src = bsrc + it * pass_stride;
                    if (scol + 3 < N) {
                        v = *(const f4_any *)src;
                    } else {
                        if (scol + 0 < N) v.x = src[0];
                        if (scol + 1 < N) v.y = src[1];
                        if (scol + 2 < N) v.z = src[2];
                    }
                }
                stage[it] = v;
            }
            bsrc += tile_stride;
        }
    };
    float *const bdst = &Bs[0][srow][(threadIdx.x % F4_PER_ROW) * 4];
    float *const btdst = &Bs[0][tk][tcol];
    auto store_tile = [&](int buf) {
        if constexpr (ALDS) {
            if (threadIdx.x < A_F4) *(f4 *)&Asl[buf][a_sr][a_sq] = a_stage;
        }
        if (transB) {
#pragma unroll
            for (int it = 0; it < LOADS; ++it)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    btdst[(buf * BK + 4 * it + e) * BN] = stage[it][e];
        } else {
#pragma unroll
            for (int it = 0; it < LOADS; ++it)
                *(f4 *)(bdst + (buf * BK + it * ROWS_PER_PASS) * BN) = stage[it];
        }
    };
    auto flush = [&]() {
        if constexpr (TASK != TASK_COUNT_GT) {
#pragma unroll
            for (int r = 0; r < TM; ++r)
#pragma unroll
                for (int c = 0; c < NG * 4; ++c) {
                    mainacc[r][c] += part[r][c];
                    part[r][c] = 0;
                }
        }
    };

    const int full_tiles = K / BK;
    const int tail = K - full_tiles * BK;
    const int n_tiles = full_tiles + (tail ? 1 : 0);
    constexpr int FLUSH_TILES = (FLUSH_K / BK) > 0 ? (FLUSH_K / BK) : 1;  // tiles per partial sum

    // A values of the chunk of KA k starting at kn, for the wave's TM rows, into SGPRs: TM
    // vectors of 4.  Row-major A: vector r holds row r's KA values.  Transposed A: vector
    // kk * (TM / 4) + v holds rows 4v .. 4v + 3 of k = kn + kk, exactly as loaded; re-sorting them
    // at fetch time would make every fetch wait for its own loads instead of letting them land
    // during the chunk's arithmetic.  a_of() names element (r, kk) of either arrangement.
    av_t a_next[TM];
    auto a_of = [](const av_t (&v)[TM], int r, int kk) -> float {
        return transA ? v[kk * (TM / 4) + r / 4][r % 4] : v[r][kk];
    };
    // (the chunk at k = kt + rel: kt a tile's first k, so that a row-major A costs one address per
    // row and tile, and the chunks whose rel is a constant are loads at immediate offsets from it)
    auto fetch_a = [&](int kt, int rel) {
        const int kn = kt + rel;
        if constexpr (!transA) {
            // the byte offset of the chunk as a 32-bit scalar the compiler cannot see through:
            // left visible, loads at constant offsets from one row address are merged into
            // one load per row and tile, issued at the tile's start and waited for there
            uint32_t relb = (uint32_t)rel * 4u;
            asm volatile("" : "+s"(relb));
            typedef const __attribute__((address_space(4))) char *sptr_c;
#pragma unroll
            for (int r = 0; r < TM; ++r) a_next[r] = *(sptr_av)((sptr_c)(As + (arow[r] + kt)) + relb);
        } else if (rows_full) {
            // 4 consecutive rows of one k are contiguous in the transposed storage
#pragma unroll
            for (int kk = 0; kk < KA; ++kk)
#pragma unroll
                for (int v = 0; v < TM / 4; ++v) {
                    a_next[kk * (TM / 4) + v] = *(sptr_av)(As + (int64_t)(kn + kk) * args.lda + arow0 + 4 * v);
                }
        } else {
#pragma unroll
            for (int kk = 0; kk < KA; ++kk)
#pragma unroll
                for (int r = 0; r < TM; ++r)
                    a_next[kk * (TM / 4) + r / 4][r % 4] = As[(int64_t)(kn + kk) * args.lda + trow(r)];
        }
    };
    load_tile(full_tiles > 0 ? BK : tail);
    store_tile(0);
    if (!ALDS && full_tiles > 0) fetch_a(0, 0);
    __syncthreads();

    // The arithmetic of one chunk: KA k of the wave's TM rows against a lane's 4 NG columns.
    auto compute_chunk = [&](const av_t (&a)[TM], const f4 (&b)[KA][NG]) {
        if constexpr (PIPE) {
            // The whole chunk as one software pipeline: compare i, multiply i + 1, FMA
            // i - 1, select i.  Every compare writes the same lane-mask register (vcc,
            // the 32-bit encodings) and its select reads it two instructions later, with
            // one fill and one drain per chunk.  (Through fold4 and a fence per k the
            // compiler finds the same order inside each k, but fills and drains four
            // times per chunk.)
            constexpr int NP = KA * TM * 4;
            float t4[TM][4];
#pragma unroll
            for (int r = 0; r < TM; ++r) thres4(r, 0, t4[r]);
            float p[NP + 1], sel[NP];
            p[0] = a_of(a, 0, 0) * b[0][0][0];
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const bool m = p[i] > t4[(i / 4) % TM][i % 4];
                __builtin_amdgcn_sched_barrier(0);
                if (i + 1 < NP) p[i + 1] = a_of(a, ((i + 1) / 4) % TM, (i + 1) / (4 * TM)) * b[(i + 1) / (4 * TM)][0][(i + 1) % 4];
                __builtin_amdgcn_sched_barrier(0);
                if (i > 0) part[((i - 1) / 4) % TM][(i - 1) % 4] = __builtin_fmaf(p[i - 1], sel[i - 1], part[((i - 1) / 4) % TM][(i - 1) % 4]);
                __builtin_amdgcn_sched_barrier(0);
                sel[i] = m ? q[i % 4] : 1.0f;
                __builtin_amdgcn_sched_barrier(0);
            }
            part[((NP - 1) / 4) % TM][(NP - 1) % 4] = __builtin_fmaf(p[NP - 1], sel[NP - 1], part[((NP - 1) / 4) % TM][(NP - 1) % 4]);
        } else {
            // one k at a time through fold4, rows in order
#pragma unroll
            for (int kk = 0; kk < KA; ++kk) {
#pragma unroll
                for (int r = 0; r < TM; ++r) {
#pragma unroll
                    for (int g = 0; g < NG; ++g) {
                        float t4[4];
                        thres4(r, g, t4);
                        fold4<TASK>(a_of(a, r, kk), b[kk][g], t4, &q[g * 4], &part[r][g * 4]);
                    }
                    // At most 4 rows of one k between fences: left alone, the scheduler may
                    // gather the compares of the whole chunk, and their lane masks (a scalar
                    // register pair each) overflow the scalar register file into spills.
                    // (The 8-row micro-tiles spill their A values regardless and lose more
                    // from the fence than they gain: they are left to the scheduler.  The
                    // count task has no masks but measured 3 % faster with the fence.)
                    if constexpr ((TASK == TASK_DISCOUNT || TASK == TASK_COUNT_GT) && TM == 4)
                        if (r == 3) __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };

    const float *bs_lane = &Bs[0][0][lane * 4];
    // Workgroups 256 apart in launch order tend to share a compute unit (8 XCDs x 32 CUs are
    // filled round-robin).  Their wave priority rotates with the tile step so that they take
    // turns being served first: left at equal priority the oldest wave always wins the issue
    // slots, the workgroups of a round finish one after the other and the round's tail runs
    // with too few waves to fill both slots (measured: +5 % when a launch is one or two rounds
    // of workgroups, +0-2 % at sixteen).
    const int prio_phase = block >> 8;
    for (int t = 0; t < n_tiles; ++t) {
        const int buf = t & 1;
        const int k0 = t * BK;
        switch ((t + prio_phase) & 3) {
        case 0: __builtin_amdgcn_s_setprio(0); break;
        case 1: __builtin_amdgcn_s_setprio(1); break;
        case 2: __builtin_amdgcn_s_setprio(2); break;
        default: __builtin_amdgcn_s_setprio(3); break;
        }
        if (t + 1 < n_tiles)
            load_tile((t + 1 < full_tiles) ? BK : tail);
        const float *bs = bs_lane + buf * (BK * BN);

        if constexpr (BPRE) {
          if (t < full_tiles) {
            // The B values of a chunk are read from LDS while the chunk before it computes: the
            // wave waits for LDS once per tile (its first chunk) instead of once per chunk.
            f4 bq[2][KA][NG];
#pragma unroll
            for (int kk = 0; kk < KA; ++kk)
#pragma unroll
                for (int g = 0; g < NG; ++g) bq[0][kk][g] = *(const f4 *)(bs + kk * BN + g * 256);
#pragma unroll
            for (int c = 0; c < BK / KA; ++c) {
                const int kc = c * KA;
                av_t a[TM];
#pragma unroll
                for (int r = 0; r < TM; ++r) a[r] = a_next[r];
                __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this chunk's B and A values have landed
                __builtin_amdgcn_sched_barrier(0);
                if (c + 1 < BK / KA) {
#pragma unroll
                    for (int kk = 0; kk < KA; ++kk)
#pragma unroll
                        for (int g = 0; g < NG; ++g) bq[(c + 1) & 1][kk][g] = *(const f4 *)(bs + (kc + KA + kk) * BN + g * 256);
                }
                // the next chunk's A values: inside this (full) tile, or the next tile's first chunk
                // (past the last full chunk: this one again)
                if (c + 1 < BK / KA) fetch_a(k0, kc + KA);
                else fetch_a(k0, k0 + BK + KA <= K ? BK : BK - KA);
                __builtin_amdgcn_sched_barrier(0);
                compute_chunk(a, bq[c & 1]);
            }
          }
        }
        if (!BPRE && t < full_tiles) {
#pragma unroll 1
            for (int kc = 0; kc < BK; kc += KA) {
                // B values of the whole chunk first, so that one wait covers them ...
                f4 b[KA][NG];
#pragma unroll
                for (int kk = 0; kk < KA; ++kk)
#pragma unroll
                    for (int g = 0; g < NG; ++g)
                        b[kk][g] = *(const f4 *)(bs + (kc + kk) * BN + g * 256);
                av_t a[TM];
                if constexpr (ALDS) {
                    // the wave's four rows of this chunk: one broadcast 16-byte LDS read each
#pragma unroll
                    for (int r = 0; r < TM; ++r) a[r] = *(const f4 *)&Asl[buf][wave * TM + r][kc];
                } else {
#pragma unroll
                    for (int r = 0; r < TM; ++r) a[r] = a_next[r];
                    // ... and the scalar fetch of the next chunk's A values is issued only after
                    // that wait: scalar loads return out of order, so any later LDS wait would
                    // have to drain them too.  Here they have the whole chunk's arithmetic to land.
                    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0), vmcnt and expcnt untouched
                    __builtin_amdgcn_sched_barrier(0);
                    fetch_a(k0, k0 + kc + 2 * KA <= K ? kc + KA : kc);   // past the last full chunk: re-read this one
                    __builtin_amdgcn_sched_barrier(0);
                }
                compute_chunk(a, b);
            }
        } else if (t >= full_tiles) {
            // K remainder: k by k, so no padded product is ever evaluated.
            for (int kk = 0; kk < tail; ++kk) {
                float a1[TM];
#pragma unroll
                for (int r = 0; r < TM; ++r)
                    a1[r] = ALDS ? Asl[ALDS ? buf : 0][ALDS ? wave * TM + r : 0][ALDS ? kk : 0]
                                 : transA ? As[(int64_t)(k0 + kk) * args.lda + trow(r)] : As[arow[transA ? 0 : r] + k0 + kk];
                f4 b[NG];
#pragma unroll
                for (int g = 0; g < NG; ++g)
                    b[g] = *(const f4 *)(bs + kk * BN + g * 256);
#pragma unroll
                for (int r = 0; r < TM; ++r)
#pragma unroll
                    for (int g = 0; g < NG; ++g) {
                        float t4[4];
                        thres4(r, g, t4);
                        fold4<TASK>(a1[r], b[g], t4, &q[g * 4], &part[r][g * 4]);
                    }
            }
        }

        // fold the partial sums into the main accumulators every FLUSH_K products
        if ((t + 1) % FLUSH_TILES == 0)
            flush();

        if (t + 1 < n_tiles)
            store_tile(buf ^ 1);
        __syncthreads();
    }
    flush();

    // ---- write-back: R += acc, once per tile ---------------------------------
    // The aligned 16-byte pieces of R are all read before the first sum is stored: as one
    // read-modify-write after the other the compiler must keep every store behind the load before
    // it (the pointers might alias), a chain of TM x NG round trips to memory.
    f4 old[TM][NG];
    bool fast[TM][NG];
#pragma unroll
    for (int r = 0; r < TM; ++r)
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int col = col0 + g * 256 + lane * 4;
            fast[r][g] = !ksplit && VEC && row0 + r < M && col + 3 < N;
            old[r][g] = f4{0.0f, 0.0f, 0.0f, 0.0f};
            if (fast[r][g]) old[r][g] = *(const f4 *)(args.R + (int64_t)(row0 + r) * args.ldr + col);
        }
#pragma unroll
    for (int r = 0; r < TM; ++r) {
        const int row = row0 + r;
        if (row >= M) continue;
        float *dst_row = args.R + (int64_t)row * args.ldr;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            const int col = col0 + g * 256 + lane * 4;
            float v[4];
#pragma unroll
            for (int c = 0; c < 4; ++c)
                v[c] = (TASK == TASK_COUNT_GT) ? (float)part[r][g * 4 + c] : mainacc[r][g * 4 + c];
            if (ksplit) {
                // several workgroups own this tile: hardware float adds, in whatever order
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (col + c < N) unsafeAtomicAdd(dst_row + col + c, v[c]);
            } else if (fast[r][g]) {
                f4 o = old[r][g];
                o.x += v[0]; o.y += v[1]; o.z += v[2]; o.w += v[3];
                *(f4 *)(dst_row + col) = o;
            } else if (col + 3 < N) {
                f4 o = *(f4_any *)(dst_row + col);
                o.x += v[0]; o.y += v[1]; o.z += v[2]; o.w += v[3];
                *(f4_any *)(dst_row + col) = o;
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (col + c < N) dst_row[col + c] += v[c];
            }
        }
    }
}

template <int TASK, int TF, int TM, int NG, int NW, int BK, int KA>
static hipError_t launch_one(const MmlikeArgs &a, hipStream_t s)
{
    const int64_t tiles_m = (a.M + NW * TM - 1) / (NW * TM);
    const int64_t tiles_n = (a.N + 256 * NG - 1) / (256 * NG);
    const int64_t wgs = xcd_grid(tiles_m, tiles_n);
    if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    // Tiles for at most half of the waves the chip holds at once (small M x N, e.g. an
    // aggregation over a long K): split K over as many workgroups per tile as still fit, at
    // least 64 k each; each adds its part to R with hardware float atomics (the sum order is
    // free, Sec. 4.1).  A SIMD with two waves runs a wave's work 20 % slower than one with four.
    MmlikeArgs b = a;
    int splits = 1;
    b.kchunk = a.K;
    const int64_t waves = tiles_m * tiles_n * NW;
    if (a.force_splits > 1) {
        // a k-axis point of the shape grid: every tile's K in (up to) force_splits parts of whole
        // partial-sum periods; nothing to split in the deterministic mode or when K is short
        if (k_split_allowed() && a.K >= 128) {
            int64_t want = a.force_splits;
            if (want > a.K / 64) want = a.K / 64;
            const int64_t chunk = ((a.K + want - 1) / want + 63) / 64 * 64;
            b.kchunk = (int)chunk;
            splits = (int)((a.K + chunk - 1) / chunk);
        }
    } else if (k_split_allowed() && waves <= 2048 && a.K >= 128) {
        // As many parts as fill the chip to three waves per SIMD (four when the tiles alone fill one),
        // of at least 64 k each and, from K = 512 on, of about 192: every part pays a first load of
        // B, a pipeline fill and a tile of atomic adds, and parts of one tile that finish together
        // queue on the same lines of R.  Measured over forced counts 1 ... 64, us, this rule / as many
        // parts of 64 k as fit at four waves per SIMD (the earlier rule) / best forced: 512^3 40 / 55 / 40,
        // 640^3 49 / 55 / 46, 768^3 63 / 73 / 61, 512^2 x 1024 58 / 86 / 54, 768^2 x 384 43 / 59 / 43,
        // 128 x 4096 x 512 42 / 64 / 42, 256^2 x 4096 56 / 85 / 55, 512^2 x 2048 80 / 93 / 78,
        // 1024^2 x 512 71 / 76 / 65; 256^3, 384^3, 896^3, 1024^3 unchanged (17, 24, 78, 97).
        int64_t want = (waves >= 1024 ? 4096 : 3072) / waves;
        const int64_t most = a.K < 512 ? a.K / 64 : (a.K + 96) / 192;
        if (want > most) want = most;
        if (want < 1) want = 1;
        if (want > 1024) want = 1024;
        const int64_t chunk = ((a.K + want - 1) / want + 63) / 64 * 64;   // whole partial-sum periods
        b.kchunk = (int)chunk;
        splits = (int)((a.K + chunk - 1) / chunk);
    }
    b.tail_base = 0; b.tail_blocks = 0; b.tail_splits = 1;
    // Discount task.  With 16-deep staging and A on the scalar path the kernel runs a chunk as one
    // compare / multiply / FMA / select pipeline whose B values were read from LDS a chunk ahead,
    // at every size (8192^3 31.9 -> 34.2 TFLOP/s, 4096^3 32.8 -> 33.9, 16384 x 2048 x 8192 33.1 ->
    // 34.0: the pipeline alone was no faster at 8192^3, the earlier reads alone gave +1.5 %).
    // The other discount instantiations (8-deep staging, A through LDS) keep the pipeline without
    // the earlier reads up to 4096 workgroups, where it measured 2-4 % faster, and the k-by-k form
    // above that.
    const bool pipe = TASK == TASK_DISCOUNT && TM == 4 && NG == 1 && wgs <= 4096;
    // Rows of a row-major A whose pitch collides in the memory system go through LDS; at other
    // pitches the scalar path is as fast or faster for every task (measured at 2048^3 ... 8192^3,
    // A through LDS against A through the scalar cache: discount 30.4-31.0 against 31.3-31.9
    // TFLOP/s, count 36.4-37.2 against 36.9-40.4, boost within +-4 % either way).
    const bool a_through_lds = !a.transA && !a.transB && pitch_collides(a.lda, 4);
    constexpr bool DPIPE = TASK == TASK_DISCOUNT && TM == 4 && NG == 1 && BK == 16;
    constexpr bool BAHEAD = (TASK == TASK_DISCOUNT || TASK == TASK_BOOST) && TM == 4 && NG == 1 && BK == 16;   // B values a chunk ahead
    auto launch = [&](int64_t n_blocks, int n_splits) -> hipError_t {
        return launch_row_of_blocks(b, n_blocks, 64 * NW, [&](unsigned n) {
            const dim3 grid(n, (unsigned)n_splits), block(64 * NW);
            switch ((a.transA ? 1 : 0) | (a.transB ? 2 : 0)) {
            case 0:
                if constexpr (TASK == TASK_DISCOUNT && TM == 4 && NG == 1 && BK == 16) {
                    // the chunk-wide pipeline fed with B values read a chunk ahead: at every size
                    if (!a_through_lds) {
                        hipLaunchKernelGGL((mmlike_valu_kernel<TASK, TF, 0, TM, NG, NW, BK, KA, false, true, true>), grid, block, 0, s, b);
                        break;
                    }
                }
                if constexpr (TASK == TASK_BOOST && TM == 4 && NG == 1 && BK == 16) {
                    // B values read a chunk ahead (no chunk pipeline: the boost has no lane mask
                    // to keep at a distance): +0.5-1.5 %
                    if (!a_through_lds) {
                        hipLaunchKernelGGL((mmlike_valu_kernel<TASK, TF, 0, TM, NG, NW, BK, KA, false, false, true>), grid, block, 0, s, b);
                        break;
                    }
                }
                if constexpr (TASK == TASK_DISCOUNT && TM == 4 && NG == 1) {
                    if (pipe) {
                        if (a_through_lds)
                            hipLaunchKernelGGL((mmlike_valu_kernel<TASK, TF, 0, TM, NG, NW, BK, KA, true, true>), grid, block, 0, s, b);
                        else
                            hipLaunchKernelGGL((mmlike_valu_kernel<TASK, TF, 0, TM, NG, NW, BK, KA, false, true>), grid, block, 0, s, b);
                        break;
                    }
                }
                if constexpr (TM == 4 && NG == 1) {
                    if (a_through_lds) {
                        hipLaunchKernelGGL((mmlike_valu_kernel<TASK, TF, 0, TM, NG, NW, BK, KA, true>), grid, block, 0, s, b);
                        break;
                    }
                }
                hipLaunchKernelGGL((mmlike_valu_kernel<TASK, TF, 0, TM, NG, NW, BK, KA, false>), grid, block, 0, s, b);
                break;
            // (transposed layouts: the discount task's pipelined form; with B a chunk ahead where A
            // is row-major -- with a transposed A the unrolled tile keeps the A values of all its
            // chunks in scalar registers at once and spills 80-130 of them)
            case 1: hipLaunchKernelGGL((mmlike_valu_kernel<TASK, TF, 1, TM, NG, NW, BK, KA, false, DPIPE, false>), grid, block, 0, s, b); break;
            case 2: hipLaunchKernelGGL((mmlike_valu_kernel<TASK, TF, 2, TM, NG, NW, BK, KA, false, DPIPE, BAHEAD>), grid, block, 0, s, b); break;
            default: hipLaunchKernelGGL((mmlike_valu_kernel<TASK, TF, 3, TM, NG, NW, BK, KA, false, DPIPE, false>), grid, block, 0, s, b); break;
            }
        });
    };
    // a last round of workgroups that would leave most of the chip idle: its tiles are launched
    // once per k range instead (choose_tail_split in amulet_internal.h)
    TailSplit t;
    if (splits == 1 && a.force_splits <= 1 && choose_tail_split(tiles_m * tiles_n, wgs, (int64_t)compute_units() * (16 / NW), a.K, 64, t)) {
        b.tail_base = (int)t.base;
        b.tail_blocks = (int)t.blocks;
        b.tail_splits = t.splits;
        b.kchunk = t.chunk;
        return launch(t.grid, 1);
    }
    return launch(wgs, splits);
}

// Shape id = k-axis index * VALU_TILES + tile index (see amulet_internal.h).
template <int TASK, int TF>
hipError_t launch_mmlike_valu_task(int shape, const MmlikeArgs &args, hipStream_t s)
{
    if (shape < 0 || shape >= VALU_SHAPE_COUNT) return hipErrorInvalidValue;
    MmlikeArgs a = args;
    a.force_splits = kValuShapes[shape].splits;
    const int tile = shape % VALU_TILES;
    if (kValuShapes[shape].BK == 8) {
        switch (tile) {
        case 0: return launch_one<TASK, TF, 4, 1, 4, 8, 4>(a, s);
        case 1: return launch_one<TASK, TF, 4, 1, 8, 8, 4>(a, s);
        case 2: return launch_one<TASK, TF, 8, 1, 8, 8, 4>(a, s);
        default: return launch_one<TASK, TF, 4, 2, 8, 8, 4>(a, s);
        }
    }
    switch (tile) {
    case 0: return launch_one<TASK, TF, 4, 1, 4, 16, 4>(a, s);
    case 1: return launch_one<TASK, TF, 4, 1, 8, 16, 4>(a, s);
    case 2: return launch_one<TASK, TF, 8, 1, 8, 16, 4>(a, s);
    default: return launch_one<TASK, TF, 4, 2, 8, 16, 4>(a, s);
    }
}

}  // namespace amulet
#endif
