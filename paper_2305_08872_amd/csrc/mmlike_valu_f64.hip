// The predicate tasks (discount, boost, count over threshold) in the paper's own element
// type, double (its listings declare double A[M][K], B[K][N], C[M][N]; Sec. 3,
// Sec. 4.3.3).  Same mapping as
// the fp32 vector-ALU kernels (mmlike_valu_impl.h): a lane owns columns, a wave owns TM rows
// whose A values arrive through the scalar cache into SGPR pairs, the B tile goes through
// LDS, the thresholds stay in registers, the K remainder is computed k by k.  One tile
// shape: 16 x 128 per workgroup (4 waves x 4 rows, 2 columns per lane), 16 k per barrier.
// fp64 accumulation needs no second level: K * 2^-53 stays far below the tolerance.
// (The identity task, a dense contraction, has its own matrix-core kernel: identity_mfma_f64.hip.)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "amulet_internal.h"

namespace amulet {

typedef double d2 __attribute__((ext_vector_type(2)));
// the same two doubles at any double address: still one 16-byte access (global accesses
// take any address on this target), used where rows are not 16-byte aligned
typedef d2 d2_any __attribute__((aligned(8)));
typedef d2 d2_a8 __attribute__((aligned(8)));
typedef const __attribute__((address_space(4))) double *sptr_d;     // read through the scalar cache
typedef const __attribute__((address_space(4))) d2_a8 *sptr_d2;
typedef double d4r __attribute__((ext_vector_type(4)));
typedef d4r d4_a8 __attribute__((aligned(8)));
typedef const __attribute__((address_space(4))) d4_a8 *sptr_d4;

// (the workgroup has D_NW = 4 or 8 waves, a template parameter: tile 16 x 128 or 32 x 128)
constexpr int D_TM = 4, D_BK = 16, D_BN = 128;

template <int TASK> struct AccD { typedef double type; };
template <> struct AccD<TASK_COUNT_GT> { typedef int type; };

// One k of the micro-tile: the D_TM x 2 products of the wave's A values with a lane's two B
// values, written stage by stage over all eight products so that no instruction waits on the
// one just issued.  The multiply is a separately rounded fp64 operation wherever a comparison
// depends on it (contraction is off).
template <int TASK>
__device__ __forceinline__ void fold_rows(const double (&a)[D_TM], d2 b, const double (&th)[D_TM][2],
                                          const double *q, typename AccD<TASK>::type (&acc)[D_TM][2])
{
    static_assert(TASK == TASK_DISCOUNT || TASK == TASK_BOOST || TASK == TASK_COUNT_GT, "predicate tasks only");
    if constexpr (TASK == TASK_DISCOUNT) {
        // A 64-bit select is two instructions, so the discount is applied under the execution
        // mask instead: the compare writes the mask, the lanes whose product is over the
        // threshold multiply it by q = 1 - dis[j], the mask is put back (a scalar move), and
        // every lane adds its term: 4 vector instructions per product instead of 5.
        const uint64_t active = __builtin_amdgcn_read_exec();   // the lanes running here: put back after each compare
        double p[D_TM][2];
#pragma unroll
        for (int r = 0; r < D_TM; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c) p[r][c] = a[r] * b[c];
#pragma unroll
        for (int r = 0; r < D_TM; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c)
                asm volatile("v_cmpx_gt_f64_e32 vcc, %0, %1\n\tv_mul_f64 %0, %0, %2\n\ts_mov_b64 exec, %3"
                             : "+v"(p[r][c])
                             : "v"(th[r][c]), "v"(q[c]), "s"(active)
                             : "vcc");
#pragma unroll
        for (int r = 0; r < D_TM; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c) acc[r][c] += p[r][c];
    } else if constexpr (TASK == TASK_BOOST) {
        // p + max(p - th, 0): continuous in p, so the fused product is within tolerance
        double d[D_TM][2];
#pragma unroll
        for (int r = 0; r < D_TM; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c) d[r][c] = __builtin_fma(a[r], b[c], -th[r][c]);
#pragma unroll
        for (int r = 0; r < D_TM; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c) acc[r][c] = __builtin_fma(a[r], b[c], acc[r][c]);
#pragma unroll
        for (int r = 0; r < D_TM; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c) d[r][c] = __builtin_fmax(d[r][c], 0.0);
#pragma unroll
        for (int r = 0; r < D_TM; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c) acc[r][c] += d[r][c];
    } else {
        // (the sign bit of th - p, which replaces compare and select in the fp32 kernel, measured
        // 10 % slower here: the subtraction is a second full-width fp64 operation)
        double p[D_TM][2];
#pragma unroll
        for (int r = 0; r < D_TM; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c) p[r][c] = a[r] * b[c];
#pragma unroll
        for (int r = 0; r < D_TM; ++r)
#pragma unroll
            for (int c = 0; c < 2; ++c) acc[r][c] += (int)(p[r][c] > th[r][c]);
    }
}

// TRANS (bit 0: a(i,k) at A[k*lda + i], bit 1: b(k,j) at B[j*ldb + k]) is a compile-time choice:
// each layout's addressing state would otherwise cost the others scalar registers in the hot loop.
// ALDS: the workgroup's rows of A go through LDS (vector loads a whole tile ahead, broadcast
// reads) instead of through the scalar cache; used when the row pitch of A collides in the memory
// system (as in the fp32 kernels, where the reason is given).
template <int TASK, int TF, int TRANS, bool ALDS, int D_NW>
__global__ void __launch_bounds__(64 * D_NW)
mmlike_valu_f64_kernel(const MmlikeArgsF64 args)
{
    static_assert(!ALDS || TRANS == 0, "A through LDS: row-major operands");
    static_assert(D_NW == 4 || D_NW == 8, "4 or 8 waves");
    constexpr int D_NT = 64 * D_NW;
    typedef typename AccD<TASK>::type acc_t;
    constexpr int D2_PER_ROW = D_BN / 2;                     // 16-byte slots in one LDS row
    constexpr int ROWS_PER_PASS = D_NT / D2_PER_ROW;         // 4 or 8
    constexpr int LOADS = D_BK / ROWS_PER_PASS;              // 4 or 2 slots staged per thread per tile
    constexpr int KA = 2;                                    // A is fetched two k at a time (one 16-byte scalar load per row)

    __shared__ __attribute__((aligned(16))) double Bs[2][D_BK][D_BN];
    constexpr int A_ROWS = D_NW * D_TM, A_PITCH = D_BK + 2;   // rows of the workgroup; padded row of the LDS A tile
    constexpr int A_D2 = A_ROWS * D_BK / 2;                   // 16-byte slots of one A tile
    static_assert(A_D2 <= D_NT, "one staging slot per thread at most");
    __shared__ __attribute__((aligned(16))) double Asl[ALDS ? 2 : 1][ALDS ? A_ROWS : 1][ALDS ? A_PITCH : 2];

    const int M = args.M, N = args.N;
    int K = args.K;
    const bool VEC = args.vec != 0;   // B and R rows are 16-byte aligned
    constexpr bool transA = (TRANS & 1) != 0, transB = (TRANS & 2) != 0;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // XCD-aware tile order, as in the fp32 kernels
    const int tiles_m = (M + D_NW * D_TM - 1) / (D_NW * D_TM);
    const int tiles_n = (N + D_BN - 1) / D_BN;
    int tm, tn;
    // place in the tile order, and which k range of it (tail split, see choose_tail_split)
    int block = (int)blockIdx.x + args.block_base, ksplit_idx = (int)blockIdx.y;
    const bool tail_part = args.tail_splits > 1 && block >= args.tail_base;
    if (tail_part) {
        const int rel = block - args.tail_base;
        block = args.tail_base + rel % args.tail_blocks;
        ksplit_idx = rel / args.tail_blocks;
    }
    if (!xcd_tile(block, tiles_m, tiles_n, tm, tn)) return;   // padding: the whole workgroup leaves
    const int row0 = tm * (D_NW * D_TM) + wave * D_TM;
    const int col0 = tn * D_BN;

    // Split K (gridDim.y > 1; chosen by the host for problems with too few tiles to fill the
    // chip): this workgroup sums k in [kb, kb + kchunk) only and adds its part to R atomically.
    const bool ksplit = gridDim.y > 1 || tail_part;
    sptr_d As = (sptr_d)args.A;
    const double *Bg = args.B;
    if (ksplit) {
        const int kb = ksplit_idx * args.kchunk;
        As += transA ? (int64_t)kb * args.lda : (int64_t)kb;
        Bg += transB ? (int64_t)kb : (int64_t)kb * args.ldb;
        K = (K - kb < args.kchunk) ? K - kb : args.kchunk;
    }
    auto rowc = [&](int r) { const int row = row0 + r; return row < M ? row : M - 1; };
    // a(i,k) lives at arow[r] + k * kstride (elements)
    int64_t arow[D_TM];
#pragma unroll
    for (int r = 0; r < D_TM; ++r) arow[r] = transA ? (int64_t)rowc(r) : (int64_t)rowc(r) * args.lda;
    const bool rows_full = row0 + D_TM <= M;   // the wave's 4 rows exist: contiguous in a transposed A

    // parameters in registers for the whole K loop (threshold in the operand form TF)
    double q[2];
    double th_col[TF == THRES_COL ? 2 : 1];
    double th_row[TF == THRES_ROW ? D_TM : 1];
    double th_el[TF == THRES_ELEM ? D_TM : 1][TF == THRES_ELEM ? 2 : 1];
    double th_const = __builtin_inf();
    {
        if constexpr (TF == THRES_CONST) th_const = ((sptr_d)args.thres)[0];
        if constexpr (TF == THRES_ROW) {
#pragma unroll
            for (int r = 0; r < D_TM; ++r) th_row[r] = ((sptr_d)args.thres)[rowc(r)];
        }
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int col = col0 + lane * 2 + c;
        q[c] = 1.0;
        if constexpr (TF == THRES_COL) th_col[c] = __builtin_inf();
        if (col < N) {
            if constexpr (TF == THRES_COL) th_col[c] = args.thres[col];
            if (TASK == TASK_DISCOUNT) q[c] = 1.0 - args.dis[col];
        }
        if constexpr (TF == THRES_ELEM) {
#pragma unroll
            for (int r = 0; r < D_TM; ++r)
                th_el[r][c] = (col < N) ? args.thres[(int64_t)rowc(r) * args.ldt + col] : __builtin_inf();
        }
    }
    // the micro-tile's thresholds as one table (copies of the same registers: the forms differ
    // only in which registers repeat)
    double th[D_TM][2];
#pragma unroll
    for (int r = 0; r < D_TM; ++r)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            if constexpr (TF == THRES_COL) th[r][c] = th_col[c];
            else if constexpr (TF == THRES_ROW) th[r][c] = th_row[r];
            else if constexpr (TF == THRES_CONST) th[r][c] = th_const;
            else th[r][c] = th_el[r][c];
        }

    acc_t acc[D_TM][2];
#pragma unroll
    for (int r = 0; r < D_TM; ++r)
#pragma unroll
        for (int c = 0; c < 2; ++c) acc[r][c] = 0;

    // ---- B tile staging: global -> registers -> LDS ---------------------------------------
    const int srow = threadIdx.x / D2_PER_ROW;
    const int scol = col0 + (threadIdx.x % D2_PER_ROW) * 2;
    const bool fast_cols = VEC && (col0 + D_BN <= N);
    const double *bsrc = Bg + (int64_t)srow * args.ldb + scol;
    const int64_t pass_stride = (int64_t)ROWS_PER_PASS * args.ldb;
    const int64_t tile_stride = (int64_t)D_BK * args.ldb;
    d2 stage[LOADS];
    // B stored transposed: a thread owns one column of the tile and 2 LOADS (8 or 4) consecutive
    // k of it, read as 16-byte pieces along k and scattered into the same [k][n] LDS tile
    // (neighbouring lanes hit neighbouring banks).
    static_assert((D_NT / D_BN) * 2 * LOADS == D_BK, "transposed-B slot mapping");
    const int tcol = threadIdx.x % D_BN;
    const int tk = (threadIdx.x / D_BN) * 2 * LOADS;
    const double *btsrc = Bg + (int64_t)(col0 + tcol < N ? col0 + tcol : N - 1) * args.ldb + tk;
    // A tile staging (ALDS): thread t < A_D2 stages slot (row t / (D_BK / 2), k pair t % (D_BK / 2))
    const int a_sr = threadIdx.x / (D_BK / 2), a_sq = (threadIdx.x % (D_BK / 2)) * 2;
    const double *asrc = nullptr;
    d2 a_stage = {0.0, 0.0};
    if constexpr (ALDS) {
        const int wg_row0 = tm * A_ROWS;
        const int arow_c = wg_row0 + a_sr < M ? wg_row0 + a_sr : M - 1;   // rows past M are never written back
        asrc = args.A + (ksplit ? (int64_t)ksplit_idx * args.kchunk : 0) + (int64_t)arow_c * args.lda + a_sq;
    }
    auto load_tile = [&](int krows) {
        if constexpr (ALDS) {
            if (threadIdx.x < A_D2) {
                if (krows == D_BK) {
                    a_stage = *(const d2_any *)asrc;
                } else {
                    a_stage = d2{0.0, 0.0};
                    if (a_sq + 0 < krows) a_stage.x = asrc[0];
                    if (a_sq + 1 < krows) a_stage.y = asrc[1];
                }
                asrc += D_BK;
            }
        }
        if (transB) {
            const bool colok = col0 + tcol < N;
#pragma unroll
            for (int it = 0; it < LOADS; ++it) {
                d2 v = {0.0, 0.0};
                const int kk = tk + 2 * it;
                if (colok) {
                    const double *src = btsrc + 2 * it;
                    if (kk + 1 < krows) {
                        v = *(const d2_any *)src;
                    } else {
                        if (kk + 0 < krows) v.x = src[0];
                        if (kk + 1 < krows) v.y = src[1];
                    }
                }
                stage[it] = v;
            }
            btsrc += D_BK;
        } else if (fast_cols && krows == D_BK) {
#pragma unroll
            for (int it = 0; it < LOADS; ++it) stage[it] = *(const d2 *)(bsrc + it * pass_stride);
        } else {
#pragma unroll
            for (int it = 0; it < LOADS; ++it) {
                d2 v = {0.0, 0.0};
                if (srow + it * ROWS_PER_PASS < krows) {
                    const double *src = bsrc + it * pass_stride;
                    if (scol + 1 < N) v = *(const d2_any *)src;
                    else if (scol < N) v.x = src[0];
                }
                stage[it] = v;
            }
        }
        bsrc += tile_stride;
    };
    double *const bdst = &Bs[0][srow][(threadIdx.x % D2_PER_ROW) * 2];
    double *const btdst = &Bs[0][tk][tcol];
    auto store_tile = [&](int buf) {
        if constexpr (ALDS) {
            if (threadIdx.x < A_D2) *(d2 *)&Asl[buf][a_sr][a_sq] = a_stage;
        }
        if (transB) {
#pragma unroll
            for (int it = 0; it < LOADS; ++it)
#pragma unroll
                for (int e = 0; e < 2; ++e) btdst[(buf * D_BK + 2 * it + e) * D_BN] = stage[it][e];
        } else {
#pragma unroll
            for (int it = 0; it < LOADS; ++it)
                *(d2 *)(bdst + (buf * D_BK + it * ROWS_PER_PASS) * D_BN) = stage[it];
        }
    };

    const int full_tiles = K / D_BK;
    const int tail = K - full_tiles * D_BK;
    const int n_tiles = full_tiles + (tail ? 1 : 0);

    // A values of the chunk of KA k starting at kn, for the wave's D_TM rows, into SGPR pairs
    // (row-major A: a_next[r] holds row r's KA values; transposed A: a_next_t[kk] holds the four
    // rows of k = kn + kk, exactly as loaded: re-sorting them at fetch time would make every fetch
    // wait for its own loads instead of letting them land during the chunk's arithmetic)
    d2_a8 a_next[transA ? 1 : D_TM];
    d4_a8 a_next_t[transA ? KA : 1];
    // (the chunk at k = kt + rel, kt a tile's first k: a row-major A costs one address per row and
    // tile, and the chunk is a 32-bit scalar offset of the load -- kept opaque to the compiler, which
    // would otherwise merge a tile's loads into one per row, issued and waited for at the tile's start)
    auto fetch_a = [&](int kt, int rel) {
        const int kn = kt + rel;
        if constexpr (!transA) {
            uint32_t relb = (uint32_t)rel * 8u;
            asm volatile("" : "+s"(relb));
            typedef const __attribute__((address_space(4))) char *sptr_c;
#pragma unroll
            for (int r = 0; r < D_TM; ++r) a_next[r] = *(sptr_d2)((sptr_c)(As + (arow[r] + kt)) + relb);
        } else if (rows_full) {
            // the 4 rows of one k are contiguous in the transposed storage
#pragma unroll
            for (int kk = 0; kk < KA; ++kk)
                a_next_t[kk] = *(sptr_d4)(As + (int64_t)(kn + kk) * args.lda + arow[0]);
        } else {
#pragma unroll
            for (int kk = 0; kk < KA; ++kk)
#pragma unroll
                for (int r = 0; r < D_TM; ++r) a_next_t[kk][r] = As[(int64_t)(kn + kk) * args.lda + arow[r]];
        }
    };
    load_tile(full_tiles > 0 ? D_BK : tail);
    store_tile(0);
    if (!ALDS && full_tiles > 0) fetch_a(0, 0);
    __syncthreads();

    const double *bs_lane = &Bs[0][0][lane * 2];
    // Wave priority rotates with the tile step, offset by the workgroup's place among those that
    // tend to share a compute unit (256 apart in launch order), so that co-resident workgroups
    // take turns being served first, as in the fp32 kernel (where the reason is given).  Measured
    // with / without: discount 2048^3 16.3 / 15.9 TFLOP/s, 1536^2 x 4096 16.8 / 16.2, 4096^3 16.5 /
    // 16.4; boost 2048^3 16.5 / 16.3; the count task 22.3 / 22.5, so it is left out there.
    const int prio_phase = block >> 8;
    for (int t = 0; t < n_tiles; ++t) {
        const int buf = t & 1;
        const int k0 = t * D_BK;
        if constexpr (TASK != TASK_COUNT_GT) {
            switch ((t + prio_phase) & 3) {
            case 0: __builtin_amdgcn_s_setprio(0); break;
            case 1: __builtin_amdgcn_s_setprio(1); break;
            case 2: __builtin_amdgcn_s_setprio(2); break;
            default: __builtin_amdgcn_s_setprio(3); break;
            }
        }
        if (t + 1 < n_tiles) load_tile((t + 1 < full_tiles) ? D_BK : tail);
        const double *bs = bs_lane + buf * (D_BK * D_BN);

        if (ALDS && t < full_tiles) {
            // The B values (and, through LDS, the A values) of a chunk are read while the chunk
            // before it computes: a chunk is only 16 products per lane here, so a wait for LDS at
            // the start of every chunk left the wave idle for a good part of it.  Now the wave
            // waits for LDS once per tile, for its first chunk.  (A through LDS only: unrolled over
            // the tile's chunks, the scalar-path variants spill scalar registers.)
            constexpr int NCH = D_BK / KA;
            d2 bq[2][KA];
            d2_a8 aq[2][ALDS ? D_TM : 1];
            auto read_chunk = [&](int c, int slot) {
#pragma unroll
                for (int kk = 0; kk < KA; ++kk) bq[slot][kk] = *(const d2 *)(bs + (c * KA + kk) * D_BN);
                if constexpr (ALDS) {
                    // the wave's four rows of the chunk: one broadcast 16-byte LDS read each
#pragma unroll
                    for (int r = 0; r < D_TM; ++r) aq[slot][r] = *(const d2 *)&Asl[buf][wave * D_TM + r][c * KA];
                }
            };
            read_chunk(0, 0);
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int kc = c * KA;
                d2_a8 a[transA ? 1 : D_TM];
                d4_a8 a_t[transA ? KA : 1];
                if constexpr (!ALDS) {
                    if constexpr (!transA) {
#pragma unroll
                        for (int r = 0; r < D_TM; ++r) a[r] = a_next[r];
                    } else {
#pragma unroll
                        for (int kk = 0; kk < KA; ++kk) a_t[kk] = a_next_t[kk];
                    }
                }
                // this chunk's values have landed; the reads of the next chunk and the scalar fetch
                // of its A values go out right after the wait (scalar loads return out of order:
                // any later LDS wait would drain them too)
                __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
                __builtin_amdgcn_sched_barrier(0);
                if (c + 1 < NCH) read_chunk(c + 1, (c + 1) & 1);
                if constexpr (!ALDS) fetch_a(k0, k0 + kc + 2 * KA <= K ? kc + KA : kc);   // past the last full chunk: this one again
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kk = 0; kk < KA; ++kk) {
                    double ak[D_TM];
#pragma unroll
                    for (int r = 0; r < D_TM; ++r)
                        ak[r] = ALDS ? aq[c & 1][ALDS ? r : 0][kk] : transA ? a_t[transA ? kk : 0][r] : a[transA ? 0 : r][kk];
                    fold_rows<TASK>(ak, bq[c & 1][kk], th, q, acc);
                }
            }
        } else if (!ALDS && t < full_tiles) {
            // A on the scalar path.  The B values of a chunk are read from LDS while the chunk before
            // it computes (two chunks per turn of the rolled loop, so that the two sets of B registers
            // need no copies): the wave waits for LDS with work queued, except for a tile's first chunk.
            d2 b0[KA], b1[KA];
#pragma unroll
            for (int kk = 0; kk < KA; ++kk) b0[kk] = *(const d2 *)(bs + kk * D_BN);
            auto chunk = [&](int kc, const d2 (&b)[KA], d2 (&bn)[KA], bool read_next) {
                d2_a8 a[transA ? 1 : D_TM];
                d4_a8 a_t[transA ? KA : 1];
                if constexpr (!transA) {
#pragma unroll
                    for (int r = 0; r < D_TM; ++r) a[r] = a_next[r];
                } else {
#pragma unroll
                    for (int kk = 0; kk < KA; ++kk) a_t[kk] = a_next_t[kk];
                }
                // this chunk's values have landed; the LDS reads of the next chunk and the scalar
                // fetch of its A values go out right after the wait (scalar loads return out of
                // order: any later LDS wait would drain them too)
                __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
                __builtin_amdgcn_sched_barrier(0);
                if (read_next) {
#pragma unroll
                    for (int kk = 0; kk < KA; ++kk) bn[kk] = *(const d2 *)(bs + (kc + KA + kk) * D_BN);
                }
                fetch_a(k0, k0 + kc + 2 * KA <= K ? kc + KA : kc);   // past the last full chunk: this one again
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int kk = 0; kk < KA; ++kk) {
                    double ak[D_TM];
#pragma unroll
                    for (int r = 0; r < D_TM; ++r) ak[r] = transA ? a_t[transA ? kk : 0][r] : a[transA ? 0 : r][kk];
                    fold_rows<TASK>(ak, b[kk], th, q, acc);
                }
            };
            static_assert((D_BK / KA) % 2 == 0, "the chunks of a tile are taken in pairs");
#pragma unroll 1
            for (int kc = 0; kc < D_BK; kc += 2 * KA) {
                chunk(kc, b0, b1, true);
                chunk(kc + KA, b1, b0, kc + 2 * KA < D_BK);
            }
        } else if (t < full_tiles) {
#pragma unroll 1
            for (int kc = 0; kc < D_BK; kc += KA) {
                d2 b[KA];
#pragma unroll
                for (int kk = 0; kk < KA; ++kk) b[kk] = *(const d2 *)(bs + (kc + kk) * D_BN);
                d2_a8 a[transA ? 1 : D_TM];
                d4_a8 a_t[transA ? KA : 1];
                if constexpr (ALDS) {
                    // the wave's four rows of this chunk: one broadcast 16-byte LDS read each
#pragma unroll
                    for (int r = 0; r < D_TM; ++r) a[r] = *(const d2 *)&Asl[buf][wave * D_TM + r][kc];
                } else {
                    if constexpr (!transA) {
#pragma unroll
                        for (int r = 0; r < D_TM; ++r) a[r] = a_next[r];
                    } else {
#pragma unroll
                        for (int kk = 0; kk < KA; ++kk) a_t[kk] = a_next_t[kk];
                    }
                    // the scalar fetch of the next chunk goes out right after the LDS wait (scalar
                    // loads return out of order: any later LDS wait would drain them too)
                    __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
                    __builtin_amdgcn_sched_barrier(0);
                    fetch_a(k0, k0 + kc + 2 * KA <= K ? kc + KA : kc);   // past the last full chunk: this one again
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int kk = 0; kk < KA; ++kk) {
                    double ak[D_TM];
#pragma unroll
                    for (int r = 0; r < D_TM; ++r) ak[r] = transA ? a_t[transA ? kk : 0][r] : a[transA ? 0 : r][kk];
                    fold_rows<TASK>(ak, b[kk], th, q, acc);
                }
            }
        } else {
            // K remainder: k by k, never zero-padded (g(0) is not 0 in general)
            for (int kk = 0; kk < tail; ++kk) {
                const d2 b = *(const d2 *)(bs + kk * D_BN);
                double ak[D_TM];
#pragma unroll
                for (int r = 0; r < D_TM; ++r)
                    ak[r] = ALDS ? Asl[ALDS ? buf : 0][ALDS ? wave * D_TM + r : 0][ALDS ? kk : 0]
                                 : transA ? As[(int64_t)(k0 + kk) * args.lda + arow[r]] : As[arow[r] + k0 + kk];
                fold_rows<TASK>(ak, b, th, q, acc);
            }
        }
        if (t + 1 < n_tiles) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- write-back: R += acc ------------------------------------------------------------
    // The aligned 16-byte pieces of R are all read before the first sum is stored (one
    // read-modify-write after the other is a chain of round trips to memory: the compiler must
    // keep every store behind the load before it).
    d2 old[D_TM];
    bool fast[D_TM];
#pragma unroll
    for (int r = 0; r < D_TM; ++r) {
        const int col = col0 + lane * 2;
        fast[r] = !ksplit && VEC && row0 + r < M && col + 1 < N;
        old[r] = d2{0.0, 0.0};
        if (fast[r]) old[r] = *(const d2 *)(args.R + (int64_t)(row0 + r) * args.ldr + col);
    }
#pragma unroll
    for (int r = 0; r < D_TM; ++r) {
        const int row = row0 + r;
        if (row >= M) continue;
        double *dst_row = args.R + (int64_t)row * args.ldr;
        const int col = col0 + lane * 2;
        const double v0 = (double)acc[r][0], v1 = (double)acc[r][1];
        if (ksplit) {
            // several workgroups own this tile: hardware fp64 adds, in whatever order
            if (col + 0 < N) unsafeAtomicAdd(dst_row + col + 0, v0);
            if (col + 1 < N) unsafeAtomicAdd(dst_row + col + 1, v1);
        } else if (fast[r]) {
            d2 o = old[r];
            o.x += v0; o.y += v1;
            *(d2 *)(dst_row + col) = o;
        } else if (col + 1 < N) {
            d2 o = *(d2_any *)(dst_row + col);
            o.x += v0; o.y += v1;
            *(d2_any *)(dst_row + col) = o;
        } else if (col < N) {
            dst_row[col] += v0;
        }
    }
}

template <int TASK, int TRANS, bool ALDS, int D_NW>
static hipError_t launch_f64_form(int form, const MmlikeArgsF64 &args, dim3 whole, hipStream_t s)
{
    constexpr int D_NT = 64 * D_NW;
    MmlikeArgsF64 a = args;
    return launch_row_of_blocks(a, whole.x, D_NT, [&](unsigned n) {
        const dim3 grid(n, whole.y);
        switch (form) {
        case THRES_COL: hipLaunchKernelGGL((mmlike_valu_f64_kernel<TASK, THRES_COL, TRANS, ALDS, D_NW>), grid, dim3(D_NT), 0, s, a); break;
        case THRES_ROW: hipLaunchKernelGGL((mmlike_valu_f64_kernel<TASK, THRES_ROW, TRANS, ALDS, D_NW>), grid, dim3(D_NT), 0, s, a); break;
        case THRES_CONST: hipLaunchKernelGGL((mmlike_valu_f64_kernel<TASK, THRES_CONST, TRANS, ALDS, D_NW>), grid, dim3(D_NT), 0, s, a); break;
        default: hipLaunchKernelGGL((mmlike_valu_f64_kernel<TASK, THRES_ELEM, TRANS, ALDS, D_NW>), grid, dim3(D_NT), 0, s, a); break;
        }
    });
}

template <int TASK, int D_NW>
static hipError_t launch_f64_layout(int trans, int form, const MmlikeArgsF64 &a, dim3 grid, hipStream_t s)
{
    switch (trans) {
    case 0: {
        // Rows of a row-major A go through LDS when their pitch collides in the memory system, and
        // in fp64 nearly always otherwise too: measured at 1024^3 ... 4096^3, A through LDS against
        // A through the scalar cache: count 17.6-22.2 against 14.7-19.4 TFLOP/s, discount 14.8-15.9
        // against 11.8-13.0; boost 14.0 / 15.6 against 12.7 / 14.9 at 1024^3 / 2048^3 but 15.8
        // against 16.1 at 4096^3, so large boost problems keep the scalar path.
        const bool lds = pitch_collides(a.lda, 8) || TASK != TASK_BOOST || (int64_t)a.M * a.N <= 2048LL * 2048LL;
        return lds ? launch_f64_form<TASK, 0, true, D_NW>(form, a, grid, s) : launch_f64_form<TASK, 0, false, D_NW>(form, a, grid, s);
    }
    case 1: return launch_f64_form<TASK, 1, false, D_NW>(form, a, grid, s);
    case 2: return launch_f64_form<TASK, 2, false, D_NW>(form, a, grid, s);
    default: return launch_f64_form<TASK, 3, false, D_NW>(form, a, grid, s);
    }
}

// force_splits > 1: every tile's K in that many parts (a k-axis point of the shape grid)
template <int D_NW>
static hipError_t launch_mmlike_f64_waves(int task, int form, int force_splits, const MmlikeArgsF64 &a, hipStream_t s)
{
    const int64_t tiles_m = (a.M + D_NW * D_TM - 1) / (D_NW * D_TM);
    const int64_t tiles_n = (a.N + D_BN - 1) / D_BN;
    const int64_t wgs = xcd_grid(tiles_m, tiles_n);
    if (wgs > 0x7fffffffLL) return hipErrorInvalidValue;
    // tiles for at most half of the waves the chip holds at once (4 per SIMD): split K over
    // as many workgroups per tile as still fit (at least 64 k each), which add their parts
    // to R with hardware fp64 atomics
    MmlikeArgsF64 b = a;
    int splits = 1;
    b.kchunk = a.K;
    const int64_t waves = tiles_m * tiles_n * D_NW;
    const bool forced = force_splits > 1 && k_split_allowed() && a.K >= 128;
    if (forced || (k_split_allowed() && waves <= 2048 && a.K >= 128)) {
        int64_t want = forced ? force_splits : 4096 / waves;
        if (want > a.K / 64) want = a.K / 64;
        if (want > 1024) want = 1024;
        const int64_t chunk = ((a.K + want - 1) / want + D_BK - 1) / D_BK * D_BK;
        b.kchunk = (int)chunk;
        splits = (int)((a.K + chunk - 1) / chunk);
    }
    b.tail_base = 0; b.tail_blocks = 0; b.tail_splits = 1;
    dim3 grid((unsigned)wgs, (unsigned)splits);
    // a last round of workgroups that would leave most of the chip idle: its tiles are launched
    // once per k range instead (choose_tail_split in amulet_internal.h)
    TailSplit t;
    if (splits == 1 && !forced && choose_tail_split(tiles_m * tiles_n, wgs, (int64_t)compute_units() * (16 / D_NW), a.K, D_BK, t)) {
        b.tail_base = (int)t.base;
        b.tail_blocks = (int)t.blocks;
        b.tail_splits = t.splits;
        b.kchunk = t.chunk;
        grid = dim3((unsigned)t.grid, 1u);
    }
    const int trans = (a.transA ? 1 : 0) | (a.transB ? 2 : 0);
    switch (task) {
    case TASK_DISCOUNT: return launch_f64_layout<TASK_DISCOUNT, D_NW>(trans, form, b, grid, s);
    case TASK_BOOST: return launch_f64_layout<TASK_BOOST, D_NW>(trans, form, b, grid, s);
    case TASK_COUNT_GT: return launch_f64_layout<TASK_COUNT_GT, D_NW>(trans, form, b, grid, s);
    default: return hipErrorInvalidValue;
    }
}

// shape = k-axis index * F64_TILES + tile; tile 0: 16 x 128 (4 waves), tile 1: 32 x 128 (8 waves);
// k axis 0: K split only where the launcher's own rule asks for it, 1, 2: every tile's K in 2, 4
// parts.  The identity task, a dense contraction, runs on the matrix cores whatever the shape, and
// only the shape's tile index means something to it: 0 = 64 x 64 tiles, 1 = 128 x 128.
hipError_t launch_mmlike_f64(int task, int form, int shape, const MmlikeArgsF64 &a, hipStream_t s)
{
    if (shape < 0 || shape >= F64_SHAPE_COUNT) return hipErrorInvalidValue;
    if (task == TASK_IDENTITY) return launch_identity_mfma_f64(a, shape % F64_TILES == 0 ? 64 : 128, s);
    const int force = shape / F64_TILES == 0 ? 0 : 1 << (shape / F64_TILES);
    return shape % F64_TILES == 1 ? launch_mmlike_f64_waves<8>(task, form, force, a, s)
                                  : launch_mmlike_f64_waves<4>(task, form, force, a, s);
}

}  // namespace amulet
