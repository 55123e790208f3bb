// Identity task (g = p, plain matmul; paper Sec. 6.1) in the paper's own element type,
// on the fp64 matrix cores: v_mfma_f64_16x16x4_f64.
//
// Workgroup: 512 threads = 8 waves in a 4 x 2 grid, R tile 128 x 128, each wave a 32 x 64
// sub-tile = 2 x 4 MFMA blocks of 16 x 16 (64 accumulator registers).  K is staged 16 at a
// time: A tile 128 x 16 (k contiguous, row pitch 18 doubles) and B tile 16 x 128 (as in
// global memory, row pitch 132 doubles), global -> registers -> LDS, double buffered, one
// barrier per stage.  The pitches put the 16 rows a quarter-wave reads, and the k rows the
// four quarter-waves read, in different banks.
//
// Fragment mapping (measured in-bounds on the device): lane l supplies row i = l % 16 (A) or
// column j = l % 16 (B) and k-slot h = l / 16; the result block holds, in element v of lane
// l, R[4 v + l / 16][l % 16].  The hardware multiplies A's slot h with B's slot h, so which
// k a slot carries is free as long as both operands agree: slot h of MFMA t carries
// k = 4 h + t, and a lane reads its four A values of a stage as two 16-byte LDS reads.
//
// Transposed operands (template parameters TA, TB; paper Sec. 6.3), as in the fp32 kernel: an
// operand keeps its global layout in LDS, k-minor (128 x 16, k contiguous: row-major A,
// transposed B; a lane's four values of a stage are two 16-byte reads) or k-major (16 x 128:
// row-major B, transposed A; one 8-byte read per MFMA step).
//
// Rows/columns beyond M/N and the K remainder are zero-filled in LDS: for the identity task
// a zero product adds nothing (NOT true of the predicate tasks, which never take this path).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "amulet_internal.h"

namespace amulet {

typedef double d2 __attribute__((ext_vector_type(2)));
typedef d2 d2_any __attribute__((aligned(8)));   // two doubles at any double address
typedef double d4 __attribute__((ext_vector_type(4)));

constexpr int DI_BM = 128, DI_BN = 128, DI_BK = 16, DI_NT = 512;
constexpr int DI_APITCH = DI_BK + 2;    // doubles
constexpr int DI_BPITCH = DI_BN + 4;    // doubles
constexpr int DI_KMINOR_DOUBLES = DI_BM * DI_APITCH;   // one k-minor tile: 128 x 18
constexpr int DI_KMAJOR_DOUBLES = DI_BK * DI_BPITCH;   // one k-major tile: 16 x 132

template <bool TA, bool TB>
struct DiLayout {
    static constexpr int A_TILE = TA ? DI_KMAJOR_DOUBLES : DI_KMINOR_DOUBLES;
    static constexpr int B_TILE = TB ? DI_KMINOR_DOUBLES : DI_KMAJOR_DOUBLES;
    static constexpr int LDS_BYTES = 2 * (A_TILE + B_TILE) * 8;   // 66-72 KB: two workgroups per compute unit
};

template <bool TA, bool TB>
__global__ void __launch_bounds__(DI_NT) __attribute__((amdgpu_waves_per_eu(4, 4)))
identity_mfma_f64_kernel(const MmlikeArgsF64 args)
{
    constexpr int A_TILE = DiLayout<TA, TB>::A_TILE, B_TILE = DiLayout<TA, TB>::B_TILE;
    extern __shared__ __attribute__((aligned(16))) double di_smem[];
    double *const As = di_smem;                  // [2][A_TILE]
    double *const Bs = di_smem + 2 * A_TILE;     // [2][B_TILE]

    const int M = args.M, N = args.N;
    int K = args.K;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int li = lane & 15, lh = lane >> 4;

    // XCD-aware tile order (xcd_tile in amulet_internal.h)
    const int tiles_m = (M + DI_BM - 1) / DI_BM;
    const int tiles_n = (N + DI_BN - 1) / DI_BN;
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
    const int row0 = tm * DI_BM, col0 = tn * DI_BN;
    // 16-byte loads allowed along the operand's contiguous axis
    const bool vecA = args.vecA != 0, vecB = TB ? args.vecBt != 0 : args.vec != 0;

    // Split K (gridDim.y > 1, chosen by the host when the tiles are too few to fill the chip):
    // this workgroup multiplies k in [kb, kb + kchunk) only and adds its part to R atomically.
    const bool ksplit = gridDim.y > 1 || tail_part;
    const double *Ag = args.A, *Bg = args.B;
    if (ksplit) {
        const int kb = ksplit_idx * args.kchunk;
        Ag += TA ? (int64_t)kb * args.lda : (int64_t)kb;
        Bg += TB ? (int64_t)kb : (int64_t)kb * args.ldb;
        K = (K - kb < args.kchunk) ? K - kb : args.kchunk;
    }

    // staging slots of 16 bytes, u = tid + 512 * it:
    //   k-minor tile, 128 lines x 8 slots: line = u / 8, k pair = u % 8
    //   k-major tile,  16 k x 64 slots:    k = u / 64, line pair = u % 64
    d2 sa[2], sb[2];
    auto load_stage = [&](int k0) {
        auto load_kminor = [&](const double *base, int64_t ld, int line0, int n_lines, bool vec, d2 (&dst)[2]) {
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int u = tid + DI_NT * it;
                const int r = line0 + (u >> 3);
                const int k = k0 + (u & 7) * 2;
                d2 v = {0.0, 0.0};
                if (r < n_lines) {
                    const double *src = base + (int64_t)r * ld + k;
                    if (k + 1 < K) {
                        v = *(const d2_any *)src;   // one 16-byte load at any double address
                    } else {
                        if (k + 0 < K) v.x = src[0];
                        if (k + 1 < K) v.y = src[1];
                    }
                }
                dst[it] = v;
            }
        };
        auto load_kmajor = [&](const double *base, int64_t ld, int line0, int n_lines, bool vec, d2 (&dst)[2]) {
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int u = tid + DI_NT * it;
                const int k = k0 + (u >> 6);
                const int c = line0 + (u & 63) * 2;
                d2 v = {0.0, 0.0};
                if (k < K) {
                    const double *src = base + (int64_t)k * ld + c;
                    if (c + 1 < n_lines) {
                        v = *(const d2_any *)src;
                    } else {
                        if (c + 0 < n_lines) v.x = src[0];
                        if (c + 1 < n_lines) v.y = src[1];
                    }
                }
                dst[it] = v;
            }
        };
        if constexpr (TA) load_kmajor(Ag, args.lda, row0, M, vecA, sa);
        else load_kminor(Ag, args.lda, row0, M, vecA, sa);
        if constexpr (TB) load_kminor(Bg, args.ldb, col0, N, vecB, sb);
        else load_kmajor(Bg, args.ldb, col0, N, vecB, sb);
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int u = tid + DI_NT * it;
            const int kminor = (u >> 3) * DI_APITCH + (u & 7) * 2;
            const int kmajor = (u >> 6) * DI_BPITCH + (u & 63) * 2;
            *(d2 *)(As + buf * A_TILE + (TA ? kmajor : kminor)) = sa[it];
            *(d2 *)(Bs + buf * B_TILE + (TB ? kminor : kmajor)) = sb[it];
        }
    };

    d4 acc[2][4];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[mi][ni][v] = 0.0;

    const int n_stages = (K + DI_BK - 1) / DI_BK;
    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int s = 0; s < n_stages; ++s) {
        const int buf = s & 1;
        if (s + 1 < n_stages) load_stage((s + 1) * DI_BK);
        const double *at = As + buf * A_TILE, *bt = Bs + buf * B_TILE;
        const int arow = wr * 32 + li, bcol = wc * 64 + li;   // + 16 per further block
        // k-minor operands: the lane's values of the stage, k = 4 lh .. 4 lh + 3 of its line
        double a4[2][4], b4[4][4];
        if constexpr (!TA) {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const double *p = at + (arow + mi * 16) * DI_APITCH + 4 * lh;
                const d2 lo = *(const d2 *)p, hi = *(const d2 *)(p + 2);
                a4[mi][0] = lo.x; a4[mi][1] = lo.y; a4[mi][2] = hi.x; a4[mi][3] = hi.y;
            }
        }
        if constexpr (TB) {
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) {
                const double *p = bt + (bcol + ni * 16) * DI_APITCH + 4 * lh;
                const d2 lo = *(const d2 *)p, hi = *(const d2 *)(p + 2);
                b4[ni][0] = lo.x; b4[ni][1] = lo.y; b4[ni][2] = hi.x; b4[ni][3] = hi.y;
            }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            double a[2], b[4];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
                a[mi] = TA ? at[(4 * lh + t) * DI_BPITCH + arow + mi * 16] : a4[mi][t];
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
                b[ni] = TB ? b4[ni][t] : bt[(4 * lh + t) * DI_BPITCH + bcol + ni * 16];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
        }
        if (s + 1 < n_stages) store_stage(buf ^ 1);
        __syncthreads();
    }

    // element v of lane l is R[4 v + l / 16][l % 16] of its 16 x 16 block.  R += acc.  A whole tile:
    // the 8 values of two blocks are all read before the first is written back (as "*dst += acc"
    // per element the write-back is a chain of 32 round trips to memory).  An edge tile adds the
    // elements that exist with atomics, like a tile whose K is split: R has one owner there, so
    // the sum is the same single rounding, and reads under a per-element mask would be that chain
    // of round trips again.
    const bool whole = row0 + DI_BM <= M && col0 + DI_BN <= N;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int np = 0; np < 2; ++np) {
            if (ksplit || !whole) {
#pragma unroll
                for (int nq = 0; nq < 2; ++nq)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int ni = 2 * np + nq;
                        const int col = col0 + wc * 64 + ni * 16 + li;
                        const int row = row0 + wr * 32 + mi * 16 + 4 * v + lh;
                        if (row < M && col < N) unsafeAtomicAdd(args.R + (int64_t)row * args.ldr + col, acc[mi][ni][v]);
                    }
                continue;
            }
            double old[2][4];
#pragma unroll
            for (int nq = 0; nq < 2; ++nq)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int ni = 2 * np + nq;
                    const int col = col0 + wc * 64 + ni * 16 + li;
                    const int row = row0 + wr * 32 + mi * 16 + 4 * v + lh;
                    old[nq][v] = args.R[(int64_t)row * args.ldr + col];
                }
#pragma unroll
            for (int nq = 0; nq < 2; ++nq)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int ni = 2 * np + nq;
                    const int col = col0 + wc * 64 + ni * 16 + li;
                    const int row = row0 + wr * 32 + mi * 16 + 4 * v + lh;
                    args.R[(int64_t)row * args.ldr + col] = old[nq][v] + acc[mi][ni][v];
                }
        }
}

template <bool TA, bool TB>
static hipError_t launch_di_layout(const MmlikeArgsF64 &a, unsigned grid, int64_t n_tiles, hipStream_t s)
{
    constexpr int LDS = DiLayout<TA, TB>::LDS_BYTES;
    MmlikeArgsF64 b = a;
    int splits = 1;
    b.kchunk = a.K;
    // The streamed kernel where the problem allows it (aligned rows, any layout, any M, N and K >= 8): two
    // workgroups to a compute unit.
    bool streamed = false;
    streamed = identity_f64_dma_eligible(b);
    // Register-staged kernel, tiles for at most half of the compute units: split K over several
    // workgroups per tile (at least 128 k each), which add their parts to R with hardware fp64
    // atomics
    const int64_t waves = (int64_t)n_tiles * (DI_NT / 64);
    if (!streamed && k_split_allowed() && 2 * n_tiles <= compute_units() && a.K >= 256) {
        int64_t want = (2048 + waves - 1) / waves;
        if (want > a.K / 128) want = a.K / 128;
        if (want > 1024) want = 1024;
        const int64_t chunk = ((a.K + want - 1) / want + DI_BK - 1) / DI_BK * DI_BK;
        b.kchunk = (int)chunk;
        splits = (int)((a.K + chunk - 1) / chunk);
    }
    b.tail_base = 0; b.tail_blocks = 0; b.tail_splits = 1;
    dim3 launch_grid(grid, (unsigned)splits);
    // Streamed kernel: with at most two rounds of tiles every tile is launched once per k range
    // (choose_stream_split in amulet_internal.h).
    if (streamed && splits == 1 && n_tiles <= 4 * (int64_t)compute_units()) {
        static const double rate2[2] = {0.93, 1.0};
        const int sp = choose_stream_split(grid / 8, compute_units() / 8, a.K, 2, rate2, 30.0, 0.34);
        if (sp > 1) {
            const int64_t chunk = chunk_with_a_whole_last_stage(a.K, ((a.K + sp - 1) / sp + DI_BK - 1) / DI_BK * DI_BK, DI_BK);
            b.kchunk = (int)chunk;
            splits = (int)((a.K + chunk - 1) / chunk);
            launch_grid = dim3(grid, (unsigned)splits);
        }
    }
    // Register-staged kernel, up to four tiles per compute unit: every tile once per k range, as
    // many ranges as the occupancy model likes best (choose_full_split in amulet_internal.h).
    if (!streamed && splits == 1 && n_tiles <= 4 * (int64_t)compute_units() && a.K >= 512) {
        static const double rate[2] = {0.86, 1.0};
        const int sp = choose_full_split(grid / 8, compute_units() / 8, a.K, rate, 2);
        if (sp > 1) {
            const int64_t chunk = ((a.K + sp - 1) / sp + DI_BK - 1) / DI_BK * DI_BK;
            b.kchunk = (int)chunk;
            splits = (int)((a.K + chunk - 1) / chunk);
            launch_grid = dim3(grid, (unsigned)splits);
        }
    }
    // more tiles than that: the launch runs in rounds (about one tile per compute unit for the
    // register-staged kernel, as in the fp32 kernel; two for the streamed one); the tiles of a
    // nearly empty last round are launched once per k range instead (choose_tail_split in
    // amulet_internal.h)
    TailSplit t;
    if (splits == 1 && n_tiles > 4 * (int64_t)compute_units() &&
        choose_tail_split(n_tiles, grid, (streamed ? 2 : 1) * (int64_t)compute_units(), a.K, DI_BK, t)) {
        if (streamed) {
            t.chunk = (int)chunk_with_a_whole_last_stage(a.K, t.chunk, DI_BK);
            t.splits = (int)((a.K + t.chunk - 1) / t.chunk);
            t.grid = t.base + t.blocks * t.splits;
        }
        b.tail_base = (int)t.base;
        b.tail_blocks = (int)t.blocks;
        b.tail_splits = t.splits;
        b.kchunk = t.chunk;
        launch_grid = dim3((unsigned)t.grid, 1u);
    }
    if (streamed)
        return launch_row_of_blocks(b, launch_grid.x, DI_NT, [&](unsigned n) {
            (void)enqueue_identity_f64_dma(b, 128, n, launch_grid.y, s);
        });
    static hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void *>(&identity_mfma_f64_kernel<TA, TB>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (granted != hipSuccess) return granted;
    return launch_row_of_blocks(b, launch_grid.x, DI_NT, [&](unsigned n) {
        hipLaunchKernelGGL((identity_mfma_f64_kernel<TA, TB>), dim3(n, launch_grid.y), dim3(DI_NT), LDS, s, b);
    });
}

// The streamed 64 x 64 tile, for problems with fewer 128 x 128 tiles than compute units (the fp64
// counterpart of the fp32 kernel's small tile, identity_mfma.hip, where the reasons are given):
// K split by the streamed kernels' model with four workgroups (rings of 32 KB) to a unit.
static hipError_t launch_di_small(const MmlikeArgsF64 &a, hipStream_t s)
{
    MmlikeArgsF64 b = a;
    b.kchunk = a.K;
    b.tail_base = 0; b.tail_blocks = 0; b.tail_splits = 1;
    const int64_t tiles_m = (a.M + 63) / 64, tiles_n = (a.N + 63) / 64;
    const int64_t grid = xcd_grid(tiles_m, tiles_n);
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    int splits = 1;
    const int cap = 4;   // rings of 32 KB; the kernel is built for four waves per SIMD
    if (tiles_m * tiles_n <= 2 * cap * (int64_t)compute_units()) {
        static const double rate[4] = {0.80, 0.93, 1.0, 1.0};
        const int sp = choose_stream_split(grid / 8, compute_units() / 8, a.K, cap, rate, 100.0, 0.34);
        if (sp > 1) {
            const int64_t chunk = chunk_with_a_whole_last_stage(a.K, ((a.K + sp - 1) / sp + DI_BK - 1) / DI_BK * DI_BK, DI_BK);
            b.kchunk = (int)chunk;
            splits = (int)((a.K + chunk - 1) / chunk);
        }
    }
    return launch_row_of_blocks(b, grid, 256, [&](unsigned n) {
        (void)enqueue_identity_f64_dma(b, 64, n, (unsigned)splits, s);
    });
}

// tile: 64 = the streamed 64 x 64 tile where the streamed kernel takes the problem; else 128 x 128
hipError_t launch_identity_mfma_f64(const MmlikeArgsF64 &a, int tile, hipStream_t s)
{
    if (tile == 64) {
        MmlikeArgsF64 b = a;
        b.kchunk = a.K;
        if (identity_f64_dma_eligible(b)) return launch_di_small(a, s);
    }
    const int64_t tiles_m = (a.M + DI_BM - 1) / DI_BM;
    const int64_t tiles_n = (a.N + DI_BN - 1) / DI_BN;
    const int64_t grid = xcd_grid(tiles_m, tiles_n);
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.transA && a.transB) return launch_di_layout<true, true>(a, (unsigned)grid, tiles_m * tiles_n, s);
    if (a.transA) return launch_di_layout<true, false>(a, (unsigned)grid, tiles_m * tiles_n, s);
    if (a.transB) return launch_di_layout<false, true>(a, (unsigned)grid, tiles_m * tiles_n, s);
    return launch_di_layout<false, false>(a, (unsigned)grid, tiles_m * tiles_n, s);
}

}  // namespace amulet
