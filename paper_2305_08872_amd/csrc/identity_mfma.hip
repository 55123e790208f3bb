// Identity task (g = p, plain matmul; paper Sec. 6.1) on the fp32 matrix cores.
// With no per-product step this one task is a dense contraction, so it runs as
// v_mfma_f32_32x32x2_f32 tiles instead of the vector-ALU micro-tiles.
//
// Workgroup: G x G waves (template parameter G = 2 or 4), R tile 64 G x 64 G (128 x 128 with
// 4 waves, or 256 x 256 with 16 waves: half the operand traffic per multiply-add, for large
// problems), each wave a 64 x 64 sub-tile = 2x2 MFMA blocks of 32 x 32 (64 accumulator registers).
// K is staged 16 at a time: A tile 128 x 16 (k contiguous, row pitch padded to
// 20 floats so 16-byte fragment reads spread over all banks) and B tile
// 16 x 128 (as in global memory), global -> registers -> LDS, double buffered,
// one barrier per stage.
//
// Fragment mapping: lane l supplies row i = l % 32 (A) or column j = l % 32 (B)
// and k-slot h = l / 32.  The hardware multiplies A's slot h with B's slot h,
// so which k a slot carries is free as long as both operands agree: per group
// of 8 k, slot h of MFMA t carries k = 4h + t.  A lane then reads its four A
// values of a group as one ds_read_b128.
//
// Transposed operands (template parameters TA, TB; paper Sec. 6.3): an operand is staged either
// "k-minor" (a tile of 128 rows or columns x 16 k, k contiguous: row-major A, transposed B) or
// "k-major" (16 k x 128, as row-major B and transposed A are stored).  Both keep their global
// layout in LDS; a k-minor operand's fragment values come from one ds_read_b128 per 4 k, a
// k-major operand's from one ds_read_b32 per MFMA step, read one step ahead.
//
// Rows/columns beyond M/N and the K remainder are zero-filled in LDS: for the
// identity task a zero product adds nothing (this is NOT true of the predicate
// tasks, which never take this path).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "amulet_internal.h"

namespace amulet {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef f4 f4_any __attribute__((aligned(4)));   // four floats at any float address
typedef float f16v __attribute__((ext_vector_type(16)));
typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int MI_BK = 16;
constexpr int MI_APITCH = MI_BK + 4;   // floats

// 4 waves per SIMD (at most 128 registers): four 128 x 128 workgroups per compute unit, which is
// what lets a 4096 x 4096 result (1024 tiles on 256 compute units) run as one full round.
template <int G, bool TA, bool TB>
struct MiLayout {
    static constexpr int BM = 64 * G, BN = 64 * G, NT = 64 * G * G;
    static constexpr int KMINOR_FLOATS = BM * MI_APITCH;   // one k-minor tile: BM x 20
    static constexpr int KMAJOR_FLOATS = MI_BK * BN;       // one k-major tile: 16 x BN
    static constexpr int A_TILE = TA ? KMAJOR_FLOATS : KMINOR_FLOATS;
    static constexpr int B_TILE = TB ? KMINOR_FLOATS : KMAJOR_FLOATS;
    static constexpr int LDS_BYTES = 2 * (A_TILE + B_TILE) * 4;   // 32-40 KB (G = 2), 64-80 KB (G = 4)
    static constexpr int ITERS = 4 / G;                    // 16-byte staging slots per thread and operand
};

template <int G, bool TA, bool TB>
__global__ void __launch_bounds__(64 * G * G) __attribute__((amdgpu_waves_per_eu(4, 4)))
identity_mfma_kernel(const MmlikeArgs args)
{
    typedef MiLayout<G, TA, TB> L;
    constexpr int MI_BM = L::BM, MI_BN = L::BN, NT = L::NT, ITERS = L::ITERS;
    constexpr int A_TILE = L::A_TILE, B_TILE = L::B_TILE;
    constexpr int QB = MI_BN / 4;   // float4 slots in one k-major row
    extern __shared__ __attribute__((aligned(16))) float mi_smem[];
    float *const As = mi_smem;                 // [2][A_TILE]
    float *const Bs = mi_smem + 2 * A_TILE;    // [2][B_TILE]

    const int M = args.M, N = args.N;
    int K = args.K;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr = wave / G, wc = wave % G;
    const int li = lane & 31, lh = lane >> 5;

    // XCD-aware tile order (xcd_tile in amulet_internal.h): each XCD walks its own rectangular
    // part of the tile grid, so its resident workgroups share A rows and B columns through its L2
    const int tiles_m = (M + MI_BM - 1) / MI_BM;
    const int tiles_n = (N + MI_BN - 1) / MI_BN;
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
    const int row0 = tm * MI_BM, col0 = tn * MI_BN;
    const bool vecA = args.vecA != 0, vecB = args.vec != 0;
    // Interior tiles with 16-byte aligned rows are staged as (wave-uniform base that advances
    // with k) + (fixed 32-bit per-thread offset): the address arithmetic stays on the scalar
    // unit, which matters because vector-ALU instructions share the issue port with the MFMAs.
    const bool interior = !TA && !TB && vecA && vecB && row0 + MI_BM <= M && col0 + MI_BN <= N &&
                          (int64_t)MI_BM * args.lda * 4 < 0x7fffffffLL && (int64_t)MI_BK * args.ldb * 4 < 0x7fffffffLL;
    // Split K (gridDim.y > 1, chosen by the host when the tiles are too few to fill the chip):
    // this workgroup multiplies k in [kb, kb + kchunk) only and adds its part to R atomically.
    const bool ksplit = gridDim.y > 1 || tail_part;
    const float *Ag = args.A, *Bg = args.B;
    if (ksplit) {
        const int kb = ksplit_idx * args.kchunk;
        Ag += TA ? (int64_t)kb * args.lda : (int64_t)kb;
        Bg += TB ? (int64_t)kb : (int64_t)kb * args.ldb;
        K = (K - kb < args.kchunk) ? K - kb : args.kchunk;
    }
    const float *const a_base = Ag + (int64_t)row0 * args.lda;
    const float *const b_base = Bg + col0;
    // staging slots of 16 bytes, u = tid + NT * it:
    //   k-minor tile, BM lines x 4 slots:  line = u / 4, k quad = u % 4
    //   k-major tile, 16 k x BN/4 slots:   k = u / (BN/4), line quad = u % (BN/4)
    unsigned offa[ITERS], offb[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int u = tid + NT * it;
        // byte offsets
        offa[it] = ((unsigned)(u >> 2) * (unsigned)args.lda + (unsigned)(u & 3) * 4u) * 4u;
        offb[it] = ((unsigned)(u / QB) * (unsigned)args.ldb + (unsigned)(u % QB) * 4u) * 4u;
    }

    // Edge workgroups of aligned row-major operands whose N is a whole number of 16-byte units take
    // the same loader with the buffers' extents set to where the operands end: a unit of a row
    // of A past M lies past the extent and reads as zero, a unit of B past N reads values of the
    // next row, or zero past the last one, and either only feeds outputs that do not exist.
    // (Every unit that feeds an existing output is whole and inside the extent: full stages
    // only, and N % 4 == 0.)
    const bool edge_fast = !interior && !TA && !TB && vecA && vecB && (N & 3) == 0 &&
                           (int64_t)MI_BM * args.lda * 4 < 0x7fffffffLL && (int64_t)MI_BK * args.ldb * 4 < 0x7fffffffLL;
    auto extent = [](int64_t bytes) { return (int)(bytes < 0 ? 0 : bytes > 0x7fffffffLL ? 0x7fffffffLL : bytes); };

    f4 sa[ITERS], sb[ITERS];
    auto load_stage = [&](int k0) {
        if ((interior || edge_fast) && k0 + MI_BK <= K) {
            // buffer loads: scalar resource (uniform base) + 32-bit per-thread byte offset;
            // extent = bytes from the stage's first element to the end of the operand's last row
            const int ext_a = interior ? 0x7fffffff : extent(((int64_t)(M - 1 - row0) * args.lda + (K - k0)) * 4);
            const int ext_b = interior ? 0x7fffffff : extent(((int64_t)(K - 1 - k0) * args.ldb + (N - col0)) * 4);
            const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(a_base + k0), 0, ext_a, 0x00020000);
            const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(b_base + (int64_t)k0 * args.ldb), 0, ext_b, 0x00020000);
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                sa[it] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(ra, offa[it], 0, 0));
                sb[it] = __builtin_bit_cast(f4, __builtin_amdgcn_raw_buffer_load_b128(rb, offb[it], 0, 0));
            }
            return;
        }
        auto load_kminor = [&](const float *base, int64_t ld, int line0, int n_lines, bool vec, f4 (&dst)[ITERS]) {
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int u = tid + NT * it;
                const int r = line0 + (u >> 2);
                const int k = k0 + (u & 3) * 4;
                f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (r < n_lines) {
                    const float *src = base + (int64_t)r * ld + k;
                    if (k + 3 < K) {
                        v = *(const f4_any *)src;   // one 16-byte load whether or not the row is aligned
                    } else {
                        if (k + 0 < K) v.x = src[0];
                        if (k + 1 < K) v.y = src[1];
                        if (k + 2 < K) v.z = src[2];
                        if (k + 3 < K) v.w = src[3];
                    }
                }
                dst[it] = v;
            }
        };
        auto load_kmajor = [&](const float *base, int64_t ld, int line0, int n_lines, bool vec, f4 (&dst)[ITERS]) {
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int u = tid + NT * it;
                const int k = k0 + u / QB;
                const int c = line0 + (u % QB) * 4;
                f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
                if (k < K) {
                    const float *src = base + (int64_t)k * ld + c;
                    if (c + 3 < n_lines) {
                        v = *(const f4_any *)src;   // one 16-byte load whether or not the row is aligned
                    } else {
                        if (c + 0 < n_lines) v.x = src[0];
                        if (c + 1 < n_lines) v.y = src[1];
                        if (c + 2 < n_lines) v.z = src[2];
                        if (c + 3 < n_lines) v.w = src[3];
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
        for (int it = 0; it < ITERS; ++it) {
            const int u = tid + NT * it;
            const int kminor = (u >> 2) * MI_APITCH + (u & 3) * 4;
            const int kmajor = (u / QB) * MI_BN + (u % QB) * 4;
            *(f4 *)&As[buf * A_TILE + (TA ? kmajor : kminor)] = sa[it];
            *(f4 *)&Bs[buf * B_TILE + (TB ? kminor : kmajor)] = sb[it];
        }
    };

    f16v acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.0f;

    const int n_stages = (K + MI_BK - 1) / MI_BK;
    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int s = 0; s < n_stages; ++s) {
        const int buf = s & 1;
        if (s + 1 < n_stages) load_stage((s + 1) * MI_BK);
        // The 8 k-steps of the stage.  A k-minor operand's values of the whole stage are read
        // first (4 x ds_read_b128); a k-major operand's values of step t+1 are read from LDS
        // before the four MFMAs of step t are issued, so the matrix pipe never waits on an LDS
        // round trip.
        const float *at = As + buf * A_TILE, *bt = Bs + buf * B_TILE;
        f4 a4[2][2], b4[2][2];
        float aq[2][2], bq[2][2];
        const int arow = wr * 64 + li, bcol = wc * 64 + li;   // + 32 for the second block
        if constexpr (!TA) {
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
                    a4[g][mi] = *(const f4 *)&at[(arow + mi * 32) * MI_APITCH + 8 * g + 4 * lh];
        } else {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) aq[0][mi] = at[(4 * lh) * MI_BN + arow + mi * 32];
        }
        if constexpr (TB) {
#pragma unroll
            for (int g = 0; g < 2; ++g)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    b4[g][ni] = *(const f4 *)&bt[(bcol + ni * 32) * MI_APITCH + 8 * g + 4 * lh];
        } else {
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) bq[0][ni] = bt[(4 * lh) * MI_BN + bcol + ni * 32];
        }
#pragma unroll
        for (int step = 0; step < 8; ++step) {
            const int g = step >> 2, t = step & 3, cur = step & 1;
            if (step + 1 < 8) {
                const int g1 = (step + 1) >> 2, t1 = (step + 1) & 3;
                if constexpr (TA) {
#pragma unroll
                    for (int mi = 0; mi < 2; ++mi)
                        aq[cur ^ 1][mi] = at[(8 * g1 + 4 * lh + t1) * MI_BN + arow + mi * 32];
                }
                if constexpr (!TB) {
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
                        bq[cur ^ 1][ni] = bt[(8 * g1 + 4 * lh + t1) * MI_BN + bcol + ni * 32];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    const float av = TA ? aq[cur][mi] : a4[g][mi][t];
                    const float bv = TB ? b4[g][ni][t] : bq[cur][ni];
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[mi][ni], 0, 0, 0);
                }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (s + 1 < n_stages) store_stage(buf ^ 1);
        __syncthreads();
    }

    // accumulator element v of lane l is R[8*(v/4) + 4*(l/32) + v%4][l%32] of its 32x32 block.
    // R += acc.  A whole tile: eight values of a block at a time are all read before the first is
    // written back (as "*dst += acc" per element the compiler must keep every store behind the
    // load before it, and the write-back is a chain of 64 round trips to memory).  An edge tile
    // adds the elements that exist with atomics, like a tile whose K is split: R has one owner
    // there, so the sum is the same single rounding, and reads under a per-element mask would be
    // that chain of round trips again.
    const bool whole = row0 + L::BM <= M && col0 + L::BN <= N;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int col = col0 + wc * 64 + ni * 32 + li;
            if (ksplit || !whole) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = row0 + wr * 64 + mi * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (row < M && col < N) unsafeAtomicAdd(args.R + (int64_t)row * args.ldr + col, acc[mi][ni][v]);
                }
                continue;
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float old[8];
#pragma unroll
                for (int w = 0; w < 8; ++w) {
                    const int v = 8 * h + w;
                    const int row = row0 + wr * 64 + mi * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    old[w] = args.R[(int64_t)row * args.ldr + col];
                }
#pragma unroll
                for (int w = 0; w < 8; ++w) {
                    const int v = 8 * h + w;
                    const int row = row0 + wr * 64 + mi * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    args.R[(int64_t)row * args.ldr + col] = old[w] + acc[mi][ni][v];
                }
            }
        }
}

// `dma_stages` > 0: run the streamed kernel (identity_mfma_dma.hip) with a ring of that many
// stages where the problem allows it (128 x 128 tile; aligned rows, any layout, any M, N and K >= 16).
template <int G, bool TA, bool TB>
static hipError_t launch_identity_layout(const MmlikeArgs &a, int dma_stages, hipStream_t s)
{
    typedef MiLayout<G, TA, TB> L;
    const int64_t tiles_m = (a.M + L::BM - 1) / L::BM;
    const int64_t tiles_n = (a.N + L::BN - 1) / L::BN;
    const int64_t grid = xcd_grid(tiles_m, tiles_n);
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    MmlikeArgs b = a;
    int splits = 1;
    b.kchunk = a.K;
    // The streamed kernel where the problem allows it: three workgroups (ring of 3 stages) or
    // two (4 stages) to a compute unit.
    bool streamed = false;
    if constexpr (G == 2) streamed = dma_stages > 0 && identity_dma_eligible(b);
    // Register-staged kernel, tiles for at most half of the compute units: split K over several
    // workgroups per tile (at least 128 k each), which add their parts to R with hardware float
    // atomics
    const int64_t waves = tiles_m * tiles_n * G * G;
    if (!streamed && k_split_allowed() && 2 * tiles_m * tiles_n <= compute_units() && a.K >= 256) {
        int64_t want = (2048 + waves - 1) / waves;
        if (want > a.K / 128) want = a.K / 128;
        if (want > 1024) want = 1024;
        const int64_t chunk = ((a.K + want - 1) / want + MI_BK - 1) / MI_BK * MI_BK;
        b.kchunk = (int)chunk;
        splits = (int)((a.K + chunk - 1) / chunk);
    }
    b.tail_base = 0; b.tail_blocks = 0; b.tail_splits = 1;
    dim3 launch_grid((unsigned)grid, (unsigned)splits);
    const int64_t tiles = tiles_m * tiles_n;
    const int per_unit = streamed ? (dma_stages == 3 ? 3 : 2) : 4;
    if (streamed && splits == 1 && tiles <= 2 * per_unit * (int64_t)compute_units()) {
        // at most two rounds of tiles: every tile once per k range (choose_stream_split)
        static const double rate3[3] = {0.92, 0.985, 1.0}, rate2[2] = {0.93, 1.0};
        const int sp = choose_stream_split(grid / 8, compute_units() / 8, a.K, per_unit, per_unit == 3 ? rate3 : rate2);
        if (sp > 1) {
            const int64_t chunk = chunk_with_a_whole_last_stage(a.K, ((a.K + sp - 1) / sp + MI_BK - 1) / MI_BK * MI_BK, MI_BK);
            b.kchunk = (int)chunk;
            splits = (int)((a.K + chunk - 1) / chunk);
            launch_grid = dim3((unsigned)grid, (unsigned)splits);
        }
    }
    // Register-staged kernel, up to four tiles per compute unit: every tile once per k range, as
    // many ranges as the occupancy model likes best (choose_full_split in amulet_internal.h).
    if (!streamed && splits == 1 && tiles <= 4 * (int64_t)compute_units() && a.K >= 512) {
        static const double rate[3] = {0.72, 0.81, 1.0};
        const int sp = choose_full_split(grid / 8, compute_units() / 8, a.K, rate, 3);
        if (sp > 1) {
            const int64_t chunk = ((a.K + sp - 1) / sp + MI_BK - 1) / MI_BK * MI_BK;
            b.kchunk = (int)chunk;
            splits = (int)((a.K + chunk - 1) / chunk);
            launch_grid = dim3((unsigned)grid, (unsigned)splits);
        }
    }
    // More tiles than that: the launch runs in rounds (one tile per compute unit for the
    // register-staged kernel: rounds of 1, 2, 3 and 4 workgroups per unit were tried in the
    // model and 1 is never worse; as many as a unit holds for the streamed one), and a last round
    // with few tiles leaves most of the chip idle for a whole K loop: its tiles are launched once
    // per k range instead (choose_tail_split in amulet_internal.h).
    TailSplit t;
    const int64_t round = streamed ? per_unit * (int64_t)compute_units() : (int64_t)compute_units();
    if (splits == 1 && tiles > (streamed ? 2 * per_unit : 4) * (int64_t)compute_units() &&
        choose_tail_split(tiles, grid, round, a.K, MI_BK, t)) {
        if (streamed) {
            t.chunk = (int)chunk_with_a_whole_last_stage(a.K, t.chunk, MI_BK);
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
        return launch_row_of_blocks(b, launch_grid.x, L::NT, [&](unsigned n) {
            (void)enqueue_identity_dma(b, 128, dma_stages, n, launch_grid.y, s);
        });
    static hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void *>(&identity_mfma_kernel<G, TA, TB>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, L::LDS_BYTES);
    if (granted != hipSuccess) return granted;
    return launch_row_of_blocks(b, launch_grid.x, L::NT, [&](unsigned n) {
        hipLaunchKernelGGL((identity_mfma_kernel<G, TA, TB>), dim3(n, launch_grid.y), dim3(L::NT), L::LDS_BYTES, s, b);
    });
}

template <int G>
static hipError_t launch_identity_grid(const MmlikeArgs &a, int dma_stages, hipStream_t s)
{
    if (a.transA && a.transB) return launch_identity_layout<G, true, true>(a, dma_stages, s);
    if (a.transA) return launch_identity_layout<G, true, false>(a, dma_stages, s);
    if (a.transB) return launch_identity_layout<G, false, true>(a, dma_stages, s);
    return launch_identity_layout<G, false, false>(a, dma_stages, s);
}

// The streamed 64 x 64 tile (a problem the streamed kernel does not take: the 128 x 128 shapes).
// Four times the tiles of the 128 x 128 shape, so a problem with fewer of those than compute units
// fills the chip without a K split or with a smaller one, and more of its write-back is plain
// stores instead of atomic adds; a workgroup streams twice the operand bytes per operation and
// has 8 matrix instructions per wave between barriers instead of 32, which is why the larger tile
// is ahead where both tile counts suit the chip equally (2048^3: 128.5 against 131 us; 1024^3: 31
// against 21).  Ring of 4 stages, 32 KB, five workgroups to a compute unit (rings of 6 and 8:
// level at one workgroup per unit, 1-5 % behind with more; of 3: 1024^3 31 us).
// K split: the streamed kernels' model; checked against forced splits of 1 ... 12 at 512^3 ...
// 1792^3 and K up to 8192: the best or within 7 %.
static hipError_t launch_identity_small(const MmlikeArgs &a, hipStream_t s)
{
    MmlikeArgs b = a;
    b.kchunk = a.K;
    b.tail_base = 0; b.tail_blocks = 0; b.tail_splits = 1;
    if (!identity_dma_eligible(b)) return launch_identity_grid<2>(a, 3, s);
    const int64_t tiles_m = (a.M + 63) / 64, tiles_n = (a.N + 63) / 64;
    const int64_t grid = xcd_grid(tiles_m, tiles_n);
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    int splits = 1;
    const int cap = 5;
    if (tiles_m * tiles_n <= 2 * cap * (int64_t)compute_units()) {
        static const double rate[5] = {0.80, 0.93, 1.0, 1.0, 1.0};
        const int sp = choose_stream_split(grid / 8, compute_units() / 8, a.K, cap, rate, 200.0);
        if (sp > 1) {
            const int64_t chunk = chunk_with_a_whole_last_stage(a.K, ((a.K + sp - 1) / sp + MI_BK - 1) / MI_BK * MI_BK, MI_BK);
            b.kchunk = (int)chunk;
            splits = (int)((a.K + chunk - 1) / chunk);
        }
    }
    return launch_row_of_blocks(b, grid, 256, [&](unsigned n) {
        (void)enqueue_identity_dma(b, 64, ID_SMALL_STAGES, n, (unsigned)splits, s);
    });
}

// variant 0: 128 x 128 tile (4 waves), register staged; 1: 256 x 256 tile (16 waves); 2, 3: the
// 128 x 128 tile streamed through a ring of 3 or 4 LDS stages where the problem allows it; 4: the
// streamed 64 x 64 tile
hipError_t launch_identity_mfma(const MmlikeArgs &a, int variant, hipStream_t s)
{
    switch (variant) {
    case 4: return launch_identity_small(a, s);
    case 0: return launch_identity_grid<2>(a, 0, s);
    case 1: return launch_identity_grid<4>(a, 0, s);
    case 2: return launch_identity_grid<2>(a, 3, s);
    case 3: return launch_identity_grid<2>(a, 4, s);
    }
    return hipErrorInvalidValue;
}

}  // namespace amulet
