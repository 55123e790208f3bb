// Identity task (g = p, plain matmul; paper Sec. 6.1) in fp64 on the matrix cores, operands
// streamed HBM -> LDS directly (global_load_lds_dwordx4, gfx950) through a ring of NSTAGE LDS
// stages: the fp64 counterpart of identity_mfma_dma_kernel (identity_mfma_dma.hip), where the
// reasons are given.
//
// Same arithmetic, tile (128 x 128, 8 waves of 32 x 64 = 2 x 4 blocks of v_mfma_f64_16x16x4_f64)
// and result layout as identity_mfma_f64_kernel.  A stage is 8 k deep (A 128 x 8 and B 8 x 128
// doubles, 16 KB); a ring of 4 stages is 64 KB, two workgroups per compute unit.  (Also as a
// 64 x 64 tile, 4 waves of 32 x 32, 8 KB stages, for problems of few tiles: the template's T.  The
// layouts below are given for T = 128; with 64 a slice has half the lines.)  The hardware
// pairs k-slot h (= lane / 16) of A with k-slot h of B, so which k a slot carries is free: the
// stage's first matrix step takes k = h, the second k = 4 + h.
//
// LDS layout of a stage, un-padded and XOR-swizzled at 16-byte granularity by choosing what each
// lane fetches:
//   A tile [128 rows][4 units of 2 k]: row r keeps logical unit u at u ^ ((r >> 2) & 3); a fragment
//     read (ds_read_b64) takes 16 neighbouring rows x 2 k-slots per clock, which then fall in 32
//     distinct 8-byte bank pairs;
//   B tile [8 k][64 units of 2 columns]: k-row k keeps logical unit u at u ^ (8 * (k & 1)); a
//     fragment read takes 16 columns of rows k and k + 1 per clock, which land on the two halves
//     of the banks.
// One barrier per stage, between its two matrix steps.
//
// Used for row-major or transposed operands of any alignment and size with at least one stage of K
// (and two lines in an operand whose lines run across k); everything else runs
// identity_mfma_f64_kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "amulet_internal.h"

// the LDS-DMA asm below sets M0 itself and says so in its clobber list
#pragma clang diagnostic ignored "-Winline-asm"

namespace amulet {

typedef double d4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void *lds_void_ptr;

constexpr int DD_BK = 8;
constexpr int DD_LOADS = 2;                         // DMA instructions per wave per stage
// T: rows and columns of a tile.  128: 8 waves of 32 x 64; 64: 4 waves of 32 x 32, for problems with
// fewer 128 x 128 tiles than compute units (same code: a wave loads 1 KB of each operand's slice
// per stage either way).
template <int T>
struct DdTile {
    static constexpr int NT = T * 4;                    // threads: one wave per 16 lines of a slice
    static constexpr int NB = T / 32;                   // 16-column blocks per wave
    static constexpr int OP_BYTES = T * DD_BK * 8;      // one operand's 8-k slice: 8 KB / 4 KB
    static constexpr int STAGE_BYTES = 2 * OP_BYTES;
    static constexpr int ROW_BYTES = T * 8;             // a k-row of a k-major slice
    static constexpr int ROW_UNITS = T / 2;             // its 16-byte units
};

template <int N>
__device__ __forceinline__ void wait_vmcnt_f64()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

extern __shared__ __attribute__((aligned(16))) char dd_smem[];

// TA / TB: the operand is stored transposed (A as K x M, B as N x K; paper Sec. 6.3).  An operand's
// 8-k slice of the tile keeps its global layout in LDS, "k-minor" (128 lines x 8 k, k contiguous:
// row-major A, transposed B) or "k-major" (8 k x 128 lines: row-major B, transposed A), with the
// swizzles given above for A and B respectively.
template <int NSTAGE, bool TA, bool TB, int T>
__global__ void __launch_bounds__(T * 4) __attribute__((amdgpu_waves_per_eu(4, 4)))
identity_mfma_f64_dma_kernel(const MmlikeArgsF64 args)
{
    static_assert(NSTAGE >= 3 && NSTAGE <= 8, "the wait counts are written for rings of 3 to 8 stages");
    typedef DdTile<T> TL;
    constexpr int DD_BM = T, DD_BN = T, DD_A_BYTES = TL::OP_BYTES, DD_STAGE_BYTES = TL::STAGE_BYTES;
    constexpr int NB = TL::NB, WC = 16 * NB, ROWB = TL::ROW_BYTES, NM = 2 * NB, READS = 2 + NB;
    constexpr bool A_KMINOR = !TA, B_KMINOR = TB;
    const int M = args.M, N = args.N;
    int K = args.K;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    const int li = lane & 15, lh = lane >> 4;

    // place in the XCD-aware tile order, and which k range of it (same conventions as
    // identity_mfma_f64_kernel: split K over gridDim.y, tail split from tail_base on)
    const int tiles_m = (M + DD_BM - 1) / DD_BM, tiles_n = (N + DD_BN - 1) / DD_BN;
    int tm, tn;
    int block = (int)blockIdx.x + args.block_base, ksplit_idx = (int)blockIdx.y;
    const bool tail_part = args.tail_splits > 1 && block >= args.tail_base;
    if (tail_part) {
        const int rel = block - args.tail_base;
        block = args.tail_base + rel % args.tail_blocks;
        ksplit_idx = rel / args.tail_blocks;
    }
    if (!xcd_tile(block, tiles_m, tiles_n, tm, tn)) return;   // padding: the whole workgroup leaves
    // (wave-uniform by construction; said so explicitly, so that everything derived from them --
    // the operand bases the loads take in scalar registers among it -- stays on the scalar unit)
    const int row0 = __builtin_amdgcn_readfirstlane(tm * DD_BM), col0 = __builtin_amdgcn_readfirstlane(tn * DD_BN);
    const bool ksplit = gridDim.y > 1 || tail_part;
    int kb = 0;
    if (ksplit) {
        kb = ksplit_idx * args.kchunk;
        K = (K - kb < args.kchunk) ? K - kb : args.kchunk;
    }
    // whole stages stream through LDS; the k that remain (fewer than a stage, in the last k range
    // only: the others are whole stages) are multiplied from values each lane fetches itself
    const int n_stages = K > 0 ? K / DD_BK : 0;
    const int ktail = K > 0 ? K - n_stages * DD_BK : 0;
    if (n_stages <= 0) return;   // (the host never makes a k range shorter than a stage)

    // ---- what each lane fetches: one A slot and one B slot per stage -----------------------
    // wave w owns the 1 KB slot group w of each operand's slice:
    //   k-minor slice: slot 64 w + lane -> line 16 w + lane / 4, physical unit lane % 4
    //   k-major slice: slot 64 w + lane -> k and physical unit = quotient and remainder by the units of a k-row
    // `lines` of the tile exist (128 but in an edge tile), and every load stays inside the operand.
    // k-minor: a line past them is replaced by the last one inside.  k-major: a unit of two lines
    // that would end past them is fetched as the two lines that end AT the edge (a 16-byte piece
    // may start at any 8-byte aligned address), so the unit an odd edge cuts holds its existing
    // line one place further up -- the fragment reads of that line look there (`edge_shift`
    // below).  A tile of one line takes the line before it in as well (`lead`: the base moves
    // back; the operand has at least two, the host checks).  What the lanes past the edge bring
    // only reaches rows and columns that are not written back.
    auto lane_offset = [&](bool kminor, int64_t ld, int lines) {
        if (kminor) {
            const int line = 16 * wave + (lane >> 2);
            const int u = (lane & 3) ^ ((line >> 2) & 3);
            const int line_in = line < lines ? line : lines - 1;
            return ((uint32_t)line_in * (uint32_t)ld + (uint32_t)(u * 2)) * 8u;
        }
        const int slot = 64 * wave + lane;
        const int k = slot / TL::ROW_UNITS;
        const int u = (slot % TL::ROW_UNITS) ^ ((k & 1) << 3);
        const int lead = lines < 2 ? 2 - lines : 0;
        const int start = 2 * u + 2 <= lines ? 2 * u + lead : lines - 2 + lead;
        return ((uint32_t)k * (uint32_t)ld + (uint32_t)start) * 8u;
    };
    const int rows_in = M - row0 < DD_BM ? M - row0 : DD_BM, cols_in = N - col0 < DD_BN ? N - col0 : DD_BN;
    const int a_lead = !A_KMINOR && rows_in < 2 ? 2 - rows_in : 0, b_lead = !B_KMINOR && cols_in < 2 ? 2 - cols_in : 0;
    const uint32_t a_voff = lane_offset(A_KMINOR, args.lda, rows_in), b_voff = lane_offset(B_KMINOR, args.ldb, cols_in);
    // the tile's first stage, and what a stage adds (doubles): 8 k along a k-minor operand's rows,
    // 8 rows of a k-major one
    const double *const a_base = A_KMINOR ? args.A + (int64_t)row0 * args.lda + kb : args.A + (int64_t)kb * args.lda + row0 - a_lead;
    const double *const b_base = B_KMINOR ? args.B + (int64_t)col0 * args.ldb + kb : args.B + (int64_t)kb * args.ldb + col0 - b_lead;
    const int64_t a_stage = A_KMINOR ? (int64_t)DD_BK : (int64_t)DD_BK * args.lda;
    const int64_t b_stage = B_KMINOR ? (int64_t)DD_BK : (int64_t)DD_BK * args.ldb;

    // The loads are asm so that the compiler's wait-count pass does not see a vector-memory
    // instruction writing LDS (it would drain all outstanding loads before every LDS read);
    // completion is tracked by hand: s_waitcnt vmcnt(n) before the stage's barrier.  M0 carries
    // the wave-uniform LDS destination; each lane's 16 bytes land at M0 + 16 * lane.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_ptr)dd_smem;
    auto dma16 = [&](const double *base, uint32_t voff, uint32_t lds_addr) {
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(voff), "s"(base), "s"(lds_addr)
                     : "memory", "m0");
    };
    // load i (0: A, 1: B) of a stage whose operands start at (ap, bp), into ring slot `buf`
    auto issue_one = [&](const double *ap, const double *bp, int buf, int i) {
        const uint32_t dst = lds_base + (uint32_t)(buf * DD_STAGE_BYTES) + (uint32_t)(wave * 1024);
        if (i & 1) dma16(bp, b_voff, dst + (uint32_t)DD_A_BYTES);
        else dma16(ap, a_voff, dst);
    };

    // ---- where each lane reads its fragments (byte offsets inside an operand's slice) --------
    // matrix step g of the stage multiplies k = 4g + lh; the lane's line is wr*32 + mi*16 + li of
    // A, wc*WC + ni*16 + li of B; one 8-byte read per block in either layout:
    //   k-minor: line * 64 + swizzled unit of k, per step g (+ 1024 per block)
    //   k-major: k-row * ROWB + swizzled unit of the line, per block (+ 4 ROWB per step)
    auto minor_off = [&](int line, int g) {
        const int k = 4 * g + lh;
        return line * 64 + (((k >> 1) ^ ((line >> 2) & 3)) * 16) + (k & 1) * 8;
    };
    auto major_off = [&](int line0, int blk, int lines) {
        const int unit = (line0 >> 1) + blk * 8 + (li >> 1);
        // (the line of the unit an odd edge cuts sits one place further up)
        const int edge_shift = (lines & 1) && line0 + blk * 16 + li >= (lines & ~1) ? 1 : 0;
        return lh * ROWB + ((unit ^ ((lh & 1) << 3)) * 16) + ((li & 1) + edge_shift) * 8;
    };
    int a_off[2], b_off[NB];   // k-minor: per step g; k-major: per block
#pragma unroll
    for (int x = 0; x < 2; ++x) a_off[x] = A_KMINOR ? minor_off(wr * 32 + li, x) : major_off(wr * 32, x, rows_in);
#pragma unroll
    for (int x = 0; x < NB; ++x)
        b_off[x] = DD_A_BYTES + (B_KMINOR ? minor_off(wc * WC + li, x & 1) : major_off(wc * WC, x, cols_in));
    // fragment read i (0 .. READS-1) of matrix step g of the stage in slot `buf`: 0, 1 = A (mi), then B (ni)
    auto read_one = [&](int buf, int g, int i, double (&a)[2], double (&b)[NB]) {
        const char *st = dd_smem + buf * DD_STAGE_BYTES;
        if (i < 2) a[i] = *(const double *)(st + (A_KMINOR ? a_off[g] + i * 1024 : a_off[i] + g * 4 * ROWB));
        else b[i - 2] = *(const double *)(st + (B_KMINOR ? b_off[g] + (i - 2) * 1024 : b_off[i - 2] + g * 4 * ROWB));
    };
    d4 acc[2][NB];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < NB; ++ni)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[mi][ni][v] = 0.0;
    // The NM matrix instructions of one matrix step, with `side(i)` issued right after
    // instruction i: a wave issues in order and a matrix instruction occupies the matrix core for
    // 64 cycles during which the wave may issue other instructions, so the stage's LDS reads and
    // loads are spread over those gaps instead of standing between two runs of matrix
    // instructions.
    auto mma_with = [&](const double (&a)[2], const double (&b)[NB], auto side) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < NB; ++ni) {
                acc[mi][ni] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
                side(mi * NB + ni);
                __builtin_amdgcn_sched_barrier(0);
            }
    };
    // Wait until this wave's loads of stage t have landed, `upto` being the last stage requested
    // so far: vector memory operations retire in order, so at most the DD_LOADS per later stage
    // may still be outstanding.  (The count is an immediate: one instruction per value.)
    auto wait_stage = [&](int t, int upto) {
        switch (upto - t) {
        case 1: wait_vmcnt_f64<DD_LOADS>(); break;
        case 2: wait_vmcnt_f64<2 * DD_LOADS>(); break;
        case 3: wait_vmcnt_f64<3 * DD_LOADS>(); break;
        case 4: wait_vmcnt_f64<4 * DD_LOADS>(); break;
        case 5: wait_vmcnt_f64<5 * DD_LOADS>(); break;
        case 6: wait_vmcnt_f64<6 * DD_LOADS>(); break;
        default: wait_vmcnt_f64<0>(); break;   // never too little
        }
    };

    // The barrier of a stage sits BETWEEN its two matrix steps: a wave reaches barrier s with the
    // fragments of step 1 of stage s in registers, and after it runs step 1 of stage s while it
    // requests a later stage and reads the fragments of step 0 of stage s+1.  Barrier s certifies
    // for all waves: the loads of stage s+1 have landed, and every read of stage s-1 is complete
    // (its last fragments were consumed by matrix instructions before the barrier), so the slot of
    // stage s-1 is refilled after it with stage s+NSTAGE-1.
    int requested = 0;
    const double *ap = a_base, *bp = b_base;        // operands of the next stage to request
#pragma unroll
    for (int d = 0; d < NSTAGE - 1; ++d)
        if (d < n_stages) {
#pragma unroll
            for (int i = 0; i < DD_LOADS; ++i) issue_one(ap, bp, d, i);
            ap += a_stage;
            bp += b_stage;
            requested = d + 1;
        }
    // While the first stages are on their way and few registers are live: the k past the last whole
    // stage (1 .. 7 of them, in the last k range only).  Matrix instruction `step` multiplies
    // k = kt + 4 step + lh, and each lane reads its own A and B values of that k from memory (its
    // row and column clamped into the tile's existing ones, a k past the end read at the last k
    // and replaced by zero).
    if (ktail > 0) {
        const int kt = kb + n_stages * DD_BK, kend = kb + K;
#pragma unroll
        for (int step = 0; step < 2; ++step) {
            if (4 * step >= ktail) break;
            const int k = kt + 4 * step + lh;
            const bool ok = k < kend;
            const int64_t kc = ok ? k : kend - 1;
            double av[2], bv[NB];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi) {
                const int r = wr * 32 + mi * 16 + li;
                const int64_t line = row0 + (r < rows_in ? r : rows_in - 1);
                const double a = TA ? args.A[kc * args.lda + line] : args.A[line * args.lda + kc];
                av[mi] = ok ? a : 0.0;
            }
#pragma unroll
            for (int ni = 0; ni < NB; ++ni) {
                const int c = wc * WC + ni * 16 + li;
                const int64_t line = col0 + (c < cols_in ? c : cols_in - 1);
                const double b = TB ? args.B[line * args.ldb + kc] : args.B[kc * args.ldb + line];
                bv[ni] = ok ? b : 0.0;
            }
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < NB; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[mi], bv[ni], acc[mi][ni], 0, 0, 0);
        }
    }
    wait_stage(0, requested - 1);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    double fa0[2], fa1[2], fb0[NB], fb1[NB];
    int buf = 0, ibuf = NSTAGE - 1;
#pragma unroll
    for (int i = 0; i < READS; ++i) read_one(0, 0, i, fa0, fb0);
    // the fragment reads of step g of the stage in `slot`, spread over the matrix instructions of
    // the step before.  (The 64 x 64 tile has 4 matrix instructions of 32 cycles a step: its four
    // reads go behind the first two, in the order of their use -- a0 b0, b1 a1 -- so that each is
    // at least two matrix instructions ahead of it.)
    auto side_reads = [&](int i, int slot, int g, double (&a)[2], double (&b)[NB]) {
        if constexpr (T == 64) {
            if (i == 0) { read_one(slot, g, 0, a, b); read_one(slot, g, 2, a, b); }
            if (i == 1) { read_one(slot, g, 3, a, b); read_one(slot, g, 1, a, b); }
        } else {
#pragma unroll
            for (int p = i; p < READS; p += NM) read_one(slot, g, p, a, b);
        }
    };
    auto iteration = [&](int s, auto steady) {
        constexpr bool STEADY = decltype(steady)::value;
        const int nbuf = buf == NSTAGE - 1 ? 0 : buf + 1;
        // step 0 of stage s; the fragments of step 1 are read meanwhile
        mma_with(fa0, fb0, [&](int i) { side_reads(i, buf, 1, fa1, fb1); });
        if constexpr (STEADY) {
            // stages up to s+NSTAGE-2 are requested; s+1 must have landed
            wait_vmcnt_f64<(NSTAGE - 3) * DD_LOADS>();
        } else {
            const int last = s + NSTAGE - 2 < n_stages - 1 ? s + NSTAGE - 2 : n_stages - 1;
            wait_stage(s + 1, last);
        }
        __builtin_amdgcn_s_barrier();   // bare: the fence of __syncthreads() would drain the loads in flight
        asm volatile("" ::: "memory");
        // step 1 of stage s; meanwhile the request for stage s+NSTAGE-1 (into the slot stage s-1
        // has left) and the fragment reads of step 0 of stage s+1
        const bool more = STEADY || s + NSTAGE - 1 < n_stages;
        mma_with(fa1, fb1, [&](int i) {
            if constexpr (T == 64) {
                side_reads(i, nbuf, 0, fa0, fb0);
                if (i >= 2 && more) issue_one(ap, bp, ibuf, i - 2);
            } else {
#pragma unroll
                for (int p = i; p < DD_LOADS + READS; p += NM) {
                    if (p < DD_LOADS) { if (more) issue_one(ap, bp, ibuf, p); }
                    else read_one(nbuf, 0, p - DD_LOADS, fa0, fb0);
                }
            }
        });
        ap += a_stage;
        bp += b_stage;
        ibuf = buf;
        buf = nbuf;
    };
    const int steady_end = n_stages - (NSTAGE - 1);   // first s that requests nothing more
    int s = 0;
    for (; s < steady_end; ++s) iteration(s, std::true_type());
    for (; s + 1 < n_stages; ++s) iteration(s, std::false_type());
    mma_with(fa0, fb0, [&](int i) { side_reads(i, buf, 1, fa1, fb1); });
    mma_with(fa1, fb1, [&](int) {});

    // element v of lane l is R[4 v + l / 16][l % 16] of its 16 x 16 block.  R += acc: the 16 values
    // of a row of blocks are all read before the first is written back (as "*dst += acc" per
    // element the compiler must keep every store behind the load before it, a chain of 32 round
    // trips to memory).
    const bool edge = rows_in < DD_BM || cols_in < DD_BN;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
        double *dst[4];
#pragma unroll
        for (int v = 0; v < 4; ++v)
            dst[v] = args.R + (int64_t)(row0 + wr * 32 + mi * 16 + 4 * v + lh) * args.ldr + col0 + wc * WC + li;
        if (ksplit || edge) {
            // (an edge tile adds with atomics too, the elements that exist: R has one owner here, so
            // the sum is the same single rounding, and an atomic needs no round trip to memory
            // before the store, which under a per-element mask would be one after the other)
#pragma unroll
            for (int ni = 0; ni < NB; ++ni)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = wr * 32 + mi * 16 + 4 * v + lh, col = wc * WC + ni * 16 + li;
                    if (row < rows_in && col < cols_in) unsafeAtomicAdd(dst[v] + ni * 16, acc[mi][ni][v]);
                }
        } else {
            double old[NB][4];
#pragma unroll
            for (int ni = 0; ni < NB; ++ni)
#pragma unroll
                for (int v = 0; v < 4; ++v) old[ni][v] = dst[v][ni * 16];
#pragma unroll
            for (int ni = 0; ni < NB; ++ni)
#pragma unroll
                for (int v = 0; v < 4; ++v) dst[v][ni * 16] = old[ni][v] + acc[mi][ni][v];
        }
    }
}

// At least one stage of K, at least two lines in an operand whose lines run across k (its 16-byte
// pieces are two lines wide), per-lane byte offsets that fit 31 bits, and k ranges (`kchunk`, when
// the launch splits K) of whole stages.  Rows need not be 16-byte aligned: a direct-to-LDS load of
// 16 bytes takes any 8-byte aligned address.
bool identity_f64_dma_eligible(const MmlikeArgsF64 &a)
{
    if (a.M <= 0 || a.N <= 0 || a.K < DD_BK || (a.kchunk < a.K && a.kchunk % DD_BK)) return false;
    if ((a.transA && a.M < 2) || (!a.transB && a.N < 2)) return false;
    // a k-minor slice spans up to 128 lines of the operand's storage, a k-major one 8
    const int64_t minor_max = (0x7FFFFFFFLL / 8 - 8) / 128, major_max = (0x7FFFFFFFLL / 8 - 128) / DD_BK;
    if (a.lda > (a.transA ? major_max : minor_max) || a.ldb > (a.transB ? minor_max : major_max)) return false;
    return true;
}

template <int NSTAGE, bool TA, bool TB, int T>
static hipError_t enqueue_f64_layout(const MmlikeArgsF64 &a, unsigned grid_x, unsigned grid_y, hipStream_t s)
{
    constexpr int LDS = NSTAGE * DdTile<T>::STAGE_BYTES;
    static hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void *>(&identity_mfma_f64_dma_kernel<NSTAGE, TA, TB, T>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (granted != hipSuccess) return granted;
    hipLaunchKernelGGL((identity_mfma_f64_dma_kernel<NSTAGE, TA, TB, T>), dim3(grid_x, grid_y), dim3(DdTile<T>::NT), LDS, s, a);
    return hipSuccess;
}

template <int NSTAGE, int T>
static hipError_t enqueue_f64_tile(const MmlikeArgsF64 &a, unsigned grid_x, unsigned grid_y, hipStream_t s)
{
    if (a.transA && a.transB) return enqueue_f64_layout<NSTAGE, true, true, T>(a, grid_x, grid_y, s);
    if (a.transA) return enqueue_f64_layout<NSTAGE, true, false, T>(a, grid_x, grid_y, s);
    if (a.transB) return enqueue_f64_layout<NSTAGE, false, true, T>(a, grid_x, grid_y, s);
    return enqueue_f64_layout<NSTAGE, false, false, T>(a, grid_x, grid_y, s);
}

// Enqueues grid.x x grid.y workgroups of the streamed kernel: tiles of 128 rows and columns (512
// threads, ring of 4 stages) or of 64 (256 threads, ring of ID_SMALL_STAGES).  The caller has
// checked identity_f64_dma_eligible and fills the split fields of `a` as for
// identity_mfma_f64_kernel.
hipError_t enqueue_identity_f64_dma(const MmlikeArgsF64 &a, int tile, unsigned grid_x, unsigned grid_y, hipStream_t s)
{
    if (tile == 128) return enqueue_f64_tile<4, 128>(a, grid_x, grid_y, s);
    if (tile == 64) return enqueue_f64_tile<ID_SMALL_STAGES, 64>(a, grid_x, grid_y, s);
    return hipErrorInvalidValue;
}

}  // namespace amulet
