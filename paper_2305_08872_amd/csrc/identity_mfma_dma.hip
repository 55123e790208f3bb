// Identity task (g = p, plain matmul; paper Sec. 6.1) on the fp32 matrix cores, operands
// streamed HBM -> LDS directly (global_load_lds_dwordx4, gfx950) through a ring of NSTAGE
// LDS stages.
//
// Same arithmetic, tile (128 x 128, 4 waves of 64 x 64) and fragment conventions as
// identity_mfma_kernel (identity_mfma.hip); what differs is the operand path.  (Also as a 64 x 64
// tile, 4 waves of 32 x 32, for problems of few tiles: the template's BLK.  The layouts below are
// given for the 128 x 128 tile; with 64 x 64 a slice has half the lines.)  That kernel
// stages a 16-k slice through registers one stage ahead, which is less than the memory latency:
// it reaches its rate only with three or four workgroups per compute unit covering for each
// other, and a problem of one or two tiles per unit runs at 0.72-0.81 of it.  Here a
// workgroup has NSTAGE - 1 stages in flight by itself, needs no staging registers and no
// ds_write, and the per-lane global addresses are fixed offsets from a scalar base.
//
// LDS layout of a stage (16 KB), un-padded and XOR-swizzled at 16-byte granularity by choosing
// what each lane fetches:
//   A tile [128 rows][4 units of 4 k]: row r keeps logical unit u at physical unit
//     u ^ ((r >> 2) & 3); the 16 lanes a ds_read_b128 is served per clock (16 neighbouring
//     rows, one unit each) then fall in 16 distinct 16-byte bank groups.
//   B tile [16 k][32 units of 4 columns]: k-row k keeps logical unit u at u ^ (8 * ((k >> 2) & 1));
//     a fragment read (ds_read_b32) takes 32 columns of row k in lanes 0-31 and of row k + 4
//     in lanes 32-63, which land on the two halves of the 64 banks.
// One barrier per stage, between the stage's two groups of 8 k (see the loop).
//
// Used for row-major or transposed operands of any alignment and size with at least one stage of
// K (and four lines in an operand whose lines run across k); everything else runs identity_mfma_kernel.  K need not be a whole number of stages (the k
// past the last whole one are multiplied from values each lane fetches itself, see the kernel's
// end), nor M and N whole tiles: a lane
// whose line (or 16-byte unit of lines) lies past the edge fetches the last one inside instead, so
// every load stays inside the operand, what it brings only reaches rows and columns of the tile
// that do not exist, and those are not written back.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "amulet_internal.h"

// the LDS-DMA asm below sets M0 itself and says so in its clobber list
#pragma clang diagnostic ignored "-Winline-asm"

namespace amulet {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void *lds_void_ptr;

constexpr int ID_BK = 16;
// BLK: 32 x 32 blocks per wave and direction.  2: the 128 x 128 tile; 1: a 64 x 64 tile for problems
// with fewer 128 x 128 tiles than compute units (same code, half the lines per operand slice).
template <int BLK>
struct IdTile {
    static constexpr int T = 64 * BLK;                  // rows of A and columns of B in a tile
    static constexpr int OP_BYTES = T * ID_BK * 4;      // one operand's 16-k slice: 8 KB / 4 KB
    static constexpr int STAGE_BYTES = 2 * OP_BYTES;
    static constexpr int LOADS = 2 * BLK;               // DMA instructions per wave per stage
    static constexpr int ROW_BYTES = T * 4;             // a k-row of a k-major slice
    static constexpr int ROW_UNITS = T / 4;             // its 16-byte units
    static constexpr int WAVE_LINES = 32 * BLK;         // lines of a wave's part of the tile
    static constexpr int NACC = BLK == 1 ? 2 : 1;       // accumulator sets (see mma_with)
};

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

extern __shared__ __attribute__((aligned(16))) char id_smem[];

// TA / TB: the operand is stored transposed (A as K x M, B as N x K; paper Sec. 6.3).  An operand's
// 16-k slice of the tile keeps its global layout in LDS, "k-minor" (128 lines x 16 k, k contiguous:
// row-major A, transposed B) or "k-major" (16 k x 128 lines: row-major B, transposed A), with the
// swizzles given above for A and B respectively.
template <int NSTAGE, bool TA, bool TB, int BLK>
__global__ void __launch_bounds__(256) identity_mfma_dma_kernel(const MmlikeArgs args)
{
    static_assert(NSTAGE >= 3 && NSTAGE <= 8, "the wait counts are written for rings of 3 to 8 stages");
    typedef IdTile<BLK> TL;
    constexpr int ID_BM = TL::T, ID_BN = TL::T, ID_A_BYTES = TL::OP_BYTES, ID_STAGE_BYTES = TL::STAGE_BYTES;
    constexpr int ID_LOADS = TL::LOADS, ROWB = TL::ROW_BYTES, WL = TL::WAVE_LINES, NACC = TL::NACC;
    constexpr bool A_KMINOR = !TA, B_KMINOR = TB;
    const int M = args.M, N = args.N;
    int K = args.K;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave >> 1, wc = wave & 1;
    const int li = lane & 31, lh = lane >> 5;

    // place in the XCD-aware tile order, and which k range of it (same conventions as
    // identity_mfma_kernel: split K over gridDim.y, tail split from tail_base on)
    const int tiles_m = (M + ID_BM - 1) / ID_BM, tiles_n = (N + ID_BN - 1) / ID_BN;
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
    const int row0 = __builtin_amdgcn_readfirstlane(tm * ID_BM), col0 = __builtin_amdgcn_readfirstlane(tn * ID_BN);
    const bool ksplit = gridDim.y > 1 || tail_part;
    int kb = 0;
    if (ksplit) {
        kb = ksplit_idx * args.kchunk;
        K = (K - kb < args.kchunk) ? K - kb : args.kchunk;
    }
    // whole stages stream through LDS; the k that remain (fewer than a stage, in the last k range
    // only: the others are whole stages) are multiplied from values each lane fetches itself
    const int n_stages = K > 0 ? K / ID_BK : 0;
    const int ktail = K > 0 ? K - n_stages * ID_BK : 0;
    if (n_stages <= 0) return;   // (the host never makes a k range shorter than a stage)

    // ---- what each lane fetches: two A slots and two B slots per stage ---------------------
    // wave w owns the 1 KB slot groups j = w (and w + 4 in the 128-line tile) of each operand's tile:
    //   k-minor tile: slot 64 j + lane -> line 16 j + lane / 4, physical unit lane % 4
    //   k-major tile: slot 64 j + lane -> k and physical unit = quotient and remainder by the units of a k-row
    // `lines` of the tile exist (128 but in an edge tile).  k-minor: a line past them is replaced
    // by the last one inside.  k-major: a unit of four lines that would end past them is fetched
    // as the four lines that end AT the edge (a 16-byte piece may start at any 4-byte aligned
    // address), so a unit the edge cuts holds its existing lines shifted up by 4 - lines % 4
    // places -- the fragment reads of those lines look there (`edge_shift` below) -- and nothing
    // is read past a row's last element.  A tile with fewer than four lines takes the lines before
    // it in as well (`lead`: the base moves back; the operand has at least four, the host checks).
    auto lane_offset = [&](bool kminor, int j, int64_t ld, int lines) {
        if (kminor) {
            const int line = 16 * j + (lane >> 2);
            const int u = (lane & 3) ^ ((line >> 2) & 3);
            const int line_in = line < lines ? line : lines - 1;
            return ((uint32_t)line_in * (uint32_t)ld + (uint32_t)(u * 4)) * 4u;
        }
        const int slot = 64 * j + lane;
        const int k = slot / TL::ROW_UNITS;
        const int u = (slot % TL::ROW_UNITS) ^ (((k >> 2) & 1) << 3);
        const int lead = lines < 4 ? 4 - lines : 0;
        const int start = 4 * u + 4 <= lines ? 4 * u + lead : lines - 4 + lead;
        return ((uint32_t)k * (uint32_t)ld + (uint32_t)start) * 4u;
    };
    const int rows_in = M - row0 < ID_BM ? M - row0 : ID_BM, cols_in = N - col0 < ID_BN ? N - col0 : ID_BN;
    const int a_lead = !A_KMINOR && rows_in < 4 ? 4 - rows_in : 0, b_lead = !B_KMINOR && cols_in < 4 ? 4 - cols_in : 0;
    uint32_t a_voff[BLK], b_voff[BLK];
#pragma unroll
    for (int q = 0; q < BLK; ++q) {
        a_voff[q] = lane_offset(A_KMINOR, wave + 4 * q, args.lda, rows_in);
        b_voff[q] = lane_offset(B_KMINOR, wave + 4 * q, args.ldb, cols_in);
    }
    // the tile's first stage, and what a stage adds (floats): 16 k along a k-minor operand's rows,
    // 16 rows of a k-major one
    const float *const a_base = A_KMINOR ? args.A + (int64_t)row0 * args.lda + kb : args.A + (int64_t)kb * args.lda + row0 - a_lead;
    const float *const b_base = B_KMINOR ? args.B + (int64_t)col0 * args.ldb + kb : args.B + (int64_t)kb * args.ldb + col0 - b_lead;
    const int64_t a_stage = A_KMINOR ? (int64_t)ID_BK : (int64_t)ID_BK * args.lda;
    const int64_t b_stage = B_KMINOR ? (int64_t)ID_BK : (int64_t)ID_BK * args.ldb;

    // The loads are asm so that the compiler's wait-count pass does not see a vector-memory
    // instruction writing LDS (it would drain all outstanding loads before every LDS read);
    // completion is tracked by hand: s_waitcnt vmcnt(n) before the stage's barrier.  M0 carries
    // the wave-uniform LDS destination; each lane's 16 bytes land at M0 + 16 * lane.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_ptr)id_smem;
    auto dma16 = [&](const float *base, uint32_t voff, uint32_t lds_addr) {
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(voff), "s"(base), "s"(lds_addr)
                     : "memory", "m0");
    };
    // load i (0 .. ID_LOADS-1) of a stage whose operands start at (ap, bp), into ring slot `buf`
    auto issue_one = [&](const float *ap, const float *bp, int buf, int i) {
        const int q = i >> 1;
        const uint32_t dst = lds_base + (uint32_t)(buf * ID_STAGE_BYTES) + (uint32_t)((wave + 4 * q) * 1024);
        if (i & 1) dma16(bp, b_voff[q], dst + (uint32_t)ID_A_BYTES);
        else dma16(ap, a_voff[q], dst);
    };

    // ---- where each lane reads its fragments (byte offsets inside an operand's slice) --------
    // The lane's line is wr*WL + blk*32 + li of A, wc*WL + blk*32 + li of B (blk = mi, ni), and
    // matrix instruction t of group g multiplies k = 8g + 4 lh + t:
    //   k-minor: the four k of a group are one 16-byte read per block;
    //   k-major: one 4-byte read per (t, block).
    auto minor_off = [&](int line, int g) { return line * 64 + (((2 * g + lh) ^ ((line >> 2) & 3)) * 16); };   // + blk * 2048
    auto major_off = [&](int line0, int blk, int lines) {
        const int unit = (line0 >> 2) + blk * 8 + (li >> 2);
        // (a line of the unit the tile's edge cuts sits 4 - lines % 4 places further up)
        const int edge_shift = (lines & 3) && line0 + blk * 32 + li >= (lines & ~3) ? 4 - (lines & 3) : 0;
        return (4 * lh) * ROWB + ((unit ^ (lh << 3)) * 16) + ((li & 3) + edge_shift) * 4;   // + (8g + t) * ROWB
    };
    int a_off[2], b_off[2];   // k-minor: per group g; k-major: per block
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        a_off[x] = A_KMINOR ? minor_off(wr * WL + li, x) : major_off(wr * WL, x < BLK ? x : 0, rows_in);
        b_off[x] = ID_A_BYTES + (B_KMINOR ? minor_off(wc * WL + li, x) : major_off(wc * WL, x < BLK ? x : 0, cols_in));
    }
    // One group's fragments of an operand: a k-minor operand's as one 16-byte value per block
    // (component t), a k-major one's as 4 x BLK floats (t, block).
    struct Frag {
        f4 v4[BLK];
        float v1[4][BLK];
    };
    constexpr int A_READS = A_KMINOR ? BLK : 4 * BLK, B_READS = B_KMINOR ? BLK : 4 * BLK, READS = A_READS + B_READS;
    // fragment read i (0 .. READS-1) of group g of the stage in slot `buf`: A's first, then B's
    auto read_one = [&](int buf, int g, int i, Frag &a, Frag &b) {
        const char *st = id_smem + buf * ID_STAGE_BYTES;
        if (i < A_READS) {
            if constexpr (A_KMINOR) a.v4[i] = *(const f4 *)(st + a_off[g] + i * 2048);
            else a.v1[i / BLK][i % BLK] = *(const float *)(st + a_off[i % BLK] + (8 * g + i / BLK) * ROWB);
        } else {
            const int j = i - A_READS;
            if constexpr (B_KMINOR) b.v4[j] = *(const f4 *)(st + b_off[g] + j * 2048);
            else b.v1[j / BLK][j % BLK] = *(const float *)(st + b_off[j % BLK] + (8 * g + j / BLK) * ROWB);
        }
    };
    // (the 64 x 64 tile has one block per wave: two accumulator sets, for even and odd t, so that
    // consecutive matrix instructions do not wait for each other's result; added up at the end)
    f16v acc[NACC][BLK][BLK];
#pragma unroll
    for (int c = 0; c < NACC; ++c)
#pragma unroll
        for (int mi = 0; mi < BLK; ++mi)
#pragma unroll
            for (int ni = 0; ni < BLK; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[c][mi][ni][v] = 0.0f;
    constexpr int NM = 4 * BLK * BLK;   // matrix instructions of a group
    // The NM matrix instructions of one group of 8 k (the hardware pairs k-slot h = lane / 32 of
    // A with k-slot h of B: instruction t of group g multiplies k = 8g + 4h + t), with `side(i)`
    // issued right after instruction i.  A wave issues in order, and a matrix instruction
    // occupies the matrix core for 64 cycles during which the wave may issue other instructions:
    // the stage's LDS reads, loads and scalar bookkeeping are spread over those gaps, a piece or
    // two per matrix instruction, instead of standing between two runs of matrix instructions,
    // where the matrix core idles while they issue.
    auto mma_with = [&](const Frag &a, const Frag &b, auto side) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int mi = 0; mi < BLK; ++mi)
#pragma unroll
                for (int ni = 0; ni < BLK; ++ni) {
                    const float av = A_KMINOR ? a.v4[mi][t] : a.v1[t][mi];
                    const float bv = B_KMINOR ? b.v4[ni][t] : b.v1[t][ni];
                    acc[t % NACC][mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[t % NACC][mi][ni], 0, 0, 0);
                    side((t * BLK + mi) * BLK + ni);
                    __builtin_amdgcn_sched_barrier(0);
                }
    };
    // Wait until this wave's loads of stage t have landed, `upto` being the last stage requested
    // so far: vector memory operations retire in order, so at most the ID_LOADS per later stage
    // may still be outstanding.  (The count is an immediate: one instruction per value.)
    auto wait_stage = [&](int t, int upto) {
        switch (upto - t) {
        case 1: wait_vmcnt<ID_LOADS>(); break;
        case 2: wait_vmcnt<2 * ID_LOADS>(); break;
        case 3: wait_vmcnt<3 * ID_LOADS>(); break;
        case 4: wait_vmcnt<4 * ID_LOADS>(); break;
        case 5: wait_vmcnt<5 * ID_LOADS>(); break;
        case 6: wait_vmcnt<6 * ID_LOADS>(); break;
        default: wait_vmcnt<0>(); break;   // never too little
        }
    };

    // The barrier of a stage sits BETWEEN its two groups of 8 k, so that the wait for the other
    // waves and the latency of the LDS reads that follow it are covered by matrix-core work
    // already queued: a wave reaches barrier s with the fragments of group 1 of stage s in
    // registers, and after it runs group 1 of stage s while it requests a later stage and reads
    // the fragments of group 0 of stage s+1.  Barrier s certifies for all waves: the loads of
    // stage s+1 have landed, and every read of stage s-1 is complete (its last fragments were
    // consumed by matrix instructions before the barrier), so the slot of stage s-1 is refilled
    // after it with stage s+NSTAGE-1.
    int requested = 0;
    const float *ap = a_base, *bp = b_base;        // operands of the next stage to request
#pragma unroll
    for (int d = 0; d < NSTAGE - 1; ++d)
        if (d < n_stages) {
#pragma unroll
            for (int i = 0; i < ID_LOADS; ++i) issue_one(ap, bp, d, i);
            ap += a_stage;
            bp += b_stage;
            requested = d + 1;
        }
    // While the first stages are on their way and few registers are live: the k past the last whole
    // stage (1 .. 15 of them, in the last k range only).  Each matrix instruction `step` multiplies
    // k = kt + 2 step + lh, and each lane reads its own A and B values of that k from memory (its
    // row and column clamped into the tile's existing ones, a k past the end read at the last k
    // and replaced by zero), eight k at a time.
    if (ktail > 0) {
        const int kt = kb + n_stages * ID_BK, kend = kb + K;
        int64_t a_line[BLK], b_line[BLK];
#pragma unroll
        for (int x = 0; x < BLK; ++x) {
            const int r = wr * WL + x * 32 + li, c = wc * WL + x * 32 + li;
            a_line[x] = row0 + (r < rows_in ? r : rows_in - 1);
            b_line[x] = col0 + (c < cols_in ? c : cols_in - 1);
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if (8 * half >= ktail) break;
            float av[4][BLK], bv[4][BLK];
#pragma unroll
            for (int step = 0; step < 4; ++step) {
                const int k = kt + 8 * half + 2 * step + lh;
                const bool ok = k < kend;
                const int64_t kc = ok ? k : kend - 1;
#pragma unroll
                for (int x = 0; x < BLK; ++x) {
                    const float a = TA ? args.A[kc * args.lda + a_line[x]] : args.A[a_line[x] * args.lda + kc];
                    const float b = TB ? args.B[b_line[x] * args.ldb + kc] : args.B[kc * args.ldb + b_line[x]];
                    av[step][x] = ok ? a : 0.0f;
                    bv[step][x] = ok ? b : 0.0f;
                }
            }
#pragma unroll
            for (int step = 0; step < 4; ++step)
#pragma unroll
                for (int mi = 0; mi < BLK; ++mi)
#pragma unroll
                    for (int ni = 0; ni < BLK; ++ni)
                        acc[step % NACC][mi][ni] =
                            __builtin_amdgcn_mfma_f32_32x32x2f32(av[step][mi], bv[step][ni], acc[step % NACC][mi][ni], 0, 0, 0);
        }
    }

    wait_stage(0, requested - 1);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    Frag fa0, fb0, fa1, fb1;
    int buf = 0, ibuf = NSTAGE - 1;
#pragma unroll
    for (int i = 0; i < READS; ++i) read_one(0, 0, i, fa0, fb0);
    // the fragment reads of group 1 of the stage in `slot`, spread over the matrix instructions of
    // group 0
    auto side_reads = [&](int i, int slot) {
#pragma unroll
        for (int p = i; p < READS; p += NM) read_one(slot, 1, p, fa1, fb1);
    };
    auto iteration = [&](int s, auto steady) {
        constexpr bool STEADY = decltype(steady)::value;
        const int nbuf = buf == NSTAGE - 1 ? 0 : buf + 1;
        // group 0 of stage s; the fragments of group 1 are read meanwhile
        mma_with(fa0, fb0, [&](int i) { side_reads(i, buf); });
        if constexpr (STEADY) {
            // stages up to s+NSTAGE-2 are requested; s+1 must have landed
            wait_vmcnt<(NSTAGE - 3) * ID_LOADS>();
        } else {
            const int last = s + NSTAGE - 2 < n_stages - 1 ? s + NSTAGE - 2 : n_stages - 1;
            wait_stage(s + 1, last);
        }
        __builtin_amdgcn_s_barrier();   // bare: the fence of __syncthreads() would drain the loads in flight
        asm volatile("" ::: "memory");
        // group 1 of stage s; meanwhile the request for stage s+NSTAGE-1 (into the slot stage s-1
        // has left) and the fragment reads of group 0 of stage s+1: ID_LOADS + READS pieces over NM
        // matrix instructions, the first few of which take one more than the rest
        const bool more = STEADY || s + NSTAGE - 1 < n_stages;
        mma_with(fa1, fb1, [&](int i) {
            if constexpr (BLK == 1) {
                // (four matrix instructions a group: the reads first, each a whole group ahead of its
                // use; the two loads behind the last two instructions)
#pragma unroll
                for (int p = i; p < READS; p += NM) read_one(nbuf, 0, p, fa0, fb0);
                if (i >= NM - ID_LOADS && more) issue_one(ap, bp, ibuf, i - (NM - ID_LOADS));
            } else {
#pragma unroll
                for (int p = i; p < ID_LOADS + READS; p += NM) {
                    if (p < ID_LOADS) { if (more) issue_one(ap, bp, ibuf, p); }
                    else read_one(nbuf, 0, p - ID_LOADS, fa0, fb0);
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
    mma_with(fa0, fb0, [&](int i) { side_reads(i, buf); });
    mma_with(fa1, fb1, [&](int) {});
    if constexpr (NACC == 2) {
#pragma unroll
        for (int mi = 0; mi < BLK; ++mi)
#pragma unroll
            for (int ni = 0; ni < BLK; ++ni) acc[0][mi][ni] += acc[1][mi][ni];
    }

    // accumulator element v of lane l is R[8*(v/4) + 4*(l/32) + v%4][l%32] of its 32x32 block.
    // R += acc: the 32 values of a row block are all read before the first is written back (as
    // "*dst += acc" per element the compiler must keep every store behind the load before it and
    // the write-back is a chain of 64 round trips to memory, 15 us of a tile).
    const bool edge = rows_in < ID_BM || cols_in < ID_BN;
#pragma unroll
    for (int mi = 0; mi < BLK; ++mi) {
        float *dst[BLK][16];
        float old[BLK][16];
#pragma unroll
        for (int ni = 0; ni < BLK; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int col = wc * WL + ni * 32 + li;
                const int row = wr * WL + mi * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                dst[ni][v] = args.R + (int64_t)(row0 + row) * args.ldr + col0 + col;
            }
        if (ksplit || edge) {
            // (an edge tile adds with atomics too, the elements that exist: R has one owner here, so
            // the sum is the same single rounding, and an atomic needs no round trip to memory
            // before the store, which under a per-element mask would be one after the other)
#pragma unroll
            for (int ni = 0; ni < BLK; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int col = wc * WL + ni * 32 + li;
                    const int row = wr * WL + mi * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    if (row < rows_in && col < cols_in) unsafeAtomicAdd(dst[ni][v], acc[0][mi][ni][v]);
                }
        } else {
#pragma unroll
            for (int ni = 0; ni < BLK; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) old[ni][v] = *dst[ni][v];
#pragma unroll
            for (int ni = 0; ni < BLK; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) *dst[ni][v] = old[ni][v] + acc[0][mi][ni][v];
        }
    }
}

// At least one stage of K, at least four lines in an operand whose lines run across k (its 16-byte
// pieces are four lines wide), per-lane byte offsets that fit 31 bits, and k ranges (`kchunk`, when
// the launch splits K) of whole stages.  Rows need not be 16-byte aligned: a direct-to-LDS load
// of 16 bytes takes any 4-byte aligned address.
bool identity_dma_eligible(const MmlikeArgs &a)
{
    if (a.M <= 0 || a.N <= 0 || a.K < ID_BK || (a.kchunk < a.K && a.kchunk % ID_BK)) return false;
    if ((a.transA && a.M < 4) || (!a.transB && a.N < 4)) return false;
    // a k-minor slice spans up to 128 lines of the operand's storage, a k-major one 16
    const int64_t minor_max = (0x7FFFFFFFLL / 4 - 16) / 128, major_max = (0x7FFFFFFFLL / 4 - 128) / ID_BK;
    if (a.lda > (a.transA ? major_max : minor_max) || a.ldb > (a.transB ? minor_max : major_max)) return false;
    return true;
}

template <int NSTAGE, bool TA, bool TB, int BLK>
static hipError_t enqueue_layout(const MmlikeArgs &a, unsigned grid_x, unsigned grid_y, hipStream_t s)
{
    constexpr int LDS = NSTAGE * IdTile<BLK>::STAGE_BYTES;
    static hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void *>(&identity_mfma_dma_kernel<NSTAGE, TA, TB, BLK>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (granted != hipSuccess) return granted;
    hipLaunchKernelGGL((identity_mfma_dma_kernel<NSTAGE, TA, TB, BLK>), dim3(grid_x, grid_y), dim3(256), LDS, s, a);
    return hipSuccess;
}

template <int NSTAGE, int BLK>
static hipError_t enqueue_stages(const MmlikeArgs &a, unsigned grid_x, unsigned grid_y, hipStream_t s)
{
    if (a.transA && a.transB) return enqueue_layout<NSTAGE, true, true, BLK>(a, grid_x, grid_y, s);
    if (a.transA) return enqueue_layout<NSTAGE, true, false, BLK>(a, grid_x, grid_y, s);
    if (a.transB) return enqueue_layout<NSTAGE, false, true, BLK>(a, grid_x, grid_y, s);
    return enqueue_layout<NSTAGE, false, false, BLK>(a, grid_x, grid_y, s);
}

// Enqueues grid.x x grid.y workgroups of the streamed kernel (the caller has checked
// identity_dma_eligible and fills the split fields of `a` as for identity_mfma_kernel): tiles of
// `tile` = 128 rows and columns through a ring of 3 or 4 stages, or of 64 through a ring of
// ID_SMALL_STAGES.
hipError_t enqueue_identity_dma(const MmlikeArgs &a, int tile, int nstage, unsigned grid_x, unsigned grid_y, hipStream_t s)
{
    if (tile == 128 && nstage == 3) return enqueue_stages<3, 2>(a, grid_x, grid_y, s);
    if (tile == 128 && nstage == 4) return enqueue_stages<4, 2>(a, grid_x, grid_y, s);
    if (tile == 64 && nstage == ID_SMALL_STAGES) return enqueue_stages<ID_SMALL_STAGES, 1>(a, grid_x, grid_y, s);
    return hipErrorInvalidValue;
}

}  // namespace amulet
