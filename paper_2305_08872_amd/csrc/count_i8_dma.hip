// Join count on the int8 matrix cores, operands streamed HBM -> LDS directly
// (global_load_lds_dwordx4, gfx950) through a ring of NSTAGE LDS stages.
//
// Same arithmetic and fragment conventions as count_i8_mfma_kernel (count_i8.hip);
// what differs is the operand path.  No staging registers and no ds_write: each
// wave-level load instruction drops 64 x 16 bytes at LDS base + 16*lane, and every
// lane may fetch from any global address, so the LDS tiles are un-padded and
// XOR-swizzled at 16-byte granularity instead of padded:
//   A tile [128 rows][64 B]: row r keeps its logical 16-byte unit u at physical unit
//     u ^ ((r >> 2) & 3).  A ds_read_b128 is served 16 lanes (256 bytes, all 64 banks) per
//     clock, and 16 neighbouring rows fall in 16 distinct 16-byte bank groups:
//     4 * (r & 3) + (u ^ ((r >> 2) & 3)) runs through 0..15;
//   B tile [64 k][256 B]: row k keeps logical unit u at u ^ (2 * (k & 7)).  A 16-lane block of a
//     ds_read_b64_tr_b8 reads one logical unit of 8 consecutive rows and its neighbour block
//     the unit next to it (u ^ 1): the 16 (row, unit) pairs of two blocks fall in 16 distinct
//     bank groups.
// One barrier per stage, placed between the stage's two k-steps (see the main loop), with the
// loads of NSTAGE-2 later stages in flight behind it.
//
// Used only when the whole problem is interior: M a multiple of the tile height (128 or
// 256), N % 256 == 0, K % 64 == 0 and 16-byte aligned rows of A, B and R; every other case
// runs count_i8_mfma_kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "amulet_internal.h"

// the LDS-DMA asm below sets M0 itself and says so in its clobber list
#pragma clang diagnostic ignored "-Winline-asm"

namespace amulet {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) v2i *lds_v2i_ptr;
typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *glb_void_ptr;

constexpr int DM_BN = 256, DM_BK = 64;
constexpr int DM_B_BYTES = DM_BK * DM_BN;          // 16 KB = 16 wave-loads

// WR = rows of the 4-wide wave grid: the workgroup has 4 * WR waves, each owning a 64 x 64
// block of the (64 * WR) x 256 tile.  WR = 2: 128 x 256, 8 waves, 72 KB ring (two workgroups
// per compute unit); WR = 4: 256 x 256, 16 waves, 96 KB ring (one workgroup per compute unit,
// a third less operand traffic out of the L2 per multiply-add).
template <int WR, int NSTAGE>
struct DmaTile {
    static constexpr int BM = 64 * WR, NW = 4 * WR, NT = 64 * NW;
    static constexpr int A_BYTES = BM * DM_BK;          // one wave-load (1 KB) per 16 rows
    static constexpr int STAGE_BYTES = A_BYTES + DM_B_BYTES;
    static constexpr int B_LOADS = 16 / NW;             // B wave-loads per wave per stage
    static constexpr int LOADS = 1 + B_LOADS;           // DMA instructions per wave per stage
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
};

// the operand ring (and, after the K loop, the image the result tile is transposed through)
extern __shared__ __attribute__((aligned(16))) int8_t dma_smem[];

// What a persistent workgroup knows of the item it will run after the current one.
struct NextItem {
    int row0, col0, kb, K;   // K == 0: there is none
};

// One work item: the product of rows [row0, row0 + 64 WR) of A with columns [col0, col0 + 256) of B
// over k in [kb, kb + K), K a multiple of 64, added to that tile of R.  `ksplit`: several
// workgroups own the tile at once (split K) and add their parts with integer atomics.  All waves
// of the workgroup call it together.
// A persistent workgroup chains items: `ring0` is the ring slot that holds this item's stage 0,
// `pre` the number of its stages the item before already requested (0 for a first item), and
// when `next` names an item, this one requests the first stages of it (PREFETCH of them) into
// the half of the ring its own write-back does not use, right after its K loop, so that they
// arrive during the write-back instead of after it (`pre_assign`: the item before stored its sums
// without reading R, see the write-back).  Returns how many stages it requested for `next`.
template <int WR, int NSTAGE>
__device__ __forceinline__ int dma_item(const CountArgs &args, const int row0, const int col0, const int kb,
                                        const int K, const bool ksplit, const int ring0 = 0, const int pre = 0,
                                        const NextItem next = NextItem{0, 0, 0, 0}, const bool pre_assign = false)
{
    typedef DmaTile<WR, NSTAGE> T;
    static_assert(NSTAGE >= 3 && NSTAGE <= 5, "the wait counts are written for rings of 3 to 5 stages");
    constexpr int DM_A_BYTES = T::A_BYTES, DM_STAGE_BYTES = T::STAGE_BYTES;
    constexpr int NW = T::NW, B_LOADS = T::B_LOADS;
    static_assert(WR == 2 || WR == 4, "wave grid is 2 x 4 or 4 x 4");

    // The thread index is made opaque per item: everything derived from it is then recomputed at
    // the start of each item (a few vector instructions) instead of being hoisted out of a
    // persistent workgroup's item loop and held in registers, or spilled, across the K loop.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // WR x 4 grid
    const int wr = wave >> 2, wc = wave & 3;
    const int li = lane & 31, lh = lane >> 5;

    // ---- what each lane fetches: one A slot and B_LOADS B slots per stage ----------------
    // An address is a wave-uniform base in scalar registers (tile origin and stage, advanced on
    // the scalar unit) plus a 32-bit byte offset per lane that never changes (the launcher runs
    // this kernel only where those offsets fit: count_i8_dma_eligible).
    // A: wave w owns LDS slots [64w, 64w+64): slot s = 64w + lane -> row s/4, physical unit s%4
    const int a_row = wave * 16 + (lane >> 2);
    const int a_log = (lane & 3) ^ ((a_row >> 2) & 3);
    const uint32_t a_voff = (uint32_t)a_row * (uint32_t)args.lda + (uint32_t)(a_log * 16);
    const int8_t *const a_base = args.A + (int64_t)row0 * args.lda + kb;
    // B: wave w owns slot groups j = w (+ NW): slot s = 64j + lane -> k row s/16, physical unit s%16
    uint32_t b_voff[B_LOADS];
#pragma unroll
    for (int q = 0; q < B_LOADS; ++q) {
        const int krow = (wave + NW * q) * 4 + (lane >> 4);
        const int blog = (lane & 15) ^ ((krow & 7) << 1);
        b_voff[q] = (uint32_t)krow * (uint32_t)args.ldb + (uint32_t)(blog * 16);
    }
    const int8_t *const b_base = args.B + (int64_t)kb * args.ldb + col0;
    const int64_t b_stage = (int64_t)DM_BK * args.ldb;

    // The loads are written as asm so that the compiler's wait-count pass does not see a
    // vector-memory instruction writing LDS: it would otherwise drain ALL outstanding loads
    // (vmcnt(0)) before every LDS read, which serialises the ring.  Completion is tracked by
    // hand below: s_waitcnt vmcnt(loads per stage) / vmcnt(0) before the stage's barrier.  M0 carries the
    // wave-uniform LDS destination; each lane's 16 bytes land at M0 + 16 * lane.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_ptr)dma_smem;
    auto dma16 = [&](const int8_t *base, uint32_t voff, uint32_t lds_addr) {
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(voff), "s"(base), "s"(lds_addr)
                     : "memory", "m0");
    };
    auto issue_from = [&](const int8_t *abase, const int8_t *bbase, int stage, int buf) {
        const uint32_t base = lds_base + (uint32_t)(buf * DM_STAGE_BYTES);
        dma16(abase + (int64_t)stage * DM_BK, a_voff, base + (uint32_t)wave * 1024u);
#pragma unroll
        for (int q = 0; q < B_LOADS; ++q)
            dma16(bbase + (int64_t)stage * b_stage, b_voff[q], base + (uint32_t)(DM_A_BYTES + (wave + NW * q) * 1024));
    };
    auto slot_of = [&](int stage) { return (ring0 + stage) % NSTAGE; };   // ring slot of a stage of this item
    auto issue = [&](int stage) { issue_from(a_base, b_base, stage, slot_of(stage)); };

    // ---- where each lane reads its fragments (byte offsets inside a stage) -----------------
    int a_off[2];   // per k-step of 32; the second row block is + 32 rows = + 2048 bytes
#pragma unroll
    for (int ksi = 0; ksi < 2; ++ksi) {
        const int row = wr * 64 + li;
        const int phys = (2 * ksi + lh) ^ ((row >> 2) & 3);
        a_off[ksi] = row * DM_BK + phys * 16;
    }
    const int tb = lane >> 4, ts = lane & 15;   // transpose-read block and slot (see count_i8.hip)
    int b_off[2];   // per column block; + 8 k rows = + 2048, + 32 k rows (next k-step) = + 8192
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        const int krow = 16 * (tb >> 1) + (ts >> 1);
        const int colbyte = (wc * 2 + ni) * 32 + 16 * (tb & 1) + 8 * (ts & 1);
        const int phys = (colbyte >> 4) ^ ((krow & 7) << 1);
        b_off[ni] = DM_A_BYTES + krow * DM_BN + phys * 16 + (colbyte & 15);
    }

    v16i acc[2][2];

    // One fragment set = the operands of one k-step of 32: two A row blocks, two B column blocks.
    auto read_frags = [&](int buf, int ksi, v4i (&a)[2], v4i (&b)[2]) {
        const int8_t *st = dma_smem + buf * DM_STAGE_BYTES;
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
            a[mi] = *(const v4i *)(st + a_off[ksi] + mi * 2048);
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int8_t *p = st + b_off[ni] + ksi * 8192;
            const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)p);
            const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(p + 2048));
            b[ni] = v4i{lo.x, lo.y, hi.x, hi.y};
        }
    };
    auto mma = [&](const v4i (&a)[2], const v4i (&b)[2]) {
#pragma unroll
        for (int mi = 0; mi < 2; ++mi)
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                acc[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
    };
    // Wait until the loads of stage `t` of this item have landed.  Vector memory operations
    // retire in the order they were issued, so this is a wait until at most as many are
    // outstanding as were issued after that stage's: T::LOADS per later stage requested so far
    // (`upto`: the last one), and, for a stage the item before requested, the EXTRA operations
    // of that item's write-back, all of which came after the request.
    constexpr int PREFETCH = 2;                     // stages requested for the next item
    // (the write-back reads R in groups of WB_GROUP rows per wave, WB_DEPTH groups ahead; 8 waves
    // have registers for one group only)
    constexpr int WB_GROUP = 4, WB_DEPTH = WR == 4 ? 2 : 1;
    constexpr int EXTRA = 2 * WR * (64 / NW) - WB_DEPTH * WB_GROUP;   // per wave: a tile's loads and stores of R rows, less the loads that precede the request
    constexpr int EXTRA_ASSIGN = WR * (64 / NW);                      // the stores alone, when the item before did not read R
    static_assert(T::LOADS * (NSTAGE - 2) + EXTRA <= 63, "the wait count is a 6-bit field");
    auto wait_stage = [&](int t, int upto) {
        const int n = T::LOADS * (upto - t) + (t < pre ? (pre_assign ? EXTRA_ASSIGN : EXTRA) : 0);
        // (the count is an immediate operand: one instruction per value that can occur)
        switch (n) {
        case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
#define AMULET_WAIT_CASE(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
        AMULET_WAIT_CASE(2) AMULET_WAIT_CASE(3) AMULET_WAIT_CASE(4) AMULET_WAIT_CASE(6) AMULET_WAIT_CASE(9)
        AMULET_WAIT_CASE(16) AMULET_WAIT_CASE(18) AMULET_WAIT_CASE(19) AMULET_WAIT_CASE(20) AMULET_WAIT_CASE(22)
        AMULET_WAIT_CASE(24) AMULET_WAIT_CASE(26) AMULET_WAIT_CASE(28) AMULET_WAIT_CASE(30)
        AMULET_WAIT_CASE(56) AMULET_WAIT_CASE(59) AMULET_WAIT_CASE(62)
#undef AMULET_WAIT_CASE
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;   // never too little: waits for everything
        }
    };

    // The barrier of a stage sits BETWEEN its two k-steps, so that the wait for the other
    // waves and the latency of the LDS reads that follow it are covered by matrix-core work
    // already queued: when a wave reaches barrier s it holds the fragments of k-step 1 of
    // stage s in registers, and right after the barrier it issues the reads of k-step 0 of
    // stage s+1 and then runs k-step 1 of stage s while they land.
    // Barrier s certifies for all waves: the loads of stage s+1 have landed, and every read
    // of stage s-1 is complete (its last fragments were consumed before the barrier), so the
    // buffer of stage s-1 is refilled right after it with stage s+NSTAGE-1.
    const int n_stages = K / DM_BK;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0;
    int requested = pre;                          // stages of this item requested so far
#pragma unroll
    for (int d = 0; d < NSTAGE - 1; ++d)
        if (d >= pre && d < n_stages) { issue(d); requested = d + 1; }
    wait_stage(0, requested - 1);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    v4i fa0[2], fb0[2], fa1[2], fb1[2];
    int buf = ring0;                              // ring slot of stage s
    int ibuf = ring0 == 0 ? NSTAGE - 1 : ring0 - 1;   // ring slot the next request goes to: the one stage s-1 has left
    read_frags(buf, 0, fa0, fb0);
    // One iteration: k-step 0 of stage s, the wait for stage s+1 and the barrier, the request for
    // stage s+NSTAGE-1, k-step 1 of stage s.  STEADY: the common iteration (stage s+1 is this
    // item's own request, a later stage is still to be requested: one constant wait count, no
    // case distinction), kept apart from the few first and last ones so that the loop that runs
    // nearly all of K stays short.
    auto iteration = [&](int s, auto steady) {
        constexpr bool STEADY = decltype(steady)::value;
        const int nbuf = buf == NSTAGE - 1 ? 0 : buf + 1;
        read_frags(buf, 1, fa1, fb1);
        mma(fa0, fb0);
        __builtin_amdgcn_sched_barrier(0);
        // requested so far: stages up to min(s+NSTAGE-2, n_stages-1); stage s+1 must have landed
        if constexpr (STEADY) {
            if constexpr (T::LOADS * (NSTAGE - 3) == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
            else if constexpr (T::LOADS * (NSTAGE - 3) == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            else wait_stage(s + 1, s + NSTAGE - 2);
        } else {
            const int last = s + NSTAGE - 2 < n_stages - 1 ? s + NSTAGE - 2 : n_stages - 1;
            wait_stage(s + 1, last);
        }
        // A bare s_barrier: the full fence of __syncthreads() would drain the loads in flight.
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (STEADY || s + NSTAGE - 1 < n_stages) issue_from(a_base, b_base, s + NSTAGE - 1, ibuf);   // into the slot stage s-1 has left
        read_frags(nbuf, 0, fa0, fb0);
        __builtin_amdgcn_sched_barrier(0);
        mma(fa1, fb1);
        ibuf = buf;
        buf = nbuf;
    };
    const int steady_end = n_stages - (NSTAGE - 1);   // first s that requests nothing more
    int s = 0;
    for (; s < pre && s + 1 < n_stages; ++s) iteration(s, std::false_type());
    for (; s < steady_end; ++s) iteration(s, std::true_type());
    for (; s + 1 < n_stages; ++s) iteration(s, std::false_type());
    // last stage: nothing left to wait for or to fetch
    read_frags(buf, 1, fa1, fb1);
    mma(fa0, fb0);
    mma(fa1, fb1);

    // ---- write-back through LDS: R += acc as whole 1 KB rows ----------------------------------
    // Accumulator element v of lane l is R[8*(v/4) + 4*(l/32) + v%4][l%32] of its 32x32 block: a
    // lane holds one column.  The operand ring is free now, so the tile is transposed through it
    // in WR parts of 64 rows x 256 columns: the waves owning the part scatter their accumulators
    // into a row-major image, then all waves add it to R with 16-byte accesses, one full 1 KB
    // tile row per wave instruction.
    // The image has no padding (64 rows x 1 KB: the first 64 KB of the ring, which leaves the rest
    // of the ring to the next item's first stages): the two half-waves of a scatter store write
    // rows 4 apart, which fall on the same banks, so every other group of four rows is kept with
    // its two 128-byte halves of each 256-byte bank row exchanged (column ^ 32): the 64 lanes of a
    // store hit 64 distinct banks, and a row is still read back as whole 16-byte units.
    constexpr int IMG_PITCH = DM_BN;
    static_assert(64 * IMG_PITCH * 4 <= NSTAGE * DM_STAGE_BYTES, "the image must fit in the ring");
    static_assert(64 * IMG_PITCH * 4 + PREFETCH * DM_STAGE_BYTES <= NSTAGE * DM_STAGE_BYTES || WR == 2,
                  "the image and the next item's first stages share the ring");
    auto img_swz = [](int r) { return ((r >> 2) & 1) << 5; };
    constexpr int ROWS_PER_WAVE = 64 / NW;
    int32_t *const img = (int32_t *)dma_smem;
    // The write-back is a chain of round trips to HBM (read the rows of R, add, store), and it is
    // short only if many of them are in flight at once.  R has one owner, so its rows may be read
    // as early as registers allow: the fragment registers are free once the last matrix
    // instruction has issued, which is room for DEPTH groups of four rows per wave.  Those are
    // requested before the first part's scatter and barriers, and each group's registers are
    // refilled with the rows DEPTH groups later as soon as its sums are formed.
    constexpr int GROUP = WB_GROUP, GROUPS = ROWS_PER_WAVE / GROUP, NGROUPS = WR * GROUPS, DEPTH = WB_DEPTH;
    static_assert(ROWS_PER_WAVE % GROUP == 0, "a wave's rows of a part come in groups of four");
    v4i rbuf[DEPTH][GROUP];
    // group q of the tile: part q / GROUPS, rows (q % GROUPS) * GROUP .. + GROUP - 1 of this wave's share.
    // A row's address is a wave-uniform base (scalar registers) plus 16 bytes per lane.
    const uint32_t lane16 = (uint32_t)lane * 16u;
    auto r_row = [&](int q, int j) {
        const int row = (q / GROUPS) * 64 + wave * ROWS_PER_WAVE + (q % GROUPS) * GROUP + j;
        char *base = (char *)(args.R + (int64_t)(row0 + row) * args.ldr + col0);   // uniform over the wave
        return (v4i *)(base + lane16);
    };
    // R = the counts (no R +=): this item's sums replace what R holds, when it owns the tile alone
    // and starts the tile's k range (a persistent workgroup's second pass over its first tile adds
    // to what its first pass stored).  The rows of R are then not read at all; the item after this
    // one is told so (`pre_assign`), because the waits for the stages requested below count the
    // vector memory operations issued behind the request.
    const bool assign = args.assign && kb == 0 && !ksplit;
    if (!ksplit && !assign) {
#pragma unroll
        for (int q = 0; q < DEPTH && q < NGROUPS; ++q)
#pragma unroll
            for (int j = 0; j < GROUP; ++j) rbuf[q][j] = __builtin_nontemporal_load(r_row(q, j));
    }
    int next_requested = 0;
#pragma unroll
    for (int part = 0; part < WR; ++part) {
        __builtin_amdgcn_s_barrier();          // the ring (or the previous part's image) is no longer read
        asm volatile("" ::: "memory");
        if (part == 0 && next.K > 0) {
            // the next item's first stages, into the ring slots behind the image; that item
            // then starts at slot NSTAGE - PREFETCH
            const int8_t *const an = args.A + (int64_t)next.row0 * args.lda + next.kb;
            const int8_t *const bn = args.B + (int64_t)next.kb * args.ldb + next.col0;
#pragma unroll
            for (int d = 0; d < PREFETCH; ++d)
                if (d * DM_BK < next.K) { issue_from(an, bn, d, NSTAGE - PREFETCH + d); next_requested = d + 1; }
        }
        if (wr == part) {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int r = mi * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                        img[r * IMG_PITCH + (((wc * 2 + ni) * 32 + li) ^ img_swz(r))] = acc[mi][ni][v];
                    }
        }
        // The image is complete for everyone once each wave's LDS writes are done: wait for those
        // only.  (__syncthreads() is a full fence: it would also wait for the rows of R already
        // requested from HBM, and put their latency back into every part.)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (ksplit) {
#pragma unroll
            for (int j = 0; j < ROWS_PER_WAVE; ++j) {
                const int r = wave * ROWS_PER_WAVE + j;           // row of the part this wave adds
                // several workgroups own this tile: integer atomic adds (exact in any order),
                // 256 contiguous bytes per wave instruction
                int32_t *drow = args.R + (int64_t)(row0 + part * 64 + r) * args.ldr + col0;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    atomicAdd(drow + e * 64 + lane, img[r * IMG_PITCH + ((e * 64 + lane) ^ img_swz(r))]);
            }
            continue;
        }
#pragma unroll
        for (int grp = 0; grp < GROUPS; ++grp) {
            const int q = part * GROUPS + grp;
#pragma unroll
            for (int j = 0; j < GROUP; ++j) {
                const int ir = wave * ROWS_PER_WAVE + grp * GROUP + j;
                const v4i part4 = *(const v4i *)(img + ir * IMG_PITCH + ((lane * 4) ^ img_swz(ir)));
                if (assign) {
                    __builtin_nontemporal_store(part4, r_row(q, j));
                    continue;
                }
                v4i cur = rbuf[q % DEPTH][j];
                cur.x = (int)((uint32_t)cur.x + (uint32_t)part4.x);
                cur.y = (int)((uint32_t)cur.y + (uint32_t)part4.y);
                cur.z = (int)((uint32_t)cur.z + (uint32_t)part4.z);
                cur.w = (int)((uint32_t)cur.w + (uint32_t)part4.w);
                __builtin_nontemporal_store(cur, r_row(q, j));
                if (q + DEPTH < NGROUPS) rbuf[q % DEPTH][j] = __builtin_nontemporal_load(r_row(q + DEPTH, j));   // this register's next row
            }
        }
    }
    return next_requested;
}

template <int WR, int NSTAGE>
__global__ void __launch_bounds__(256 * WR) __attribute__((amdgpu_waves_per_eu(4, 4)))
count_i8_dma_kernel(const CountArgs args)
{
    typedef DmaTile<WR, NSTAGE> T;
    // Split K (gridDim.y > 1, chosen by the host when the tiles are too few to fill the chip):
    // this workgroup multiplies k in [kb, kb + kchunk) only and adds its part to R atomically.
    const bool ksplit = gridDim.y > 1;
    const int kb = ksplit ? (int)blockIdx.y * args.kchunk : 0;
    const int K = ksplit ? ((args.K - kb < args.kchunk) ? args.K - kb : args.kchunk) : args.K;
    // XCD-aware tile order (xcd_tile in amulet_internal.h)
    const int tiles_m = args.M / T::BM, tiles_n = args.N / DM_BN;
    int tm, tn;
    if (!xcd_tile((int)blockIdx.x + args.block_base, tiles_m, tiles_n, tm, tn)) return;   // padding: the whole workgroup leaves
    (void)dma_item<WR, NSTAGE>(args, tm * T::BM, tn * DM_BN, kb, K, ksplit);
}

// Persistent form: one launch of as many workgroups as the chip holds at once (a compute unit
// holds one 256 x 256 workgroup or two 128 x 256 ones), each walking its share of its XCD's part
// of the tile order: workgroup b (XCD b % 8, slot b / 8 of n_slots) takes the places slot,
// slot + n_slots, ... of that part, so the workgroups resident on an XCD at any moment still
// form the compact block of R that shares A rows and B columns through that L2.
//
// What the loop is for: all tiles take equally long, so workgroups launched together reach their
// write-back together, and the launch alternates between a phase in which only the matrix cores
// work and one in which only the memory system does (the read-modify-write of R ran at HBM
// speed for a third of the launch, with the matrix cores idle).  Here a workgroup's first item is
// only a leading part of its first tile's k range, and the rest of that range is its last item
// (same owner, plain adds: "+=" makes a tile in two passes as good as in one), so that from then
// on workgroups of different phases write back at different times.  The phases: odd XCDs half a
// tile behind even ones, and within an XCD the slots in eight groups two stages (about a
// microsecond) apart -- close enough in k that the groups still find each other's operand lines
// in the L2 (workgroups half a tile apart do not: the L2 holds about twenty stages of an XCD's
// traffic), far enough that their write-backs do not start together.  Measured (ms; no phases /
// halves of an XCD's slots half a tile apart and XCD pairs a quarter / this arrangement):
// 8192 x 8192 x 4096 0.236 / 0.2215 / 0.2125, x 1024 0.132 / 0.135 / 0.124, x 8192 0.373 / 0.356 / 0.343,
// 16384 x 8192 x 4096 0.447 / 0.430 / 0.395, 16384 x 16384 x 4096 0.834 / 0.820 / 0.832.
template <int WR, int NSTAGE>
__global__ void __launch_bounds__(256 * WR) __attribute__((amdgpu_waves_per_eu(4, 4)))
count_i8_dma_persistent_kernel(const CountArgs args)
{
    typedef DmaTile<WR, NSTAGE> T;
    const int tiles_m = args.M / T::BM, tiles_n = args.N / DM_BN;
    const int xcd = (int)blockIdx.x & 7, slot = (int)blockIdx.x >> 3, n_slots = (int)gridDim.x >> 3;
    const int places = (int)xcd_places(tiles_m, tiles_n);   // places of one XCD's share (the last may hold no tile)
    auto tile_at = [&](int place, int &row0, int &col0) {
        int tm, tn;
        const bool real = xcd_tile(place * 8 + xcd, tiles_m, tiles_n, tm, tn);
        row0 = tm * T::BM;
        col0 = tn * DM_BN;
        return real;
    };
    const int n_st = args.K / DM_BK;             // stages of a tile's k range
    int phase = (slot * args.pers_groups / n_slots) * args.pers_group_stages;   // in stages
    if (args.pers_xcds > 1) phase += (int)((int64_t)n_st * ((xcd % args.pers_xcds) * args.pers_xcd_span / args.pers_xcds) / 16);
    const int kq = (phase % n_st) * DM_BK;
    int row0, col0;
    const int n_mine = slot < places ? (places - slot + n_slots - 1) / n_slots : 0;   // places slot, slot + n_slots, ...
    const bool split_first = kq > 0 && n_mine > 0 && tile_at(slot, row0, col0);
    const int n_steps = n_mine + (split_first ? 1 : 0);
    // item `step` of this workgroup (false: that place is padding)
    auto item_at = [&](int step, NextItem &it) {
        int place = slot + step * n_slots;
        it.kb = 0;
        it.K = args.K;
        if (split_first && step == 0) it.K = kq;
        if (split_first && step == n_mine) { place = slot; it.kb = kq; it.K = args.K - kq; }
        return tile_at(place, it.row0, it.col0);
    };
    auto next_real = [&](int step, NextItem &it) {   // first real item from `step` on, or n_steps
        while (step < n_steps && !item_at(step, it)) ++step;
        if (step >= n_steps) it.K = 0;
        return step;
    };
    NextItem cur, nxt;
    int step = next_real(0, cur);
    int ring0 = 0, pre = 0;
    bool pre_assign = false;
    while (step < n_steps) {
        const int nstep = next_real(step + 1, nxt);
        const int req = dma_item<WR, NSTAGE>(args, cur.row0, cur.col0, cur.kb, cur.K, false, ring0, pre, nxt, pre_assign);
        pre_assign = args.assign && cur.kb == 0;
        __builtin_amdgcn_s_barrier();            // every wave is done with the image: the ring is the next item's
        ring0 = req > 0 ? NSTAGE - 2 : 0;
        pre = req;
        cur = nxt;
        step = nstep;
    }
}

// True when the direct-to-LDS kernel with a (64 * wr) x 256 tile may run this problem
// (everything interior and aligned).
bool count_i8_dma_eligible(const CountArgs &a, int wr)
{
    // a lane's fixed byte offset from its tile's origin must fit 31 bits (kept clear of the sign
    // bit): the tile's last row of A, the stage's last k row of B
    const bool offsets_fit = a.lda <= (int64_t)(0x7FFFFFFF - 64) / (64 * wr) && a.ldb <= (int64_t)(0x7FFFFFFF - 256) / DM_BK;
    return offsets_fit && a.vecA && a.vecB && a.vecR && a.M % (64 * wr) == 0 && a.N % DM_BN == 0 && a.K % DM_BK == 0;
}

template <int WR, int NSTAGE>
static hipError_t launch_dma(const CountArgs &a, hipStream_t s)
{
    typedef DmaTile<WR, NSTAGE> T;
    const int64_t tiles_m = a.M / T::BM, tiles_n = a.N / DM_BN;
    const int64_t grid = xcd_grid(tiles_m, tiles_n);
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    static hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void *>(&count_i8_dma_kernel<WR, NSTAGE>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    if (granted != hipSuccess) return granted;
    // too few tiles to give every SIMD two waves: split K over several workgroups per tile
    // (at least 512 k each), which add their parts to R with integer atomics
    CountArgs b = a;
    int splits = 1;
    b.kchunk = a.K;
    const int64_t waves = tiles_m * tiles_n * T::NW;
    if (waves < 2048 && a.K >= 1024) {
        int64_t want = (2048 + waves - 1) / waves;
        if (want > a.K / 512) want = a.K / 512;
        if (want > 1024) want = 1024;
        const int64_t chunk = ((a.K + want - 1) / want + DM_BK - 1) / DM_BK * DM_BK;
        b.kchunk = (int)chunk;
        splits = (int)((a.K + chunk - 1) / chunk);
    }
    if (splits > 1 && a.assign) {   // several workgroups add into a tile: from zero
        const hipError_t ez = launch_zero_r_i32(a, s);
        if (ez != hipSuccess) return ez;
        b.assign = 0;
    }
    return launch_row_of_blocks(b, grid, T::NT, [&](unsigned n) {
        hipLaunchKernelGGL((count_i8_dma_kernel<WR, NSTAGE>), dim3(n, (unsigned)splits), dim3(T::NT), T::LDS_BYTES, s, b);
    });
}

// Workgroups of the persistent form: what one XCD holds at once (its share of the compute units
// times the workgroups one unit holds: one of 256 x 256, two of 128 x 256), times 8.  Zero when the
// persistent form does not apply: every workgroup should have at least two tiles to walk, and the
// launch must fit one grid.
template <int WR>
static int64_t persistent_grid(const CountArgs &a)
{
    const int64_t tiles_m = a.M / (64 * WR), tiles_n = a.N / DM_BN;
    const int64_t places = xcd_places(tiles_m, tiles_n);
    const int64_t slots = (int64_t)(compute_units() / 8) * (WR == 4 ? 1 : 2);
    if (slots <= 0 || places < 2 * slots || a.K < 2 * DM_BK) return 0;
    return 8 * slots;
}

template <int WR, int NSTAGE>
static hipError_t launch_dma_persistent(const CountArgs &a, hipStream_t s)
{
    typedef DmaTile<WR, NSTAGE> T;
    const int64_t grid = persistent_grid<WR>(a);
    if (grid == 0) return launch_dma<WR, NSTAGE>(a, s);
    static hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void *>(&count_i8_dma_persistent_kernel<WR, NSTAGE>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    if (granted != hipSuccess) return granted;
    CountArgs b = a;
    b.kchunk = a.K;
    b.block_base = 0;
    if (forced_launch_failure()) return hipErrorLaunchFailure;
    hipLaunchKernelGGL((count_i8_dma_persistent_kernel<WR, NSTAGE>), dim3((unsigned)grid), dim3(T::NT), T::LDS_BYTES, s, b);
    return hipGetLastError();
}

hipError_t launch_count_i8_dma(const CountArgs &a, int wr, hipStream_t s, bool persistent)
{
    if (wr == 4) return persistent ? launch_dma_persistent<4, 4>(a, s) : launch_dma<4, 4>(a, s);
    return launch_dma<2, 3>(a, s);
}

}  // namespace amulet
