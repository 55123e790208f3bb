// Join count on the int8 matrix cores, operands streamed HBM -> LDS directly
// (global_load_lds_dwordx4, gfx950) through a ring of NSTAGE LDS stages.
//
// Same arithmetic and fragment conventions as count_i8_mfma_kernel (count_i8.hip);
// what differs is the operand path.  No staging registers and no ds_write: each
// wave-level load instruction drops 64 x 16 bytes at LDS base + 16*lane, and every
// lane may fetch from any global address, so the LDS tiles are un-padded and
// XOR-swizzled at 16-byte granularity instead of padded:
//   A tile [128 rows][64 B]: row r keeps its logical 16-byte unit u at physical unit
//     u ^ ((r >> 1) & 3), so the ds_read_b128 of 8 neighbouring rows fall in 8 distinct
//     bank groups;
//   B tile [64 k][256 B]: row k keeps logical unit u at u ^ (k & 7), so the 8 rows a
//     ds_read_b64_tr_b8 block reads (same logical unit) fall in 8 distinct bank groups.
// With the loads of NSTAGE-1 stages in flight and one barrier per stage, the wait for a
// stage's data is the wait for loads issued two stages of arithmetic earlier.
//
// Used only when the whole problem is interior: M % 128 == 0, N % 256 == 0,
// K % 64 == 0 and 16-byte aligned rows of A, B and R; every other case runs
// count_i8_mfma_kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

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

constexpr int DM_BM = 128, DM_BN = 256, DM_BK = 64;
constexpr int DM_A_BYTES = DM_BM * DM_BK;          // 8 KB  = 8 wave-loads
constexpr int DM_B_BYTES = DM_BK * DM_BN;          // 16 KB = 16 wave-loads
constexpr int DM_STAGE_BYTES = DM_A_BYTES + DM_B_BYTES;

template <int NSTAGE>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4, 4)))
count_i8_dma_kernel(const CountArgs args)
{
    static_assert(NSTAGE == 3, "the wait counts below are written for a ring of three stages");
    extern __shared__ __attribute__((aligned(16))) int8_t dma_smem[];

    const int K = args.K;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // 0..7, 2 x 4 grid
    const int wr = wave >> 2, wc = wave & 3;
    const int li = lane & 31, lh = lane >> 5;

    // XCD-aware tile order (see count_i8.hip)
    const int tiles_m = args.M / DM_BM, tiles_n = args.N / DM_BN;
    const int band = (tiles_n + 7) / 8;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int tn = xcd * band + slot % band;
    const int tm = slot / band;
    if (tn >= tiles_n || tm >= tiles_m) return;
    const int row0 = tm * DM_BM, col0 = tn * DM_BN;

    // ---- what each lane fetches: one A slot and two B slots per stage ------------------
    // A: wave w owns LDS slots [64w, 64w+64): slot s = 64w + lane -> row s/4, physical unit s%4
    const int a_row = wave * 16 + (lane >> 2);
    const int a_log = (lane & 3) ^ ((a_row >> 1) & 3);
    const int8_t *ga = args.A + (int64_t)(row0 + a_row) * args.lda + a_log * 16;
    // B: wave w owns slot groups j = w and w + 8: slot s = 64j + lane -> k row s/16, physical unit s%16
    const int8_t *gb[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int krow = (wave + 8 * q) * 4 + (lane >> 4);
        const int blog = (lane & 15) ^ (krow & 7);
        gb[q] = args.B + (int64_t)krow * args.ldb + col0 + blog * 16;
    }
    const int64_t b_stage = (int64_t)DM_BK * args.ldb;

    // The loads are written as asm so that the compiler's wait-count pass does not see a
    // vector-memory instruction writing LDS: it would otherwise drain ALL outstanding loads
    // (vmcnt(0)) before every LDS read, which serialises the ring.  Completion is tracked by
    // hand below: s_waitcnt vmcnt(3) / vmcnt(0) before the stage's barrier.  M0 carries the
    // wave-uniform LDS destination; each lane's 16 bytes land at M0 + 16 * lane.
    const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_void_ptr)dma_smem;
    auto dma16 = [&](const int8_t *g, uint32_t lds_addr) {
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                     :
                     : "v"(g), "s"(lds_addr)
                     : "memory", "m0");
    };
    auto issue = [&](int stage, int buf) {
        const uint32_t base = lds_base + (uint32_t)(buf * DM_STAGE_BYTES);
        dma16(ga + (int64_t)stage * DM_BK, base + (uint32_t)wave * 1024u);
#pragma unroll
        for (int q = 0; q < 2; ++q)
            dma16(gb[q] + (int64_t)stage * b_stage, base + (uint32_t)(DM_A_BYTES + (wave + 8 * q) * 1024));
    };

    // ---- where each lane reads its fragments (byte offsets inside a stage) -----------------
    int a_off[2];   // per k-step of 32; the second row block is + 32 rows = + 2048 bytes
#pragma unroll
    for (int ksi = 0; ksi < 2; ++ksi) {
        const int row = wr * 64 + li;
        const int phys = (2 * ksi + lh) ^ ((row >> 1) & 3);
        a_off[ksi] = row * DM_BK + phys * 16;
    }
    const int tb = lane >> 4, ts = lane & 15;   // transpose-read block and slot (see count_i8.hip)
    int b_off[2];   // per column block; + 8 k rows = + 2048, + 32 k rows (next k-step) = + 8192
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
        const int krow = 16 * (tb >> 1) + (ts >> 1);
        const int colbyte = (wc * 2 + ni) * 32 + 16 * (tb & 1) + 8 * (ts & 1);
        const int phys = (colbyte >> 4) ^ (krow & 7);
        b_off[ni] = DM_A_BYTES + krow * DM_BN + phys * 16 + (colbyte & 15);
    }

    v16i acc[2][2];
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0;

    const int n_stages = K / DM_BK;
    issue(0, 0);
    if (n_stages > 1) issue(1, 1);

    int buf = 0;
    for (int s = 0; s < n_stages; ++s) {
        // this wave's loads of stage s have landed once at most the 3 loads of stage s+1 are pending
        if (s + 1 < n_stages)
            asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
        else
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        // ... and so have every other wave's after the barrier.  A bare s_barrier: every LDS read
        // of the previous stage was already waited for by the MFMAs that consumed it, and the
        // full fence of __syncthreads() would drain the loads in flight for the next stages.
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // the buffer of stage s-1 is free now (all waves are past its arithmetic): refill it
        if (s + 2 < n_stages) issue(s + 2, buf == 0 ? 2 : buf - 1);
        const int8_t *st = dma_smem + buf * DM_STAGE_BYTES;
#pragma unroll
        for (int ksi = 0; ksi < 2; ++ksi) {
            v4i a[2], b[2];
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
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
        }
        buf = buf == 2 ? 0 : buf + 1;
    }

    // ---- write-back through LDS: R += acc as whole 1 KB rows ----------------------------------
    // Accumulator element v of lane l is R[8*(v/4) + 4*(l/32) + v%4][l%32] of its 32x32 block: a
    // lane holds one column.  The operand ring is free now, so the tile is transposed through it
    // in two halves of 64 rows x 256 columns (64 KB): the waves owning the half scatter their
    // accumulators into a row-major image, then all 8 waves add it to R with 16-byte accesses,
    // one full 1 KB tile row per wave instruction.
    int32_t *const img = (int32_t *)dma_smem;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        __builtin_amdgcn_s_barrier();          // the ring (or the previous half's image) is no longer read
        asm volatile("" ::: "memory");
        if (wr == half) {
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int r = mi * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                        img[r * DM_BN + (wc * 2 + ni) * 32 + li] = acc[mi][ni][v];
                    }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = wave * 8 + j;           // row of the half this wave adds
            const v4i part = *(const v4i *)(img + r * DM_BN + lane * 4);
            v4i *dst = (v4i *)(args.R + (int64_t)(row0 + half * 64 + r) * args.ldr + col0 + lane * 4);
            v4i cur = *dst;
            cur.x = (int)((uint32_t)cur.x + (uint32_t)part.x);
            cur.y = (int)((uint32_t)cur.y + (uint32_t)part.y);
            cur.z = (int)((uint32_t)cur.z + (uint32_t)part.z);
            cur.w = (int)((uint32_t)cur.w + (uint32_t)part.w);
            *dst = cur;
        }
    }
}

// True when the direct-to-LDS kernel may run this problem (everything interior and aligned).
bool count_i8_dma_eligible(const CountArgs &a)
{
    return a.vecA && a.vecB && a.vecR && a.M % DM_BM == 0 && a.N % DM_BN == 0 && a.K % DM_BK == 0;
}

hipError_t launch_count_i8_dma(const CountArgs &a, hipStream_t s)
{
    constexpr int LDS = 3 * DM_STAGE_BYTES;   // 72 KB: two workgroups per compute unit
    const int64_t tiles_m = a.M / DM_BM, tiles_n = a.N / DM_BN;
    const int64_t grid = 8 * ((tiles_n + 7) / 8) * tiles_m;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    static hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void *>(&count_i8_dma_kernel<3>),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (granted != hipSuccess) return granted;
    hipLaunchKernelGGL((count_i8_dma_kernel<3>), dim3((unsigned)grid), dim3(512), LDS, s, a);
    return hipGetLastError();
}

}  // namespace amulet
