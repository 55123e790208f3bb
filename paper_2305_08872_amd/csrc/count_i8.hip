// Join count as a matrix product on int8 indicator matrices:
// R[i][j] += sum_k A[i][k]*B[k][j], int32, exact (the join-as-matmul
// translation cited in the paper's introduction).  This is a dense
// contraction, so it runs on the int8 matrix cores
// (v_mfma_i32_32x32x32_i8: a 32 x 32 block of R advances 32 k per instruction).
//
// Workgroup = WR x WC waves; each wave owns MB x NB MFMA blocks.  K is
// staged 64 bytes at a time, global -> registers -> LDS, double buffered:
//   A tile [BM][64] keeps its global layout (k contiguous), row pitch 80 B so
//     the 16-byte fragment reads of 8 neighbouring lanes fall in distinct banks;
//   B tile [64][BN] ALSO keeps its global layout (n contiguous).  The matrix
//     core wants, per column, 16 consecutive k in one lane; that transposition
//     is done by the LDS itself with ds_read_b64_tr_b8 (gfx950): in each block
//     of 16 lanes, lane t supplies the address of 8 bytes and receives byte
//     t%8 of the 8 lanes of parity t/8.  Even lanes point at columns c..c+7 and
//     odd lanes at c+8..c+15 of 8 consecutive k rows, so lane t gets column
//     c+t, rows k..k+7: two such reads give a lane its 16 k.  No VALU work
//     and no scattered LDS writes are spent on the transpose.
//
// Fragment convention: lane l supplies row/column l % 32 and k-slot h = l / 32;
// byte t of slot h is k = 16h + t for both operands.
// Rows, columns and k beyond the matrix are zero-filled in LDS (a zero product
// adds nothing to an integer dot product).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "amulet_internal.h"

namespace amulet {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) v2i *lds_v2i_ptr;


// 16 bytes of a row starting at src; n_valid of them exist (the rest read as 0).
__device__ __forceinline__ v4i load16_i8(const int8_t *src, bool vec, int n_valid)
{
    v4i v = {0, 0, 0, 0};
    if (n_valid <= 0) return v;
    if (n_valid >= 16) {
        // 16 whole bytes in range: one vector load either way.  The second form tells the
        // compiler nothing about alignment; the target's global loads accept any address,
        // so it still becomes one 16-byte load (slower than an aligned one, far faster
        // than sixteen byte loads).
        if (vec) return *(const v4i *)src;
        typedef v4i v4i_anyaddr __attribute__((aligned(1)));
        return *(const v4i_anyaddr *)src;
    }
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    for (int t = 0; t < 16; ++t)
        if (t < n_valid) w[t >> 2] |= (uint32_t)(uint8_t)src[t] << (8 * (t & 3));
    v.x = (int)w[0]; v.y = (int)w[1]; v.z = (int)w[2]; v.w = (int)w[3];
    return v;
}

// The 16 bytes of v moved down by `shift` bytes (1 .. 15, the same for every lane), zeros coming
// in at the top.  A row's last, partial unit is loaded as the 16 bytes that end at the row's
// last byte (all inside the row) and moved down by the bytes it lacks.  (Byte by byte that unit
// costs up to fifteen loads, and a workgroup on the right-hand edge of B has one per k row: an
// 8192 x 8191 x 4096 count took 1.16 ms against 0.40 ms for 8192 x 8192.)
__device__ __forceinline__ v4i shift_down_i8(v4i l, int shift)
{
    const uint64_t lo = (uint64_t)(uint32_t)l.x | ((uint64_t)(uint32_t)l.y << 32);
    const uint64_t hi = (uint64_t)(uint32_t)l.z | ((uint64_t)(uint32_t)l.w << 32);
    const int sb = 8 * shift;                // 8 .. 120 bits
    uint64_t nlo, nhi;
    if (sb < 64) {
        nlo = (lo >> sb) | (hi << (64 - sb));
        nhi = hi >> sb;
    } else {
        nlo = hi >> (sb - 64);
        nhi = 0;
    }
    return v4i{(int)(uint32_t)nlo, (int)(uint32_t)(nlo >> 32), (int)(uint32_t)nhi, (int)(uint32_t)(nhi >> 32)};
}

// BK = bytes of k staged per barrier
template <int MB, int NB, int WR, int WC, int BK>
struct CountTile {
    static constexpr int CI_BK = BK, CI_APITCH = BK + 16;
    static constexpr int NT = 64 * WR * WC;
    static constexpr int BM = WR * MB * 32, BN = WC * NB * 32;
    static constexpr int BPITCH = BN + 32;
    static constexpr int A_BYTES = BM * CI_APITCH, B_BYTES = CI_BK * BPITCH;
    static constexpr int LDS_BYTES = 2 * (A_BYTES + B_BYTES);
};

// WPE: resident waves per SIMD the register allocation is held to (512 / WPE registers per lane)
template <int MB, int NB, int WR, int WC, int WPE, int BK>
__global__ void __launch_bounds__(64 * WR * WC)
__attribute__((amdgpu_waves_per_eu(WPE, WPE)))
count_i8_mfma_kernel(const CountArgs args)
{
    typedef CountTile<MB, NB, WR, WC, BK> T;
    constexpr int NT = T::NT, BM = T::BM, BN = T::BN, BPITCH = T::BPITCH;
    constexpr int CI_BK = BK, CI_APITCH = T::CI_APITCH;
    constexpr int AU = BK / 16;   // 16-byte slots per A row
    constexpr int A_UNITS = BM * (CI_BK / 16) / NT;   // 16-byte slots per thread per stage
    constexpr int B_UNITS = CI_BK * (BN / 16) / NT;
    static_assert(A_UNITS >= 1 && B_UNITS >= 1, "tile too small for the workgroup");
    static_assert(BM * (CI_BK / 16) % NT == 0 && CI_BK * (BN / 16) % NT == 0, "slots must split evenly");

    // dynamic LDS: [2][BM][CI_APITCH] for A, then [2][CI_BK][BPITCH] for B
    extern __shared__ __attribute__((aligned(16))) int8_t count_smem[];
    int8_t *const As = count_smem;
    int8_t *const Bs = count_smem + 2 * T::A_BYTES;

    const int M = args.M, N = args.N;
    int K = args.K;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wr = wave / WC, wc = wave % WC;
    const int li = lane & 31, lh = lane >> 5;

    // XCD-aware tile order (xcd_tile in amulet_internal.h): each XCD walks its own rectangular
    // part of the tile grid, so its resident workgroups share A rows and B columns through its L2
    const int tiles_m = (M + BM - 1) / BM;
    const int tiles_n = (N + BN - 1) / BN;
    int tm, tn;
    if (!xcd_tile((int)blockIdx.x + args.block_base, tiles_m, tiles_n, tm, tn)) return;   // padding: the whole workgroup leaves
    const int row0 = tm * BM, col0 = tn * BN;
    const bool vecA = args.vecA != 0, vecB = args.vecB != 0;

    // Staging slots: thread t, pass `it` handles 16-byte slot u = t + 256*it of each tile.
    // Interior workgroups (tile inside the matrix, 16-byte aligned rows) run a branch-free
    // loader off pointers that only advance by one stage per iteration; edge tiles and
    // unaligned operands take the guarded byte-wise loader.
    const bool interior = vecA && vecB && row0 + BM <= args.Mload && col0 + BN <= args.Nload &&
                          (int64_t)BM * args.lda < 0x7fffffffLL && (int64_t)CI_BK * args.ldb < 0x7fffffffLL;
    // interior path: buffer loads off a wave-uniform base that advances with k plus a fixed
    // 32-bit per-thread byte offset, so the address arithmetic stays on the scalar unit
    // (vector-ALU instructions share the issue port with the MFMAs)
    // Split K (gridDim.y > 1, chosen by the host when the tiles are too few to fill the chip):
    // this workgroup multiplies k in [kb, kb + kchunk) only and adds its part to R atomically.
    const bool ksplit = gridDim.y > 1;
    const int8_t *Ag = args.A, *Bg = args.B;
    if (ksplit) {
        const int kb = (int)blockIdx.y * args.kchunk;
        Ag += kb;
        Bg += (int64_t)kb * args.ldb;
        K = (K - kb < args.kchunk) ? K - kb : args.kchunk;
    }
    // bytes in the last, partial 16-byte unit of a row of B, for the workgroups whose tile holds it
    const int tail_n = __builtin_amdgcn_readfirstlane(col0 + BN > N ? (N & 15) : 0);
    const int8_t *const a_base = Ag + (int64_t)row0 * args.lda;
    const int8_t *const b_base = Bg + col0;
    unsigned offa[A_UNITS], offb[B_UNITS];
    int8_t *la[A_UNITS];
    int8_t *lb[B_UNITS];
#pragma unroll
    for (int it = 0; it < A_UNITS; ++it) {
        const int u = tid + it * NT;
        offa[it] = (unsigned)(u / AU) * (unsigned)args.lda + (unsigned)(u % AU) * 16u;
        la[it] = As + (u / AU) * CI_APITCH + (u % AU) * 16;
    }
#pragma unroll
    for (int it = 0; it < B_UNITS; ++it) {
        const int u = tid + it * NT;
        offb[it] = (unsigned)(u / (BN / 16)) * (unsigned)args.ldb + (unsigned)(u % (BN / 16)) * 16u;
        lb[it] = Bs + (u / (BN / 16)) * BPITCH + (u % (BN / 16)) * 16;
    }

    // Edge workgroups of aligned operands whose N is a whole number of 16-byte units take the
    // same loader with the buffers' extents set to where the operands end: a unit of a row of A
    // past M lies past the extent and reads as zero, a unit of B past N reads bytes of the next
    // row, or zero past the last one, and either only feeds outputs that do not exist.  (Every
    // unit that feeds an existing output is whole and inside the extent: full stages only, and
    // N % 16 == 0.)
    const bool edge_fast = !interior && vecA && vecB && (N & 15) == 0 &&
                           (int64_t)BM * args.lda < 0x7fffffffLL && (int64_t)CI_BK * args.ldb < 0x7fffffffLL;
    auto extent = [](int64_t bytes) { return (int)(bytes < 0 ? 0 : bytes > 0x7fffffffLL ? 0x7fffffffLL : bytes); };

    v4i sa[A_UNITS], sb[B_UNITS];
    auto load_stage = [&](int k0) {
        if ((interior || edge_fast) && k0 + CI_BK <= K) {
            // bytes from the stage's first byte to the end of the operand's last row
            const int ext_a = interior ? 0x7fffffff : extent((int64_t)(M - 1 - row0) * args.lda + (K - k0));
            const int ext_b = interior ? 0x7fffffff : extent((int64_t)(K - 1 - k0) * args.ldb + (N - col0));
            const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(a_base + k0), 0, ext_a, 0x00020000);
            const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(b_base + (int64_t)k0 * args.ldb), 0, ext_b, 0x00020000);
#pragma unroll
            for (int it = 0; it < A_UNITS; ++it) sa[it] = __builtin_amdgcn_raw_buffer_load_b128(ra, offa[it], 0, 0);
#pragma unroll
            for (int it = 0; it < B_UNITS; ++it) sb[it] = __builtin_amdgcn_raw_buffer_load_b128(rb, offb[it], 0, 0);
        } else {
#pragma unroll
            for (int it = 0; it < A_UNITS; ++it) {
                const int u = tid + it * NT;
                const int r = row0 + u / AU, k = k0 + (u % AU) * 16;
                sa[it] = (r < M) ? load16_i8(Ag + (int64_t)r * args.lda + k, vecA, K - k) : v4i{0, 0, 0, 0};
            }
#pragma unroll
            for (int it = 0; it < B_UNITS; ++it) {
                const int u = tid + it * NT;
                const int k = k0 + u / (BN / 16), c = col0 + (u % (BN / 16)) * 16;
                // a row's last, partial unit (not the row's first unit): the 16 bytes ending at
                // the row's end, moved down afterwards
                const int nv = N - c;
                const bool part = tail_n != 0 && nv > 0 && nv < 16 && c >= 16;
                const int8_t *src = Bg + (int64_t)k * args.ldb + c - (part ? 16 - tail_n : 0);
                v4i x = (k < K) ? load16_i8(src, vecB && tail_n == 0, part ? 16 : nv) : v4i{0, 0, 0, 0};
                if (tail_n != 0) {
                    const v4i y = shift_down_i8(x, 16 - tail_n);
                    x = part ? y : x;
                }
                sb[it] = x;
            }
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int it = 0; it < A_UNITS; ++it) *(v4i *)(la[it] + buf * T::A_BYTES) = sa[it];
#pragma unroll
        for (int it = 0; it < B_UNITS; ++it) *(v4i *)(lb[it] + buf * T::B_BYTES) = sb[it];
    };

    v16i acc[MB][NB];
#pragma unroll
    for (int mi = 0; mi < MB; ++mi)
#pragma unroll
        for (int ni = 0; ni < NB; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0;

    // transpose-read addressing inside a 16-lane block (see the header comment)
    const int tb = lane >> 4;                 // block 0..3: column half tb%2, k-slot tb/2 (= lh)
    const int ts = lane & 15;
    const int b_krow = 16 * (tb >> 1) + (ts >> 1);             // + 8 for the second read, + 32 per k-step
    const int b_col = 16 * (tb & 1) + 8 * (ts & 1);            // + 32*ni + the wave's column offset

    const int n_stages = (K + CI_BK - 1) / CI_BK;
    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int s = 0; s < n_stages; ++s) {
        const int buf = s & 1;
        if (s + 1 < n_stages) load_stage((s + 1) * CI_BK);
#pragma unroll
        for (int ks = 0; ks < CI_BK; ks += 32) {
            v4i a[MB], b[NB];
#pragma unroll
            for (int mi = 0; mi < MB; ++mi)
                a[mi] = *(const v4i *)(As + buf * T::A_BYTES + ((wr * MB + mi) * 32 + li) * CI_APITCH + ks + 16 * lh);
#pragma unroll
            for (int ni = 0; ni < NB; ++ni) {
                const int8_t *p = Bs + buf * T::B_BYTES + (ks + b_krow) * BPITCH + (wc * NB + ni) * 32 + b_col;
                const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)p);
                const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i_ptr)(p + 8 * BPITCH));
                b[ni] = v4i{lo.x, lo.y, hi.x, hi.y};
            }
#pragma unroll
            for (int mi = 0; mi < MB; ++mi)
#pragma unroll
                for (int ni = 0; ni < NB; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
        }
        if (s + 1 < n_stages) store_stage(buf ^ 1);
        __syncthreads();
    }

    // accumulator element v of lane l is R[8*(v/4) + 4*(l/32) + v%4][l%32] of its 32x32 block.
    // R += acc: eight values of a block at a time are all read before the first is written back
    // (as "*dst += acc" per element the compiler must keep every store behind the load before it,
    // and the write-back is a chain of serial round trips to memory).
#pragma unroll
    for (int mi = 0; mi < MB; ++mi)
#pragma unroll
        for (int ni = 0; ni < NB; ++ni) {
            const int col = col0 + (wc * NB + ni) * 32 + li;
            if (col >= N) continue;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                uint32_t old[8];
#pragma unroll
                for (int w = 0; w < 8; ++w) {
                    const int v = 8 * h + w;
                    const int row = row0 + (wr * MB + mi) * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                    int32_t *dst = args.R + (int64_t)row * args.ldr + col;
                    if (ksplit) {
                        if (row < M) atomicAdd(dst, acc[mi][ni][v]);
                    } else {
                        old[w] = row < M && !args.assign ? (uint32_t)*dst : 0u;
                    }
                }
                if (!ksplit) {
#pragma unroll
                    for (int w = 0; w < 8; ++w) {
                        const int v = 8 * h + w;
                        const int row = row0 + (wr * MB + mi) * 32 + 8 * (v >> 2) + 4 * lh + (v & 3);
                        if (row < M) args.R[(int64_t)row * args.ldr + col] = (int32_t)(old[w] + (uint32_t)acc[mi][ni][v]);
                    }
                }
            }
        }
}

// Shape 0: one output per thread, plain k loop.  Kept as the simplest exact
// form; every other shape is checked against the same oracle.
__global__ void __launch_bounds__(256)
count_i8_simple_kernel(const CountArgs args)
{
    const int j = blockIdx.x * 64 + (threadIdx.x & 63);
    const int i = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (i >= args.M || j >= args.N) return;
    const int8_t *a = args.A + (int64_t)i * args.lda;
    const int8_t *b = args.B + j;
    int acc = 0;
    for (int k = 0; k < args.K; ++k)
        acc += (int)a[k] * (int)b[(int64_t)k * args.ldb];
    int32_t *dst = args.R + (int64_t)i * args.ldr + j;
    *dst = args.assign ? acc : (int32_t)((uint32_t)*dst + (uint32_t)acc);
}

__global__ void __launch_bounds__(256) zero_r_i32_kernel(int32_t *R, int64_t ldr, int M, int N)
{
    const int64_t row = blockIdx.y;
    for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < N; j += (int64_t)gridDim.x * 256)
        if (row < M) R[row * ldr + j] = 0;
}

hipError_t launch_zero_r_i32(const CountArgs &a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    const unsigned gx = (unsigned)((a.N + 255) / 256 < 1024 ? (a.N + 255) / 256 : 1024);
    for (int64_t r0 = 0; r0 < a.M; r0 += 65535) {
        const int64_t rows = a.M - r0 < 65535 ? a.M - r0 : 65535;
        hipLaunchKernelGGL(zero_r_i32_kernel, dim3(gx, (unsigned)rows), dim3(256), 0, s, a.R + r0 * a.ldr, a.ldr, (int)rows, a.N);
    }
    return hipGetLastError();
}

template <int MB, int NB, int WR, int WC, int WPE, int BK>
static hipError_t launch_mfma(const CountArgs &a, hipStream_t s)
{
    typedef CountTile<MB, NB, WR, WC, BK> T;
    const int64_t tiles_m = (a.M + T::BM - 1) / T::BM, tiles_n = (a.N + T::BN - 1) / T::BN;
    const int64_t grid = xcd_grid(tiles_m, tiles_n);
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if (T::LDS_BYTES > 65536) {
        // more than 64 KB of LDS per workgroup has to be granted once per kernel
        static hipError_t granted = hipFuncSetAttribute(
            reinterpret_cast<const void *>(&count_i8_mfma_kernel<MB, NB, WR, WC, WPE, BK>),
            hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
        if (granted != hipSuccess) return granted;
    }
    // too few tiles to give every SIMD two waves: split K over several workgroups per tile
    // (at least 512 k each), which add their parts to R with integer atomics
    CountArgs b = a;
    int splits = 1;
    b.kchunk = a.K;
    const int64_t waves = tiles_m * tiles_n * WR * WC;
    if (waves < 2048 && a.K >= 1024) {
        int64_t want = (2048 + waves - 1) / waves;
        if (want > a.K / 512) want = a.K / 512;
        if (want > 1024) want = 1024;
        const int64_t chunk = ((a.K + want - 1) / want + BK - 1) / BK * BK;
        b.kchunk = (int)chunk;
        splits = (int)((a.K + chunk - 1) / chunk);
    }
    if (splits > 1 && a.assign) {   // several workgroups add into a tile: from zero
        const hipError_t ez = launch_zero_r_i32(a, s);
        if (ez != hipSuccess) return ez;
        b.assign = 0;
    }
    return launch_row_of_blocks(b, grid, T::NT, [&](unsigned n) {
        hipLaunchKernelGGL((count_i8_mfma_kernel<MB, NB, WR, WC, WPE, BK>), dim3(n, (unsigned)splits), dim3(T::NT),
                           T::LDS_BYTES, s, b);
    });
}

hipError_t launch_count_i8(int shape, const CountArgs &a, hipStream_t s)
{
    switch (shape) {
    case 0: {
        // grid.y is limited to 65535 and grid.x to 2^32 - 1 work-items: walk rows and columns in slabs
        const int64_t col_slab = 64LL * (0xFFFFFFFFLL / 256);
        for (int64_t c0 = 0; c0 < a.N; c0 += col_slab)
            for (int64_t r0 = 0; r0 < a.M; r0 += 65535LL * 4) {
                CountArgs sub = a;
                const int64_t rows = (a.M - r0 < 65535LL * 4) ? a.M - r0 : 65535LL * 4;
                const int64_t cols = (a.N - c0 < col_slab) ? a.N - c0 : col_slab;
                sub.A = a.A + r0 * a.lda;
                sub.B = a.B + c0;
                sub.R = a.R + r0 * a.ldr + c0;
                sub.M = (int)rows;
                sub.N = (int)cols;
                hipLaunchKernelGGL(count_i8_simple_kernel, dim3((unsigned)((cols + 63) / 64), (unsigned)((rows + 3) / 4)),
                                   dim3(256), 0, s, sub);
            }
        return hipGetLastError();
    }
    case 1: return launch_mfma<2, 2, 2, 2, 3, 64>(a, s);   // 128 x 128 tile, 4 waves
    case 2: return launch_mfma<4, 2, 2, 4, 2, 64>(a, s);   // 256 x 256 tile, 8 waves of 128 x 64
    case 3: return launch_mfma<2, 2, 2, 4, 4, 64>(a, s);   // 128 x 256 tile, 8 waves of 64 x 64
    case 4: return launch_mfma<2, 1, 2, 4, 4, 128>(a, s);  // 128 x 128 tile, 8 waves of 64 x 32, 128-byte stages
    case 5: return launch_mfma<2, 2, 4, 4, 4, 64>(a, s);   // 256 x 256 tile, 16 waves of 64 x 64
    case 6:   // 128 x 256 tile streamed HBM -> LDS directly
    case 7:   // 256 x 256 tile, 16 waves, streamed HBM -> LDS directly
    case 8: { // the same tile with persistent workgroups (one per compute unit) walking the tile order
        // The streamed kernels take whole tiles of aligned operands with K % 64 == 0.  A problem
        // with ragged M or N is cut into its interior (whole tiles, streamed) and up to two edge
        // strips (bottom rows, right-hand columns) that the register-staged kernel of the same
        // tile handles: the three launches write disjoint parts of R.
        // (and rows short enough for the streamed kernels' 32-bit lane offsets: 256 rows of A,
        // 64 k rows of B)
        const bool aligned = a.vecA && a.vecB && a.vecR && a.K % 64 == 0 &&
                             a.lda <= (int64_t)(0x7FFFFFFF - 64) / 256 && a.ldb <= (int64_t)(0x7FFFFFFF - 256) / 64;
        int wr = shape == 6 ? 2 : 4;
        const bool persistent = shape == 8;
        if (wr == 4 && a.M < 256) wr = 2;
        const int bm = 64 * wr;
        const int Mi = aligned ? a.M - a.M % bm : 0, Ni = aligned ? a.N - a.N % 256 : 0;
        if (Mi == 0 || Ni == 0) return launch_mfma<2, 2, 2, 4, 4, 64>(a, s);
        CountArgs in = a;
        in.M = Mi; in.N = Ni;
        hipError_t e = launch_count_i8_dma(in, wr, s, persistent && wr == 4);
        if (e == hipSuccess && a.M > Mi) {          // bottom strip: rows Mi.., all columns
            CountArgs bot = a;
            bot.A = a.A + (int64_t)Mi * a.lda; bot.R = a.R + (int64_t)Mi * a.ldr; bot.M = a.M - Mi;
            bot.Mload = a.Mload - Mi;
            e = launch_mfma<2, 2, 2, 4, 4, 64>(bot, s);
        }
        if (e == hipSuccess && a.N > Ni) {          // right-hand strip: rows 0..Mi, columns Ni..
            CountArgs right = a;
            right.B = a.B + Ni; right.R = a.R + Ni; right.M = Mi; right.N = a.N - Ni;
            right.Nload = a.Nload - Ni;
            e = launch_mfma<2, 2, 2, 4, 4, 64>(right, s);
        }
        return e;
    }
    default:
        return hipErrorInvalidValue;
    }
}

}  // namespace amulet
