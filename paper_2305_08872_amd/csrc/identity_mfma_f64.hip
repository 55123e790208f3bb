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
// Rows/columns beyond M/N and the K remainder are zero-filled in LDS: for the identity task
// a zero product adds nothing (NOT true of the predicate tasks, which never take this path).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "amulet_internal.h"

namespace amulet {

typedef double d2 __attribute__((ext_vector_type(2)));
typedef double d4 __attribute__((ext_vector_type(4)));

constexpr int DI_BM = 128, DI_BN = 128, DI_BK = 16, DI_NT = 512;
constexpr int DI_APITCH = DI_BK + 2;    // doubles
constexpr int DI_BPITCH = DI_BN + 4;    // doubles
constexpr int DI_A_DOUBLES = DI_BM * DI_APITCH, DI_B_DOUBLES = DI_BK * DI_BPITCH;
constexpr int DI_LDS_BYTES = 2 * (DI_A_DOUBLES + DI_B_DOUBLES) * 8;   // 70 656: two workgroups per compute unit

__global__ void __launch_bounds__(DI_NT) __attribute__((amdgpu_waves_per_eu(4, 4)))
identity_mfma_f64_kernel(const MmlikeArgsF64 args)
{
    extern __shared__ __attribute__((aligned(16))) double di_smem[];
    double *const As = di_smem;                        // [2][DI_BM][DI_APITCH]
    double *const Bs = di_smem + 2 * DI_A_DOUBLES;     // [2][DI_BK][DI_BPITCH]

    const int M = args.M, N = args.N, K = args.K;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int li = lane & 15, lh = lane >> 4;

    // XCD-aware tile order (xcd_tile in amulet_internal.h)
    const int tiles_m = (M + DI_BM - 1) / DI_BM;
    const int tiles_n = (N + DI_BN - 1) / DI_BN;
    int tm, tn;
    if (!xcd_tile((int)blockIdx.x, tiles_m, tiles_n, tm, tn)) return;   // padding: the whole workgroup leaves
    const int row0 = tm * DI_BM, col0 = tn * DI_BN;
    const bool vecA = args.vecA != 0, vecB = args.vec != 0;

    // staging slots of 16 bytes, u = tid + 512 * it:
    //   A tile 128 rows x 8 slots: row = u / 8, k pair = u % 8
    //   B tile  16 rows x 64 slots: k = u / 64, column pair = u % 64
    d2 sa[2], sb[2];
    auto load_stage = [&](int k0) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int u = tid + DI_NT * it;
            const int r = row0 + (u >> 3);
            const int k = k0 + (u & 7) * 2;
            d2 v = {0.0, 0.0};
            if (r < M) {
                const double *src = args.A + (int64_t)r * args.lda + k;
                if (vecA && k + 1 < K) {
                    v = *(const d2 *)src;
                } else {
                    if (k + 0 < K) v.x = src[0];
                    if (k + 1 < K) v.y = src[1];
                }
            }
            sa[it] = v;
        }
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int u = tid + DI_NT * it;
            const int k = k0 + (u >> 6);
            const int c = col0 + (u & 63) * 2;
            d2 v = {0.0, 0.0};
            if (k < K) {
                const double *src = args.B + (int64_t)k * args.ldb + c;
                if (vecB && c + 1 < N) {
                    v = *(const d2 *)src;
                } else {
                    if (c + 0 < N) v.x = src[0];
                    if (c + 1 < N) v.y = src[1];
                }
            }
            sb[it] = v;
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            const int u = tid + DI_NT * it;
            *(d2 *)(As + buf * DI_A_DOUBLES + (u >> 3) * DI_APITCH + (u & 7) * 2) = sa[it];
            *(d2 *)(Bs + buf * DI_B_DOUBLES + (u >> 6) * DI_BPITCH + (u & 63) * 2) = sb[it];
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
        const double *as = As + buf * DI_A_DOUBLES + (wr * 32 + li) * DI_APITCH + 4 * lh;
        const double *bs = Bs + buf * DI_B_DOUBLES + (4 * lh) * DI_BPITCH + wc * 64 + li;
        // the lane's A values of the stage: k = 4 lh .. 4 lh + 3 of its row in both row blocks
        double a[2][4];
#pragma unroll
        for (int mi = 0; mi < 2; ++mi) {
            const d2 lo = *(const d2 *)(as + mi * 16 * DI_APITCH);
            const d2 hi = *(const d2 *)(as + mi * 16 * DI_APITCH + 2);
            a[mi][0] = lo.x; a[mi][1] = lo.y; a[mi][2] = hi.x; a[mi][3] = hi.y;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            double b[4];
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) b[ni] = bs[t * DI_BPITCH + ni * 16];
#pragma unroll
            for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[mi][t], b[ni], acc[mi][ni], 0, 0, 0);
        }
        if (s + 1 < n_stages) store_stage(buf ^ 1);
        __syncthreads();
    }

    // element v of lane l is R[4 v + l / 16][l % 16] of its 16 x 16 block
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
            const int col = col0 + wc * 64 + ni * 16 + li;
            if (col >= N) continue;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = row0 + wr * 32 + mi * 16 + 4 * v + lh;
                if (row < M) {
                    double *dst = args.R + (int64_t)row * args.ldr + col;
                    *dst += acc[mi][ni][v];
                }
            }
        }
}

hipError_t launch_identity_mfma_f64(const MmlikeArgsF64 &a, hipStream_t s)
{
    const int64_t tiles_m = (a.M + DI_BM - 1) / DI_BM;
    const int64_t tiles_n = (a.N + DI_BN - 1) / DI_BN;
    const int64_t grid = xcd_grid(tiles_m, tiles_n);
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    static hipError_t granted = hipFuncSetAttribute(reinterpret_cast<const void *>(&identity_mfma_f64_kernel),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, DI_LDS_BYTES);
    if (granted != hipSuccess) return granted;
    hipLaunchKernelGGL(identity_mfma_f64_kernel, dim3((unsigned)grid), dim3(DI_NT), DI_LDS_BYTES, s, a);
    return hipGetLastError();
}

}  // namespace amulet
