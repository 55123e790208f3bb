// Join count as a matrix product on int8 indicator matrices:
// R[i][j] += sum_k A[i][k]*B[k][j], int32, exact (the join-as-matmul
// translation cited in the paper's introduction).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "amulet_internal.h"

namespace amulet {

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
    *dst = (int32_t)((uint32_t)*dst + (uint32_t)acc);
}

hipError_t launch_count_i8(int shape, const CountArgs &a, hipStream_t s)
{
    switch (shape) {
    case 0: {
        const int64_t gx = (a.N + 63) / 64, gy = (a.M + 3) / 4;
        if (gy > 65535) {
            // grid.y is limited: walk the rows in slabs
            for (int64_t r0 = 0; r0 < a.M; r0 += 65535LL * 4) {
                CountArgs sub = a;
                const int64_t rows = (a.M - r0 < 65535LL * 4) ? a.M - r0 : 65535LL * 4;
                sub.A = a.A + r0 * a.lda;
                sub.R = a.R + r0 * a.ldr;
                sub.M = (int)rows;
                hipLaunchKernelGGL(count_i8_simple_kernel, dim3((unsigned)gx, (unsigned)((rows + 3) / 4)),
                                   dim3(256), 0, s, sub);
            }
        } else {
            hipLaunchKernelGGL(count_i8_simple_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, s, a);
        }
        return hipGetLastError();
    }
    default:
        return hipErrorInvalidValue;
    }
}

}  // namespace amulet
