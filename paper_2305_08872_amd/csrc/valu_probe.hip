// Register-only issue-rate probe: what the vector ALU of this chip sustains on
// the instruction mix of a task when nothing but arithmetic is in the way (no
// LDS, no global memory, no barriers).  The bench reports it beside the kernel's
// rate, so the roofline fraction can also be read against a measured ceiling.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "amulet.h"
#include "amulet_internal.h"

namespace amulet {

// mix 0: fused multiply-add only (the identity task's inner operation)
// mix 1: multiply, compare, select, fused multiply-add (the discount task), interleaved as in the kernel
// mix 2: fma, fma, max, add (the boost task), one product at a time as in the kernel
// mix 3: multiply, subtract, then the sign bit of the difference added to an integer count (the count task)
template <int MIX>
__global__ void __launch_bounds__(256) valu_probe_kernel(float *out, float a0, int iters)
{
    float acc[16], b[16], th[16], q[16];
    int cnt[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        cnt[i] = 0;
        acc[i] = threadIdx.x * 0.001f + i;
        b[i] = 1.0f + i * 0.01f + threadIdx.x * 1e-6f;
        // per-lane values, as in the kernels: a wave-uniform threshold would be kept in a scalar
        // register, and a compare with a scalar threshold operand issues slower
        th[i] = 1.5f + i + threadIdx.x * 1e-4f;
        q[i] = 0.9f - i * 0.01f - threadIdx.x * 1e-5f;
    }
    float a = a0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (MIX == 1) {
                // in the order the kernel's inner loop runs them: compare i, multiply i + 1, FMA
                // i - 1, select i, so that every compare can write the same lane-mask register and
                // its select reads it two instructions later
                float p[17], s[16];
                p[0] = a * b[0];
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const bool m = p[i] > th[i];
                    __builtin_amdgcn_sched_barrier(0);
                    if (i + 1 < 16) p[i + 1] = a * b[i + 1];
                    __builtin_amdgcn_sched_barrier(0);
                    if (i > 0) acc[i - 1] = __builtin_fmaf(p[i - 1], s[i - 1], acc[i - 1]);
                    __builtin_amdgcn_sched_barrier(0);
                    s[i] = m ? q[i] : 1.0f;
                    __builtin_amdgcn_sched_barrier(0);
                }
                acc[15] = __builtin_fmaf(p[15], s[15], acc[15]);
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (MIX == 0) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[g * 4 + c] = __builtin_fmaf(a, b[g * 4 + c], acc[g * 4 + c]);
                } else if (MIX == 1) {
                    // (above)
                } else if (MIX == 3) {
                    float p[4], d[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) p[c] = a * b[g * 4 + c];
#pragma unroll
                    for (int c = 0; c < 4; ++c) d[c] = th[g * 4 + c] - p[c];
#pragma unroll
                    for (int c = 0; c < 4; ++c) cnt[g * 4 + c] += (int)(__builtin_bit_cast(unsigned, d[c]) >> 31);
                } else {
                    // one product at a time, as the kernel runs them
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        float d = __builtin_fmaf(a, b[g * 4 + c], -th[g * 4 + c]);
                        acc[g * 4 + c] = __builtin_fmaf(a, b[g * 4 + c], acc[g * 4 + c]);
                        d = __builtin_fmaxf(d, 0.0f);
                        acc[g * 4 + c] += d;
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            a += 1e-7f;
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i] + (float)cnt[i];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

typedef int probe_v4i __attribute__((ext_vector_type(4)));
typedef int probe_v16i __attribute__((ext_vector_type(16)));

// Register-only loop of the join count's matrix-core instruction (v_mfma_i32_32x32x32_i8)
// on four independent accumulators, as in the kernel's 2 x 2 block.
__global__ void __launch_bounds__(256) mfma_i8_probe_kernel(int *out, int iters)
{
    const int lane = threadIdx.x;
    const probe_v4i a = {lane, lane * 3, lane * 5, lane * 7}, b = {lane * 11, lane ^ 0x55, lane + 9, lane * 13};
    probe_v16i acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[i], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace amulet

using namespace amulet;

extern "C" int amulet_probe_mfma_i8(int waves_per_simd, double *macs_per_second, void *stream)
{
    if (waves_per_simd < 1 || waves_per_simd > 8) return AMULET_ERR_DIM;
    if (!macs_per_second) return AMULET_ERR_NULL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return AMULET_ERR_LAUNCH;
    const int iters = 2000;
    const int grid = cus * waves_per_simd;  // 256 threads = one wave per SIMD per workgroup
    int *out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipStream_t s = (hipStream_t)stream;
    int rc = AMULET_ERR_LAUNCH;
    if (hipMalloc(&out, (size_t)grid * 256 * sizeof(int)) == hipSuccess &&
        hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess) {
        for (int rep = 0; rep < 2; ++rep) {  // first repetition is the warm-up
            (void)hipEventRecord(e0, s);
            hipLaunchKernelGGL(mfma_i8_probe_kernel, dim3(grid), dim3(256), 0, s, out, iters);
            (void)hipEventRecord(e1, s);
        }
        float ms = 0.0f;
        if (hipGetLastError() == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
            hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.0f) {
            // per wave and iteration: 16 instructions of 32 x 32 x 32 multiply-adds
            *macs_per_second = (double)grid * 4.0 * iters * 16.0 * 32768.0 / (ms * 1e-3);
            rc = AMULET_OK;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (out) (void)hipFree(out);
    return rc;
}

extern "C" int amulet_probe_valu(int mix, int waves_per_simd, double *products_per_second, void *stream)
{
    if (mix < 0 || mix > 3) return AMULET_ERR_TASK;
    if (waves_per_simd < 1 || waves_per_simd > 8) return AMULET_ERR_DIM;
    if (!products_per_second) return AMULET_ERR_NULL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return AMULET_ERR_LAUNCH;
    const int iters = 10000;
    const int grid = cus * waves_per_simd;  // 256 threads = 4 waves = one wave per SIMD per workgroup
    float *out = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipStream_t s = (hipStream_t)stream;
    int rc = AMULET_ERR_LAUNCH;
    if (hipMalloc(&out, (size_t)grid * 256 * sizeof(float)) == hipSuccess &&
        hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess) {
        for (int rep = 0; rep < 2; ++rep) {  // first repetition is the warm-up
            (void)hipEventRecord(e0, s);
            switch (mix) {
            case 0: hipLaunchKernelGGL(valu_probe_kernel<0>, dim3(grid), dim3(256), 0, s, out, 1.0f, iters); break;
            case 1: hipLaunchKernelGGL(valu_probe_kernel<1>, dim3(grid), dim3(256), 0, s, out, 1.0f, iters); break;
            case 2: hipLaunchKernelGGL(valu_probe_kernel<2>, dim3(grid), dim3(256), 0, s, out, 1.0f, iters); break;
            default: hipLaunchKernelGGL(valu_probe_kernel<3>, dim3(grid), dim3(256), 0, s, out, 1.0f, iters); break;
            }
            (void)hipEventRecord(e1, s);
        }
        float ms = 0.0f;
        if (hipGetLastError() == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
            hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.0f) {
            // 16 accumulators x 4 unrolled passes = 64 products per lane per iteration
            *products_per_second = (double)grid * 256.0 * iters * 64.0 / (ms * 1e-3);
            rc = AMULET_OK;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (out) (void)hipFree(out);
    return rc;
}
