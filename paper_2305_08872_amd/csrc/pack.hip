// Packing (paper Sec. 3.1): copy an operand once into storage whose layout suits the kernels'
// access order.  On this GPU "suits" means one thing only: a row pitch that does not put the
// rows a workgroup reads at one k into the same L2 sets and memory channel.  The copy is a
// strided 2-D copy into rows spaced by amulet_packed_ld(); the compute kernels then read it
// in place like any other row-major operand.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "amulet.h"
#include "amulet_internal.h"

namespace amulet {

typedef unsigned int pk_u4 __attribute__((ext_vector_type(4)));

// One workgroup row of 256 threads copies `row_units` 16-byte units of a row per pass; rows are
// walked with a grid stride in y, so any row count fits the grid limits.
__global__ void __launch_bounds__(256)
pack_rows16_kernel(const uint8_t *src, int64_t pitch_src, uint8_t *dst, int64_t pitch_dst,
                   int64_t rows, int64_t row_units)
{
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) {
        const pk_u4 *s = (const pk_u4 *)(src + r * pitch_src);
        pk_u4 *d = (pk_u4 *)(dst + r * pitch_dst);
        for (int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x; u < row_units; u += (int64_t)gridDim.x * 256)
            d[u] = s[u];
    }
}

// Same walk, one element per thread and pass: for rows that are not 16-byte aligned.
template <typename T>
__global__ void __launch_bounds__(256)
pack_rows_elem_kernel(const T *src, int64_t ld_src, T *dst, int64_t ld_dst, int64_t rows, int64_t cols)
{
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) {
        const T *s = src + r * ld_src;
        T *d = dst + r * ld_dst;
        for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < cols; c += (int64_t)gridDim.x * 256)
            d[c] = s[c];
    }
}

// dst[c][r] = src[r][c] for a rows x cols matrix of bytes: 64 x 64 tiles through LDS, so that
// both the reads (along src rows) and the writes (along dst rows) are contiguous runs of 64
// bytes (16 per lane: one 16-byte access where the tile is interior and `vec` says both
// matrices are 16-byte aligned).  Pitches in bytes.  Tiles are walked with a grid stride.
__global__ void __launch_bounds__(256)
transpose_i8_kernel(const int8_t *src, int64_t pitch_src, int8_t *dst, int64_t pitch_dst, int64_t rows,
                    int64_t cols, int vec)
{
    __shared__ __attribute__((aligned(16))) int8_t tile[64][64 + 16];
    const int64_t tiles_c = (cols + 63) / 64, tiles_r = (rows + 63) / 64;
    const int lr = threadIdx.x >> 2, lq = (threadIdx.x & 3) * 16;   // row of the tile, 16-byte quarter of it
    for (int64_t t = blockIdx.x; t < tiles_r * tiles_c; t += gridDim.x) {
        const int64_t r0 = (t / tiles_c) * 64, c0 = (t % tiles_c) * 64;
        const bool interior = vec && r0 + 64 <= rows && c0 + 64 <= cols;
        if (interior) {
            *(pk_u4 *)&tile[lr][lq] = *(const pk_u4 *)(src + (r0 + lr) * pitch_src + c0 + lq);
        } else {
            const int64_t r = r0 + lr;
            for (int e = 0; e < 16; ++e) {
                const int64_t c = c0 + lq + e;
                tile[lr][lq + e] = (r < rows && c < cols) ? src[r * pitch_src + c] : (int8_t)0;
            }
        }
        __syncthreads();
        {
            // row c0 + lr of dst, bytes lq .. lq + 15 of it: column lr of the tile, rows lq ...
            unsigned int w[4] = {0u, 0u, 0u, 0u};
            for (int e = 0; e < 16; ++e) w[e >> 2] |= (unsigned int)(uint8_t)tile[lq + e][lr] << (8 * (e & 3));
            const int64_t c = c0 + lr;
            if (interior) {
                pk_u4 v = {w[0], w[1], w[2], w[3]};
                *(pk_u4 *)(dst + c * pitch_dst + r0 + lq) = v;
            } else if (c < cols) {
                for (int e = 0; e < 16; ++e) {
                    const int64_t r = r0 + lq + e;
                    if (r < rows) dst[c * pitch_dst + r] = (int8_t)(w[e >> 2] >> (8 * (e & 3)));
                }
            }
        }
        __syncthreads();
    }
}

// Copy of a rows x cols byte matrix into rows_p x cols_p (cols_p a multiple of 16, dst 16-byte
// aligned rows), zero beyond the source: a thread writes one aligned 16-byte unit and reads its
// 16 source bytes with one load at whatever address they have (global accesses take any
// address on this target), bytewise only across the source's right-hand edge.
typedef pk_u4 pk_u4_any __attribute__((aligned(1)));
__global__ void __launch_bounds__(256)
pack_pad_i8_kernel(const int8_t *src, int64_t pitch_src, int64_t rows, int64_t cols, int8_t *dst, int64_t pitch_dst,
                   int64_t rows_p, int64_t units)
{
    for (int64_t r = blockIdx.y; r < rows_p; r += gridDim.y) {
        const int8_t *srow = src + r * pitch_src;
        for (int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x; u < units; u += (int64_t)gridDim.x * 256) {
            const int64_t c0 = u * 16;
            pk_u4 v = {0u, 0u, 0u, 0u};
            if (r < rows) {
                if (c0 + 16 <= cols) {
                    v = *(const pk_u4_any *)(srow + c0);
                } else {
                    unsigned int w[4] = {0u, 0u, 0u, 0u};
                    for (int e = 0; e < 16; ++e)
                        if (c0 + e < cols) w[e >> 2] |= (unsigned int)(uint8_t)srow[c0 + e] << (8 * (e & 3));
                    v = pk_u4{w[0], w[1], w[2], w[3]};
                }
            }
            *(pk_u4 *)(dst + r * pitch_dst + c0) = v;
        }
    }
}

// Zero the bytes [col0, col0 + ncols) of rows [row0, row0 + nrows): the padding around a
// transposed copy (a fill kernel rather than a memset, so that a caller may capture the call).
__global__ void __launch_bounds__(256)
zero_block_i8_kernel(int8_t *dst, int64_t pitch, int64_t row0, int64_t nrows, int64_t col0, int64_t ncols)
{
    for (int64_t r = blockIdx.y; r < nrows; r += gridDim.y)
        for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < ncols; c += (int64_t)gridDim.x * 256)
            dst[(row0 + r) * pitch + col0 + c] = 0;
}

hipError_t launch_pack_pad_i8(int64_t rows, int64_t cols, const int8_t *src, int64_t ld_src, int8_t *dst,
                              int64_t ld_dst, int64_t rows_p, int64_t cols_p, hipStream_t s)
{
    const int64_t units = cols_p / 16;
    int64_t gx = (units + 255) / 256;
    if (gx > 64) gx = 64;
    const int64_t gy = rows_p < 65535 ? rows_p : 65535;
    hipLaunchKernelGGL(pack_pad_i8_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, s, src, ld_src, rows, cols,
                       dst, ld_dst, rows_p, units);
    return hipGetLastError();
}

hipError_t launch_zero_block_i8(int8_t *dst, int64_t ld, int64_t row0, int64_t nrows, int64_t col0, int64_t ncols,
                                hipStream_t s)
{
    if (nrows <= 0 || ncols <= 0) return hipSuccess;
    int64_t gx = (ncols + 255) / 256;
    if (gx > 64) gx = 64;
    const int64_t gy = nrows < 65535 ? nrows : 65535;
    hipLaunchKernelGGL(zero_block_i8_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, s, dst, ld, row0, nrows,
                       col0, ncols);
    return hipGetLastError();
}

hipError_t launch_transpose_i8(int64_t rows, int64_t cols, const int8_t *src, int64_t ld_src, int8_t *dst,
                               int64_t ld_dst, hipStream_t s)
{
    const int64_t tiles = ((rows + 63) / 64) * ((cols + 63) / 64);
    const int64_t grid = tiles < 65536 ? tiles : 65536;
    const int vec = ((((uintptr_t)src | (uintptr_t)dst) & 15u) == 0 && ld_src % 16 == 0 && ld_dst % 16 == 0) ? 1 : 0;
    hipLaunchKernelGGL(transpose_i8_kernel, dim3((unsigned)grid), dim3(256), 0, s, src, ld_src, dst, ld_dst, rows,
                       cols, vec);
    return hipGetLastError();
}

hipError_t launch_pack(int elem_bytes, int64_t rows, int64_t cols, const void *src, int64_t ld_src,
                       void *dst, int64_t ld_dst, hipStream_t s)
{
    const int64_t row_bytes = cols * elem_bytes;
    const bool vec = (((uintptr_t)src | (uintptr_t)dst) & 15u) == 0 && (ld_src * elem_bytes) % 16 == 0 &&
                     (ld_dst * elem_bytes) % 16 == 0 && row_bytes % 16 == 0;
    const int64_t units = vec ? row_bytes / 16 : cols;
    int64_t gx = (units + 255) / 256;
    if (gx > 64) gx = 64;                       // a row of up to 256 KiB in one pass, longer rows in several
    const int64_t gy = rows < 65535 ? rows : 65535;
    const dim3 grid((unsigned)gx, (unsigned)gy), block(256);
    if (vec) {
        hipLaunchKernelGGL(pack_rows16_kernel, grid, block, 0, s, (const uint8_t *)src, ld_src * elem_bytes,
                           (uint8_t *)dst, ld_dst * elem_bytes, rows, units);
    } else if (elem_bytes == 8) {
        hipLaunchKernelGGL(pack_rows_elem_kernel<uint64_t>, grid, block, 0, s, (const uint64_t *)src, ld_src,
                           (uint64_t *)dst, ld_dst, rows, cols);
    } else if (elem_bytes == 4) {
        hipLaunchKernelGGL(pack_rows_elem_kernel<uint32_t>, grid, block, 0, s, (const uint32_t *)src, ld_src,
                           (uint32_t *)dst, ld_dst, rows, cols);
    } else {
        hipLaunchKernelGGL(pack_rows_elem_kernel<uint8_t>, grid, block, 0, s, (const uint8_t *)src, ld_src,
                           (uint8_t *)dst, ld_dst, rows, cols);
    }
    return hipGetLastError();
}

}  // namespace amulet
