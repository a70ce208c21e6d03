// Kernels of the traditional ABFT technique at the GEMM level, the comparison system of Sec. 5.3 of the
// paper (row + column checksums, Sec. 2.1): data movement into the larger operands, checksum
// generation, verification of the larger product by reading it once along rows and once along columns,
// and the copy back.  The larger GEMM itself is the library's unchecked 1x1 convolution.
// All sums are 32-bit and wrap; integer atomics make the accumulation order irrelevant.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace abed {

// Task 2 / task 6: rows of `w_src` elements copied into rows of `w_dst` elements (the first min(w_src, w_dst) of each),
// element size eb; the rest of a destination row is left alone.  16 bytes per thread when everything is aligned.
__global__ void abft_copy_rows_kernel(const unsigned char *src, unsigned char *dst, long long rows, long long w_src_bytes,
                                      long long w_dst_bytes, long long w_copy_bytes)
{
    const long long per_row = w_copy_bytes / 16;
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * per_row) return;
    const long long r = i / per_row, c = i - r * per_row;
    *reinterpret_cast<uint4 *>(dst + r * w_dst_bytes + c * 16) = *reinterpret_cast<const uint4 *>(src + r * w_src_bytes + c * 16);
}

// Task 6 where the rows are not whole 16-byte pieces: one 32-bit word per thread.
__global__ void abft_copy_words_kernel(const int *src, int *dst, long long rows, int ld_src, int w)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows * w) return;
    const long long r = i / w;
    dst[i] = src[r * ld_src + (i - r * w)];
}

// Column sums of a row-major matrix, 16 bytes per thread and row: sums[c] += sum over this block's chunk of rows of
// m[row][c].  EB = bytes per element (1: int8, task 3; 4: int32, the second pass of task 5).  A block covers up to
// 256 consecutive 16-byte units of a row; narrower matrices put several row phases side by side.  Per-thread
// registers, then LDS atomics across the phases, then one global atomic per column and block.
template <int EB>
__global__ __launch_bounds__(256) void abft_colsum_kernel(const unsigned char *m, long long rows, int units, long long row_bytes,
                                                          int rows_per_block, int *sums)
{
    constexpr int CPU = 16 / EB;                     // columns per unit
    __shared__ int lsum[256 * CPU];
    const int t = threadIdx.x;
    const int ublock = units < 256 ? units : 256;    // units this block covers
    const int phases = 256 / ublock;
    const int u_local = t % ublock, phase = t / ublock;
    const int unit = blockIdx.x * 256 + u_local;
    const bool active = phase < phases && unit < units;
    for (int i = t; i < 256 * CPU; i += 256) lsum[i] = 0;
    __syncthreads();
    const long long r0 = (long long)blockIdx.y * rows_per_block;
    long long r1 = r0 + rows_per_block; if (r1 > rows) r1 = rows;
    int s[CPU];
#pragma unroll
    for (int q = 0; q < CPU; ++q) s[q] = 0;
    if (active) {
#pragma unroll 4
        for (long long r = r0 + phase; r < r1; r += phases) {
            const int4 v = *reinterpret_cast<const int4 *>(m + r * row_bytes + (long long)unit * 16);
            const int w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (EB == 1) {
                    s[4 * j + 0] += (w[j] << 24) >> 24; s[4 * j + 1] += (w[j] << 16) >> 24;
                    s[4 * j + 2] += (w[j] << 8) >> 24; s[4 * j + 3] += w[j] >> 24;
                } else {
                    s[j] += w[j];
                }
            }
        }
#pragma unroll
        for (int q = 0; q < CPU; ++q) atomicAdd(&lsum[u_local * CPU + q], s[q]);
    }
    __syncthreads();
    for (int i = t; i < ublock * CPU; i += 256) {
        const int col = blockIdx.x * 256 * CPU + i;
        if (col < units * CPU) atomicAdd(&sums[col], lsum[i]);
    }
}

// Task 3, second half: balanced base-256 digits (Sec. 4.1) of sums[k] into d rows of `cols` int8 values.
__global__ void abft_digits_kernel(const int *sums, int cols, int d, int8_t *rows_out)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= cols) return;
    int s = sums[k];
    for (int i = 0; i < d; ++i) {
        const int dig = ((s + 128) & 255) - 128;
        s = (s - dig) >> 8;
        rows_out[(long long)i * cols + k] = (int8_t)dig;
    }
}

// Task 5, first pass over the larger output C' [rows_total][ld]: every data row's sum over the data columns against
// its recombined checksum entries.  One wave per row at a time.  part[block] = the sum of the block's rows' checksum
// values (for the corner).  flags: [0] bit 0, [1] number of bad rows, [3] largest bad row index.
__global__ __launch_bounds__(256) void abft_row_check_kernel(const int *cp, long long M, int Ng, int d_b, int ld, uint32_t *flags, int *part)
{
    __shared__ unsigned wsum[4];
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = (long long)gridDim.x * 4;
    unsigned chk_total = 0;
    for (long long i = wave; i < M; i += nwaves) {
        const int *row = cp + i * ld;
        unsigned s = 0;
        for (int j = lane * 4; j < Ng; j += 256) {          // rows start on 16-byte boundaries (ld is a multiple of 4)
            const int4 v = *reinterpret_cast<const int4 *>(row + j);
            s += (unsigned)v.x + (j + 1 < Ng ? (unsigned)v.y : 0u) + (j + 2 < Ng ? (unsigned)v.z : 0u) + (j + 3 < Ng ? (unsigned)v.w : 0u);
        }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) s += (unsigned)__shfl_xor((int)s, m, 64);
        unsigned c = 0;
        for (int d = 0; d < d_b; ++d) c += (unsigned)row[Ng + d] << (8 * d);
        chk_total += c;
        if (lane == 0 && s != c) {
            atomicOr(&flags[0], 1u);
            atomicAdd(&flags[1], 1u);
            atomicMax(&flags[3], (uint32_t)i);
        }
    }
    if (lane == 0) wsum[threadIdx.x >> 6] = chk_total;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (int)(wsum[0] + wsum[1] + wsum[2] + wsum[3]);
}

// Task 5, second pass: abft_colsum_kernel<4> over the data rows of C'.

// ... and the comparison of the column sums with the recombined checksum rows.  part[block] = the sum of the block's
// columns' checksum values.  flags: [0] bit 1, [2] number of bad columns, [4] largest bad column index.
__global__ __launch_bounds__(256) void abft_col_check_kernel(const int *cp, long long M, int Ng, int d_a, int ld, const int *sums, uint32_t *flags, int *part)
{
    __shared__ unsigned wsum[4];
    const int j = blockIdx.x * 256 + threadIdx.x;
    unsigned c = 0;
    if (j < Ng) {
        for (int d = 0; d < d_a; ++d) c += (unsigned)cp[(M + d) * ld + j] << (8 * d);
        if ((unsigned)sums[j] != c) {
            atomicOr(&flags[0], 2u);
            atomicAdd(&flags[2], 1u);
            atomicMax(&flags[4], (uint32_t)j);
        }
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) c += (unsigned)__shfl_xor((int)c, m, 64);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = (int)(wsum[0] + wsum[1] + wsum[2] + wsum[3]);
}

// The corner: digit rows x digit columns, against the sum of the checksum column (row_part) and of the checksum row (col_part).
__global__ __launch_bounds__(256) void abft_corner_kernel(const int *cp, long long M, int Ng, int d_a, int d_b, int ld,
                                                          const int *row_part, int n_row_part, const int *col_part, int n_col_part, uint32_t *flags)
{
    __shared__ unsigned wsum[2][4];
    unsigned a = 0, b = 0;
    for (int i = threadIdx.x; i < n_row_part; i += 256) a += (unsigned)row_part[i];
    for (int i = threadIdx.x; i < n_col_part; i += 256) b += (unsigned)col_part[i];
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) { a += (unsigned)__shfl_xor((int)a, m, 64); b += (unsigned)__shfl_xor((int)b, m, 64); }
    if ((threadIdx.x & 63) == 0) { wsum[0][threadIdx.x >> 6] = a; wsum[1][threadIdx.x >> 6] = b; }
    __syncthreads();
    if (threadIdx.x != 0) return;
    a = wsum[0][0] + wsum[0][1] + wsum[0][2] + wsum[0][3];
    b = wsum[1][0] + wsum[1][1] + wsum[1][2] + wsum[1][3];
    unsigned c = 0;
    for (int i = 0; i < d_a; ++i)
        for (int j = 0; j < d_b; ++j) c += (unsigned)cp[(M + i) * ld + Ng + j] << (8 * (i + j));
    if (a != c || b != c) atomicOr(&flags[0], 4u);
}

}  // namespace abed
