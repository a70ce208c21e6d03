// Kernels of the FIC scheme (Sec. 3.3) that have a launch of their own: the offline filter checksum,
// the input checksum kernel, the output fmap checksum pass of the unfused option, and the final
// sum-and-compare of the unfused option.  The device code they share with the convolution kernel
// (which hosts the input checksum workgroups in the fused option) is in fic_device.h.
#pragma once
#include "fic_device.h"

namespace abed {

// Offline step: the filter checksum as int32.  Grid ceil(crs / 64) x 1024 threads (16 slices share the filters).
__global__ __launch_bounds__(1024) void fic_filter_checksum_i8_kernel(const int8_t *w, int32_t *wsum, int K, int crs)
{
    __shared__ int red[16][64];
    const int slice = threadIdx.x >> 6, l = threadIdx.x & 63;
    const int e = blockIdx.x * 64 + l;
    int s = 0;
    if (e < crs) {
#pragma unroll 4
        for (int k = slice; k < K; k += 16) s += w[(long long)k * crs + e];
    }
    red[slice][l] = s;
    __syncthreads();
    if (slice == 0 && e < crs) {
        int t = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) t += red[q][l];
        wsum[e] = t;
    }
}

// Offline step of the in-loop option: the same filter checksum as three balanced base-256 digits (each in
// [-128, 127], value = d0 + 256 d1 + 65536 d2, exact while |checksum| < 2^23), int8 [3][gpad] with
// gpad = 64 * ceil(crs / 64) and zeros from crs on.  Grid gpad / 64 x 1024 threads.
__global__ __launch_bounds__(1024) void fic_filter_digits_i8_kernel(const int8_t *w, int8_t *wdig, int K, int crs, int gpad)
{
    __shared__ int red[16][64];
    const int slice = threadIdx.x >> 6, l = threadIdx.x & 63;
    const int e = blockIdx.x * 64 + l;
    int s = 0;
    if (e < crs) {
#pragma unroll 4
        for (int k = slice; k < K; k += 16) s += w[(long long)k * crs + e];
    }
    red[slice][l] = s;
    __syncthreads();
    if (slice == 0) {
        int t = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) t += red[q][l];
        for (int d = 0; d < 3; ++d) {
            const int dig = ((t + 128) & 255) - 128;
            t = (t - dig) >> 8;                   // exact: t - dig is a multiple of 256
            wdig[d * gpad + e] = (int8_t)dig;
        }
    }
}

template <int SMAX>
__global__ __launch_bounds__(256) void fic_input_rows_i8_kernel(const FicRowsParams p)
{
    __shared__ __attribute__((aligned(16))) int cols[64][64];
    __shared__ unsigned char meets[SMAX][64];
    __shared__ long long dsum[4];
    fic_rows_body<SMAX>(p, (int)blockIdx.x, (int)threadIdx.x, cols, meets, dsum);
}

// Output fmap checksum of the unfused option: one more pass over the stored int32 ConvOut; one
// partial sum per workgroup.
__global__ __launch_bounds__(256) void fic_output_sum_kernel(const int32_t *y, long long total, long long *partial)
{
    __shared__ long long part[4];
    long long s = 0;
    const long long stride = (long long)gridDim.x * 256 * 4;
    for (long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 4; i < total; i += stride) {
        if (i + 4 <= total) {
            const int4 v = *reinterpret_cast<const int4 *>(y + i);
            s += (long long)v.x + v.y + v.z + v.w;
        } else {
            for (long long j = i; j < total; ++j) s += y[j];
        }
    }
    for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

struct FicVerifyParams {
    const long long *dotpart;   // partial dot products, one per workgroup of the input checksum kernel
    const long long *partial;   // output checksum partials, one per producer workgroup
    long long *result;          // [0] output checksum, [1] dot product
    uint32_t *flag;             // 1 = the two differ
    int ndot, npartial;
};

// Tasks 3 and 7 of Sec. 4.3, last step: add up the partial dot products and the partial output
// checksums and compare the two 64-bit values.  One workgroup of 1024 threads per layer.
__device__ __forceinline__ void fic_verify_body(const FicVerifyParams &p)
{
    __shared__ long long part[2][16];
    long long dot = 0, ocs = 0;
    for (int i = threadIdx.x; i < p.ndot; i += 1024) dot += p.dotpart[i];
    for (int i = threadIdx.x; i < p.npartial; i += 1024) ocs += p.partial[i];
    for (int m = 32; m >= 1; m >>= 1) { dot += __shfl_xor(dot, m, 64); ocs += __shfl_xor(ocs, m, 64); }
    if ((threadIdx.x & 63) == 0) { part[0][threadIdx.x >> 6] = dot; part[1][threadIdx.x >> 6] = ocs; }
    __syncthreads();
    if (threadIdx.x == 0) {
        long long d = 0, o = 0;
        for (int i = 0; i < 16; ++i) { d += part[0][i]; o += part[1][i]; }
        p.result[0] = o;
        p.result[1] = d;
        *p.flag = (o != d) ? 1u : 0u;
    }
}

__global__ __launch_bounds__(1024) void fic_verify_kernel(const FicVerifyParams p) { fic_verify_body(p); }

// The same for several layers in one launch (the comparison deferred to the end of a group of
// layers): workgroup b verifies layer b.
constexpr int kFicVerifyBatch = 32;
struct FicVerifyBatchParams { FicVerifyParams layer[kFicVerifyBatch]; };
__global__ __launch_bounds__(1024) void fic_verify_batch_kernel(const FicVerifyBatchParams p) { fic_verify_body(p.layer[blockIdx.x]); }

}  // namespace abed
