// Kernels of the FIC scheme (filter and input fmap checksums, Sec. 3.3 of the paper) around the
// convolution kernel: the offline filter checksum, the online input checksum, the output fmap
// checksum of the unfused option, and the dot product + comparison.
//
//   filter checksum  wsum[r,s,c] = sum_k w[k,r,s,c]                       int32, offline (Sec. 4.2)
//   input checksum   X[r,s,c]    = sum over n and over all output positions (p,q) of the input
//                                  element that filter element (r,s,c) meets there      int32
//   dot product      sum_{r,s,c} X * wsum                                 int64
//   output checksum  sum of all ConvOut accumulators                       int64
// and the two int64 values must be equal (bit widths: Sec. 4.1).
//
// The input checksum is separable: the set of input rows that filter row r meets and the set of
// input columns that filter column s meets do not depend on each other.  So it is made in two
// steps: xrows[h,s,c] = sum over n and over the input columns w that filter column s meets of
// x[n,h,w,c] (one pass over x, the ICG kernel), then X[r,s,c] = sum over the input rows h that
// filter row r meets of xrows[h,s,c], which is so small that it rides in the kernel that also
// takes the dot product and compares.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace abed {

__global__ void fic_filter_checksum_i8_kernel(const int8_t *w, int32_t *wsum, int K, int crs)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= crs) return;
    int s = 0;
    for (int k = 0; k < K; ++k) s += w[(long long)k * crs + e];
    wsum[e] = s;
}

struct FicRowsParams {
    const int8_t *x;
    int32_t *xrows;               // [H][S][C]
    unsigned long long *zero_me;  // a word to clear (the output checksum accumulator), or null
    int N, H, W, C, S, Q, sw, pw;
};

// One workgroup per (input row h, group of 64 channels).  Lane t: 16-byte channel chunk t & 3 of the
// group, slot t >> 2 of 64 slots that stride over the (image, column) pairs of the row.
template <int SMAX>
__global__ __launch_bounds__(256) void fic_input_rows_i8_kernel(const FicRowsParams p)
{
    __shared__ int red[4][SMAX][64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cgroups = (p.C + 63) / 64;
    const int h = blockIdx.x / cgroups, cg = blockIdx.x - h * cgroups;
    if (blockIdx.x == 0 && tid == 0 && p.zero_me) *p.zero_me = 0ull;
    const int chunk = tid & 3, slot = tid >> 2;
    const int c0 = cg * 64 + chunk * 16;
    int acc[SMAX][16];
#pragma unroll
    for (int s = 0; s < SMAX; ++s)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[s][i] = 0;
    if (c0 < p.C) {
        const int pairs = p.N * p.W;
        for (int idx = slot; idx < pairs; idx += 64) {
            const int n = idx / p.W, w = idx - n * p.W;
            const int4 v = *reinterpret_cast<const int4 *>(p.x + (((long long)n * p.H + h) * p.W + w) * p.C + c0);
            const int words[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int s = 0; s < SMAX; ++s) {
                // does filter column s meet input column w at some output column q?  w = q*sw - pw + s
                const int t = w + p.pw - s;
                const bool hit = s < p.S && t >= 0 && t % p.sw == 0 && t / p.sw < p.Q;
                if (hit) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[s][i] += (int)(int8_t)(words[i >> 2] >> (8 * (i & 3)));
                }
            }
        }
    }
    // sum over the 16 slots of a wave (lanes with the same chunk: lane bits 2..5), then over the 4 waves
#pragma unroll
    for (int s = 0; s < SMAX; ++s)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            int v = acc[s][i];
            v += __shfl_xor(v, 4, 64); v += __shfl_xor(v, 8, 64); v += __shfl_xor(v, 16, 64); v += __shfl_xor(v, 32, 64);
            if (lane < 4) red[wave][s][lane * 16 + i] = v;
        }
    __syncthreads();
    for (int i = tid; i < p.S * 64; i += 256) {
        const int s = i >> 6, c = i & 63;
        if (cg * 64 + c < p.C)
            p.xrows[((long long)h * p.S + s) * p.C + cg * 64 + c] = red[0][s][c] + red[1][s][c] + red[2][s][c] + red[3][s][c];
    }
}

// Output fmap checksum of the unfused option: one more pass over the stored int32 ConvOut.
__global__ __launch_bounds__(256) void fic_output_sum_kernel(const int32_t *y, long long total, unsigned long long *ocs)
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
    if (threadIdx.x == 0) atomicAdd(ocs, (unsigned long long)(part[0] + part[1] + part[2] + part[3]));
}

struct FicVerifyParams {
    const int32_t *xrows;   // [H][S][C]
    const int32_t *wsum;    // [R][S][C]
    long long *result;      // [0] output checksum (read), [1] dot product (written)
    uint32_t *flag;         // 1 = the two differ
    int H, C, R, S, P, sh, ph;
};

// X[r,s,c] = sum over the input rows that filter row r meets, dot product with wsum, comparison.
// One workgroup; the tensors have C*R*S entries (at most 64K).
__global__ __launch_bounds__(1024) void fic_verify_kernel(const FicVerifyParams p)
{
    __shared__ long long part[16];
    const int sc = p.S * p.C;
    long long dot = 0;
    for (int e = threadIdx.x; e < p.R * sc; e += 1024) {
        const int r = e / sc, rest = e - r * sc;          // rest = s*C + c
        int X = 0;
        for (int q = 0; q < p.P; ++q) {
            const int h = q * p.sh - p.ph + r;
            if (h >= 0 && h < p.H) X += p.xrows[(long long)h * sc + rest];
        }
        dot += (long long)X * p.wsum[e];
    }
    for (int m = 32; m >= 1; m >>= 1) dot += __shfl_xor(dot, m, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = dot;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long d = 0;
        for (int i = 0; i < 16; ++i) d += part[i];
        p.result[1] = d;
        *p.flag = (p.result[0] != d) ? 1u : 0u;
    }
}

__global__ void fill_u64_kernel(unsigned long long *p, unsigned long long v) { *p = v; }

}  // namespace abed
