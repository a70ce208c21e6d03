// Kernels of IC option 2 (Sec. 3.2 of the paper): the input fmaps are reduced to a checksum tensor of
// the size of one filter, that tensor is convolved with the K filters, and the K results must equal the
// output fmaps reduced over batch, height and width.
//
// The input checksum is the one the FIC scheme uses, in its row-wise form xrows[j,h,s,c] (fic_device.h):
// X[r,s,c] is the sum of xrows over the batch parts j and over the input rows h that filter row r
// meets.  Here X is materialised once (a small kernel), because all K dot products
//   chk[k] = sum_{r,s,c} X[r,s,c] * w[k,r,s,c]
// need it.  The dot products and the output sums are 64-bit (Sec. 4.1).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace abed {

// Output fmap checksum generation of the unfused option: one more pass over the stored int32 ConvOut
// [rows][K]; workgroup b sums rows b, b + gridDim.x, ... and writes one partial per filter.
// Dynamic LDS: K * 8 bytes.
__global__ __launch_bounds__(256) void ic2_output_sums_kernel(const int32_t *y, long long rows, int K, long long *part)
{
    extern __shared__ unsigned long long colsum[];
    const int tid = threadIdx.x;
    for (int k = tid; k < K; k += 256) colsum[k] = 0;
    __syncthreads();
    const int cp = K < 256 ? K : 256;            // columns taken side by side
    const int rows_par = 256 / cp;               // rows taken side by side
    const int c0 = tid % cp, slot = tid / cp;
    if (slot < rows_par) {
        for (int c = c0; c < K; c += cp) {
            long long s = 0;
            for (long long r = (long long)blockIdx.x * rows_par + slot; r < rows; r += (long long)gridDim.x * rows_par)
                s += y[r * K + c];
            atomicAdd(&colsum[c], (unsigned long long)s);
        }
    }
    __syncthreads();
    for (int k = tid; k < K; k += 256) part[(long long)blockIdx.x * K + k] = (long long)colsum[k];
}

struct Ic2FoldParams {
    const int32_t *xrows;       // [parts][H][S][C]
    int32_t *X;                 // [R][S][C]
    int H, C, R, S, P, sh, ph, parts;
};

// The filter-sized input checksum from its row-wise form: X[r,s,c] = sum of xrows[j,h,s,c] over the batch
// parts j and over the input rows h = p*sh - ph + r that filter row r meets at some output row p.
// (int32 suffices: the host has checked 8 + log2(PQN) <= 31 bits, Sec. 4.1.)
// A workgroup takes 64 consecutive (r,s,c) elements; its 16 slices of 64 threads share the (j, p) pairs.
__global__ __launch_bounds__(1024) void ic2_fold_kernel(const Ic2FoldParams p)
{
    __shared__ int red[16][64];
    const int tid = threadIdx.x, slice = tid >> 6, l = tid & 63;
    const int sc = p.S * p.C, rsc = p.R * sc;
    const int e = blockIdx.x * 64 + l;
    int sum = 0;
    if (e < rsc) {
        const int r = e / sc, rest = e - r * sc;
        const long long hsc = (long long)p.H * sc;
#pragma unroll 4
        for (int i = slice; i < p.parts * p.P; i += 16) {
            const int j = i / p.P, op = i - j * p.P;
            const int h = op * p.sh - p.ph + r;
            if (h >= 0 && h < p.H) sum += p.xrows[j * hsc + (long long)h * sc + rest];
        }
    }
    red[slice][l] = sum;
    __syncthreads();
    if (slice == 0 && e < rsc) {
        int t = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) t += red[q][l];
        p.X[e] = t;
    }
}

struct Ic2VerifyParams {
    const int8_t *w;            // [K][R][S][C]
    const int32_t *X;           // [R][S][C] input checksum
    const long long *part;      // [nrows][kstride] partial per-filter output sums
    long long *result;          // [0..K) reduced outputs, [K..2K) checksum tensor convolved with the filters
    uint32_t *flags;            // [K]: 1 = the two differ
    int K, crs, nrows, kstride;
};

// One workgroup per filter k: the checksum convolution's value for k (the checksum tensor has the
// extent of one filter, so that is one dot product), the sum of the partial output sums of k, and the
// comparison (the element-wise verification of Sec. 3.2 option 2).
__global__ __launch_bounds__(256) void ic2_verify_kernel(const Ic2VerifyParams p)
{
    __shared__ long long red[2][4];
    const int k = blockIdx.x, tid = threadIdx.x;
    const int8_t *wk = p.w + (long long)k * p.crs;
    long long chk = 0;
#pragma unroll 4
    for (int e = tid; e < p.crs; e += 256) chk += (long long)p.X[e] * wk[e];
    long long osum = 0;
#pragma unroll 4
    for (int i = tid; i < p.nrows; i += 256) osum += p.part[(long long)i * p.kstride + k];
    for (int m = 32; m >= 1; m >>= 1) { chk += __shfl_xor(chk, m, 64); osum += __shfl_xor(osum, m, 64); }
    if ((tid & 63) == 0) { red[0][tid >> 6] = chk; red[1][tid >> 6] = osum; }
    __syncthreads();
    if (tid == 0) {
        const long long c = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        const long long o = red[1][0] + red[1][1] + red[1][2] + red[1][3];
        p.result[k] = o;
        p.result[p.K + k] = c;
        p.flags[k] = (o != c) ? 1u : 0u;
    }
}

}  // namespace abed
