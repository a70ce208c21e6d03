// Kernels of IC option 2 (Sec. 3.2 of the paper): the input fmaps are reduced to a checksum tensor of
// the size of one filter, that tensor is convolved with the K filters, and the K results must equal the
// output fmaps reduced over batch, height and width.
//
// The input checksum is the one the FIC scheme uses, in its row-wise form xrows[j,h,s,c] (fic_device.h):
// X[r,s,c] is the sum of xrows over the batch parts j and over the input rows h that filter row r
// meets.  As there, X is never materialised:
//   chk[k] = sum_{r,s,c} X[r,s,c] * w[k,r,s,c] = sum_{h,s,c} (sum_j xrows[j,h,s,c]) * (sum of w[k,r,s,c] over the r that meet h).
// All sums are 64-bit (Sec. 4.1).
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

struct Ic2VerifyParams {
    const int8_t *w;            // [K][R][S][C]
    const int32_t *xrows;       // [parts][H][S][C]
    const long long *part;      // [nrows][kstride] partial per-filter output sums
    long long *result;          // [0..K) reduced outputs, [K..2K) checksum tensor convolved with the filters
    uint32_t *flags;            // [K]: 1 = the two differ
    int K, H, C, R, S, P, sh, ph, parts, nrows, kstride;
};

// One workgroup per filter k: the checksum convolution's value for k, the sum of the partial output
// sums of k, and the comparison (the element-wise verification of Sec. 3.2 option 2).
__global__ __launch_bounds__(256) void ic2_verify_kernel(const Ic2VerifyParams p)
{
    __shared__ long long red[2][4];
    const int k = blockIdx.x, tid = threadIdx.x;
    const int sc = p.S * p.C;
    const long long hsc = (long long)p.H * sc;
    const int8_t *wk = p.w + (long long)k * p.R * sc;
    long long chk = 0;
    for (long long e = tid; e < hsc; e += 256) {
        const int h = (int)(e / sc), rest = (int)(e - (long long)h * sc);
        int wsum = 0;                             // filter rows r that meet input row h:  h = q*sh - ph + r
        for (int r = 0; r < p.R; ++r) {
            const int t = h + p.ph - r;
            if (t >= 0 && t % p.sh == 0 && t / p.sh < p.P) wsum += wk[r * sc + rest];
        }
        if (wsum != 0) {
            long long xr = 0;
            for (int j = 0; j < p.parts; ++j) xr += p.xrows[j * hsc + e];
            chk += xr * wsum;
        }
    }
    long long osum = 0;
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
