// Small kernels around the convolution: offline filter checksum (Sec. 3.1, 4.1,
// 4.2), online input checksum generation ICG (Sec. 3.2 option 1), the verify
// kernel of the variants that check from memory, the finish kernel of the
// partial-reduction variant, the separate epilog (Sec. 4.3), the compare kernel
// of the duplication baseline, and a one-bit flip for fault-injection tests.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace abed {

typedef int i32x4a __attribute__((ext_vector_type(4)));

// balanced base-256 digit: d in [-128,127], d == s (mod 256); rest = (s - d) / 256
__device__ __forceinline__ int take_digit(int &s)
{
    const int d = ((s + 128) & 255) - 128;
    s = (s - d) >> 8;   // exact: s - d is a multiple of 256
    return d;
}

// wsum[e] = sum_k w[k][e]; digits to wchk[d][e].  One thread per element (offline step).
__global__ void filter_checksum_i8_kernel(const int8_t *w, int8_t *wchk, int K, int crs, int d_f)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= crs) return;
    int s = 0;
    for (int k = 0; k < K; ++k) s += w[(long long)k * crs + e];
    for (int d = 0; d < d_f; ++d) wchk[(long long)d * crs + e] = (int8_t)take_digit(s);
}

// xsum[e] = sum_n x[n][e] for 16 consecutive elements per thread group of 4 lanes
// (each lane sums a quarter of the images); digits to xchk[d][e].
__global__ __launch_bounds__(256) void batch_checksum_i8_kernel(const int8_t *x, int8_t *xchk, int N, long long hwc, int d_i)
{
    const long long chunk = (long long)blockIdx.x * 64 + (threadIdx.x >> 2);
    const int part = threadIdx.x & 3;
    const long long e0 = chunk * 16;
    const bool live = e0 < hwc;
    int s[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0;
    if (live) {
        for (int n = part; n < N; n += 4) {
            const i32x4a v = *reinterpret_cast<const i32x4a *>(x + n * hwc + e0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                s[4 * j + 0] += (v[j] << 24) >> 24;
                s[4 * j + 1] += (v[j] << 16) >> 24;
                s[4 * j + 2] += (v[j] << 8) >> 24;
                s[4 * j + 3] += v[j] >> 24;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        s[i] += __shfl_xor(s[i], 1, 64);
        s[i] += __shfl_xor(s[i], 2, 64);
    }
    if (live && part == 0) {
        for (int d = 0; d < d_i; ++d) {
            i32x4a o;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                unsigned pk = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) pk |= ((unsigned)take_digit(s[4 * j + b]) & 0xffu) << (8 * b);
                o[j] = (int)pk;
            }
            *reinterpret_cast<i32x4a *>(xchk + d * hwc + e0) = o;
        }
    }
}

struct VerifyParams {
    const int32_t *y;     // ConvOut [N][PQ][K]
    const int32_t *yf;    // [N][PQ][d_f]   digit fmaps of the checksum filters
    const int32_t *yi;    // [d_i][PQ][K]   digit fmaps of the checksum images
    const int32_t *yfi;   // [d_i][PQ][d_f]
    uint32_t *flags;
    int N, PQ, K, d_f, d_i, tp, tile_n, grid_n;
};

// Variants that verify from memory (Sec. 4.3, unfused option): read ConvOut back,
// reduce over filters and over the batch, compare with the checksum fmaps.
// One workgroup per tile-row (tp pixels, all images, all filters).
__global__ __launch_bounds__(256) void verify_i8_kernel(const VerifyParams p)
{
    extern __shared__ int vs[];
    int *cs = vs;                       // [tp][K]   sum over images
    int *syf = cs + p.tp * p.K;         // [tp]      sum over images of the FC fmap
    int *fl = syf + p.tp;               // [grid_n]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int mt = blockIdx.x;
    for (int i = tid; i < p.tp * p.K + p.tp + p.grid_n; i += 256) vs[i] = 0;
    __syncthreads();
    const int rows = p.tp * p.N;
    for (int r = wave; r < rows; r += 4) {
        const int t = r / p.N, n = r - t * p.N;
        const int pix = mt * p.tp + t;
        if (pix >= p.PQ) continue;
        const int32_t *row = p.y + ((long long)n * p.PQ + pix) * p.K;
        unsigned s = 0;
        for (int k = lane; k < p.K; k += 64) {
            const int v = row[k];
            s += (unsigned)v;
            atomicAdd(&cs[t * p.K + k], v);
        }
        for (int m = 32; m >= 1; m >>= 1) s += (unsigned)__shfl_xor((int)s, m, 64);
        if (lane == 0) {
            unsigned c = 0;
            for (int d = 0; d < p.d_f; ++d) c += (unsigned)p.yf[((long long)n * p.PQ + pix) * p.d_f + d] << (8 * d);
            if (s != c) atomicOr(reinterpret_cast<unsigned *>(&fl[0]), 1u);
            atomicAdd(&syf[t], (int)c);
        }
    }
    __syncthreads();
    for (int i = tid; i < p.tp * p.K; i += 256) {
        const int t = i / p.K, k = i - t * p.K;
        const int pix = mt * p.tp + t;
        if (pix >= p.PQ) continue;
        unsigned c = 0;
        for (int j = 0; j < p.d_i; ++j) c += (unsigned)p.yi[((long long)j * p.PQ + pix) * p.K + k] << (8 * j);
        if ((unsigned)cs[i] != c) atomicOr(reinterpret_cast<unsigned *>(&fl[k / p.tile_n]), 2u);
    }
    // corner: sum_n yf and sum_k yi against conv(xsum, wsum)
    for (int t = wave; t < p.tp; t += 4) {
        const int pix = mt * p.tp + t;
        if (pix >= p.PQ) continue;
        unsigned sk = 0;
        for (int k = lane; k < p.K; k += 64)
            for (int j = 0; j < p.d_i; ++j) sk += (unsigned)p.yi[((long long)j * p.PQ + pix) * p.K + k] << (8 * j);
        for (int m = 32; m >= 1; m >>= 1) sk += (unsigned)__shfl_xor((int)sk, m, 64);
        if (lane == 0) {
            unsigned c = 0;
            for (int j = 0; j < p.d_i; ++j)
                for (int d = 0; d < p.d_f; ++d) c += (unsigned)p.yfi[((long long)j * p.PQ + pix) * p.d_f + d] << (8 * (j + d));
            if (sk != c || (unsigned)syf[t] != c) atomicOr(reinterpret_cast<unsigned *>(&fl[0]), 4u);
        }
    }
    __syncthreads();
    for (int i = tid; i < p.grid_n; i += 256) p.flags[(long long)mt * p.grid_n + i] = (uint32_t)fl[i];
}

struct FinishParams {
    const int32_t *rs;    // [grid_n][grid_m][tm]
    const int32_t *yf;    // [grid_m][tm]
    const int32_t *cs;    // [grid_m][8][K + 16]
    const int32_t *yi;    // [grid_m][8][K + 16]
    const int32_t *yfi;   // [grid_m][grid_n + 1][8]
    uint32_t *flags;
    int K, tm, tp, tile_n, grid_m, grid_n, d_f;
};

// Partial-reduction variant: sum the per-tile partial sums across tile columns and compare.
__global__ __launch_bounds__(256) void finish_i8_kernel(const FinishParams p)
{
    extern __shared__ int fs[];   // [grid_n]
    const int tid = threadIdx.x, mt = blockIdx.x;
    for (int i = tid; i < p.grid_n; i += 256) fs[i] = 0;
    __syncthreads();
    for (int r = tid; r < p.tm; r += 256) {
        unsigned s = 0;
        for (int kt = 0; kt < p.grid_n; ++kt) s += (unsigned)p.rs[((long long)kt * p.grid_m + mt) * p.tm + r];
        if (s != (unsigned)p.yf[(long long)mt * p.tm + r]) atomicOr(reinterpret_cast<unsigned *>(&fs[0]), 1u);
    }
    const int KA = p.K + 16;
    for (int i = tid; i < p.tp * p.K; i += 256) {
        const int t = i / p.K, k = i - t * p.K;
        const long long o = ((long long)mt * 8 + t) * KA + k;
        if (p.cs[o] != p.yi[o]) atomicOr(reinterpret_cast<unsigned *>(&fs[k / p.tile_n]), 2u);
    }
    if (tid < p.tp) {
        const int t = tid;
        unsigned s = 0;
        for (int kt = 0; kt < p.grid_n; ++kt) s += (unsigned)p.yfi[((long long)mt * (p.grid_n + 1) + kt) * 8 + t];
        const unsigned yfi = (unsigned)p.yfi[((long long)mt * (p.grid_n + 1) + p.grid_n) * 8 + t];
        unsigned a = 0, b = 0;
        for (int d = 0; d < 4; ++d) {
            const long long o = ((long long)mt * 8 + t) * KA + p.K + d;
            a += (unsigned)p.cs[o] << (8 * d);
            b += (unsigned)p.yi[o] << (8 * d);
        }
        if (s != yfi || a != b) atomicOr(reinterpret_cast<unsigned *>(&fs[0]), 4u);
    }
    __syncthreads();
    for (int i = tid; i < p.grid_n; i += 256) p.flags[(long long)mt * p.grid_n + i] = (uint32_t)fs[i];
}

// Separate epilog (Sec. 4.3): ConvOut int32 -> int8, 4 elements per thread.
__global__ void epilog_i8_kernel(const int32_t *acc, int8_t *out, const float *scale, const float *bias,
                                 int relu, long long total, int K)
{
    const long long i = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i >= total) return;
    unsigned pk = 0;
    for (int e = 0; e < 4 && i + e < total; ++e) {
        const int k = (int)((i + e) % K);
        float t = (float)acc[i + e];
        t = __fmul_rn(t, scale[k]);
        t = __fadd_rn(t, bias[k]);
        if (relu) t = fmaxf(t, 0.f);
        t = fminf(fmaxf(rintf(t), -128.f), 127.f);
        if (i + 4 <= total && (total & 3) == 0) pk |= ((unsigned)(int)t & 0xffu) << (8 * e);
        else out[i + e] = (int8_t)(int)t;
    }
    if (i + 4 <= total && (total & 3) == 0) *reinterpret_cast<unsigned *>(out + i) = pk;
}

// Duplication baseline: element-wise comparison of two outputs, 16 bytes per thread.
__global__ void compare_kernel(const void *a, const void *b, long long bytes, uint32_t *flag)
{
    const long long i = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * 16;
    if (i >= bytes) return;
    bool diff = false;
    if (i + 16 <= bytes) {
        const i32x4a va = *reinterpret_cast<const i32x4a *>((const char *)a + i);
        const i32x4a vb = *reinterpret_cast<const i32x4a *>((const char *)b + i);
        diff = (va[0] != vb[0]) | (va[1] != vb[1]) | (va[2] != vb[2]) | (va[3] != vb[3]);
    } else {
        for (long long j = i; j < bytes; ++j) diff |= ((const char *)a)[j] != ((const char *)b)[j];
    }
    if (diff) atomicOr(flag, 1u);
}

__global__ void fill_u32_kernel(uint32_t *p, long long n, uint32_t v)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

__global__ void flip_bit_u32_kernel(uint32_t *p, long long index, uint32_t mask)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) p[index] ^= mask;
}

}  // namespace abed
