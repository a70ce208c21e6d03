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
// filter row r meets of xrows[h,s,c].  The second step is folded into the dot product, whose
// partial sums the ICG kernel forms while it still holds its piece of xrows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace abed {

struct FicRowsParams {
    const int8_t *x;
    const int32_t *wsum;          // [R][S][C]
    int32_t *xrows;               // [parts][H][S][C]
    long long *dotpart;           // one partial dot product per workgroup [parts * H * ceil(C/64)], or null (then R = 0)
    int N, H, W, C, R, S, P, Q, sh, sw, ph, pw, parts;
    int from_rows;                // 0: from the images x; 1: xrows is given, only the partial dot products are
                                  // formed; 2: from the batch-summed image xsum, which is cleared after use
    int32_t *xsum;                // [H][W][C] int32 (from_rows == 2)
};

// sum of wsum[r][rest] over the filter rows r that meet input row h:  h = q*sh - ph + r for an output row q
__device__ __forceinline__ long long fic_wsum_meeting_row(const int32_t *wsum, int rest, int sc, int h, int R, int P, int sh, int ph)
{
    long long wv = 0;
    for (int r = 0; r < R; ++r) {
        const int t = h + ph - r;
        if (t >= 0 && t % sh == 0 && t / sh < P) wv += wsum[r * sc + rest];
    }
    return wv;
}

// One workgroup per (part of the batch, input row h, group of 64 channels).  Phase 1: lane t takes the
// 16-byte channel chunk t & 3 of the group and slot t >> 2 of 64 slots; a slot is one input column w
// (and, when the row is short, one of several interleaved subsets of the part's images); the lane sums
// its column over its images and leaves the 16 sums in LDS.  Phase 2: thread (s, c) adds the slots whose
// column w meets filter column s.  The workgroup then stores its piece of xrows and its share of the
// dot product with the filter checksum:
//   sum_{r,s,c} X * wsum = sum_{h,s,c} xrows[h,s,c] * (sum of wsum[r,s,c] over the filter rows r that meet h).
// LDS: cols = 64 x 64 ints (16-byte aligned), meets = SMAX x 64 bytes, dsum = 4 x 8 bytes.  256 threads;
// `block` is the workgroup's index among the input checksum workgroups
// (a multiple of 8 of them are launched).
constexpr int kFicRowsLdsBytes = 64 * 64 * 4 + 7 * 64 + 64;
template <int SMAX>
__device__ __forceinline__ void fic_rows_body(const FicRowsParams &p, const int block, const int tid,
                                              int (*cols)[64], unsigned char (*meets)[64], long long *dsum)
{
    const int cgroups = (p.C + 63) / 64;
    // Workgroups go to the 8 XCDs round-robin by index and every XCD has its own L2: index i is mapped to
    // piece (i & 7) * ceil(n / 8) + (i >> 3), so that one XCD takes a contiguous eighth of the pieces and the
    // channel groups that share 128-byte lines of x (neighbours in the list) meet in one L2.  (The launch
    // covers a multiple of 8 indices; the ones past the end leave.)
    const int nblocks = p.parts * p.H * cgroups;
    const int piece = (block & 7) * ((nblocks + 7) >> 3) + (block >> 3);
    if (piece >= nblocks) return;
    int b = piece;
    const int cg = b % cgroups; b /= cgroups;
    const int h = b % p.H;
    const int part = b / p.H;
    const int sc = p.S * p.C;
    int32_t *rows = p.xrows + ((long long)part * p.H + h) * sc;
    int acc[(SMAX * 64 + 255) / 256];                           // phase-2 sums of elements tid, tid + 256, ...
    long long wv[(SMAX * 64 + 255) / 256];                      // their factors of the dot product (fetched early)
#pragma unroll
    for (int j = 0; j < (SMAX * 64 + 255) / 256; ++j) {
        acc[j] = 0;
        const int e = tid + 256 * j;
        const int s = e >> 6, c = cg * 64 + (e & 63);
        wv[j] = (e < SMAX * 64 && s < p.S && c < p.C) ? fic_wsum_meeting_row(p.wsum, s * p.C + c, sc, h, p.R, p.P, p.sh, p.ph) : 0;
    }
    if (p.from_rows == 2) {
        // The previous layer's kernel has left sum_n x[n] here (Sec. 4.3, the option that generates the
        // next layer's input checksum): only the columns remain to be added.  Part 0 does it; the slice
        // of xsum this workgroup owns is cleared afterwards, ready for the producer's next additions.
        int32_t *src = p.xsum + (long long)h * p.W * p.C + cg * 64;
        if (part == 0) {
            for (int w0 = 0; w0 < p.W; w0 += 64) {
                for (int e = tid; e < SMAX * 64; e += 256) {
                    const int s = e >> 6, wc = w0 + (e & 63);
                    const int t = wc + p.pw - s;
                    meets[s][e & 63] = (s < p.S && wc < p.W && t >= 0 && t % p.sw == 0 && t / p.sw < p.Q) ? 1 : 0;
                }
                __syncthreads();
#pragma unroll
                for (int j = 0; j < (SMAX * 64 + 255) / 256; ++j) {
                    const int e = tid + 256 * j;
                    const int s = e >> 6, c = e & 63;
                    if (e < SMAX * 64 && s < p.S && cg * 64 + c < p.C) {
                        int a = 0;
                        for (int sl = 0; sl < 64 && w0 + sl < p.W; ++sl) a += meets[s][sl] ? src[(long long)(w0 + sl) * p.C + c] : 0;
                        acc[j] += a;
                    }
                }
                __syncthreads();
            }
            for (int i = tid; i < p.W * 64; i += 256) {
                const int wc = i >> 6, c = i & 63;
                if (cg * 64 + c < p.C) src[(long long)wc * p.C + c] = 0;
            }
        }
    } else if (!p.from_rows) {
        const int chunk = tid & 3, slot = tid >> 2;
        const int c0 = cg * 64 + chunk * 16;
        const int n_lo = p.N * part / p.parts, n_hi = p.N * (part + 1) / p.parts;
        const int nsub = p.W >= 64 ? 1 : 64 / p.W;              // image subsets side by side when the row is short
        const int sub = slot / p.W, w_first = slot - sub * p.W;
        const long long img = (long long)p.H * p.W * p.C;
        for (int w0 = 0; w0 < p.W; w0 += 64) {                  // 64 columns at a time
            const int w = w0 + w_first;
            // Sixteen int8 channels per load, summed two to a register: the bytes are made unsigned
            // (xor 0x80) and the even and odd bytes of each word are added in 16-bit fields, which hold
            // 256 additions; the bias 128 * count is taken off when the fields are unpacked.
            unsigned ev[4] = {0, 0, 0, 0}, od[4] = {0, 0, 0, 0};
            int count = 0;
            const bool live = c0 < p.C && sub < nsub && w < p.W;
            if (live) {
                const int8_t *src = p.x + ((long long)h * p.W + w) * p.C + c0;
                // (the host picks the parts so that a lane never takes more than 256 images)
#pragma unroll 4
                for (int n = n_lo + sub; n < n_hi; n += nsub) {
                    const int4 v = *reinterpret_cast<const int4 *>(src + n * img);
                    const unsigned words[4] = {(unsigned)v.x ^ 0x80808080u, (unsigned)v.y ^ 0x80808080u,
                                               (unsigned)v.z ^ 0x80808080u, (unsigned)v.w ^ 0x80808080u};
#pragma unroll
                    for (int q = 0; q < 4; ++q) { ev[q] += words[q] & 0x00ff00ffu; od[q] += (words[q] >> 8) & 0x00ff00ffu; }
                    ++count;
                }
            }
            int tot[16];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                tot[4 * q + 0] = (int)(ev[q] & 0xffffu) - 128 * count;
                tot[4 * q + 1] = (int)(od[q] & 0xffffu) - 128 * count;
                tot[4 * q + 2] = (int)(ev[q] >> 16) - 128 * count;
                tot[4 * q + 3] = (int)(od[q] >> 16) - 128 * count;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<int4 *>(&cols[slot][chunk * 16 + q * 4]) = make_int4(tot[4 * q], tot[4 * q + 1], tot[4 * q + 2], tot[4 * q + 3]);
            for (int e = tid; e < SMAX * 64; e += 256) {
                // does filter column s meet input column w at some output column q?  w = q*sw - pw + s
                const int s = e >> 6, sl = e & 63;
                const int sb = sl / p.W, wc = w0 + sl - sb * p.W;
                const int t = wc + p.pw - s;
                meets[s][sl] = (s < p.S && sb < nsub && wc < p.W && t >= 0 && t % p.sw == 0 && t / p.sw < p.Q) ? 1 : 0;
            }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < (SMAX * 64 + 255) / 256; ++j) {
                const int e = tid + 256 * j;
                if (e < SMAX * 64 && (e >> 6) < p.S) {
                    const int s = e >> 6, c = e & 63;
                    int a = 0;
#pragma unroll 4
                    for (int sl = 0; sl < 64; ++sl) a += meets[s][sl] ? cols[sl][c] : 0;
                    acc[j] += a;
                }
            }
            __syncthreads();
        }
    }
    long long dot = 0;
#pragma unroll
    for (int j = 0; j < (SMAX * 64 + 255) / 256; ++j) {
        const int e = tid + 256 * j;
        const int s = e >> 6, c = cg * 64 + (e & 63);
        if (e < SMAX * 64 && s < p.S && c < p.C) {
            int xr;
            if (p.from_rows == 1) xr = rows[s * p.C + c];
            else { xr = acc[j]; rows[s * p.C + c] = xr; }
            dot += (long long)xr * wv[j];
        }
    }
    for (int m = 32; m >= 1; m >>= 1) dot += __shfl_xor(dot, m, 64);
    if ((tid & 63) == 0) dsum[tid >> 6] = dot;
    __syncthreads();
    if (tid == 0 && p.dotpart) p.dotpart[piece] = dsum[0] + dsum[1] + dsum[2] + dsum[3];
}


}  // namespace abed
