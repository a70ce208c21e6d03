// Implicit-GEMM convolution kernel for gfx950 with the ABED checksum rows and
// columns riding in the same tile (Sec. 3.1, 3.2, 4.1, 4.3 of the paper).
//
// GEMM view: rows m = (pixel, image) pairs, image fastest; columns = filters;
// reduction index crs = (r, s, c) in the order the KRSC filter is stored.
// One workgroup = 4 waves.  Wave w owns WM blocks of 16 rows and ALL WK blocks
// of 16 filters of the tile, so the sum over filters of a row (FC) never
// leaves the wave.  A tile holds tile_pixels pixels for ALL images, so the sum
// over the batch (IC) never leaves the workgroup.
//
// MFMA operand roles are swapped with respect to the GEMM view: filters are the
// MFMA "A" operand (rows of D), output rows the "B" operand (columns of D).
// Then a lane holds 4 consecutive filters of one output row per block, and with
// the filter permutation below 16 consecutive filters per 4 blocks, which makes
// the NPQK store 16..64 contiguous bytes per lane.
//
// AUG = true appends one block of 16 checksum filters (d_f digit filters, rest
// zero) and one block of 16 checksum rows (8 pixel slots x 2 digit images).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace abed {

typedef int i32x4 __attribute__((ext_vector_type(4)));

enum Mode : int {
    MODE_PLAIN = 0,     // no checks
    MODE_WRITE = 2,     // write the checksum fmaps (digit level) to the workspace
    MODE_PARTIAL = 3,   // write per-tile reductions of both sides to the workspace
    MODE_CHECK = 4,     // reduce, compare, set flags
    MODE_CHECK_NEXT = 5 // as 4 + next layer's batch checksum
};

struct ConvParams {
    const int8_t *x, *w, *wchk, *xchk;
    void *y;                     // int32 or int8 [N][P][Q][K]
    const float *scale, *bias;   // epilog, or null
    uint32_t *flags;
    int8_t *xchk_next;
    // workspace views
    int32_t *ws_yf;   // MODE_WRITE: [N][P][Q][d_f]      MODE_PARTIAL: yf  [grid_m][tile_m]
    int32_t *ws_yi;   // MODE_WRITE: [d_i][P][Q][K]      MODE_PARTIAL: yi  [grid_m][8][K]
    int32_t *ws_yfi;  // MODE_WRITE: [d_i][P][Q][d_f]    MODE_PARTIAL: [grid_m][4][8]
    int32_t *ws_rs;   // MODE_PARTIAL / split K: rs [grid_n][grid_m][tile_m]
    int32_t *ws_cs;   // MODE_PARTIAL: cs [grid_m][8][K + 16]
    uint32_t *ws_count;  // arrival counters [grid_m]
    int N, H, W, C, K, R, S, sh, sw, ph, pw, P, Q;
    int crs;          // C*R*S
    int nsteps;       // ceil(crs / 64)
    int n_eff;        // batch padded to a power of two (< 16) or a multiple of 16
    int tp;           // pixels per tile
    int tm_used;      // tp * n_eff
    int d_f, d_i;
    int grid_m, grid_n;
    int mode;
    int out_int8, relu;
    int inj_on;       // ACC injection
    int inj_row;      // GEMM row (pixel * n_eff + n) of the injected element
    int inj_k;
    uint32_t inj_mask;
};

__device__ __forceinline__ int lds_off(int row, int chunk)
{
    // 64-byte rows; the 16-byte chunk position is swizzled with bits 2..3 of the row
    return row * 64 + (((chunk ^ (row >> 2)) & 3) << 4);
}

// LDS filter row (MFMA block kb, MFMA row i) <-> filter index inside the tile.
// Within each group of 64 filters the lane that owns MFMA rows 4g..4g+3 of blocks
// 4u..4u+3 holds filters 64u + 16g .. 64u + 16g + 15.
__device__ __forceinline__ int filter_of_ldsrow(int ldsrow)
{
    const int kb = ldsrow >> 4, i = ldsrow & 15;
    return ((kb >> 2) << 6) + ((i >> 2) << 4) + ((kb & 3) << 2) + (i & 3);
}

struct RowSlot {
    long long off;   // element offset of the window origin from the slot's base (may be negative)
    int h0, w0;      // window origin; h0 = INT_MIN/2 marks an invalid slot
};

__device__ __forceinline__ i32x4 ld16(const int8_t *p) { return *reinterpret_cast<const i32x4 *>(p); }

template <int WM, int WK, bool AUG>
__global__ __launch_bounds__(256) void conv_i8_kernel(const ConvParams p)
{
    constexpr int TM = 64 * WM;          // real rows per tile (maximum)
    constexpr int TK = 16 * WK;          // real filters per tile
    constexpr int ROWS_K = TK + (AUG ? 16 : 0);
    constexpr int ROWS_M = TM + (AUG ? 16 : 0);
    constexpr int STAGE = (ROWS_K + ROWS_M) * 64;
    constexpr int KPASS = (WK + 3) / 4;  // loader passes over filter rows
    constexpr int NCB = (WK + 3) / 4;    // checksum-row blocks per wave
    constexpr int TKA = TK + 16;
    constexpr int EPI_INTS = AUG ? (24 * TKA + 64 + 16 + 8) : 0;
    constexpr int LDS_BYTES = (2 * STAGE > EPI_INTS * 4) ? 2 * STAGE : EPI_INTS * 4;
    __shared__ __attribute__((aligned(16))) int8_t lds[LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    // wave index as a scalar, so that every wave-level condition is a scalar branch: matrix
    // instructions must never sit under a per-lane execution mask
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lg = lane >> 4, lj = lane & 15;
    const int mt = blockIdx.x / p.grid_n, kt = blockIdx.x - mt * p.grid_n;
    const int PQ = p.P * p.Q;
    const long long HWC = (long long)p.H * p.W * p.C;

    // ---------------- loader set-up ----------------
    const int ld_row = tid >> 2, ld_chunk = tid & 3;
    RowSlot slot[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int sl = ld_row + 64 * i;
        const int pl = sl / p.n_eff, n = sl - pl * p.n_eff;
        const int pix = mt * p.tp + pl;
        slot[i].h0 = INT_MIN / 2;
        slot[i].w0 = 0;
        slot[i].off = 0;
        if (sl < p.tm_used && n < p.N && pix < PQ) {
            const int pp = pix / p.Q, qq = pix - pp * p.Q;
            slot[i].h0 = pp * p.sh - p.ph;
            slot[i].w0 = qq * p.sw - p.pw;
            slot[i].off = n * HWC + ((long long)slot[i].h0 * p.W + slot[i].w0) * p.C;
        }
    }
    // checksum rows are loaded by wave 1, checksum filters by wave 2
    RowSlot cslot;
    cslot.h0 = INT_MIN / 2; cslot.w0 = 0; cslot.off = 0;
    if (AUG && wave == 1) {
        const int csl = (tid - 64) >> 2;          // 0..15 = digit * 8 + pixel slot
        const int t = csl & 7, jj = csl >> 3;
        const int pix = mt * p.tp + t;
        if (t < p.tp && jj < p.d_i && pix < PQ) {
            const int pp = pix / p.Q, qq = pix - pp * p.Q;
            cslot.h0 = pp * p.sh - p.ph;
            cslot.w0 = qq * p.sw - p.pw;
            cslot.off = jj * HWC + ((long long)cslot.h0 * p.W + cslot.w0) * p.C;
        }
    }
    long long koff[KPASS];                        // filter row offsets (elements), -1 = zero row
#pragma unroll
    for (int i = 0; i < KPASS; ++i) {
        const int ldsrow = ld_row + 64 * i;
        const int k = kt * TK + (WK >= 4 ? filter_of_ldsrow(ldsrow) : ldsrow);
        koff[i] = (ldsrow < TK && k < p.K) ? (long long)k * p.crs : -1;
    }
    long long ckoff = -1;
    if (AUG && wave == 2) {
        const int i = (tid - 128) >> 2;           // checksum filter row 0..15
        if (i < p.d_f && kt == p.grid_n - 1) ckoff = (long long)i * p.crs;
    }
    const bool has_fchk = AUG && (kt == p.grid_n - 1);

    // position of this thread's 16-byte chunk in (r, s, c)
    int crs_pos = ld_chunk * 16;                  // byte offset in the crs axis
    int tap_r = 0, tap_s = 0, ch = crs_pos;
    while (ch >= p.C) { ch -= p.C; if (++tap_s == p.S) { tap_s = 0; ++tap_r; } }

    i32x4 stage_m[WM], stage_k[KPASS], stage_c;
    const i32x4 zero4 = {0, 0, 0, 0};

    auto global_load = [&]() {
        const bool in_crs = crs_pos < p.crs;
        const long long tap_off = ((long long)tap_r * p.W + tap_s) * p.C + ch;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const unsigned h = (unsigned)(slot[i].h0 + tap_r), w_ = (unsigned)(slot[i].w0 + tap_s);
            stage_m[i] = (in_crs && h < (unsigned)p.H && w_ < (unsigned)p.W) ? ld16(p.x + slot[i].off + tap_off) : zero4;
        }
#pragma unroll
        for (int i = 0; i < KPASS; ++i)
            stage_k[i] = (in_crs && koff[i] >= 0) ? ld16(p.w + koff[i] + crs_pos) : zero4;
        if (AUG) {
            stage_c = zero4;
            if (wave == 1) {
                const unsigned h = (unsigned)(cslot.h0 + tap_r), w_ = (unsigned)(cslot.w0 + tap_s);
                if (in_crs && h < (unsigned)p.H && w_ < (unsigned)p.W) stage_c = ld16(p.xchk + cslot.off + tap_off);
            } else if (wave == 2) {
                if (in_crs && ckoff >= 0) stage_c = ld16(p.wchk + ckoff + crs_pos);
            }
        }
        // advance to the next step
        crs_pos += 64;
        ch += 64;
        while (ch >= p.C) { ch -= p.C; if (++tap_s == p.S) { tap_s = 0; ++tap_r; } }
    };
    auto lds_store = [&](int buf) {
        int8_t *base = lds + buf * STAGE;
#pragma unroll
        for (int i = 0; i < KPASS; ++i) {
            const int row = ld_row + 64 * i;
            if (row < TK) *reinterpret_cast<i32x4 *>(base + lds_off(row, ld_chunk)) = stage_k[i];
        }
#pragma unroll
        for (int i = 0; i < WM; ++i)
            *reinterpret_cast<i32x4 *>(base + ROWS_K * 64 + lds_off(ld_row + 64 * i, ld_chunk)) = stage_m[i];
        if (AUG) {
            if (wave == 1) *reinterpret_cast<i32x4 *>(base + ROWS_K * 64 + lds_off(TM + ((tid - 64) >> 2), ld_chunk)) = stage_c;
            if (wave == 2) *reinterpret_cast<i32x4 *>(base + lds_off(TK + ((tid - 128) >> 2), ld_chunk)) = stage_c;
        }
    };

    // ---------------- accumulators ----------------
    i32x4 acc[WM][WK];
    i32x4 accF[WM];      // checksum filters x this wave's rows
    i32x4 accC[NCB];     // checksum rows x filter blocks kb = 4c + wave
    i32x4 accX = zero4;  // corner block (wave 3)
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        accF[i] = zero4;
#pragma unroll
        for (int k = 0; k < WK; ++k) acc[i][k] = zero4;
    }
#pragma unroll
    for (int c = 0; c < NCB; ++c) accC[c] = zero4;

    // ---------------- main loop ----------------
    global_load();
    lds_store(0);
    __syncthreads();
    for (int step = 0; step < p.nsteps; ++step) {
        const int buf = step & 1;
        const bool more = step + 1 < p.nsteps;
        if (more) global_load();
        const int8_t *ldsK = lds + buf * STAGE;
        const int8_t *ldsM = ldsK + ROWS_K * 64;
        i32x4 bfr[WM], bchk = zero4;
#pragma unroll
        for (int i = 0; i < WM; ++i)
            bfr[i] = *reinterpret_cast<const i32x4 *>(ldsM + lds_off((wave * WM + i) * 16 + lj, lg));
        if (AUG) bchk = *reinterpret_cast<const i32x4 *>(ldsM + lds_off(TM + lj, lg));
#pragma unroll
        for (int kb = 0; kb < WK; ++kb) {
            const i32x4 a = *reinterpret_cast<const i32x4 *>(ldsK + lds_off(kb * 16 + lj, lg));
#pragma unroll
            for (int i = 0; i < WM; ++i)
                acc[i][kb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bfr[i], acc[i][kb], 0, 0, 0);
            if (AUG && (kb & 3) == wave)
                accC[kb >> 2] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bchk, accC[kb >> 2], 0, 0, 0);
        }
        if (AUG && has_fchk) {
            const i32x4 a = *reinterpret_cast<const i32x4 *>(ldsK + lds_off(TK + lj, lg));
#pragma unroll
            for (int i = 0; i < WM; ++i)
                accF[i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bfr[i], accF[i], 0, 0, 0);
            if (wave == 3) accX = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bchk, accX, 0, 0, 0);
        }
        if (more) lds_store(buf ^ 1);
        __syncthreads();
    }

    // ---------------- epilogue ----------------
    // Output row of lane column lj in this wave's block i.
    const long long PQK = (long long)PQ * p.K;
    int row_slot[WM];
    long long row_out[WM];        // element offset of y[n][pix][0], or -1
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int sl = (wave * WM + i) * 16 + lj;
        const int pl = sl / p.n_eff, n = sl - pl * p.n_eff;
        const int pix = mt * p.tp + pl;
        row_slot[i] = sl;
        row_out[i] = (sl < p.tm_used && n < p.N && pix < PQ) ? n * PQK + (long long)pix * p.K : -1;
    }
    // filter index (inside the tile) of register v of block kb in this lane
    auto filt = [&](int kb, int v) {
        return WK >= 4 ? ((kb >> 2) << 6) + (lg << 4) + ((kb & 3) << 2) + v : kb * 16 + lg * 4 + v;
    };

    // (1) accumulator fault injection (tests)
    if (p.inj_on) {
        const int row0 = mt * p.tm_used, k0 = kt * TK;
        if (p.inj_row >= row0 && p.inj_row < row0 + p.tm_used && p.inj_k >= k0 && p.inj_k < k0 + TK) {
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int kb = 0; kb < WK; ++kb)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (row0 + row_slot[i] == p.inj_row && k0 + filt(kb, v) == p.inj_k)
                            acc[i][kb][v] ^= (int)p.inj_mask;
        }
    }

    int *e_cs = reinterpret_cast<int *>(lds);     // [8 pixel slots][TKA]  sum over images
    int *e_yi = e_cs + 8 * TKA;                   // [16 checksum slots][TKA] digit fmaps of the checksum rows
    int *e_crs = e_yi + 16 * TKA;                 // [4 waves][16] partial sums over filters of the checksum rows
    int *e_cyf = e_crs + 64;                      // [16] corner block recombined over filter digits
    int *e_flag = e_cyf + 16;                     // [1]
    uint32_t my_flag = 0;

    if (AUG) {
        for (int i = tid; i < 8 * TKA; i += 256) e_cs[i] = 0;
        if (tid == 0) e_flag[0] = 0;
        if (tid < 16) e_cyf[tid] = 0;
        __syncthreads();

        // (2) FC: row sums over the tile's filters (Sec. 3.1), in-lane then across the 4 lane groups
        int rs[WM], yf[WM];
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            int s = 0;
#pragma unroll
            for (int kb = 0; kb < WK; ++kb) s += acc[i][kb][0] + acc[i][kb][1] + acc[i][kb][2] + acc[i][kb][3];
            s += __shfl_xor(s, 16, 64);
            s += __shfl_xor(s, 32, 64);
            rs[i] = s;
            // digit fmaps of the checksum filters sit in lane group 0, registers 0..d_f-1 (Sec. 4.1 shifts)
            yf[i] = (int)((unsigned)accF[i][0] + ((unsigned)accF[i][1] << 8) + ((unsigned)accF[i][2] << 16) + ((unsigned)accF[i][3] << 24));
        }
        // (3) checksum rows: digit fmaps to LDS, partial sums over filters
        {
            int s = 0;
#pragma unroll
            for (int c = 0; c < NCB; ++c) {
                const int kb = 4 * c + wave;
                if (kb < WK) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        e_yi[lj * TKA + filt(kb, v)] = accC[c][v];
                        s += accC[c][v];
                    }
                }
            }
            s += __shfl_xor(s, 16, 64);
            s += __shfl_xor(s, 32, 64);
            if (lg == 0) e_crs[wave * 16 + lj] = s;
            if (wave == 3) {
#pragma unroll
                for (int v = 0; v < 4; ++v) e_yi[lj * TKA + TK + lg * 4 + v] = accX[v];
                if (lg == 0)
                    e_cyf[lj] = (int)((unsigned)accX[0] + ((unsigned)accX[1] << 8) + ((unsigned)accX[2] << 16) + ((unsigned)accX[3] << 24));
            }
        }
        if (p.mode == MODE_CHECK || p.mode == MODE_CHECK_NEXT) {
            if (p.grid_n == 1) {
#pragma unroll
                for (int i = 0; i < WM; ++i)
                    if (lg == 0 && rs[i] != yf[i]) my_flag |= 1u;
            }
        }
        if (p.mode == MODE_WRITE) {
            // digit fmaps of the checksum filters: ws_yf[n][pix][d_f]
            if (has_fchk && lg == 0) {
#pragma unroll
                for (int i = 0; i < WM; ++i)
                    if (row_out[i] >= 0)
                        for (int d = 0; d < p.d_f; ++d) p.ws_yf[row_out[i] / p.K * p.d_f + d] = accF[i][d];
            }
        }
        if (p.mode == MODE_PARTIAL || (p.grid_n > 1 && p.mode != MODE_WRITE)) {
            // per-tile row sums (and the recombined checksum fmap from the tile column that has it)
            if (lg == 0) {
#pragma unroll
                for (int i = 0; i < WM; ++i) {
                    p.ws_rs[((long long)kt * p.grid_m + mt) * TM + row_slot[i]] = rs[i];
                    if (has_fchk) p.ws_yf[(long long)mt * TM + row_slot[i]] = yf[i];
                }
            }
        }
    }

    // (4) store the outputs (trimming: checksum rows and columns are never written to y, Sec. 4.3)
    {
        const int k0 = kt * TK;
        if (WK >= 4) {
#pragma unroll
            for (int u = 0; u < WK / 4; ++u) {
                const int kbase = k0 + 64 * u + 16 * lg;      // 16 consecutive filters in this lane
                if (p.out_int8) {
                    float sc[16], bi[16];
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const bool ok = kbase + e < p.K;
                        sc[e] = ok ? p.scale[kbase + e] : 0.f;
                        bi[e] = ok ? p.bias[kbase + e] : 0.f;
                    }
#pragma unroll
                    for (int i = 0; i < WM; ++i) {
                        if (row_out[i] < 0) continue;
                        int packed[4];
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            unsigned pk = 0;
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                float t = (float)acc[i][4 * u + b][v];
                                t = __fmul_rn(t, sc[4 * b + v]);
                                t = __fadd_rn(t, bi[4 * b + v]);
                                if (p.relu) t = fmaxf(t, 0.f);
                                t = rintf(t);
                                t = fminf(fmaxf(t, -128.f), 127.f);
                                pk |= ((unsigned)(int)t & 0xffu) << (8 * v);
                            }
                            packed[b] = (int)pk;
                        }
                        int8_t *dst = reinterpret_cast<int8_t *>(p.y) + row_out[i] + kbase;
                        if (kbase + 16 <= p.K && (p.K & 15) == 0) {
                            *reinterpret_cast<i32x4 *>(dst) = i32x4{packed[0], packed[1], packed[2], packed[3]};
                        } else {
                            for (int e = 0; e < 16; ++e)
                                if (kbase + e < p.K) dst[e] = (int8_t)((packed[e >> 2] >> (8 * (e & 3))) & 0xff);
                        }
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < WM; ++i) {
                        if (row_out[i] < 0) continue;
                        int32_t *dst = reinterpret_cast<int32_t *>(p.y) + row_out[i] + kbase;
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            if (kbase + 4 * b + 4 <= p.K && (p.K & 3) == 0) {
                                *reinterpret_cast<i32x4 *>(dst + 4 * b) = acc[i][4 * u + b];
                            } else {
                                for (int v = 0; v < 4; ++v)
                                    if (kbase + 4 * b + v < p.K) dst[4 * b + v] = acc[i][4 * u + b][v];
                            }
                        }
                    }
                }
            }
        } else {
            // narrow tiles (fewer than 64 filters): 4 consecutive filters per block
#pragma unroll
            for (int kb = 0; kb < WK; ++kb) {
                const int kbase = k0 + kb * 16 + lg * 4;
#pragma unroll
                for (int i = 0; i < WM; ++i) {
                    if (row_out[i] < 0) continue;
                    for (int v = 0; v < 4; ++v) {
                        if (kbase + v >= p.K) continue;
                        if (p.out_int8) {
                            float t = (float)acc[i][kb][v];
                            t = __fmul_rn(t, p.scale[kbase + v]);
                            t = __fadd_rn(t, p.bias[kbase + v]);
                            if (p.relu) t = fmaxf(t, 0.f);
                            t = fminf(fmaxf(rintf(t), -128.f), 127.f);
                            reinterpret_cast<int8_t *>(p.y)[row_out[i] + kbase + v] = (int8_t)(int)t;
                        } else {
                            reinterpret_cast<int32_t *>(p.y)[row_out[i] + kbase + v] = acc[i][kb][v];
                        }
                    }
                }
            }
        }
    }

    if (!AUG) return;

    // (5) IC: sums over the images of each pixel (Sec. 3.2 option 1).  Rows of a block
    // are lanes lj; images of one pixel are min(16, n_eff) adjacent lanes, and n_eff/16
    // adjacent blocks when n_eff >= 16.  Butterfly inside the lane segment, then one lane
    // per segment adds into the pixel's LDS slot.
    {
        const int seg = p.n_eff < 16 ? p.n_eff : 16;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int sl0 = (wave * WM + i) * 16;
            if (sl0 >= p.tm_used) continue;                       // empty block (wave-uniform)
            const int pl = (sl0 + lj) / p.n_eff;                  // pixel slot of this lane's row
            const bool writer = ((lj & (seg - 1)) == 0) && pl < 8;
#pragma unroll
            for (int kb = 0; kb <= WK; ++kb) {
                if (kb == WK && !has_fchk) continue;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    int s = (kb < WK) ? acc[i][kb][v] : accF[i][v];
                    for (int m = 1; m < seg; m <<= 1) s += __shfl_xor(s, m, 64);
                    const int f = (kb < WK) ? filt(kb, v) : TK + lg * 4 + v;
                    if (writer) atomicAdd(&e_cs[pl * TKA + f], s);
                }
            }
        }
    }
    __syncthreads();

    // (6) compare the batch sums with the checksum rows (digits recombined, Sec. 4.1)
    if (p.mode == MODE_CHECK || p.mode == MODE_CHECK_NEXT) {
        for (int idx = tid; idx < p.tp * TK; idx += 256) {
            const int t = idx / TK, f = idx - t * TK;
            const int yi = (int)((unsigned)e_yi[t * TKA + f] + ((unsigned)e_yi[(8 + t) * TKA + f] << 8));
            if (e_cs[t * TKA + f] != yi) my_flag |= 2u;
        }
        if (tid < 8) {
            const int t = tid;
            // corner, filter side: sum over filters of the checksum rows against the corner block
            unsigned s0 = 0, s1 = 0;
            for (int w = 0; w < 4; ++w) { s0 += (unsigned)e_crs[w * 16 + t]; s1 += (unsigned)e_crs[w * 16 + 8 + t]; }
            const unsigned sum_k_yi = s0 + (s1 << 8);
            const unsigned yfi = (unsigned)e_cyf[t] + ((unsigned)e_cyf[8 + t] << 8);
            if (p.grid_n == 1) {
                if (sum_k_yi != yfi) my_flag |= 4u;
            } else {
                p.ws_yfi[((long long)mt * (p.grid_n + 1) + kt) * 8 + t] = (int)sum_k_yi;
                if (has_fchk) p.ws_yfi[((long long)mt * (p.grid_n + 1) + p.grid_n) * 8 + t] = (int)yfi;
            }
            // corner, batch side: sum over images of the checksum-filter fmaps against the corner block
            if (has_fchk) {
                unsigned a = 0, b = 0;
                for (int d = 0; d < 4; ++d) {
                    a += (unsigned)e_cs[t * TKA + TK + d] << (8 * d);
                    b += ((unsigned)e_yi[t * TKA + TK + d] + ((unsigned)e_yi[(8 + t) * TKA + TK + d] << 8)) << (8 * d);
                }
                if (a != b) my_flag |= 4u;
            }
        }
        if (my_flag) atomicOr(reinterpret_cast<unsigned *>(e_flag), my_flag);
        __syncthreads();
        if (tid == 0) p.flags[mt * p.grid_n + kt] = (uint32_t)e_flag[0];
        if (p.grid_n > 1) {
            // The filters of a row are spread over grid_n workgroups: each has written its partial
            // row sums; the workgroup that arrives last adds them up and compares (bits 0 and 2 of a
            // tile-row are reported on its first tile column).
            __threadfence();
            __syncthreads();
            if (tid == 0) {
                const unsigned old = atomicAdd(&p.ws_count[mt], 1u);
                e_flag[1] = (old == (unsigned)(p.grid_n - 1));
            }
            __syncthreads();
            if (e_flag[1]) {
                __threadfence();
                unsigned late = 0;
                for (int r = tid; r < TM; r += 256) {
                    unsigned s = 0;
                    for (int c = 0; c < p.grid_n; ++c) s += (unsigned)p.ws_rs[((long long)c * p.grid_m + mt) * TM + r];
                    if (s != (unsigned)p.ws_yf[(long long)mt * TM + r]) late |= 1u;
                }
                if (tid < 8) {
                    unsigned s = 0;
                    for (int c = 0; c < p.grid_n; ++c) s += (unsigned)p.ws_yfi[((long long)mt * (p.grid_n + 1) + c) * 8 + tid];
                    if (s != (unsigned)p.ws_yfi[((long long)mt * (p.grid_n + 1) + p.grid_n) * 8 + tid]) late |= 4u;
                }
                if (late) atomicOr(&p.flags[mt * p.grid_n], late);
                if (tid == 0) p.ws_count[mt] = 0;      // ready for the next call
            }
        }
    } else if (p.mode == MODE_WRITE) {
        // digit fmaps of the checksum rows: ws_yi[d_i][pix][K], ws_yfi[d_i][pix][d_f]
        for (int idx = tid; idx < 16 * TK; idx += 256) {
            const int csl = idx / TK, f = idx - csl * TK;
            const int t = csl & 7, jj = csl >> 3, pix = mt * p.tp + t, k = kt * TK + f;
            if (t < p.tp && jj < p.d_i && pix < PQ && k < p.K)
                p.ws_yi[((long long)jj * PQ + pix) * p.K + k] = e_yi[csl * TKA + f];
        }
        if (has_fchk && tid < 64) {
            const int csl = tid >> 2, d = tid & 3;
            const int t = csl & 7, jj = csl >> 3, pix = mt * p.tp + t;
            if (t < p.tp && jj < p.d_i && pix < PQ && d < p.d_f)
                p.ws_yfi[((long long)jj * PQ + pix) * p.d_f + d] = e_yi[csl * TKA + TK + d];
        }
    } else if (p.mode == MODE_PARTIAL) {
        for (int idx = tid; idx < 8 * TKA; idx += 256) {
            const int t = idx / TKA, f = idx - t * TKA;
            const int k = (f < TK) ? kt * TK + f : p.K + (f - TK);
            if (f < TK ? (kt * TK + f < p.K) : has_fchk) {
                const long long o = ((long long)mt * 8 + t) * (p.K + 16) + k;
                p.ws_cs[o] = e_cs[t * TKA + f];
                p.ws_yi[o] = (int)((unsigned)e_yi[t * TKA + f] + ((unsigned)e_yi[(8 + t) * TKA + f] << 8));
            }
        }
        if (tid < 8) {
            const int t = tid;
            unsigned s0 = 0, s1 = 0;
            for (int w = 0; w < 4; ++w) { s0 += (unsigned)e_crs[w * 16 + t]; s1 += (unsigned)e_crs[w * 16 + 8 + t]; }
            // [grid_m][grid_n + 1][8]: partial sums over filters of the checksum rows, then the corner value
            p.ws_yfi[((long long)mt * (p.grid_n + 1) + kt) * 8 + t] = (int)(s0 + (s1 << 8));
            if (has_fchk)
                p.ws_yfi[((long long)mt * (p.grid_n + 1) + p.grid_n) * 8 + t] = (int)((unsigned)e_cyf[t] + ((unsigned)e_cyf[8 + t] << 8));
        }
    }
}

}  // namespace abed
