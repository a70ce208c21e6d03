// Implicit-GEMM int8 convolution for gfx950 with the ABED checksum rows and
// columns riding in the same tiles (Sec. 3.1, 3.2, 4.1, 4.3 of the paper).
//
// The checked convolution is the plain convolution of an AUGMENTED problem:
//   batch entries  e = 0..N-1 real images, e = N..N+d_i-1 the int8 digit images of
//                  the batch checksum xsum = sum_n x[n]          (Sec. 3.2 option 1, 4.1)
//   filter blocks  of 16 filters: blocks 0..ceil(K/16)-1 real, then one block whose
//                  rows 0..d_f-1 are the int8 digit filters of wsum = sum_k w[k]
//                  and whose other rows are zero                  (Sec. 3.1, 4.1)
// followed by an epilogue that forms, for every output row, the FC residual
//   sum_k y[row,k] - sum_i (yf_i[row] << 8i)
// and for every (pixel, filter) the IC residual
//   sum_n y[n,pixel,k] - sum_j (yi_j[pixel,k] << 8j),
// both mod 2^32; a non-zero residual is an error.  Digit rows and the digit
// block get the same treatment, which checks the checksums against each other
// (the corner of the row+column scheme, Sec. 2.1).
// Either scheme can run alone (Table 1 of Sec. 3.4 compares them): with d_i = 0 there are no digit
// images and no IC residual, with d_f = 0 no digit block and no FC residual; the corner needs both.
// When K is not a multiple of 16 and the last real block has d_f free rows, the digit filters can
// take those rows instead of a block of their own (the caller stores them behind the K filters in
// one buffer): the layer then costs no more matrix work than without FC.
//
// Tile = 16 consecutive output pixels x MB batch entries x WK filter blocks.
// MFMA operand roles: filters are the "A" operand (rows of D), the 16 pixels of
// one batch entry the "B" operand (columns of D).  So lane (g, j) of a wave holds,
// per (entry, filter block), pixel j and filters 4g..4g+3 of the block, and
//   - the sum over filters (FC) is a sum over registers plus two cross-lane steps,
//   - the sum over the batch (IC) is a sum over registers only,
// because all entries of a tile share the same 16 pixels in the same lanes.
// Wave w owns entries [w*WM, (w+1)*WM) of the tile and all WK filter blocks.
//
// A workgroup has KG groups of 4 waves.  With KG > 1 the groups split the reduction axis: a
// pipeline stage holds KG consecutive 64-byte steps, group g loads and multiplies step g of
// the stage, and after the loop the groups' accumulators are added through LDS into group 0,
// which runs the epilogue alone.  This puts 2 or 4 waves on every SIMD (the matrix pipe
// stays busy while another wave waits for LDS or for the barrier) on layers whose grid
// is too small to fill the chip with several workgroups per CU.
//
// Operands reach LDS by direct global->LDS buffer loads (no staging registers), NST
// stages deep; out-of-image taps and out-of-range rows are masked by the buffer
// descriptor's range check.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include "fic_device.h"

namespace abed {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

enum Mode : int {
    MODE_PLAIN = 0,     // no checks (n_entries = N, no digit block)
    MODE_WRITE = 2,     // write the digit fmaps to the workspace, a verify kernel compares
    MODE_PARTIAL = 3,   // write per-tile residuals to the workspace, a finish kernel compares
    MODE_CHECK = 4,     // compare in the kernel and set the flags
    MODE_CHECK_NEXT = 5 // as 4, and emit the next layer's batch checksum digits
};

struct ConvParams {
    const int8_t *x, *w, *wchk, *xchk;
    void *y;                     // int32 or int8 [N][P][Q][K]
    const float *scale, *bias;   // epilog (Sec. 4.3), or null
    uint32_t *flags;             // [grid_m][grid_b][grid_n]
    int8_t *xchk_next;           // [d_i][PQ][K]
    int32_t *ws_yf;              // MODE_WRITE: [N][PQ][d_f]
    int32_t *ws_yi;              // MODE_WRITE: [d_i][PQ][K]
    int32_t *ws_yfi;             // MODE_WRITE: [d_i][PQ][d_f]
    int32_t *ws_fc;              // FC residual partials [grid_m][grid_b][grid_n][MB*16]
    int32_t *ws_ic;              // IC residual partials [grid_m][grid_n][grid_b][WK*256]
    int32_t *ws_nx;              // partial batch sums of the int8 output, same shape as ws_ic
    uint32_t *cnt_fc;            // arrival counters [grid_m][grid_b]
    uint32_t *cnt_ic;            // arrival counters [grid_m][grid_n]
    int N, H, W, C, K, R, S, sh, sw, ph, pw, P, Q;
    int cb;           // bytes of one filter tap: C * element size
    int crsb;         // bytes of one filter: C*R*S * element size
    int nsteps;       // ceil(crsb / 64)
    int n_entries;    // N, or N + d_i when checked
    int n_fblk;       // ceil(K/16), or that + 1 when checked
    int kblk;         // ceil(K/16): index of the digit block
    int d_f, d_i;
    int packed_df;    // d_f when the digit filters are rows K..K+d_f-1 of the last real block (and of w's buffer), else 0
    int grid_m, grid_b, grid_n;
    int kt_slowest;   // order of the tile list: 1 = filter tile slowest, 0 = pixel group slowest
    int mode;
    int out_int8, relu;
    // accumulator fault injection (tests): tile coordinates of the element
    int inj_on, inj_pg, inj_nt, inj_kt, inj_mb, inj_kb, inj_lane, inj_v;
    uint32_t inj_mask;
    int dbg;          // timing experiments (builds with ABED_ENABLE_DBG only): bit 0 ends the kernel before its stores, bit 1 skips the main loop
    int out_fp32;      // fp16 path: 1 = fp32 output
    float rtol, atol;  // fp16 path: threshold of the checks
    int l1;            // fp16 path: threshold relative to the sum of magnitudes of the reduced elements
    // FIC scheme (Sec. 3.3).  fic_ocs: per-tile sums of all accumulators [ntiles], or null.  The first
    // fic_rows_lead workgroups of the launch (the number of pieces of the input checksum, fic_parts * H *
    // ceil(C / 64), rounded up to a multiple of 8; 0 = none) make the input checksum and its partial dot
    // products instead of a tile; they depend on nothing the tiles produce and nothing waits for them
    // inside the launch.
    long long *fic_ocs;
    const int32_t *fic_wsum;       // filter checksum [R][S][C]
    int32_t *fic_xrows;            // row-wise input checksum [fic_parts][H][S][C]
    long long *fic_dotpart;        // one per piece of the input checksum (in-loop input side: one per (pixel group, batch tile))
    int fic_parts, fic_rows_lead, fic_from_rows;
    int32_t *fic_xsum_in;          // batch-summed input image [H][W][C] handed over by the previous layer (fic_from_rows == 2)
    int32_t *fic_xsum_next;        // batch sum of this layer's int8 output [P][Q][K], added to (must start at zero), or null
    // FIC with the input side formed in the main loop (int8): fic_wdig = three balanced base-256 digits of the
    // filter checksum, [3][nsteps * 64] int8 along the reduction axis (zero beyond it), or null.  The tiles of
    // filter tile 0 multiply every activation fragment they feed to the matrix units with the digits as well
    // (the sum over a tile's rows of row . filter checksum) and leave one 64-bit partial per (pixel group,
    // batch tile) in fic_dotpart.  The launch then brings 3 * nstages * KG * 64 bytes of dynamic LDS (at
    // least 128) for the digits.
    const int8_t *fic_wdig;
    // a lane's accumulators add up inside 32 bits (R*S*C * 4*WM*WK * 2^14 < 2^31) and no fault is injected: the
    // lane sums are formed in 32 bits.  A faulty accumulator can then wrap a lane's sum; the reported output
    // checksum is off by a multiple of 2^32 in that case, and still differs from the dot product.
    int fic_sum32;
    int fic_ndig;                  // digits in use: 2 while 128 K < 2^15, else 3 (the third row is zero otherwise)
    // IC option 2 (Sec. 3.2): per-filter sums of a tile's accumulators over its pixels and entries,
    // [grid_m * grid_b][grid_n * WK * 16] int64, or null
    long long *ic2_part;
};

__device__ __forceinline__ int lds_off(int row, int chunk)
{
    // 64-byte rows; the 16-byte chunk position is swizzled with bits 1..2 of the row, so that the 8
    // lanes a 16-byte-per-lane LDS read serves per cycle (8 consecutive rows, same chunk) fall into
    // 8 different 16-byte slots of the 128-byte bank window
    return row * 64 + (((chunk ^ (row >> 1)) & 3) << 4);
}

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding:
// vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
#define ABED_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | 0x0F70)

__device__ __forceinline__ int requant(int acc, float sc, float bi, int relu)
{
    float t = (float)acc;
    t = __fmul_rn(t, sc);
    t = __fadd_rn(t, bi);
    if (relu) t = fmaxf(t, 0.f);
    t = fminf(fmaxf(rintf(t), -128.f), 127.f);
    return (int)t;
}

// The epilog for four accumulators at once, packed into four bytes (first value in the low byte).  Same arithmetic as
// requant(), in fewer vector instructions: the clamp comes before the rounding (both are monotone and the bounds are
// integers, so the order does not matter; with ReLU the lower bound is 0), and the rounding to nearest even is done by
// the addition of 1.5 * 2^23, which leaves the integer, in two's complement, in the low mantissa bits.
__device__ __forceinline__ unsigned requant_pack4(const int (&acc)[4], const float (&sc)[4], const float (&bi)[4], int relu)
{
#if defined(__HIP_DEVICE_COMPILE__)
    const float lo = relu ? 0.f : -128.f;
    unsigned u[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        float t = (float)acc[v];
        t = __fmul_rn(t, sc[v]);
        t = __fadd_rn(t, bi[v]);
        t = __builtin_amdgcn_fmed3f(t, lo, 127.f);
        u[v] = __builtin_bit_cast(unsigned, __fadd_rn(t, 12582912.f));
    }
    return __builtin_amdgcn_perm(u[1], u[0], 0x0c0c0400u) | __builtin_amdgcn_perm(u[3], u[2], 0x04000c0cu);
#else
    return 0u;
#endif
}

// Residual partials that another workgroup will read: written through to device-coherent
// memory and read back past the non-coherent caches (relaxed device-scope atomics), so that no
// cache write-back fence is needed; ordering comes from waiting for the stores to complete
// before the arrival counter is bumped.
__device__ __forceinline__ void st_dev(int *p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ int ld_dev(const int *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// 16-byte versions: one write-through store / cache-bypassing load (device scope) per lane
__device__ __forceinline__ void st_dev4(int *p, i32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}
#if defined(__HIP_DEVICE_COMPILE__)
// 16 bytes per lane read past the non-coherent caches (device scope), as a buffer load so that the
// compiler keeps several of them in flight
__device__ __forceinline__ i32x4 ld_dev4(const __amdgpu_buffer_rsrc_t rs, int byte_off)
{
    return __builtin_bit_cast(i32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, byte_off, 0, 16 /* sc1 */));
}
#endif

#if defined(__HIP_DEVICE_COMPILE__)
// OR of the three flag bits over the lanes of a wave
__device__ __forceinline__ uint32_t wave_or3(uint32_t f)
{
    return (__builtin_amdgcn_ballot_w64((f & 1u) != 0) ? 1u : 0u) | (__builtin_amdgcn_ballot_w64((f & 2u) != 0) ? 2u : 0u) |
           (__builtin_amdgcn_ballot_w64((f & 4u) != 0) ? 4u : 0u);
}
#endif

// balanced base-256 digit (same rule as the ICG kernel)
__device__ __forceinline__ int next_digit(int &s)
{
    const int d = ((s + 128) & 255) - 128;
    s = (s - d) >> 8;
    return d;
}

#if defined(__HIP_DEVICE_COMPILE__)
// Sum of a 64-bit integer (magnitude below 2^46) over the 64 lanes of a wave on the matrix unit, which is idle
// in the epilogue: as doubles, exactly.  A 16x16x4 product of the lanes' values (A[i][k] = lane i + 16 k)
// with a matrix of ones leaves the sum over k of row i in every column; a lane adds the four rows it holds,
// and the same product once more adds the four groups of rows.  Every lane gets the total.  All lanes of the
// wave must be active (matrix instructions ignore the execution mask).
__device__ __forceinline__ long long wave_sum64(long long t)
{
    typedef double f64x4 __attribute__((ext_vector_type(4)));
    const f64x4 zero = {0.0, 0.0, 0.0, 0.0};
    f64x4 d = __builtin_amdgcn_mfma_f64_16x16x4f64((double)t, 1.0, zero, 0, 0, 0);
    const double rows = (d[0] + d[1]) + (d[2] + d[3]);
    d = __builtin_amdgcn_mfma_f64_16x16x4f64(rows, 1.0, zero, 0, 0, 0);
    return (long long)d[0];
}
#endif

// F16 = false: int8 data, int32 accumulators, exact checks mod 2^32.
// F16 = true: fp16 data, fp32 accumulators, threshold checks (Sec. 7); the two checksum tensors
// per side are the hi/lo pair, recombined by addition.
// FICV = true (int8 only): the build of the kernel that also forms the FIC scheme's dot product in the main
// loop (fic_wdig); kept apart so that the other launches carry none of it.
template <bool F16, int WM, int WK, int NST, int KG, bool FICV = false>
__global__ __launch_bounds__(256 * KG) void conv_kernel(const ConvParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)   // the host pass needs the signature only (the body uses device-only types)
    using acc_t = typename std::conditional<F16, f32x4, i32x4>::type;
    constexpr int MB = 4 * WM;                 // batch entries per tile
    constexpr int NB = WK + MB;                // 1 KB blocks per stage: filter blocks, then entry blocks
    constexpr int L = (NB + 3) / 4;            // direct-to-LDS loads per wave and step
    constexpr int SUB = NB * 1024;              // one 64-byte step of the tile
    constexpr int STAGE = KG * SUB;
    constexpr int EPI_BYTES = (F16 ? 12 : 4) * WK * 1024 + 128 + (F16 ? 0 : WK * 128);   // + misc words, + the tile's scale and bias
    constexpr int RED_BYTES = (KG - 1) * 4 * WM * WK * 1024;   // accumulators of groups 1..KG-1
    constexpr int FIC_BYTES = F16 ? 0 : kFicRowsLdsBytes;      // the input checksum workgroups of the FIC scheme
    constexpr int LDS_MIN0 = EPI_BYTES > RED_BYTES ? EPI_BYTES : RED_BYTES;
    constexpr int LDS_MIN = LDS_MIN0 > FIC_BYTES ? LDS_MIN0 : FIC_BYTES;
    constexpr int LDS_BYTES = (NST * STAGE > LDS_MIN) ? NST * STAGE : LDS_MIN;
    static_assert((NST - 1) * L <= 63, "vmcnt is a 6-bit counter");
    __shared__ __attribute__((aligned(1024))) int8_t lds[LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    // wave index as a scalar: every wave-level condition must be a scalar branch, matrix
    // instructions ignore the per-lane execution mask
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = KG > 1 ? wave_all >> 2 : 0;  // group along the reduction axis
    const int wave = wave_all & 3;              // position inside the group: which entries
    const int lg = lane >> 4, lj = lane & 15;
    const bool aug = p.mode != MODE_PLAIN;

    // Block index -> tile.  Workgroups go to the 8 XCDs round-robin by block index, and every XCD has
    // its own L2, so blocks b, b + 8, b + 16, ... get consecutive tiles: one XCD then works on one
    // contiguous eighth of the tile list.  The list is ordered so that this eighth shares the larger
    // operand: filter tile slowest when the filters outweigh the activations, pixel group slowest
    // otherwise.  (Only locality depends on how the hardware places blocks, never the result.)
    const int ntiles = p.grid_m * p.grid_b * p.grid_n;
    int blk = (int)blockIdx.x;
    if constexpr (!F16) {
        // FIC scheme: the leading workgroups make the input checksum (Sec. 3.3) beside the tiles
        if (blk < p.fic_rows_lead) {
            if (tid >= 256) return;               // (indices past the last piece leave inside)
            FicRowsParams rp;
            rp.x = p.x; rp.wsum = p.fic_wsum; rp.xrows = p.fic_xrows; rp.dotpart = p.fic_dotpart;
            rp.N = p.N; rp.H = p.H; rp.W = p.W; rp.C = p.C; rp.R = p.fic_wsum ? p.R : 0; rp.S = p.S; rp.P = p.P; rp.Q = p.Q;
            rp.sh = p.sh; rp.sw = p.sw; rp.ph = p.ph; rp.pw = p.pw; rp.parts = p.fic_parts; rp.from_rows = p.fic_from_rows; rp.xsum = p.fic_xsum_in;
            int (*cols)[64] = reinterpret_cast<int (*)[64]>(lds);
            unsigned char (*meets)[64] = reinterpret_cast<unsigned char (*)[64]>(lds + 64 * 64 * 4);
            long long *dsum = reinterpret_cast<long long *>(lds + 64 * 64 * 4 + 7 * 64);
            fic_rows_body<7>(rp, blk, tid, cols, meets, dsum);
            return;
        }
        blk -= p.fic_rows_lead;
    }
    const int per_xcd = (ntiles + 7) >> 3;
    int bid = (blk & 7) * per_xcd + (blk >> 3);
    if (bid >= ntiles) return;                   // the grid is rounded up to a multiple of 8
    int kt, nt, pg;
    if (p.kt_slowest) {
        pg = bid % p.grid_m; bid /= p.grid_m;
        nt = bid % p.grid_b;
        kt = bid / p.grid_b;
    } else {
        kt = bid % p.grid_n; bid /= p.grid_n;
        nt = bid % p.grid_b;
        pg = bid / p.grid_b;
    }
    const int PQ = p.P * p.Q;
    const long long HWC = (long long)p.H * p.W * p.cb;      // bytes of one image

    // ---------------- loader set-up ----------------
    // Operands are fetched with buffer loads straight into LDS: a buffer descriptor per tensor (scalar
    // registers), a per-lane byte offset, and a scalar byte offset per block.  An offset at or beyond
    // the descriptor's size reads as zero, which is how padding taps, rows past K or N and the tail of
    // the reduction axis are masked.  In a 1 KB block lane l fills row l>>2, chunk position l&3.
    constexpr int OOB = 0x7ffffff0;             // never below a descriptor's size (sizes are < 2^31 - 16)
    const int ld_row = lane >> 2;
    const int ld_chunk = (lane & 3) ^ ((ld_row >> 1) & 3);   // which 16 bytes of the 64-byte step this lane fetches
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, p.N * (int)HWC, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_xc = __builtin_amdgcn_make_buffer_rsrc((void *)p.xchk, 0, p.xchk ? p.d_i * (int)HWC : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)p.w, 0, (p.K + p.packed_df) * p.crsb, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_wc = __builtin_amdgcn_make_buffer_rsrc((void *)p.wchk, 0, p.wchk ? p.d_f * p.crsb : 0, 0x00020000);
    // pixel of this lane's row (the same for every entry block)
    int h0 = -(1 << 20), w0 = 0;                             // a pixel beyond the output: every tap test fails
    int lane_base = 0;                                       // byte offset of tap (0,0), channel chunk of this lane
    {
        const int pix = pg * 16 + ld_row;
        if (pix < PQ) {
            const int pp = pix / p.Q, qq = pix - pp * p.Q;
            h0 = pp * p.sh - p.ph;
            w0 = qq * p.sw - p.pw;
            lane_base = (h0 * p.W + w0) * p.cb + ld_chunk * 16;
        }
    }
    // the blocks this wave loads each step: block b = wave + 4 i < NB.  When NB is not a multiple of 4 the
    // waves from NB % 4 on have one load fewer (their last slot is skipped, not duplicated: every
    // vector-memory instruction per step counts on the small layers), and wait for one fewer.
    // Everything about a block that does not change from step to step is settled here: its
    // descriptor (a descriptor of size 0 masks a whole block), whether it is a filter block, the
    // scalar offset of an entry block's image, the per-lane row offset of a filter block.
    const __amdgpu_buffer_rsrc_t rs_none = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, 0, 0x00020000);
    __amdgpu_buffer_rsrc_t blk_rs[L];
    bool blk_filter[L];   // wave-uniform
    int blk_soff[L];      // wave-uniform scalar byte offset (entry blocks: the image)
    int blk_voff[L];      // per-lane byte offset of the row at step 0 (filter blocks), or OOB
#pragma unroll
    for (int i = 0; i < L; ++i) {
        int b = wave + 4 * i;
        if (b > NB - 1) b = NB - 1;                          // (slot unused, see short_wave)
        blk_rs[i] = rs_none; blk_soff[i] = 0; blk_voff[i] = OOB;
        blk_filter[i] = b < WK;
        if (b < WK) {
            const int fb = kt * WK + b;                       // global filter block
            const int f = fb * 16 + ld_row;
            if (fb < p.kblk) { blk_rs[i] = rs_w; if (f < p.K + p.packed_df) blk_voff[i] = f * p.crsb + ld_chunk * 16; }
            else if (fb == p.kblk && fb < p.n_fblk) { blk_rs[i] = rs_wc; if (ld_row < p.d_f) blk_voff[i] = ld_row * p.crsb + ld_chunk * 16; }
        } else {
            const int e = nt * MB + (b - WK);
            if (e < p.N) { blk_rs[i] = rs_x; blk_soff[i] = e * (int)HWC; }
            else if (e < p.n_entries) { blk_rs[i] = rs_xc; blk_soff[i] = (e - p.N) * (int)HWC; }
        }
    }

    // Position on the reduction axis (bytes).  Fast path: when a tap's bytes are a multiple of 64
    // (and the filter has at most 64 taps) every chunk of a step lies in one tap, so the tap, the
    // byte offset of the step inside an image and the step's offset inside a filter row live in
    // scalar registers, and each lane only keeps a bit mask of the taps that fall inside the image
    // for its pixel.  Otherwise the tap is tracked per lane.
    const bool utap = (p.cb & 63) == 0 && p.R * p.S <= 64;
    unsigned mask_lo = 0, mask_hi = 0;                       // per lane: bit t set = tap t is inside the image
    if (utap) {
        int t = 0;
        for (int r = 0; r < p.R; ++r)
            for (int c = 0; c < p.S; ++c, ++t) {
                const unsigned ok = ((unsigned)(h0 + r) < (unsigned)p.H && (unsigned)(w0 + c) < (unsigned)p.W) ? 1u : 0u;
                if (t < 32) mask_lo |= ok << t; else mask_hi |= ok << (t - 32);
            }
    }
    int s_step = 0;                                          // uniform: 64 * step
    int s_off = 0, s_ch = 0, s_tap = 0, s_col = 0;           // uniform (fast path): offset in the image, channel byte, tap, tap column
    const int row_jump = (p.W - p.S) * p.cb;                 // extra offset when the tap moves to the next filter row
    int tap_r = 0, tap_s = 0, ch = ld_chunk * 16;            // per lane (slow path)
    if (!utap)
        while (ch >= p.cb) { ch -= p.cb; if (++tap_s == p.S) { tap_s = 0; ++tap_r; } }

    // move the position one 64-byte step along the reduction axis (ut: the fast path, as a
    // compile-time tag so that the main loop is compiled once per path without branches on it)
    auto advance = [&](auto ut) {
        if constexpr (decltype(ut)::value) {
            s_off += 64; s_ch += 64;
            if (s_ch == p.cb) { s_ch = 0; ++s_tap; if (++s_col == p.S) { s_col = 0; s_off += row_jump; } }
        } else {
            ch += 64;
            while (ch >= p.cb) { ch -= p.cb; if (++tap_s == p.S) { tap_s = 0; ++tap_r; } }
        }
        s_step += 64;
    };
    for (int g = 0; g < kg; ++g) {                           // group g starts at step g
        if (utap) advance(std::true_type{}); else advance(std::false_type{});
    }

    constexpr int REM = NB % 4;
    const bool short_wave = REM != 0 && wave >= REM;         // this wave's last slot lies beyond the tile's blocks
    auto issue = [&](int stage, auto ut) {
        int voff_x;            // per-lane offset of this step's chunk inside an image, or OOB
        const bool live = s_step < p.crsb;                   // uniform: the step starts inside the reduction axis
        bool in_crs = live;    // this lane's chunk lies inside the reduction axis
        if constexpr (decltype(ut)::value) {
            const unsigned m = (s_tap & 32) ? mask_hi : mask_lo;
            const bool inb = live && ((m >> (s_tap & 31)) & 1u);
            voff_x = inb ? lane_base + s_off : OOB;
        } else {
            in_crs = s_step + ld_chunk * 16 < p.crsb;
            const bool inb = in_crs && (unsigned)(h0 + tap_r) < (unsigned)p.H && (unsigned)(w0 + tap_s) < (unsigned)p.W;
            voff_x = inb ? ((h0 + tap_r) * p.W + (w0 + tap_s)) * p.cb + ch : OOB;
        }
        int8_t *sbase = lds + stage * STAGE + kg * SUB;
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const int b = wave + 4 * i;
            if (i == L - 1 && short_wave) break;             // wave-uniform
            __attribute__((address_space(3))) void *dst = (__attribute__((address_space(3))) void *)(sbase + b * 1024);
            // filter rows: constant per-lane row offset, the step in the scalar offset (the range check
            // looks at the per-lane offset only, so a step past the end is masked explicitly)
            const int voff = blk_filter[i] ? (in_crs ? blk_voff[i] : OOB) : voff_x;
            const int soff = blk_filter[i] ? s_step : blk_soff[i];
            __builtin_amdgcn_raw_ptr_buffer_load_lds(blk_rs[i], dst, 16, voff, soff, 0, 0);
        }
#pragma unroll
        for (int g = 0; g < KG; ++g) advance(ut);            // this group's next step
    };

    // ---------------- FIC, input side in the main loop: the digits of the filter checksum into LDS ----------------
    extern __shared__ __attribute__((aligned(16))) int8_t dyn_lds[];
    bool fic_tile = false;                       // uniform over the workgroup
    int fic_pad = 0;                             // bytes of one digit row in LDS
    int fdot0 = 0, fdot1 = 0, fdot2 = 0;         // this lane's sums of fragment . digit
    if constexpr (FICV) {
        if (p.fic_wdig && kt == 0) {
            fic_tile = true;
            fic_pad = ((p.nsteps + KG - 1) / KG) * KG * 64;
        }
    }
    // 16-byte chunk c of the digits: from global memory (zeros beyond the reduction axis) / to LDS
    auto dig_load = [&](int c) {
        const int gpad = p.nsteps * 64, per_row = fic_pad >> 4;
        const int d = c / per_row, o = (c - d * per_row) << 4;
        i32x4 v = {0, 0, 0, 0};
        if (o < gpad) v = *reinterpret_cast<const i32x4 *>(p.fic_wdig + d * gpad + o);
        return v;
    };
    auto dig_store = [&](int c, i32x4 v) {
        const int per_row = fic_pad >> 4;
        const int d = c / per_row, o = (c - d * per_row) << 4;
        *reinterpret_cast<i32x4 *>(dyn_lds + d * fic_pad + o) = v;
    };

    // ---------------- accumulators ----------------
    acc_t acc[WM][WK];
    const acc_t zero4 = {0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int k = 0; k < WK; ++k) acc[i][k] = zero4;

    // ---------------- main loop ----------------
    // Stage s holds steps s*KG .. s*KG+KG-1 (s mod NST).  Loads run NST-1 stages ahead; steps past
    // the end load zeros, which keeps the per-wave load count per stage constant.
    const int rd_lane = lds_off(lj, lg);         // this lane's 16 bytes inside any 1 KB block
    const int nstages = (p.nsteps + KG - 1) / KG;
    auto main_loop = [&](auto ut) {
    // FIC, input side: a thread's first chunk of the digits is requested before the tile's loads, so that
    // it does not delay them, and put into LDS behind them; the loop's first barrier publishes it
    const int dig_chunks = fic_tile ? p.fic_ndig * (fic_pad >> 4) : 0;
    i32x4 dig_first = {0, 0, 0, 0};
    if constexpr (FICV) {
        if (tid < dig_chunks) dig_first = dig_load(tid);
    }
#pragma unroll
    for (int s = 0; s < NST - 1; ++s) issue(s, ut);
    if constexpr (FICV) {
        if (fic_tile) {
            if (tid < dig_chunks) dig_store(tid, dig_first);
            for (int c = tid + 256 * KG; c < dig_chunks; c += 256 * KG) dig_store(c, dig_load(c));
            __builtin_amdgcn_s_waitcnt(0xc07f);  // the LDS writes (lgkmcnt 0) are done before the barrier
        }
    }
    int stage = 0;
#ifdef ABED_ENABLE_DBG
    const int nloop = (p.dbg & 2) ? 0 : nstages;
#else
    const int nloop = nstages;
#endif
    for (int step = 0; step < nloop; ++step) {
        // this wave's loads of `step` have landed (the counter's limit is an immediate: one branch per count)
        if (short_wave) ABED_WAIT_VMCNT((NST - 2) * (L - 1)); else ABED_WAIT_VMCNT((NST - 2) * L);
        __builtin_amdgcn_s_barrier();            // everyone's have, and everyone is done with step-1
        {
            int st = stage + NST - 1;            // the stage that step-1 used gets refilled
            if (st >= NST) st -= NST;
            issue(st, ut);
        }
        const int8_t *ldsK = lds + stage * STAGE + kg * SUB + rd_lane;   // + 1024 * filter block
        const int8_t *ldsM = ldsK + (WK + wave * WM) * 1024;         // + 1024 * entry of this wave
        i32x4 bfr[WM];
#pragma unroll
        for (int i = 0; i < WM; ++i)
            bfr[i] = *reinterpret_cast<const i32x4 *>(ldsM + i * 1024);
#pragma unroll
        for (int kb = 0; kb < WK; ++kb) {
            const i32x4 a = *reinterpret_cast<const i32x4 *>(ldsK + kb * 1024);
#pragma unroll
            for (int i = 0; i < WM; ++i)
                if constexpr (F16)
                    acc[i][kb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, bfr[i]), acc[i][kb], 0, 0, 0);
                else
                    acc[i][kb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, bfr[i], acc[i][kb], 0, 0, 0);
        }
        // FIC, input side: the same fragments against the digits of the filter checksum, on the vector ALU
        // behind the matrix instructions (which are still executing)
        if constexpr (FICV) {
            if (fic_tile) {                      // scalar branch
                const int8_t *dg = dyn_lds + (step * KG + kg) * 64 + lg * 16;
                const i32x4 d0 = *reinterpret_cast<const i32x4 *>(dg);
                const i32x4 d1 = *reinterpret_cast<const i32x4 *>(dg + fic_pad);
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        fdot0 = __builtin_amdgcn_sdot4(bfr[i][j], d0[j], fdot0, false);
                        fdot1 = __builtin_amdgcn_sdot4(bfr[i][j], d1[j], fdot1, false);
                    }
                if (p.fic_ndig > 2) {            // scalar branch
                    const i32x4 d2 = *reinterpret_cast<const i32x4 *>(dg + 2 * fic_pad);
#pragma unroll
                    for (int i = 0; i < WM; ++i)
#pragma unroll
                        for (int j = 0; j < 4; ++j) fdot2 = __builtin_amdgcn_sdot4(bfr[i][j], d2[j], fdot2, false);
                }
            }
        }
        if (++stage == NST) stage = 0;
    }
    };
    if (utap) main_loop(std::true_type{}); else main_loop(std::false_type{});
    ABED_WAIT_VMCNT(0);                          // drain the run-ahead loads before LDS is reused
    __builtin_amdgcn_s_barrier();

    // FIC, input side: this lane's share of the dot product, recombined from the digits in 64 bits
    // (Sec. 4.1).  The waves of the groups that end here leave their sums in LDS (the digits there are no
    // longer read; the barrier of the group sum publishes them); the others carry theirs into the epilogue.
    long long fic_dot = 0;
    if constexpr (FICV) {
        if (fic_tile) {
            fic_dot = (long long)fdot0 + 256LL * fdot1 + 65536LL * fdot2;
            if (KG > 1 && kg > 0) {
                const long long t = wave_sum64(fic_dot);
                if (lane == 0) reinterpret_cast<long long *>(dyn_lds)[wave_all] = t;
            }
        }
    }

    // ---------------- sum over the groups of the reduction axis ----------------
    if constexpr (KG > 1) {
        acc_t *red = reinterpret_cast<acc_t *>(lds);             // [KG-1][4 waves][WM*WK][64 lanes]
        if (kg > 0) {
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int k = 0; k < WK; ++k)
                    red[(((kg - 1) * 4 + wave) * (WM * WK) + i * WK + k) * 64 + lane] = acc[i][k];
        }
        __syncthreads();
        if (kg > 0) return;                      // barriers from here on count the surviving waves only
#pragma unroll
        for (int g = 1; g < KG; ++g)
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int k = 0; k < WK; ++k)
                    acc[i][k] += red[(((g - 1) * 4 + wave) * (WM * WK) + i * WK + k) * 64 + lane];
        __syncthreads();                         // the epilogue reuses this memory
    }

    if constexpr (F16) {
        // ---------------- epilogue, fp16 data (Sec. 7) ----------------
        const int pix = pg * 16 + lj;
        const bool pvalid = pix < PQ;
        float *e_ic = reinterpret_cast<float *>(lds);            // [3][4 waves][WK][64 lanes][4]: sums, checksum values, sums of magnitudes
        int *e_misc = reinterpret_cast<int *>(e_ic + 12 * WK * 256);
        if (tid < 4) e_misc[tid] = 0;     // [1], [2]: "last arriver" marks, read after later barriers
        uint32_t my_flag = 0;
        // a scheme that is not selected (d_f or d_i zero) has nothing to exchange
        const bool fc_local = p.grid_n == 1 || p.d_f == 0, ic_local = p.grid_b == 1 || p.d_i == 0;
        const bool checking = p.mode == MODE_CHECK || p.mode == MODE_CHECK_NEXT;
        const bool want_next = p.mode == MODE_CHECK_NEXT && p.xchk_next != nullptr;
        // the hi/lo pair of a batch sum of fp16 outputs, into the next layer's checksum images [2][PQ][K]
        auto store_next = [&](const f32x4 s4, int fb) {
            if (!pvalid || fb >= p.kblk) return;
            _Float16 *dst = reinterpret_cast<_Float16 *>(p.xchk_next) + (long long)pix * p.K + fb * 16 + lg * 4;
            for (int v = 0; v < 4; ++v)
                if (fb * 16 + lg * 4 + v < p.K) {
                    const _Float16 hi = (_Float16)s4[v];
                    dst[v] = hi;
                    dst[(long long)PQ * p.K + v] = (_Float16)(s4[v] - (float)hi);
                }
        };
        // The threshold is relative to the larger of the two compared values or, with p.l1, to the sum of
        // magnitudes of what was reduced (Sec. 7 leaves its choice open).  NaN and infinity are mismatches.
        auto bad = [&](float sum, float chk, float mag) {
            const float tol = p.rtol * (p.l1 ? mag : fmaxf(fabsf(sum), fabsf(chk))) + p.atol;
            return !(fabsf(sum - chk) <= tol) || !(fabsf(sum) < __builtin_inff()) || !(fabsf(chk) < __builtin_inff()) ||
                   !(tol < __builtin_inff());
        };
        // (1) fault injection: one bit of the value rounded to fp16; the corrupted value takes the
        // accumulator's place in the reductions and in the store
        if (p.inj_on && pg == p.inj_pg && nt == p.inj_nt && kt == p.inj_kt) {
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int kb = 0; kb < WK; ++kb)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (wave * WM + i == p.inj_mb && kb == p.inj_kb && v == p.inj_v && lane == p.inj_lane) {
                            const _Float16 h = (_Float16)acc[i][kb][v];
                            const unsigned short bits = __builtin_bit_cast(unsigned short, h) ^ (unsigned short)p.inj_mask;
                            acc[i][kb][v] = (float)__builtin_bit_cast(_Float16, bits);
                        }
        }
        // (2) FC: sum over the real filters of every row against hi + lo of the checksum-filter fmaps
        const bool reduce = aug && p.mode != MODE_WRITE;          // sums are formed in this kernel
        if (reduce && p.d_f) {
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                const int e = nt * MB + wave * WM + i;
                float sum = 0.f, chk = 0.f, mag = 0.f;
#pragma unroll
                for (int kb = 0; kb < WK; ++kb) {
                    const int fb = kt * WK + kb;
                    const float t = (acc[i][kb][0] + acc[i][kb][1]) + (acc[i][kb][2] + acc[i][kb][3]);
                    if (fb < p.kblk) {
                        sum += t;
                        mag += (fabsf(acc[i][kb][0]) + fabsf(acc[i][kb][1])) + (fabsf(acc[i][kb][2]) + fabsf(acc[i][kb][3]));
                    } else if (fb == p.kblk) chk += t;      // rows 2..15 of the checksum block are zero filters
                }
                sum += __shfl_xor(sum, 16, 64); sum += __shfl_xor(sum, 32, 64);
                chk += __shfl_xor(chk, 16, 64); chk += __shfl_xor(chk, 32, 64);
                mag += __shfl_xor(mag, 16, 64); mag += __shfl_xor(mag, 32, 64);
                if (checking && fc_local) {
                    if (bad(sum, chk, mag)) my_flag |= (e < p.N) ? 1u : 4u;
                } else if (lg == 0) {
                    int *dst = &p.ws_fc[(((long long)pg * p.grid_b + nt) * p.grid_n + kt) * (3 * MB * 16) + (wave * WM + i) * 16 + lj];
                    st_dev(dst, __builtin_bit_cast(int, sum));
                    st_dev(dst + MB * 16, __builtin_bit_cast(int, chk));
                    st_dev(dst + 2 * MB * 16, __builtin_bit_cast(int, mag));
                }
            }
        }
#ifdef ABED_ENABLE_DBG
        if (p.dbg & 1) return;
#endif
        const bool exchange = checking && !(fc_local && ic_local);
        const long long word = ((long long)pg * p.grid_b + nt) * p.grid_n + kt;
        if (reduce) {
            // (3) IC: sum over the real images of every (pixel, filter) against hi + lo of the checksum-image fmaps
            if (p.d_i) {
#pragma unroll
            for (int kb = 0; kb < WK; ++kb) {
                f32x4 sum = {0.f, 0.f, 0.f, 0.f}, chk = {0.f, 0.f, 0.f, 0.f}, mag = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < WM; ++i) {
                    const int e = nt * MB + wave * WM + i;
                    if (e < p.N) {
                        sum += acc[i][kb];
                        mag += f32x4{fabsf(acc[i][kb][0]), fabsf(acc[i][kb][1]), fabsf(acc[i][kb][2]), fabsf(acc[i][kb][3])};
                    } else if (e < p.n_entries) chk += acc[i][kb];
                }
                *reinterpret_cast<f32x4 *>(e_ic + ((wave * WK + kb) * 64 + lane) * 4) = sum;
                *reinterpret_cast<f32x4 *>(e_ic + 4 * WK * 256 + ((wave * WK + kb) * 64 + lane) * 4) = chk;
                *reinterpret_cast<f32x4 *>(e_ic + 8 * WK * 256 + ((wave * WK + kb) * 64 + lane) * 4) = mag;
            }
            __syncthreads();
#pragma unroll
            for (int c4 = 0; c4 < (WK + 3) / 4; ++c4) {
                const int kb = 4 * c4 + wave;
                if (kb >= WK) continue;
                f32x4 sum = {0.f, 0.f, 0.f, 0.f}, chk = {0.f, 0.f, 0.f, 0.f}, mag = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    sum += *reinterpret_cast<const f32x4 *>(e_ic + ((w * WK + kb) * 64 + lane) * 4);
                    chk += *reinterpret_cast<const f32x4 *>(e_ic + 4 * WK * 256 + ((w * WK + kb) * 64 + lane) * 4);
                    mag += *reinterpret_cast<const f32x4 *>(e_ic + 8 * WK * 256 + ((w * WK + kb) * 64 + lane) * 4);
                }
                const int fb = kt * WK + kb;
                if (checking && ic_local) {
                    if (bad(sum[0], chk[0], mag[0]) || bad(sum[1], chk[1], mag[1]) || bad(sum[2], chk[2], mag[2]) || bad(sum[3], chk[3], mag[3]))
                        my_flag |= (fb < p.kblk) ? 2u : 4u;
                } else {
                    int *dst = p.ws_ic + ((((long long)pg * p.grid_n + kt) * p.grid_b + nt) * 3 * WK + kb) * 256 + lane * 4;
                    st_dev4(dst, __builtin_bit_cast(i32x4, sum));
                    st_dev4(dst + WK * 256, __builtin_bit_cast(i32x4, chk));
                    st_dev4(dst + 2 * WK * 256, __builtin_bit_cast(i32x4, mag));
                }
            }
            }
            if (want_next) {
                // (3b) the next layer's batch checksum (Sec. 4.3): the sum over the real images of the outputs as the
                // next layer will read them (rounded to fp16), in fp32; a second pass through the LDS area of (3)
                __syncthreads();
#pragma unroll
                for (int kb = 0; kb < WK; ++kb) {
                    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int i = 0; i < WM; ++i)
                        if (nt * MB + wave * WM + i < p.N)
                            sum += f32x4{(float)(_Float16)acc[i][kb][0], (float)(_Float16)acc[i][kb][1], (float)(_Float16)acc[i][kb][2], (float)(_Float16)acc[i][kb][3]};
                    *reinterpret_cast<f32x4 *>(e_ic + ((wave * WK + kb) * 64 + lane) * 4) = sum;
                }
                __syncthreads();
#pragma unroll
                for (int c4 = 0; c4 < (WK + 3) / 4; ++c4) {
                    const int kb = 4 * c4 + wave;
                    if (kb >= WK) continue;
                    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int w = 0; w < 4; ++w) sum += *reinterpret_cast<const f32x4 *>(e_ic + ((w * WK + kb) * 64 + lane) * 4);
                    if (p.grid_b == 1) store_next(sum, kt * WK + kb);
                    else st_dev4(p.ws_nx + ((((long long)pg * p.grid_n + kt) * p.grid_b + nt) * WK + kb) * 256 + lane * 4, __builtin_bit_cast(i32x4, sum));
                }
            }
            if (checking) {
                // (4) flags of this tile; when sums span several tiles, count this tile's arrival (the
                // answer is picked up after the output stores have been issued)
                // every wave leaves its bits in a word of its own (nothing to initialise, so no wave can wipe another's)
                {
                    const uint32_t wf = wave_or3(my_flag);
                    if (lane == 0) e_misc[4 + wave] = (int)wf;
                }
                __syncthreads();
                if (tid == 0) __hip_atomic_store(&p.flags[word], (uint32_t)(e_misc[4] | e_misc[5] | e_misc[6] | e_misc[7]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (exchange) {
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                    __syncthreads();
                    if (tid == 0) {
                        // a count at or beyond the number of tiles that share the counter: the workspace did not start at zero
                        // (abed_workspace_init not called, or calls overlapped); some cross-tile comparison was then made
                        // early or not at all, which the caller must learn
                        bool stale = false;
                        if (!fc_local)
                            { const unsigned c = __hip_atomic_fetch_add(&p.cnt_fc[pg * p.grid_b + nt], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); e_misc[1] = c == (unsigned)(p.grid_n - 1); stale |= c >= (unsigned)p.grid_n; }
                        if (!ic_local)
                            { const unsigned c = __hip_atomic_fetch_add(&p.cnt_ic[pg * p.grid_n + kt], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); e_misc[2] = c == (unsigned)(p.grid_b - 1); stale |= c >= (unsigned)p.grid_b; }
                        if (stale) __hip_atomic_fetch_or(&p.flags[word], 8u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
        }
        // (5) stores (checksum rows and columns are trimmed)
#pragma unroll
        for (int kb = 0; kb < WK; ++kb) {
            const int fb = kt * WK + kb;
            const int k = fb * 16 + lg * 4;
            if (p.mode == MODE_WRITE && pvalid) {
                // the checksum fmaps go to the workspace as fp32 (the verify kernel reads them back): rows of the
                // checksum images [d_i][PQ][K], columns of the checksum filters [N][PQ][d_f], their corner [d_i][PQ][d_f]
#pragma unroll
                for (int i = 0; i < WM; ++i) {
                    const int e = nt * MB + wave * WM + i;
                    if (fb < p.kblk && e >= p.N && e < p.n_entries) {
                        float *dst = reinterpret_cast<float *>(p.ws_yi) + ((long long)(e - p.N) * PQ + pix) * p.K + k;
                        for (int v = 0; v < 4; ++v)
                            if (k + v < p.K) dst[v] = acc[i][kb][v];
                    } else if (fb == p.kblk && lg == 0 && e < p.n_entries && p.d_f) {
                        float *dst = e < p.N ? reinterpret_cast<float *>(p.ws_yf) + ((long long)e * PQ + pix) * p.d_f
                                             : reinterpret_cast<float *>(p.ws_yfi) + ((long long)(e - p.N) * PQ + pix) * p.d_f;
                        for (int v = 0; v < p.d_f; ++v) dst[v] = acc[i][kb][v];
                    }
                }
            }
            if (fb >= p.kblk) continue;
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                const int e = nt * MB + wave * WM + i;
                if (!pvalid || e >= p.N) continue;
                const long long o = ((long long)e * PQ + pix) * p.K + k;
                if (p.out_fp32) {
                    float *dst = reinterpret_cast<float *>(p.y) + o;
                    if (k + 4 <= p.K && (p.K & 3) == 0) *reinterpret_cast<f32x4 *>(dst) = acc[i][kb];
                    else
                        for (int v = 0; v < 4; ++v)
                            if (k + v < p.K) dst[v] = acc[i][kb][v];
                } else {
                    _Float16 *dst = reinterpret_cast<_Float16 *>(p.y) + o;
                    typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
                    const f16x4 h = {(_Float16)acc[i][kb][0], (_Float16)acc[i][kb][1], (_Float16)acc[i][kb][2], (_Float16)acc[i][kb][3]};
                    if (k + 4 <= p.K && (p.K & 3) == 0) *reinterpret_cast<f16x4 *>(dst) = h;
                    else
                        for (int v = 0; v < 4; ++v)
                            if (k + v < p.K) dst[v] = h[v];
                }
            }
        }
        if (!exchange) return;
        // (6) sums that span several tiles are finished by the workgroup that arrives last
        __syncthreads();
        if (e_misc[1]) {
            uint32_t late = 0;
            for (int r = tid; r < MB * 16; r += 256) {
                float sum = 0.f, chk = 0.f, mag = 0.f;
                for (int c = 0; c < p.grid_n; ++c) {
                    const int *src = &p.ws_fc[(((long long)pg * p.grid_b + nt) * p.grid_n + c) * (3 * MB * 16) + r];
                    sum += __builtin_bit_cast(float, ld_dev(src));
                    chk += __builtin_bit_cast(float, ld_dev(src + MB * 16));
                    mag += __builtin_bit_cast(float, ld_dev(src + 2 * MB * 16));
                }
                if (bad(sum, chk, mag)) late |= (nt * MB + (r >> 4) < p.N) ? 1u : 4u;
            }
            if (late) __hip_atomic_fetch_or(&p.flags[((long long)pg * p.grid_b + nt) * p.grid_n], late, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (tid == 0) __hip_atomic_store(&p.cnt_fc[pg * p.grid_b + nt], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (e_misc[2]) {
            uint32_t late = 0;
            // the partials of this (pixel group, filter tile): [grid_b][3][WK][256] words
            const __amdgpu_buffer_rsrc_t rs_ic = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(p.ws_ic + (((long long)pg * p.grid_n + kt) * p.grid_b) * 3 * WK * 256), 0, p.grid_b * 3 * WK * 1024, 0x00020000);
            for (int idx = tid; idx < WK * 64; idx += 256) {
                const int kb = idx >> 6, ln = idx & 63;
                const int fb = kt * WK + kb;
                f32x4 sum = {0.f, 0.f, 0.f, 0.f}, chk = {0.f, 0.f, 0.f, 0.f}, mag = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
                for (int b = 0; b < p.grid_b; ++b) {
                    const int off = (((b * 3 * WK) + kb) * 256 + ln * 4) * 4;
                    sum += __builtin_bit_cast(f32x4, ld_dev4(rs_ic, off));
                    chk += __builtin_bit_cast(f32x4, ld_dev4(rs_ic, off + WK * 1024));
                    mag += __builtin_bit_cast(f32x4, ld_dev4(rs_ic, off + 2 * WK * 1024));
                }
                if (bad(sum[0], chk[0], mag[0]) || bad(sum[1], chk[1], mag[1]) || bad(sum[2], chk[2], mag[2]) || bad(sum[3], chk[3], mag[3]))
                    late |= (fb < p.kblk) ? 2u : 4u;
            }
            if (late) __hip_atomic_fetch_or(&p.flags[((long long)pg * p.grid_b) * p.grid_n + kt], late, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (want_next) {
                // the batch tiles' sums of the fp16 outputs, added in tile order: [grid_b][WK][256] words
                const __amdgpu_buffer_rsrc_t rs_nx = __builtin_amdgcn_make_buffer_rsrc(
                    (void *)(p.ws_nx + (((long long)pg * p.grid_n + kt) * p.grid_b) * WK * 256), 0, p.grid_b * WK * 1024, 0x00020000);
                for (int idx = tid; idx < WK * 64; idx += 256) {
                    const int kb = idx >> 6, ln = idx & 63;
                    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
                    for (int b = 0; b < p.grid_b; ++b) sum += __builtin_bit_cast(f32x4, ld_dev4(rs_nx, ((b * WK + kb) * 256 + ln * 4) * 4));
                    // (this thread's lane position may differ from ln: recompute the pixel and filter from ln)
                    const int px = pg * 16 + (ln & 15), fb = kt * WK + kb;
                    if (px < PQ && fb < p.kblk) {
                        _Float16 *dst = reinterpret_cast<_Float16 *>(p.xchk_next) + (long long)px * p.K + fb * 16 + (ln >> 4) * 4;
                        for (int v = 0; v < 4; ++v)
                            if (fb * 16 + (ln >> 4) * 4 + v < p.K) {
                                const _Float16 hi = (_Float16)sum[v];
                                dst[v] = hi;
                                dst[(long long)PQ * p.K + v] = (_Float16)(sum[v] - (float)hi);
                            }
                    }
                }
            }
            if (tid == 0) __hip_atomic_store(&p.cnt_ic[pg * p.grid_n + kt], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    } else {
    // ---------------- epilogue, int8 data ----------------
    const int pix = pg * 16 + lj;                // output pixel of this lane
    const bool pvalid = pix < PQ;
    int *e_ic = reinterpret_cast<int *>(lds);                 // [4 waves][WK][64 lanes][4]
    int *e_misc = e_ic + 4 * WK * 256;                        // [0] flag bits, [1] last for FC, [2] last for IC
    if (tid < 4) e_misc[tid] = 0;     // [1], [2]: "last arriver" marks, read after later barriers
    // the epilog's per-filter scale and bias of this tile's filters, fetched once (zeros beyond K); the first
    // barrier before their use publishes them
    float *e_scale = reinterpret_cast<float *>(e_misc + 32), *e_bias = e_scale + WK * 16;
    if (p.out_int8) {
        for (int t = tid; t < 2 * WK * 16; t += 256) {
            const int f = t < WK * 16 ? t : t - WK * 16;
            const int k = kt * WK * 16 + f;
            const float *src = t < WK * 16 ? p.scale : p.bias;
            e_scale[t] = k < p.K ? src[k] : 0.f;
        }
    }
    uint32_t my_flag = 0;
    // a scheme that is not selected (d_f or d_i zero) has nothing to exchange
    const bool fc_local = p.grid_n == 1 || p.d_f == 0, ic_local = p.grid_b == 1 || p.d_i == 0;
    const bool checking = p.mode == MODE_CHECK || p.mode == MODE_CHECK_NEXT;
    const bool reduce = aug && p.mode != MODE_WRITE;          // residuals are formed in this kernel
    const bool want_next = p.mode == MODE_CHECK_NEXT && p.out_int8 && p.xchk_next != nullptr;
    const long long tile = ((long long)pg * p.grid_b + nt) * p.grid_n + kt;

    // (1) accumulator fault injection (tests).  inj_fix: what the 32-bit sum of the faulty accumulator's group
    // of four loses when it wraps (a multiple of 2^32), so that the FIC output sum below stays exact for any bit.
    long long inj_fix = 0;
    if (p.inj_on && pg == p.inj_pg && nt == p.inj_nt && kt == p.inj_kt) {
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int kb = 0; kb < WK; ++kb)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (wave * WM + i == p.inj_mb && kb == p.inj_kb && v == p.inj_v && lane == p.inj_lane) {
                        acc[i][kb][v] ^= (int)p.inj_mask;
                        const long long g = (long long)acc[i][kb][0] + acc[i][kb][1] + acc[i][kb][2] + acc[i][kb][3];
                        inj_fix = g - (long long)(int)(unsigned)g;
                    }
    }

    // (1b) FIC scheme (Sec. 3.3): output fmap checksum = the sum of all accumulators, in 64 bits
    // (Sec. 4.1).  Rows, entries and filters beyond the problem were loaded as zeros and add nothing.
    if (p.fic_ocs) {
        // a lane's four values of one (entry, filter block) add up inside 32 bits (the host checked R*S*C <
        // 2^15: each is at most R*S*C * 2^14 in magnitude); so do all of a lane's values when fic_sum32 is set,
        // else every such group is widened to 64 bits
        long long t = 0;
        int t32 = 0;
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int kb = 0; kb < WK; ++kb) {
                t32 += (acc[i][kb][0] + acc[i][kb][1]) + (acc[i][kb][2] + acc[i][kb][3]);
                if (!p.fic_sum32) { t += t32; t32 = 0; }         // scalar branch
            }
        t += t32 + inj_fix;
        // the workgroup's output sum and, for the in-loop input side, its dot product
        long long *e64 = reinterpret_cast<long long *>(e_misc + 16);   // [0..3] output sums, [4..7] dot products of the waves
        t = wave_sum64(t);
        if (lane == 0) e64[wave] = t;
        if (fic_tile) {
            const long long d = wave_sum64(fic_dot);
            if (lane == 0) e64[4 + wave] = d;
        }
        __syncthreads();
        if (tid == 0) {
            p.fic_ocs[tile] = e64[0] + e64[1] + e64[2] + e64[3];
            if (fic_tile) {
                long long d = e64[4] + e64[5] + e64[6] + e64[7];
                for (int w = 4; w < 4 * KG; ++w) d += reinterpret_cast<const long long *>(dyn_lds)[w];
                p.fic_dotpart[pg * p.grid_b + nt] = d;
            }
        }
    }

    // (1c) IC option 2 (Sec. 3.2): the output fmaps reduced over batch, height and width, one 64-bit sum
    // per filter (Sec. 4.1); this tile's share.  Two passes through the LDS area of the IC pass, one with
    // the low and one with the high 16 bits of the accumulators (a tile sums at most 16 * MB of them,
    // so neither half overflows 32 bits): a lane adds its entries in registers; then thread (f, w) adds
    // filter f's values of wave w over the 16 pixels and the 4 threads of a filter add up across lanes.
    if (p.ic2_part) {
        constexpr int NF = WK * 16, NIT = (4 * NF + 255) / 256;
        const i32x4 low16 = {0xffff, 0xffff, 0xffff, 0xffff};
        long long total[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) total[it] = 0;
        for (int pass = 0; pass < 2; ++pass) {
#pragma unroll
            for (int kb = 0; kb < WK; ++kb) {
                i32x4 c = zero4;
#pragma unroll
                for (int i = 0; i < WM; ++i) c += pass ? (acc[i][kb] >> 16) : (acc[i][kb] & low16);
                *reinterpret_cast<i32x4 *>(e_ic + ((wave * WK + kb) * 64 + lane) * 4) = c;
            }
            __syncthreads();
#pragma unroll
            for (int it = 0; it < NIT; ++it) {
                const int idx = it * 256 + tid, w = idx & 3, f = idx >> 2;
                int sum = 0;
                if (f < NF) {
                    const int kb = f >> 4, g = (f >> 2) & 3, v = f & 3;
                    const int *src = e_ic + ((w * WK + kb) * 64 + g * 16) * 4 + v;
#pragma unroll
                    for (int j = 0; j < 16; ++j) sum += src[((j + g * 4 + w) & 15) * 4];   // rotated: the 64 lanes hit 64 banks
                }
                sum += __shfl_xor(sum, 1, 64);
                sum += __shfl_xor(sum, 2, 64);
                total[it] += pass ? (long long)sum * 65536 : (long long)sum;
            }
            __syncthreads();
        }
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int idx = it * 256 + tid, f = idx >> 2;
            if (f < NF && (idx & 3) == 0)
                p.ic2_part[((long long)pg * p.grid_b + nt) * (p.grid_n * NF) + kt * NF + f] = total[it];
        }
    }

    // (2) FC residual of every row of the tile (Sec. 3.1; digit shifts of Sec. 4.1)
    if (reduce && p.d_f) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int e = nt * MB + wave * WM + i;
            unsigned r = 0;
#pragma unroll
            for (int kb = 0; kb < WK; ++kb) {
                const int fb = kt * WK + kb;
                if (fb < p.kblk) {
                    r += (unsigned)acc[i][kb][0] + (unsigned)acc[i][kb][1] + (unsigned)acc[i][kb][2] + (unsigned)acc[i][kb][3];
                } else if (fb == p.kblk) {
                    if (lg == 0)
                        r -= (unsigned)acc[i][kb][0] + ((unsigned)acc[i][kb][1] << 8) + ((unsigned)acc[i][kb][2] << 16) + ((unsigned)acc[i][kb][3] << 24);
                }
            }
            if (p.packed_df) {
                // the digit filters share the last real block: its columns K..K+d_f-1 were added above as
                // if they were real filters; take them out again and subtract them with their shifts
#pragma unroll
                for (int kb = 0; kb < WK; ++kb)
                    if (kt * WK + kb == p.kblk - 1)
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int k = (p.kblk - 1) * 16 + lg * 4 + v;
                            if (k >= p.K && k < p.K + p.packed_df)
                                r -= (unsigned)acc[i][kb][v] + ((unsigned)acc[i][kb][v] << (8 * (k - p.K)));
                        }
            }
            r += (unsigned)__shfl_xor((int)r, 16, 64);
            r += (unsigned)__shfl_xor((int)r, 32, 64);
            if (checking && fc_local) {
                if (r != 0) my_flag |= (e < p.N) ? 1u : 4u;
            } else if (lg == 0) {
                st_dev(&p.ws_fc[tile * (MB * 16) + (wave * WM + i) * 16 + lj], (int)r);
            }
        }
    }
#ifdef ABED_ENABLE_DBG
    if (p.dbg & 1) return;
#endif

    // flag bits of a non-zero IC residual vector: a real filter's column is an IC mismatch, a digit
    // filter's column a disagreement of the checksums with each other
    // (only called for a non-zero vector of the block that real and digit filters share)
    auto ic_bits_shared = [&](const i32x4 c, int fb, int g) -> uint32_t {
        uint32_t b = 0;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (c[v] != 0) b |= (fb * 16 + g * 4 + v < p.K) ? 2u : 4u;
        return b;
    };

    // IC residual of every (pixel, filter) of the tile (Sec. 3.2 option 1), pass 0: sum over this
    // wave's entries in registers, then over the 4 waves through LDS.  Pass 1 does the same for the
    // int8 outputs (the next layer's batch checksum, Sec. 4.3).
    auto ic_pass = [&](int pass) {
#pragma unroll
        for (int kb = 0; kb < WK; ++kb) {
            i32x4 c = zero4;
            if (pass == 0) {
#pragma unroll
                for (int i = 0; i < WM; ++i) {
                    const int e = nt * MB + wave * WM + i;
                    if (e < p.N) {
                        c += acc[i][kb];
                    } else if (e < p.n_entries) {
                        const int sh = 8 * (e - p.N);
#pragma unroll
                        for (int v = 0; v < 4; ++v) c[v] -= (int)((unsigned)acc[i][kb][v] << sh);
                    }
                }
            } else {
                // batch sum of the int8 outputs: requantised again here rather than kept from the store
                // loop (16 more live registers there cost more than these few operations)
                const int k = (kt * WK + kb) * 16 + lg * 4;
                float sc[4], bi[4];
                {
                    const f32x4 s4 = *reinterpret_cast<const f32x4 *>(e_scale + kb * 16 + lg * 4);
                    const f32x4 b4 = *reinterpret_cast<const f32x4 *>(e_bias + kb * 16 + lg * 4);
#pragma unroll
                    for (int v = 0; v < 4; ++v) { sc[v] = s4[v]; bi[v] = b4[v]; }
                }
#pragma unroll
                for (int i = 0; i < WM; ++i)
                    if (pvalid && nt * MB + wave * WM + i < p.N)
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (k + v < p.K) c[v] += requant(acc[i][kb][v], sc[v], bi[v], p.relu);
            }
            *reinterpret_cast<i32x4 *>(e_ic + ((wave * WK + kb) * 64 + lane) * 4) = c;
        }
        __syncthreads();
        // wave w finishes filter blocks kb = w, w+4, ...
#pragma unroll
        for (int c4 = 0; c4 < (WK + 3) / 4; ++c4) {
            const int kb = 4 * c4 + wave;
            if (kb >= WK) continue;
            i32x4 c = *reinterpret_cast<const i32x4 *>(e_ic + ((0 * WK + kb) * 64 + lane) * 4);
#pragma unroll
            for (int w = 1; w < 4; ++w) c += *reinterpret_cast<const i32x4 *>(e_ic + ((w * WK + kb) * 64 + lane) * 4);
            const int fb = kt * WK + kb;
            const long long part = ((((long long)pg * p.grid_n + kt) * p.grid_b + nt) * WK + kb) * 256 + lane * 4;
            if (pass == 0) {
                if (checking && ic_local) {
                    if ((c[0] | c[1] | c[2] | c[3]) != 0)
                        my_flag |= (p.packed_df && fb == p.kblk - 1) ? ic_bits_shared(c, fb, lg) : ((fb < p.kblk) ? 2u : 4u);
                } else {
                    st_dev4(p.ws_ic + part, c);
                }
            } else if (pass == 2) {
                // FIC scheme, next layer's input checksum source (Sec. 4.3): the batch sum of the int8
                // outputs, added to an int32 image that starts at zero (tiles of other batch parts add too)
                const int k = fb * 16 + lg * 4;
                if (pvalid && fb < p.kblk)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (k + v < p.K && c[v] != 0)
                            __hip_atomic_fetch_add(&p.fic_xsum_next[(long long)pix * p.K + k + v], c[v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else if (fb < p.kblk) {
                if (ic_local) {
                    // digits of the next layer's batch checksum: xchk_next[d][pix][k..k+3]
                    const int k = fb * 16 + lg * 4;
                    if (pvalid) {
                        int rest[4] = {c[0], c[1], c[2], c[3]};
                        for (int d = 0; d < p.d_i; ++d) {
                            unsigned pk = 0;
#pragma unroll
                            for (int v = 0; v < 4; ++v) pk |= ((unsigned)next_digit(rest[v]) & 0xffu) << (8 * v);
                            int8_t *dst = p.xchk_next + ((long long)d * PQ + pix) * p.K + k;
                            if (k + 4 <= p.K && (p.K & 3) == 0) *reinterpret_cast<unsigned *>(dst) = pk;
                            else
                                for (int v = 0; v < 4; ++v)
                                    if (k + v < p.K) dst[v] = (int8_t)((pk >> (8 * v)) & 0xff);
                        }
                    }
                } else {
                    st_dev4(p.ws_nx + part, c);
                }
            }
        }
    };

    // Flags of this tile; when residuals span several tiles, count this tile's arrival.  The
    // partial stores are write-through, so waiting for them to complete (the release fence) is
    // enough before the arrival is counted.  The answer (was this the last tile?) is picked up
    // after the output stores have been issued, which hides the round trip of the counter.
    const bool exchange = checking && !(fc_local && ic_local);
    auto arrive = [&]() {
        // every wave leaves its bits in a word of its own (nothing to initialise, so no wave can wipe another's)
        {
            const uint32_t wf = wave_or3(my_flag);
            if (lane == 0) e_misc[4 + wave] = (int)wf;
        }
        __syncthreads();
        if (tid == 0) __hip_atomic_store(&p.flags[tile], (uint32_t)(e_misc[4] | e_misc[5] | e_misc[6] | e_misc[7]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!exchange) return;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (tid == 0) {
            // a count at or beyond the number of tiles that share the counter: the workspace did not start at zero
            // (abed_workspace_init not called, or calls overlapped); some cross-tile comparison was then made early or
            // not at all, which the caller must learn
            bool stale = false;
            if (!fc_local)
                { const unsigned c = __hip_atomic_fetch_add(&p.cnt_fc[pg * p.grid_b + nt], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); e_misc[1] = c == (unsigned)(p.grid_n - 1); stale |= c >= (unsigned)p.grid_n; }
            if (!ic_local)
                { const unsigned c = __hip_atomic_fetch_add(&p.cnt_ic[pg * p.grid_n + kt], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); e_misc[2] = c == (unsigned)(p.grid_b - 1); stale |= c >= (unsigned)p.grid_b; }
            if (stale) __hip_atomic_fetch_or(&p.flags[tile], 8u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    };

    // (3) residuals first (they are small), then the output stores, behind which the arrival counter's
    // round trip hides; variant 5 adds the pass over the requantised outputs
    if (reduce) {
        if (p.d_i) ic_pass(0);
        if (want_next) {
            __syncthreads();
            ic_pass(1);
        }
        if (checking) arrive();
        else if (tid == 0) p.flags[tile] = 0;    // partial-reduction variant: the finish kernel ORs its findings in
    }

    // (4) stores; checksum rows and columns are trimmed from y (end of Sec. 4.3).
    // int32 output with whole filter blocks: entry-major order, so that the two 64-byte halves of a
    // 128-byte line (filter blocks kb, kb + 1 of one pixel) leave in consecutive instructions, and no
    // per-element guards (3-4 % of the checked kernels, 13 % of the store-bound 64->256 1x1 layer)
    const bool whole_blocks = !p.out_int8 && p.mode != MODE_WRITE && (p.K & 15) == 0;
    if (whole_blocks) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const int e = nt * MB + wave * WM + i;
            if (!pvalid || e >= p.N) continue;
            int32_t *row = reinterpret_cast<int32_t *>(p.y) + ((long long)e * PQ + pix) * p.K + lg * 4;
#pragma unroll
            for (int kb = 0; kb < WK; ++kb) {
                const int fb = kt * WK + kb;
                if (fb < p.kblk) *reinterpret_cast<i32x4 *>(row + fb * 16) = acc[i][kb];
            }
        }
    }
    // int8 output (the epilog of Sec. 4.3).  A lane holds 4 bytes per (entry, block), far too little for a
    // store: with whole filter blocks the wave lays its requantised bytes out in LDS as
    // [entry][pixel][filter of the tile], 4 entries at a time, and writes them back 16 bytes per lane,
    // 16 * WK contiguous bytes per pixel.  Otherwise the 4 bytes are stored directly, guarded per filter.
    if (p.out_int8) {
        const bool staged = (p.K & 15) == 0;
        __syncthreads();                         // a residual pass of another wave may still be reading this memory
        int8_t *stage = lds + wave * (WK * 1024);
        constexpr int ROWB = WK * 16;            // bytes of one (entry, pixel) row of the tile
#pragma unroll
        for (int i0 = 0; i0 < WM; i0 += 4) {
#pragma unroll
            for (int kb = 0; kb < WK; ++kb) {
                const int fb = kt * WK + kb;
                const int k = fb * 16 + lg * 4;
                float sc[4], bi[4];
                {
                    const f32x4 s4 = *reinterpret_cast<const f32x4 *>(e_scale + kb * 16 + lg * 4);
                    const f32x4 b4 = *reinterpret_cast<const f32x4 *>(e_bias + kb * 16 + lg * 4);
#pragma unroll
                    for (int v = 0; v < 4; ++v) { sc[v] = s4[v]; bi[v] = b4[v]; }
                }
#pragma unroll
                for (int il = 0; il < 4; ++il) {
                    if (i0 + il >= WM) continue;
                    const int i = i0 + il < WM ? i0 + il : 0;
                    const int e = nt * MB + wave * WM + i;
                    const bool real = pvalid && e < p.N;
                    const int a4[4] = {acc[i][kb][0], acc[i][kb][1], acc[i][kb][2], acc[i][kb][3]};
                    const unsigned pk = requant_pack4(a4, sc, bi, p.relu);
                    if (staged) {
                        *reinterpret_cast<unsigned *>(stage + (il * 16 + lj) * ROWB + kb * 16 + lg * 4) = pk;
                    } else if (real) {
                        int8_t *dst = reinterpret_cast<int8_t *>(p.y) + ((long long)e * PQ + pix) * p.K + k;
                        if (k + 4 <= p.K && (p.K & 3) == 0) *reinterpret_cast<unsigned *>(dst) = pk;
                        else
                            for (int v = 0; v < 4; ++v)
                                if (k + v < p.K) dst[v] = (int8_t)((pk >> (8 * v)) & 0xff);
                    }
                }
            }
            if (staged) {
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int it = 0; it < WK; ++it) {
                    const int q = it * 64 + lane;
                    const int row = q / WK, c16 = q - row * WK;      // row = entry * 16 + pixel
                    const int il = row >> 4, px = pg * 16 + (row & 15);
                    const int e = nt * MB + wave * WM + i0 + il, fb = kt * WK + c16;
                    const i32x4 v = *reinterpret_cast<const i32x4 *>(stage + row * ROWB + c16 * 16);
                    if (i0 + il < WM && e < p.N && px < PQ && fb < p.kblk)
                        *reinterpret_cast<i32x4 *>(reinterpret_cast<int8_t *>(p.y) + ((long long)e * PQ + px) * p.K + fb * 16) = v;
                }
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                __builtin_amdgcn_wave_barrier();
            }
        }
    }
#pragma unroll
    for (int kb = 0; kb < WK; ++kb) {
        if (whole_blocks || p.out_int8) break;
        const int fb = kt * WK + kb;
        const int k = fb * 16 + lg * 4;                       // first of this lane's 4 filters
        if (fb < p.kblk) {
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                const int e = nt * MB + wave * WM + i;
                if (!pvalid) continue;
                if (e < p.N) {
                    int32_t *dst = reinterpret_cast<int32_t *>(p.y) + ((long long)e * PQ + pix) * p.K + k;
                    if (k + 4 <= p.K && (p.K & 3) == 0) *reinterpret_cast<i32x4 *>(dst) = acc[i][kb];
                    else
                        for (int v = 0; v < 4; ++v)
                            if (k + v < p.K) dst[v] = acc[i][kb][v];
                } else if (p.mode == MODE_WRITE && e < p.n_entries) {
                    int32_t *dst = p.ws_yi + ((long long)(e - p.N) * PQ + pix) * p.K + k;
                    for (int v = 0; v < 4; ++v)
                        if (k + v < p.K) dst[v] = acc[i][kb][v];
                }
            }
        } else if (fb == p.kblk && p.mode == MODE_WRITE && lg == 0 && pvalid) {
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                const int e = nt * MB + wave * WM + i;
                if (e < p.N) {
                    for (int v = 0; v < p.d_f; ++v) p.ws_yf[((long long)e * PQ + pix) * p.d_f + v] = acc[i][kb][v];
                } else if (e < p.n_entries) {
                    for (int v = 0; v < p.d_f; ++v) p.ws_yfi[((long long)(e - p.N) * PQ + pix) * p.d_f + v] = acc[i][kb][v];
                }
            }
        }
    }
    if (p.fic_xsum_next && p.out_int8) {
        __syncthreads();
        ic_pass(2);
    }
    if (!reduce) return;
    if (!exchange) return;   // MODE_PARTIAL: the finish kernel compares; local sums: done

    // (5) residuals that span several tiles are summed by the workgroup that arrives last and
    // reported on kt = 0 (FC) / nt = 0 (IC)
    __syncthreads();
    const bool last_fc = e_misc[1] != 0, last_ic = e_misc[2] != 0;
    if (!last_fc && !last_ic) return;
    if (last_fc) {
        uint32_t late = 0;
        const int *src = &p.ws_fc[(((long long)pg * p.grid_b + nt) * p.grid_n) * (MB * 16)];
        for (int r = tid; r < MB * 16; r += 256) {
            unsigned s = 0;
#pragma unroll 4
            for (int c = 0; c < p.grid_n; ++c) s += (unsigned)ld_dev(src + c * (MB * 16) + r);
            if (s != 0) late |= (nt * MB + (r >> 4) < p.N) ? 1u : 4u;
        }
        if (late) __hip_atomic_fetch_or(&p.flags[((long long)pg * p.grid_b + nt) * p.grid_n], late, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (tid == 0) __hip_atomic_store(&p.cnt_fc[pg * p.grid_b + nt], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
    }
    if (last_ic) {
        uint32_t late = 0;
        // the partials of this (pixel group, filter tile): [grid_b][WK][256] words
        const long long base = (((long long)pg * p.grid_n + kt) * p.grid_b) * WK * 256;
        const __amdgpu_buffer_rsrc_t rs_ic = __builtin_amdgcn_make_buffer_rsrc((void *)(p.ws_ic + base), 0, p.grid_b * WK * 1024, 0x00020000);
        const __amdgpu_buffer_rsrc_t rs_nx = __builtin_amdgcn_make_buffer_rsrc((void *)(want_next ? p.ws_nx + base : p.ws_ic + base), 0, p.grid_b * WK * 1024, 0x00020000);
        for (int idx = tid; idx < WK * 64; idx += 256) {      // one (filter block, lane) vector each
            const int kb = idx >> 6, ln = idx & 63;
            const int fb = kt * WK + kb;
            i32x4 s = zero4, sn = zero4;
#pragma unroll 4
            for (int b = 0; b < p.grid_b; ++b) {
                const int off = ((b * WK + kb) * 256 + ln * 4) * 4;
                s += ld_dev4(rs_ic, off);
                if (want_next) sn += ld_dev4(rs_nx, off);
            }
            if ((s[0] | s[1] | s[2] | s[3]) != 0)
                late |= (p.packed_df && fb == p.kblk - 1) ? ic_bits_shared(s, fb, ln >> 4) : ((fb < p.kblk) ? 2u : 4u);
            if (want_next && fb < p.kblk) {
                const int px = pg * 16 + (ln & 15), k = fb * 16 + (ln >> 4) * 4;
                if (px < PQ) {
                    int rest[4] = {sn[0], sn[1], sn[2], sn[3]};
                    for (int d = 0; d < p.d_i; ++d) {
                        unsigned pk = 0;
#pragma unroll
                        for (int v = 0; v < 4; ++v) pk |= ((unsigned)next_digit(rest[v]) & 0xffu) << (8 * v);
                        int8_t *dst = p.xchk_next + ((long long)d * PQ + px) * p.K + k;
                        if (k + 4 <= p.K && (p.K & 3) == 0) *reinterpret_cast<unsigned *>(dst) = pk;
                        else
                            for (int v = 0; v < 4; ++v)
                                if (k + v < p.K) dst[v] = (int8_t)((pk >> (8 * v)) & 0xff);
                    }
                }
            }
        }
        if (late) __hip_atomic_fetch_or(&p.flags[((long long)pg * p.grid_b) * p.grid_n + kt], late, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (tid == 0) __hip_atomic_store(&p.cnt_ic[pg * p.grid_n + kt], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    }  // int8 epilogue
#endif
}

}  // namespace abed
