// 3x3, stride-1 int8 convolution for gfx950 that keeps every ABED checksum local to a workgroup
// (Sec. 3.1, 3.2 option 1, 4.1, 4.3 of the paper): no checksum tensor goes through memory at run time
// except the offline filter checksums, no workgroup waits for another, and there is no separate input
// checksum kernel.
//
// Work split.  A workgroup (512 threads, 8 waves, one per CU) owns
//   - a box of 8x8 output pixels of the image plane (4 groups of 4x4 pixels),
//   - a range of batch entries, walked in batches of 8,
//   - a tile of 16*FBR filters, plus (FC) one block of 16 filters whose rows 0,1 are the two int8 digit
//     filters of THIS tile's filter checksum  sum_{k in tile} w[k]  (the scheme of Sec. 3.1 applied to
//     the tile's filters; digits as in Sec. 4.1).
// Wave w multiplies pixel group w>>1 for entries 4*(w&1) .. +3 of the batch against all FB filter
// blocks: 4*FB MFMA tiles of 16 filters x 16 pixels (v_mfma_i32_16x16x64_i8, filters = A operand).
//
// Reuse of the input.  For a chunk of 64 channels the 10x10 input pixels that the box's 3x3 windows
// touch are put into LDS once per entry and all nine taps read them from there (per-lane addresses),
// so an activation byte crosses the global->LDS path 1.56 times instead of 9.  The filters of one
// filter row (3 taps x 64 channels per filter) form a sub-stage; a barrier separates sub-stages, i.e.
// 3*FB*4 matrix instructions per wave lie between two barriers.
//
// Checks.
//   FC: per output row, sum over the tile's real filters == digit-recombined checksum-filter fmaps,
//       mod 2^32, in registers plus two cross-lane steps (as in conv_kernel.h).
//   IC: the scheme of Sec. 3.2 option 1 applied to the workgroup's range of entries: while the
//       entries stream through LDS every thread adds "its" 16 bytes of every entry's staged input
//       (bytes biased to unsigned, two 16-bit fields per register); after the last real batch the sums
//       are split into two int8 digit images (Sec. 4.1), written to LDS as two more entries, and
//       convolved like any batch.  sum_n acc[n] is kept in registers across batches (a wave's four
//       entries share their pixels) and must equal the digit-recombined fmaps of the digit images.
//   corner: FC residual of the digit images' rows, IC residual of the digit block's columns.
// One flag word per workgroup: bit 0 FC, bit 1 IC, bit 2 corner.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include "conv_kernel.h"

namespace abed {

struct BoxParams {
    const int8_t *x, *w, *wchk;   // wchk: [grid_n][2][R][S][C] digit filters of each filter tile's checksum
    void *y;                      // int32 or int8 [N][P][Q][K]
    const float *scale, *bias;    // epilog (Sec. 4.3) or null
    uint32_t *flags;              // [boxes][nranges][grid_n]
    int N, H, W, C, K, P, Q, ph, pw;
    int crsb;                     // 9 * C
    int nch;                      // C / 64
    int boxes_x, boxes_y;         // ceil(Q / 8), ceil(P / 8)
    int grid_n;                   // filter tiles
    int nranges, range_len;       // entry ranges: range i covers entries [i * range_len, min(N, (i+1) * range_len))
    int out_int8, relu;
    int inj_on, inj_box, inj_range, inj_kt, inj_batch, inj_wave, inj_i, inj_fb, inj_lane, inj_v;
    uint32_t inj_mask;
};

constexpr int kBox = 8;                       // output pixels per box side
constexpr int kHalo = kBox + 2;               // input pixels per side that a 3x3 window over the box touches
constexpr int kSlots = kHalo * kHalo;         // 100 input pixels per entry and chunk
constexpr int kEB = 8;                        // entries per batch
constexpr int kAEntry = kSlots * 64;          // bytes of one entry's staged chunk
constexpr int kAStage = kEB * kAEntry;        // 51200
constexpr int kAInstr = kAStage / 1024;       // 50 one-KB loads per stage

// s_waitcnt vmcnt(n) for a wave-uniform run-time n (the instruction takes an immediate): the largest
// compiled limit that does not exceed n.  Waiting for a smaller count than allowed is always safe.
__device__ __forceinline__ void wait_vmcnt_upto(int n)
{
#define ABED_W(k) if (n >= k) { ABED_WAIT_VMCNT(k); return; }
    ABED_W(48) ABED_W(40) ABED_W(36) ABED_W(32) ABED_W(28) ABED_W(24) ABED_W(22) ABED_W(20) ABED_W(18) ABED_W(16)
    ABED_W(14) ABED_W(12) ABED_W(11) ABED_W(10) ABED_W(9) ABED_W(8) ABED_W(7) ABED_W(6) ABED_W(5) ABED_W(4)
    ABED_W(3) ABED_W(2) ABED_W(1)
#undef ABED_W
    ABED_WAIT_VMCNT(0);
}

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// FB: filter blocks per tile incl. the digit block; FC: the last block is the digit block; XCH: 0 = no
// batch checksum, else the number of 64-channel chunks (== p.nch), one set of sum registers per chunk;
// NBR: sub-stages of the filter ring in LDS (2 or 3).
template <int FB, bool FC, int XCH, int NBR>
__global__ __launch_bounds__(512) void box_conv_kernel(const BoxParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int FBR = FB - (FC ? 1 : 0);
    constexpr bool IC = XCH > 0;
    constexpr int B_SUB = FB * 16 * 192;          // one filter row of taps: [16 FB filters][3 taps][64 B]
    constexpr int B_INSTR = B_SUB / 1024;         // 3 * FB
    constexpr int LB = (B_INSTR + 7) / 8;
    constexpr int LA = (kAInstr + 7) / 8;
    constexpr int A_OFF = 0, B_OFF = 2 * kAStage, MISC_OFF = B_OFF + NBR * B_SUB;
    constexpr int LDS_BYTES = MISC_OFF + 256 + 2 * FBR * 16 * 4;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    __shared__ __attribute__((aligned(1024))) int8_t lds[LDS_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lg = lane >> 4, lj = lane & 15;
    const int pg = wave >> 1, eh = wave & 1;

    // ---- block index -> (box, range, filter tile); blocks b, b+8, ... share an XCD and take a contiguous eighth
    const int nboxes = p.boxes_x * p.boxes_y;
    const int ntiles = nboxes * p.nranges * p.grid_n;
    const int per_xcd = (ntiles + 7) >> 3;
    int bid = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (bid >= ntiles) return;
    const int box = bid % nboxes; bid /= nboxes;
    const int range = bid % p.nranges;
    const int kt = bid / p.nranges;
    const int by = box / p.boxes_x, bx = box - by * p.boxes_x;
    const int n0 = range * p.range_len;
    const int n_end = (n0 + p.range_len < p.N) ? n0 + p.range_len : p.N;
    const int nbatch = (n_end - n0 + kEB - 1) / kEB;
    const int HWC = p.H * p.W * p.C;
    const int PQ = p.P * p.Q;

    constexpr int OOB = 0x7ffffff0;
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, n_end * HWC, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)p.w, 0, p.K * p.crsb, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_wc = __builtin_amdgcn_make_buffer_rsrc((void *)p.wchk, 0, (FC && p.wchk) ? p.grid_n * 2 * p.crsb : 0, 0x00020000);

    // ---- loader set-up: which 16 bytes each lane fetches in each of this wave's load instructions
    // A stage: piece q = instr * 64 + lane lands at LDS byte 16 q; q -> (entry e, slot, part'); the 16-byte
    // part actually fetched is part' ^ (halo row & 3), which makes the fragment reads conflict-free.
    int a_off[LA];            // byte offset inside the batch's first image, or OOB
    int a_cnt = 0;            // instructions this wave issues per stage (wave-uniform)
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        const int instr = j * 8 + wave;
        a_off[j] = OOB;
        if (instr < kAInstr) {
            ++a_cnt;
            const int q = instr * 64 + lane;
            const int e = q / (kSlots * 4), rem = q - e * (kSlots * 4);
            const int slot = rem >> 2, part = rem & 3;
            const int hy = slot / kHalo, hx = slot - hy * kHalo;
            const int iy = by * kBox - p.ph + hy, ix = bx * kBox - p.pw + hx;
            if ((unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W)
                a_off[j] = ((e * p.H + iy) * p.W + ix) * p.C + ((part ^ (hy & 3)) << 4);
        }
    }
    // B sub-stage: piece q -> (filter row f of the tile, tap t of the filter row, part'); fetched part = part' ^ ((f >> 2) & 3)
    int b_off[LB];
    bool b_chk[LB];           // wave-uniform: the instruction's rows belong to the digit block
    int b_cnt = 0;
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        const int instr = j * 8 + wave;
        b_off[j] = OOB; b_chk[j] = false;
        if (instr < B_INSTR) {
            ++b_cnt;
            const int q = instr * 64 + lane;
            const int f = q / 12, rem = q - f * 12;
            const int t = rem >> 2, part = rem & 3;
            const int inrow = t * p.C + ((part ^ ((f >> 2) & 3)) << 4);
            if (f < FBR * 16) {
                b_off[j] = (kt * FBR * 16 + f) * p.crsb + inrow;
            } else {
                b_chk[j] = true;
                const int df = f - FBR * 16;
                if (df < 2) b_off[j] = (kt * 2 + df) * p.crsb + inrow;
            }
        }
    }

    // ---- in-order model of the vector-memory counter (loads, LDS DMA and stores complete in issue order):
    // `issued` counts this wave's vector-memory instructions; a wait for "everything up to mark m" allows
    // issued - m younger ones to be outstanding.
    int issued = 0;
    int b_mark[NBR];          // value of `issued` right after the loads of the sub-stage in ring slot i
    int a_mark[2];
#pragma unroll
    for (int i = 0; i < NBR; ++i) b_mark[i] = 0;
    a_mark[0] = a_mark[1] = 0;

    auto issue_b = [&](int slot, int chunk, int r) {
        const int soff = r * 3 * p.C + chunk * 64;
        int8_t *dst0 = lds + B_OFF + slot * B_SUB;
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            const int instr = j * 8 + wave;
            if (instr < B_INSTR) {   // wave-uniform
                __attribute__((address_space(3))) void *dst = (__attribute__((address_space(3))) void *)(dst0 + instr * 1024);
                if (b_chk[j]) __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_wc, dst, 16, b_off[j], soff, 0, 0);
                else __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, dst, 16, b_off[j], soff, 0, 0);
            }
        }
        issued += b_cnt;
    };
    auto issue_a = [&](int buf, int batch, int chunk) {
        const int base = (n0 + batch * kEB) * HWC;
        int8_t *dst0 = lds + A_OFF + buf * kAStage;
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            const int instr = j * 8 + wave;
            if (instr < kAInstr) {   // wave-uniform
                __attribute__((address_space(3))) void *dst = (__attribute__((address_space(3))) void *)(dst0 + instr * 1024);
                const int voff = a_off[j] == OOB ? OOB : a_off[j] + base;   // entries at or past n_end fall outside the descriptor
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, dst, 16, voff, chunk * 64, 0, 0);
            }
        }
        issued += a_cnt;
    };

    // ---- fragment addresses
    // B: lane (lg, lj) wants part lg of row fb*16 + lj, tap s: const + fb * 3072 + s * 64
    const int b_lane = lj * 192 + (((lg ^ (lj >> 2)) & 3) << 4);
    // A: lane's pixel inside the box and its slot for tap (0,0)
    const int oy_l = (pg >> 1) * 4 + (lj >> 2), ox_l = (pg & 1) * 4 + (lj & 3);
    const int sig0 = oy_l * kHalo + ox_l;
    const int oy = by * kBox + oy_l, ox = bx * kBox + ox_l;
    const bool pvalid = oy < p.P && ox < p.Q;
    const int pix = oy * p.Q + ox;

    // ---- batch checksum state: this thread's 16 bytes (piece) of every entry's staged chunk
    const bool x_on = IC && tid < kSlots * 4;
    const int x_piece = tid * 16;            // byte offset of the piece inside an entry's stage
    constexpr int XR = IC ? XCH : 1;
    unsigned xs_lo[XR][4], xs_hi[XR][4];
#pragma unroll
    for (int c = 0; c < XR; ++c)
#pragma unroll
        for (int d = 0; d < 4; ++d) xs_lo[c][d] = xs_hi[c][d] = 0u;

    // the epilog's scale and bias of this tile's filters, once (the loop's first barrier publishes them)
    float *e_scale = reinterpret_cast<float *>(lds + MISC_OFF + 256), *e_bias = e_scale + FBR * 16;
    if (p.out_int8 && tid < 2 * FBR * 16) {
        const int f = tid < FBR * 16 ? tid : tid - FBR * 16;
        e_scale[tid] = (tid < FBR * 16 ? p.scale : p.bias)[kt * FBR * 16 + f];
    }

    i32x4 acc[4][FB];
    i32x4 icsum[FB];
    const i32x4 zero4 = {0, 0, 0, 0};
#pragma unroll
    for (int fb = 0; fb < FB; ++fb) icsum[fb] = zero4;
    uint32_t my_flag = 0;

    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.N * PQ * p.K * (p.out_int8 ? 1 : 4), 0x00020000);

    // ---- the multiply phase of one sub-step (filter row r) for NI of this wave's entries
    auto mfma_row = [&](auto ni_tag, int abuf, int bslot, int r) {
        constexpr int NI = decltype(ni_tag)::value;
        const int hy = oy_l + r;
        const int8_t *pa = lds + A_OFF + abuf * kAStage + (eh * 4) * kAEntry + (sig0 + r * kHalo) * 64 + (((lg ^ hy) & 3) << 4);
        const int8_t *pb = lds + B_OFF + bslot * B_SUB + b_lane;
#pragma unroll 1
        for (int s = 0; s < 3; ++s) {
            i32x4 bfr[NI];
#pragma unroll
            for (int i = 0; i < NI; ++i) bfr[i] = *reinterpret_cast<const i32x4 *>(pa + i * kAEntry + s * 64);
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) {
                const i32x4 afr = *reinterpret_cast<const i32x4 *>(pb + fb * 3072 + s * 64);
#pragma unroll
                for (int i = 0; i < NI; ++i) acc[i][fb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(afr, bfr[i], acc[i][fb], 0, 0, 0);
            }
        }
    };

    // ---- FC residual of one accumulator row set (Sec. 3.1 with the digit shifts of Sec. 4.1)
    auto fc_residual = [&](int i) -> unsigned {
        unsigned r = 0;
#pragma unroll
        for (int fb = 0; fb < FBR; ++fb)
            r += (unsigned)acc[i][fb][0] + (unsigned)acc[i][fb][1] + (unsigned)acc[i][fb][2] + (unsigned)acc[i][fb][3];
        if (FC && lg == 0) r -= (unsigned)acc[i][FB - 1][0] + ((unsigned)acc[i][FB - 1][1] << 8);
        r += (unsigned)__shfl_xor((int)r, 16, 64);
        r += (unsigned)__shfl_xor((int)r, 32, 64);
        return r;
    };

    // ---- main loop over steps = (batch, chunk); batch == nbatch is the digit batch (IC only)
    const int nsteps_real = nbatch * p.nch;
    const int nsteps = (nbatch + (IC ? 1 : 0)) * p.nch;
    const int nsub = nsteps * 3;
    // prologue: the first NBR-1 filter sub-stages and the first A stage
    {
#pragma unroll
        for (int u = 0; u < NBR - 1; ++u) {
            if (u < nsub) {
                const int st = u / 3, r = u - st * 3;
                issue_b(u % NBR, st % p.nch, r);
                b_mark[u % NBR] = issued;
            }
            if (u == 0) { issue_a(0, 0, 0); a_mark[0] = issued; }
        }
    }

    int usub = 0;             // running sub-step index
    int bslot = 0;            // usub % NBR
    for (int batch = 0; batch < nbatch + (IC ? 1 : 0); ++batch) {
        const bool digit = IC && batch == nbatch;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) acc[i][fb] = zero4;

        auto step = [&](auto c_tag, int chunk) {
            constexpr int CT = decltype(c_tag)::value;       // compile-time chunk for the checksum registers (0 when XCH == 0)
            const int stepi = batch * p.nch + chunk;
            const int abuf = stepi & 1;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                // (1) this sub-step's filters, and at r == 0 this step's inputs, have landed
                {
                    int need = b_mark[bslot];
                    if (r == 0 && !digit && a_mark[abuf] > need) need = a_mark[abuf];
                    wait_vmcnt_upto(issued - need);
                }
                __builtin_amdgcn_s_waitcnt(0xc07f);          // this wave's LDS writes (digit images) are done: lgkmcnt(0)
                __builtin_amdgcn_s_barrier();
                // (2) refill: the ring slot that sub-step usub-1 used, and at r == 0 the A buffer that step-1 used
                {
                    const int un = usub + NBR - 1;
                    if (un < nsub) {
                        const int st = un / 3, rr = un - st * 3;
                        int sl = bslot + NBR - 1; if (sl >= NBR) sl -= NBR;
                        issue_b(sl, st % p.nch, rr);
                        b_mark[sl] = issued;
                    }
                    if (r == 0 && stepi + 1 < nsteps_real) {
                        const int nb = (chunk + 1 == p.nch) ? batch + 1 : batch;
                        const int nc = (chunk + 1 == p.nch) ? 0 : chunk + 1;
                        issue_a(abuf ^ 1, nb, nc);
                        a_mark[abuf ^ 1] = issued;
                    }
                }
                // (3) batch checksum: add this step's staged inputs; hand the finished sums of the next
                // digit step's chunk to LDS as two digit images (Sec. 4.1)
                if constexpr (IC) {
                    if (r == 0) {
                        if (!digit && x_on) {
                            const int8_t *src = lds + A_OFF + abuf * kAStage + x_piece;
#pragma unroll
                            for (int e = 0; e < kEB; ++e) {
                                const i32x4 v = *reinterpret_cast<const i32x4 *>(src + e * kAEntry);
#pragma unroll
                                for (int d = 0; d < 4; ++d) {
                                    const unsigned u = (unsigned)v[d] ^ 0x80808080u;
                                    xs_lo[CT][d] += u & 0x00ff00ffu;
                                    xs_hi[CT][d] += (u >> 8) & 0x00ff00ffu;
                                }
                            }
                        }
                        if (stepi + 1 >= nsteps_real && stepi + 1 < nsteps && x_on) {
                            constexpr int CN = (CT + 1) % XR;        // chunk of step stepi + 1
                            const int bias = 128 * nbatch * kEB;     // every staged entry added 128 per byte (zero-filled ones too)
                            i32x4 d0, d1;
#pragma unroll
                            for (int d = 0; d < 4; ++d) {
                                int s0 = (int)(xs_lo[CN][d] & 0xffffu) - bias, s1 = (int)(xs_hi[CN][d] & 0xffffu) - bias;
                                int s2 = (int)(xs_lo[CN][d] >> 16) - bias, s3 = (int)(xs_hi[CN][d] >> 16) - bias;
                                const unsigned lo = ((unsigned)next_digit(s0) & 0xffu) | (((unsigned)next_digit(s1) & 0xffu) << 8) |
                                                    (((unsigned)next_digit(s2) & 0xffu) << 16) | (((unsigned)next_digit(s3) & 0xffu) << 24);
                                const unsigned hi = ((unsigned)s0 & 0xffu) | (((unsigned)s1 & 0xffu) << 8) | (((unsigned)s2 & 0xffu) << 16) | (((unsigned)s3 & 0xffu) << 24);
                                d0[d] = (int)lo; d1[d] = (int)hi;
                            }
                            int8_t *dst = lds + A_OFF + (abuf ^ 1) * kAStage + x_piece;
                            *reinterpret_cast<i32x4 *>(dst) = d0;
                            *reinterpret_cast<i32x4 *>(dst + kAEntry) = d1;
                        }
                    }
                }
                // (4) multiply
                if (!digit) mfma_row(std::integral_constant<int, 4>{}, abuf, bslot, r);
                else if (eh == 0) mfma_row(std::integral_constant<int, 2>{}, abuf, bslot, r);
                ++usub;
                if (++bslot == NBR) bslot = 0;
            }
        };
        if constexpr (IC) {
            // chunk loop unrolled: the checksum registers of a chunk are selected at compile time
            static_for<0, XR>([&](auto c_tag) { step(c_tag, decltype(c_tag)::value); });
        } else {
            for (int chunk = 0; chunk < p.nch; ++chunk) step(std::integral_constant<int, 0>{}, chunk);
        }

        // ---- epilogue of the batch (registers only; the next batch's loads are already in flight)
        if (!digit) {
            if (p.inj_on && box == p.inj_box && range == p.inj_range && kt == p.inj_kt && batch == p.inj_batch && wave == p.inj_wave) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int fb = 0; fb < FBR; ++fb)
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (i == p.inj_i && fb == p.inj_fb && v == p.inj_v && lane == p.inj_lane) acc[i][fb][v] ^= (int)p.inj_mask;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = n0 + batch * kEB + eh * 4 + i;
                if (FC) {
                    const unsigned r = fc_residual(i);
                    if (r != 0 && e < n_end) my_flag |= 1u;
                }
                if (IC) {
#pragma unroll
                    for (int fb = 0; fb < FB; ++fb) icsum[fb] += acc[i][fb];   // entries past the range are all zero
                }
                // stores: checksum columns are trimmed (end of Sec. 4.3); masked lanes go out of the descriptor's range
                const bool live = pvalid && e < n_end;
                if (!p.out_int8) {
                    const int o = live ? ((e * PQ + pix) * p.K + kt * FBR * 16 + lg * 4) * 4 : OOB;
#pragma unroll
                    for (int fb = 0; fb < FBR; ++fb)
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[i][fb]), rs_y, o, fb * 64, 0);
                    issued += FBR;
                } else {
                    const int o = live ? (e * PQ + pix) * p.K + kt * FBR * 16 + lg * 4 : OOB;
#pragma unroll
                    for (int fb = 0; fb < FBR; ++fb) {
                        const int k = fb * 16 + lg * 4;
                        unsigned pk = 0;
#pragma unroll
                        for (int v = 0; v < 4; ++v) pk |= ((unsigned)requant(acc[i][fb][v], e_scale[k + v], e_bias[k + v], p.relu) & 0xffu) << (8 * v);
                        __builtin_amdgcn_raw_buffer_store_b32(pk, rs_y, o, fb * 16, 0);
                    }
                    issued += FBR;
                }
            }
        }
    }

    // ---- final comparisons
    if constexpr (IC) {
        // digit batch results sit in acc[0], acc[1] of the even waves; corner: the digit images' rows under FC
        int *red = reinterpret_cast<int *>(lds);              // [4 pixel groups][FB][64 lanes][4]: the odd waves' sums
        ABED_WAIT_VMCNT(0);
        __syncthreads();                                      // all fragment reads are done; LDS is free
        if (eh == 1) {
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) *reinterpret_cast<i32x4 *>(red + ((pg * FB + fb) * 64 + lane) * 4) = icsum[fb];
        }
        __syncthreads();
        if (eh == 0) {
            if (FC) {
                if (fc_residual(0) != 0 || fc_residual(1) != 0) my_flag |= 4u;
            }
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) {
                i32x4 c = icsum[fb] + *reinterpret_cast<const i32x4 *>(red + ((pg * FB + fb) * 64 + lane) * 4);
#pragma unroll
                for (int v = 0; v < 4; ++v) c[v] -= (int)((unsigned)acc[0][fb][v] + ((unsigned)acc[1][fb][v] << 8));
                if ((c[0] | c[1] | c[2] | c[3]) != 0) my_flag |= (FC && fb == FB - 1) ? 4u : 2u;
            }
        }
    }
    if (p.flags) {
        int *misc = reinterpret_cast<int *>(lds + MISC_OFF);
        const uint32_t wf = wave_or3(my_flag);
        if (lane == 0) misc[wave] = (int)wf;
        __syncthreads();
        if (tid == 0) {
            uint32_t f = 0;
#pragma unroll
            for (int w8 = 0; w8 < 8; ++w8) f |= (uint32_t)misc[w8];
            p.flags[(box * p.nranges + range) * p.grid_n + kt] = f;
        }
    }
#endif
}

}  // namespace abed
