// 3x3, stride-1 int8 convolution for gfx950 that keeps every ABED checksum local to a workgroup
// (Sec. 3.1, 3.2 option 1, 4.1, 4.3 of the paper): no checksum tensor goes through memory at run time
// except the offline filter checksums, no workgroup waits for another, and there is no separate input
// checksum kernel.
//
// Work split.  A workgroup (512 threads, 8 waves, one per CU; template parameter EH = 1: 256 threads, 4 waves, two
// per CU, batches of 4) owns
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
    long long *dbg_ts;   // builds with ABED_ENABLE_DBG only: time stamps of two waves of one workgroup
    int dbg;   // timing experiments (builds with ABED_ENABLE_DBG only): bit 0 no loads in the loop, 1 no matrix instructions, 2 no stores, 3 no barriers
};

constexpr int kBox = 8;                       // output pixels per box side
constexpr int kHalo = kBox + 2;               // input pixels per side that a 3x3 window over the box touches
constexpr int kSlots = kHalo * kHalo;         // 100 input pixels per entry and chunk
constexpr int kAEntry = kSlots * 64;          // bytes of one entry's staged chunk

// s_waitcnt vmcnt(n) for a wave-uniform run-time n (the instruction takes an immediate): the largest
// compiled limit that does not exceed n, found by a short tree of scalar branches.  Waiting for a smaller
// count than allowed is always safe.
__device__ __forceinline__ void wait_vmcnt_upto(int n)
{
    if (n >= 6) {
        if (n >= 16) {
            if (n >= 24) ABED_WAIT_VMCNT(24); else if (n >= 20) ABED_WAIT_VMCNT(20); else ABED_WAIT_VMCNT(16);
        } else {
            if (n >= 12) ABED_WAIT_VMCNT(12); else if (n >= 8) ABED_WAIT_VMCNT(8); else ABED_WAIT_VMCNT(6);
        }
    } else {
        if (n >= 3) {
            if (n >= 5) ABED_WAIT_VMCNT(5); else if (n >= 4) ABED_WAIT_VMCNT(4); else ABED_WAIT_VMCNT(3);
        } else {
            if (n >= 2) ABED_WAIT_VMCNT(2); else if (n >= 1) ABED_WAIT_VMCNT(1); else ABED_WAIT_VMCNT(0);
        }
    }
}

// Where the 16-byte parts of a staged input pixel sit inside its 64-byte slot.  A 16-byte-per-lane LDS read serves
// 8 consecutive lanes per cycle out of a 128-byte bank window; the 8 lanes of a fragment read are 4 neighbouring
// pixels of two neighbouring halo rows, i.e. slots sigma..sigma+3 and sigma+10..sigma+13.  Slots of equal parity
// share a half of the window, so the part index is XOR-ed with (bit 1 of the slot, bit 0 of the halo row): the four
// lanes of a parity class then read four different parts.
__device__ __forceinline__ int a_swz(int slot, int hy) { return ((slot >> 1) & 1) | ((hy & 1) << 1); }

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
// NBR: sub-stages of the filter ring in LDS (2 or 3); EH: entry halves = groups of four waves.  EH = 2: 8 waves,
// batches of 8 entries, one workgroup per CU.  EH = 1: 4 waves, batches of 4 entries, at most 80 KB of LDS and 256
// registers, so that two workgroups share a CU and one's loads, barriers and stores overlap the other's matrix work.
template <int FB, bool FC, int XCH, int NBR, int EH = 2>
__global__ __launch_bounds__(256 * EH, 2 / EH) void box_conv_kernel(const BoxParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int FBR = FB - (FC ? 1 : 0);
    constexpr bool IC = XCH > 0;
    constexpr int NW = 4 * EH;                    // waves
    constexpr int kEB = 4 * EH;                   // entries per batch
    constexpr int kAStage = kEB * kAEntry;        // 51200 / 25600
    constexpr int kAInstr = kAStage / 1024;       // one-KB loads per stage
    // one filter row of taps: [16 FB filters][3 taps][64 B].  With EH = 1 the digit block keeps 1 KB (its rows 0, 1
    // are the digit filters, rows 2..4 zeros); the fragment reads of its rows 5..15 run into what follows and give
    // values nobody uses (only the lanes of filters 0..3 of the digit block are ever looked at)
    constexpr bool SHORT_DIGIT = FC && EH == 1;
    constexpr int B_SUB = SHORT_DIGIT ? FBR * 16 * 192 + 1024 : FB * 16 * 192;
    constexpr int B_INSTR = B_SUB / 1024;
    constexpr int LB = (B_INSTR + NW - 1) / NW;
    constexpr int LA = (kAInstr + NW - 1) / NW;
    constexpr int A_OFF = 0, B_OFF = 2 * kAStage, MISC_OFF = B_OFF + NBR * B_SUB + (SHORT_DIGIT ? 2048 : 0);
    constexpr int LDS_BYTES = MISC_OFF + 256 + 2 * FBR * 16 * 4;
    static_assert(LDS_BYTES <= 160 * 1024 / (3 - EH), "LDS");
    __shared__ __attribute__((aligned(1024))) int8_t lds[LDS_BYTES];

#ifdef ABED_ENABLE_DBG
    if (p.dbg & 16) return;      // launch floor
#endif
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lg = lane >> 4, lj = lane & 15;
    const int pg = wave / EH, eh = wave % EH;

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
    constexpr int kMasked = 0x40000000;     // + any offset inside x (below 2^30 bytes) stays beyond x's descriptor and below 2^31
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
        const int instr = j * NW + wave;
        a_off[j] = kMasked;
        if (instr < kAInstr) {
            ++a_cnt;
            const int q = instr * 64 + lane;
            const int e = q / (kSlots * 4), rem = q - e * (kSlots * 4);
            const int slot = rem >> 2, part = rem & 3;
            const int hy = slot / kHalo, hx = slot - hy * kHalo;
            const int iy = by * kBox - p.ph + hy, ix = bx * kBox - p.pw + hx;
            if ((unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W)
                a_off[j] = ((e * p.H + iy) * p.W + ix) * p.C + ((part ^ a_swz(slot, hy)) << 4);
        }
    }
    // B sub-stage: piece q -> (filter row f of the tile, tap t of the filter row, part'); fetched part = part' ^ ((f >> 1) & 3)
    // (rows are 192 bytes: rows of equal parity share a half of the 128-byte bank window, and the 8 lanes of a read are 8 consecutive rows)
    int b_off[LB];
    int b_cnt = 0;
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        const int instr = j * NW + wave;
        b_off[j] = OOB;
        if (instr < B_INSTR) {
            ++b_cnt;
            const int q = instr * 64 + lane;
            const int f = q / 12, rem = q - f * 12;
            const int t = rem >> 2, part = rem & 3;
            const int inrow = t * p.C + ((part ^ ((f >> 1) & 3)) << 4);
            if (f < FBR * 16) {
                b_off[j] = (kt * FBR * 16 + f) * p.crsb + inrow;
            } else {
                const int df = f - FBR * 16;
                if (df < 2) b_off[j] = (kt * 2 + df) * p.crsb + inrow;
            }
        }
    }

    // ---- which of the 3*FB load slots of a sub-step this wave uses (loop-invariant, wave-uniform bit masks):
    // filters at slots 1 + 4 J, inputs at the even slots 2 + 2 J' (r == 0: instructions J = J', r == 1: J = J' + 4)
    unsigned msk_b = 0, msk_a0 = 0, msk_a1 = 0;
#pragma unroll
    for (int j = 0; j < LB; ++j)
        if (j * NW + wave < B_INSTR) msk_b |= 1u << (1 + 4 * j);
#pragma unroll
    for (int j = 0; j < LA; ++j)
        if (j * NW + wave < kAInstr) { if (j < 4) msk_a0 |= 1u << (2 + 2 * j); else msk_a1 |= 1u << (2 + 2 * (j - 4)); }
    static_assert(1 + 4 * (LB - 1) < 3 * FB && 2 + 2 * 3 < 3 * FB && LA <= 8, "load slots");
    // the digit block's rows can only be in this wave's last filter instruction
    const bool last_chk = FC && (LB - 1) * NW + wave >= FBR * 3;
    const __amdgpu_buffer_rsrc_t rs_blast = last_chk ? rs_wc : rs_w;

    // Vector-memory instructions (loads, LDS DMA, stores) complete in issue order, so "everything issued
    // before the previous sub-step's are done" is a wait that allows as many outstanding ones as that
    // sub-step issued: vm_prev.  Filters are requested two sub-steps ahead (NBR == 3; with NBR == 2 one
    // ahead: then only the stores behind them may stay outstanding) and inputs a step ahead.
    int vm_prev = 0, st_prev = 0;   // loads / stores issued by this wave in the previous sub-step

    auto issue_b = [&](int slot, int chunk, int r) {
        static_for<0, LB>([&](auto j_tag) {
            constexpr int J = decltype(j_tag)::value;
            const int instr = J * NW + wave;
            if (instr < B_INSTR) {
                __attribute__((address_space(3))) void *dst = (__attribute__((address_space(3))) void *)(lds + B_OFF + slot * B_SUB + instr * 1024);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(J == LB - 1 ? rs_blast : rs_w, dst, 16, b_off[J], r * 3 * p.C + chunk * 64, 0, 0);
            }
        });
    };
    auto issue_a = [&](int buf, int batch, int chunk) {
        static_for<0, LA>([&](auto j_tag) {
            constexpr int J = decltype(j_tag)::value;
            const int instr = J * NW + wave;
            if (instr < kAInstr) {
                __attribute__((address_space(3))) void *dst = (__attribute__((address_space(3))) void *)(lds + A_OFF + buf * kAStage + instr * 1024);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, dst, 16, a_off[J] + (n0 + batch * kEB) * HWC, chunk * 64, 0, 0);
            }
        });
    };

    // ---- fragment addresses
    // B: lane (lg, lj) wants part lg of row fb*16 + lj, tap s: const + fb * 3072 + s * 64
    const int b_lane = lj * 192 + (((lg ^ (lj >> 1)) & 3) << 4);
    // A: lane's pixel inside the box and its slot for tap (0,0)
    const int oy_l = (pg >> 1) * 4 + (lj >> 2), ox_l = (pg & 1) * 4 + (lj & 3);
    const int sig0 = oy_l * kHalo + ox_l;
    const int oy = by * kBox + oy_l, ox = bx * kBox + ox_l;
    const bool pvalid = oy < p.P && ox < p.Q;
    const int pix = oy * p.Q + ox;

    // ---- batch checksum state: this thread's 16 bytes (piece) of every entry's staged chunk
    // (EH = 2: 400 pieces on 512 threads, one each, its eight entries added over sub-steps r = 1, 2;  EH = 1: 256
    // threads, piece tid in r = 1 and piece 256 + tid, for the first 144 threads, in r = 2, four entries each)
    constexpr int NP = IC ? 3 - EH : 1;      // pieces per thread
    const int x_piece = tid * 16;            // byte offset of the (first) piece inside an entry's stage
    constexpr int XR = IC ? XCH : 1;
    unsigned xs_lo[XR][NP][4], xs_hi[XR][NP][4];
#pragma unroll
    for (int c = 0; c < XR; ++c)
#pragma unroll
        for (int q = 0; q < NP; ++q)
#pragma unroll
            for (int d = 0; d < 4; ++d) xs_lo[c][q][d] = xs_hi[c][q][d] = 0u;

    unsigned xt_lo[4] = {0u, 0u, 0u, 0u}, xt_hi[4] = {0u, 0u, 0u, 0u};
    i32x4 x_next = {0, 0, 0, 0};

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

    // ---- the multiply phase of one sub-step (filter row r) for NI of this wave's entries: 3 FB groups of NI matrix
    // instructions, group g = (tap g / FB, filter block g % FB).  Fragments are requested ahead of their use: the
    // pixel fragments of tap s+1 at the start of tap s (two register sets), the filter fragment of group g + 3
    // before group g's matrix instructions (a ring of four), so the LDS latency hides behind matrix work.
    auto mfma_row = [&](auto ni_tag, int abuf, int bslot, int r, int ebase, auto &&mid) {
        constexpr int NI = decltype(ni_tag)::value;
        constexpr int RB = 4, G = 3 * FB;
        const int hy = oy_l + r;
        // this lane's pixel fragment of tap s: slot sig0 + 10 r + s, part lg at its swizzled place
        const int8_t *pa3[3];
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            const int slot = sig0 + r * kHalo + t;
            pa3[t] = lds + A_OFF + abuf * kAStage + ebase * kAEntry + slot * 64 + ((lg ^ a_swz(slot, hy)) << 4);
        }
        const int8_t *pb = lds + B_OFF + bslot * B_SUB + b_lane;
        i32x4 bfr[2][NI], afr[RB];
        auto fetch_a = [&](int set, int s) {
#pragma unroll
            for (int i = 0; i < NI; ++i) bfr[set][i] = *reinterpret_cast<const i32x4 *>(pa3[s] + i * kAEntry);
        };
        fetch_a(0, 0);
        static_for<0, RB - 1>([&](auto g_tag) {
            constexpr int GG = decltype(g_tag)::value;
            afr[GG % RB] = *reinterpret_cast<const i32x4 *>(pb + (GG % FB) * 3072 + (GG / FB) * 64);
        });
        static_for<0, G>([&](auto g_tag) {
            constexpr int GG = decltype(g_tag)::value;
            constexpr int S = GG / FB, F = GG % FB;
            if constexpr (F == 0 && S < 2) fetch_a((S + 1) & 1, S + 1);
            if constexpr (GG + RB - 1 < G) {
                constexpr int GN = GG + RB - 1;
                afr[GN % RB] = *reinterpret_cast<const i32x4 *>(pb + (GN % FB) * 3072 + (GN / FB) * 64);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NI; ++i) acc[i][F] = __builtin_amdgcn_mfma_i32_16x16x64_i8(afr[GG % RB], bfr[S & 1][i], acc[i][F], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            mid(g_tag);      // at most one refill load (see the sub-step)
            __builtin_amdgcn_sched_barrier(0);
        });
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

    // ---- main loop over sub-steps; a step = (batch, chunk) = three sub-steps (filter rows); batch == nbatch is
    // the digit batch (IC only)
    const int nsteps_real = nbatch * p.nch;
    const int nsteps = (nbatch + (IC ? 1 : 0)) * p.nch;
    const int nsub = nsteps * 3;
#ifdef ABED_ENABLE_DBG
    if (p.dbg & 32) { if (p.flags && tid == 0) p.flags[(box * p.nranges + range) * p.grid_n + kt] = (uint32_t)(a_off[0] + b_off[0] + msk_b) & 0u; return; }   // set-up only
#endif
    // prologue: the first filter sub-stage and the first A stage, then (NBR == 3) the second filter sub-stage
    issue_b(0, 0, 0);
    issue_a(0, 0, 0);
    if (NBR == 3) { issue_b(1, 0, 1); vm_prev = b_cnt; }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) acc[i][fb] = zero4;

    int bslot = 0;            // usub % NBR
    int r = 0, chunk = 0, batch = 0, stepi = 0;
    int pf_r = (NBR - 1) % 3, pf_chunk = ((NBR - 1) / 3) % p.nch;    // (filter row, chunk) of sub-step usub + NBR - 1
#ifdef ABED_ENABLE_DBG
    int nts = 0;
    const bool ts_on = p.dbg_ts && (int)blockIdx.x == 16 && (tid == 0 || tid == 448);
    long long *ts_buf = p.dbg_ts + (tid == 0 ? 0 : 2048);
#define ABED_TS() do { if (ts_on && nts < 2048) ts_buf[nts++] = (long long)__builtin_amdgcn_s_memtime(); } while (0)
#else
#define ABED_TS() do { } while (0)
#endif
    int usub = 0;
    // one sub-step; dig_tag: compile-time "this is the digit batch" (its own copy of the code, so that no
    // branch inside the loop decides which matrix instructions touch the accumulators)
    auto substep = [&](auto dig_tag) {
        constexpr bool digit = decltype(dig_tag)::value;
        const int abuf = stepi & 1;
        ABED_TS();
        // (1) this sub-step's filters, and at r == 0 this step's inputs, have landed.  With one chunk the filter
        // ring holds the whole tile from the second step on: then only the change of the A buffer (r == 0)
        // needs the workgroup to meet.
        const bool resident = NBR == 3 && p.nch == 1 && usub >= 3;
        if (!resident || r == 0) {
            wait_vmcnt_upto((NBR == 3 ? vm_prev : 0) + st_prev);
            ABED_TS();
            __builtin_amdgcn_s_waitcnt(0xc07f);          // this wave's LDS writes (digit images) are done: lgkmcnt(0)
#ifdef ABED_ENABLE_DBG
            if (!(p.dbg & 8))
#endif
            __builtin_amdgcn_s_barrier();
        } else {
            ABED_TS();
        }
        ABED_TS();
        // (2) refill, issued inside (4), at most one load behind every group of matrix instructions: the
        // address unit the loads go through is shared by the eight waves, and a burst from all of them stalls
        // every wave at once.  Filters of sub-step usub + NBR - 1 go into the ring slot that sub-step usub-1
        // used; inputs of step + 1 (at r == 0 and r == 1) into the A buffer that step-1 used.  With one chunk the
        // ring holds the whole filter tile after the first three sub-steps, and nothing is reloaded.
        const bool more_a = stepi + 1 < nsteps_real && r < 2;
        const bool more_b = usub + NBR - 1 < nsub && !(NBR == 3 && p.nch == 1 && usub >= 1);
        unsigned m = (more_b ? msk_b : 0u) | (more_a ? (r == 0 ? msk_a0 : msk_a1) : 0u);
#ifdef ABED_ENABLE_DBG
        if (p.dbg & 1) m = 0;
#endif
        int bsl = bslot + NBR - 1; if (bsl >= NBR) bsl -= NBR;
        const int8_t *b_dst = lds + B_OFF + bsl * B_SUB + wave * 1024;
        const int b_soff = pf_r * 3 * p.C + pf_chunk * 64;
        const int8_t *a_dst = lds + A_OFF + (abuf ^ 1) * kAStage + wave * 1024 + (r == 1 ? 4 * NW * 1024 : 0);
        const int a_soff = ((chunk + 1 == p.nch) ? 0 : chunk + 1) * 64;
        int a_voff[4];
        if (more_a) {
            const int abase = (n0 + ((chunk + 1 == p.nch) ? batch + 1 : batch) * kEB) * HWC;   // masked lanes stay beyond the descriptor, as do entries at or past n_end
#pragma unroll
            for (int j = 0; j < 4; ++j) a_voff[j] = (r == 1 ? (j + 4 < LA ? a_off[j + 4 < LA ? j + 4 : 0] : kMasked) : a_off[j]) + abase;
        }
        auto mid = [&](auto k_tag) {
            constexpr int K = decltype(k_tag)::value;
            if constexpr (K % 4 == 1 && (K - 1) / 4 < LB) {
                constexpr int J = (K - 1) / 4;
                if (m & (1u << K))
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(J == LB - 1 ? rs_blast : rs_w, (__attribute__((address_space(3))) void *)(b_dst + J * NW * 1024), 16, b_off[J], b_soff, 0, 0);
            } else if constexpr (K % 2 == 0 && K >= 2 && K <= 8) {
                constexpr int J = (K - 2) / 2;
                if (m & (1u << K))
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (__attribute__((address_space(3))) void *)(a_dst + J * NW * 1024), 16, a_voff[J], a_soff, 0, 0);
            }
        };
        ABED_TS();
        // (3) batch checksum (Sec. 3.2 option 1): this thread's 16 bytes of every staged entry are added up in the
        // load slots that sub-steps r == 1 and r == 2 leave free (one entry per slot, requested one slot ahead), so
        // the additions hide behind the matrix instructions.  xt_*: the step's sums, folded into the chunk's
        // registers at the end of r == 2.
        // the piece this sub-step adds, and whether this thread has it
        const int x_pc = EH == 1 ? r - 1 : 0;
        const bool x_on = IC && (EH == 1 ? (r >= 1 && tid + 256 * x_pc < kSlots * 4) : tid < kSlots * 4);
        const int8_t *x_src = lds + A_OFF + abuf * kAStage + x_piece + (EH == 1 ? x_pc * 4096 : 0);
        auto x_add = [&](const i32x4 v) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const unsigned u = (unsigned)v[d] ^ 0x80808080u;
                xt_lo[d] += u & 0x00ff00ffu;
                xt_hi[d] += (u >> 8) & 0x00ff00ffu;
            }
        };
        auto mid_all = [&](auto k_tag) {
            constexpr int K = decltype(k_tag)::value;
            mid(k_tag);
            if constexpr (IC && !digit) {
                // slots 0, 3, 7, 10 of r == 1 take entries 0..3, the same slots of r == 2 entries 4..7 (EH = 1: the
                // four entries of the second piece)
                constexpr int Q = K == 0 ? 0 : K == 3 ? 1 : K == 7 ? 2 : K == 10 ? 3 : -1;
                if constexpr (Q >= 0) {
                    if (r >= 1 && x_on) {
                        const int e = EH == 1 ? Q : (r - 1) * 4 + Q;
                        x_add(x_next);                          // entry e, requested one slot earlier
                        if (e + 1 < kEB) x_next = *reinterpret_cast<const i32x4 *>(x_src + (e + 1) * kAEntry);
                    }
                }
            }
        };
        if constexpr (IC && !digit) {
            if ((r == 1 || (EH == 1 && r == 2)) && x_on) {
#pragma unroll
                for (int d = 0; d < 4; ++d) xt_lo[d] = xt_hi[d] = 0u;
                x_next = *reinterpret_cast<const i32x4 *>(x_src);
            }
        }
        // (4) multiply; in the digit batch entries 0 and 1 of the stage are the two digit images: the even waves
        // take digit 0, the odd waves digit 1 of their pixel group
        ABED_TS();
#ifdef ABED_ENABLE_DBG
        if (!(p.dbg & 2)) {
#endif
        if constexpr (digit) mfma_row(std::integral_constant<int, 3 - EH>{}, abuf, bslot, r, EH == 1 ? 0 : eh, mid_all);
        else mfma_row(std::integral_constant<int, 4>{}, abuf, bslot, r, eh * 4, mid_all);
#ifdef ABED_ENABLE_DBG
        }
#endif
        ABED_TS();
        vm_prev = __builtin_popcount(m); st_prev = 0;   // (sub-steps that skip the wait issue their loads before r == 2, whose own count is then 0)
        if (++pf_r == 3) { pf_r = 0; if (++pf_chunk == p.nch) pf_chunk = 0; }
        if (++bslot == NBR) bslot = 0;
        ++usub;

        if constexpr (IC) {
            if constexpr (!digit) {
                // fold the sub-step's sums into the chunk's registers (EH = 2: after r == 2; EH = 1: a piece per sub-step)
                if ((r == 2 || (EH == 1 && r == 1)) && x_on) {
                    static_for<0, XR>([&](auto c_tag) {
                        constexpr int CT = decltype(c_tag)::value;
                        static_for<0, NP>([&](auto q_tag) {
                            constexpr int QT = decltype(q_tag)::value;
                            if (chunk == CT && x_pc == QT) {
#pragma unroll
                                for (int d = 0; d < 4; ++d) { xs_lo[CT][QT][d] += xt_lo[d]; xs_hi[CT][QT][d] += xt_hi[d]; }
                            }
                        });
                    });
                }
            }
            // the next step is a digit step: its chunk's sums are complete; split them into two int8 digit
            // images (Sec. 4.1) and put them into the free A buffer as entries 0 and 1
            if (r == 2 && stepi + 1 >= nsteps_real && stepi + 1 < nsteps) {
                const int cn = (chunk + 1 == p.nch) ? 0 : chunk + 1;     // chunk of step stepi + 1
                static_for<0, NP>([&](auto q_tag) {
                    constexpr int QT = decltype(q_tag)::value;
                    if (tid + 256 * QT < kSlots * 4) {
                        unsigned lo[4], hi[4];
                        static_for<0, XR>([&](auto c_tag) {
                            constexpr int CT = decltype(c_tag)::value;
                            if (cn == CT) {
#pragma unroll
                                for (int d = 0; d < 4; ++d) { lo[d] = xs_lo[CT][QT][d]; hi[d] = xs_hi[CT][QT][d]; }
                            }
                        });
                        const int bias = 128 * nbatch * kEB;     // every staged entry added 128 per byte (zero-filled ones too)
                        i32x4 d0, d1;
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            int s0 = (int)(lo[d] & 0xffffu) - bias, s1 = (int)(hi[d] & 0xffffu) - bias;
                            int s2 = (int)(lo[d] >> 16) - bias, s3 = (int)(hi[d] >> 16) - bias;
                            const unsigned dl = ((unsigned)next_digit(s0) & 0xffu) | (((unsigned)next_digit(s1) & 0xffu) << 8) |
                                                (((unsigned)next_digit(s2) & 0xffu) << 16) | (((unsigned)next_digit(s3) & 0xffu) << 24);
                            const unsigned dh = ((unsigned)s0 & 0xffu) | (((unsigned)s1 & 0xffu) << 8) | (((unsigned)s2 & 0xffu) << 16) | (((unsigned)s3 & 0xffu) << 24);
                            d0[d] = (int)dl; d1[d] = (int)dh;
                        }
                        int8_t *dst = lds + A_OFF + (abuf ^ 1) * kAStage + x_piece + QT * 4096;
                        *reinterpret_cast<i32x4 *>(dst) = d0;
                        *reinterpret_cast<i32x4 *>(dst + kAEntry) = d1;
                    }
                });
            }
        }
        // (5) end of a step / of a batch
        if (++r < 3) return;
        r = 0; ++stepi;
        if (++chunk < p.nch) return;
        chunk = 0;
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
                    const unsigned res = fc_residual(i);
                    if (res != 0 && e < n_end) my_flag |= 1u;
                }
                if (IC) {
#pragma unroll
                    for (int fb = 0; fb < FB; ++fb) icsum[fb] += acc[i][fb];   // entries past the range are all zero
                }
                // stores: checksum columns are trimmed (end of Sec. 4.3); masked lanes go out of the descriptor's range
#ifdef ABED_ENABLE_DBG
                const bool live = pvalid && e < n_end && !(p.dbg & 4);
#else
                const bool live = pvalid && e < n_end;
#endif
                if (!p.out_int8) {
                    const int o = live ? ((e * PQ + pix) * p.K + kt * FBR * 16 + lg * 4) * 4 : OOB;
#pragma unroll
                    for (int fb = 0; fb < FBR; ++fb)
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[i][fb]), rs_y, o, fb * 64, 0);
                } else {
                    const int o = live ? (e * PQ + pix) * p.K + kt * FBR * 16 + lg * 4 : OOB;
#pragma unroll
                    for (int fb = 0; fb < FBR; ++fb) {
                        const int k = fb * 16 + lg * 4;
                        const int a4[4] = {acc[i][fb][0], acc[i][fb][1], acc[i][fb][2], acc[i][fb][3]};
                        const float s4[4] = {e_scale[k], e_scale[k + 1], e_scale[k + 2], e_scale[k + 3]}, b4[4] = {e_bias[k], e_bias[k + 1], e_bias[k + 2], e_bias[k + 3]};
                        __builtin_amdgcn_raw_buffer_store_b32(requant_pack4(a4, s4, b4, p.relu), rs_y, o, fb * 16, 0);
                    }
                }
            }
            st_prev = 4 * FBR;
        }
        ++batch;
        if (usub < nsub) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) acc[i][fb] = zero4;
        }
    };
    const int nsub_real = nsteps_real * 3;
#pragma unroll 1
    while (usub < nsub_real) substep(std::false_type{});
    if constexpr (IC) {
#pragma unroll 1
        while (usub < nsub) substep(std::true_type{});
    }

    // ---- final comparisons
    if constexpr (IC) {
        int *red = reinterpret_cast<int *>(lds);              // [4 pixel groups][FB][64 lanes][4]: the odd waves' sums
        ABED_WAIT_VMCNT(0);
        __syncthreads();                                      // all fragment reads are done; LDS is free
        // a lane of the digit block counts only if it holds the digit filters' columns (with the short digit block
        // the other lanes multiplied bytes that are not filters)
        auto counts = [&](int fb) { return !(SHORT_DIGIT && fb == FB - 1 && lg != 0); };
        if constexpr (EH == 2) {
            // the digit batch left, in acc[0], the fmaps of digit image 0 (even waves) / digit image 1 (odd waves)
            if (FC) {
                if (fc_residual(0) != 0) my_flag |= 4u;           // corner: a digit image's row under FC
            }
            if (eh == 1) {
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) {
                    i32x4 c = icsum[fb];
#pragma unroll
                    for (int v = 0; v < 4; ++v) c[v] -= (int)((unsigned)acc[0][fb][v] << 8);
                    *reinterpret_cast<i32x4 *>(red + ((pg * FB + fb) * 64 + lane) * 4) = c;
                }
            }
            __syncthreads();
            if (eh == 0) {
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) {
                    const i32x4 c = icsum[fb] + *reinterpret_cast<const i32x4 *>(red + ((pg * FB + fb) * 64 + lane) * 4) - acc[0][fb];
                    if ((c[0] | c[1] | c[2] | c[3]) != 0 && counts(fb)) my_flag |= (FC && fb == FB - 1) ? 4u : 2u;
                }
            }
        } else {
            // one wave per pixel group: the digit batch left the fmaps of digit image 0 in acc[0], of digit image 1 in acc[1]
            if (FC) {
                if (fc_residual(0) != 0 || fc_residual(1) != 0) my_flag |= 4u;
            }
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) {
                i32x4 c = icsum[fb] - acc[0][fb];
#pragma unroll
                for (int v = 0; v < 4; ++v) c[v] -= (int)((unsigned)acc[1][fb][v] << 8);
                if ((c[0] | c[1] | c[2] | c[3]) != 0 && counts(fb)) my_flag |= (FC && fb == FB - 1) ? 4u : 2u;
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
            for (int w8 = 0; w8 < NW; ++w8) f |= (uint32_t)misc[w8];
            p.flags[(box * p.nranges + range) * p.grid_n + kt] = f;
        }
    }
#endif
}

}  // namespace abed
