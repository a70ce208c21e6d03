// 3x3, stride-1 int8 convolution (Sec. 2.2 of the paper) for gfx950, unchecked, with one wave per SIMD and the
// 32x32x32 matrix instruction: an alternative main loop to conv_box_kernel.h, built to find out what a loop that
// keeps the matrix pipe busy between barriers is worth on this part.  Opt-in (ABED_IMG=1); int32 ConvOut only.
//
// Work split.  A workgroup (256 threads, 4 waves, one per SIMD and per CU: up to 512 registers a lane) owns
//   - a region of RH x RW output positions of the image plane, flattened row by row into NB = 4 / IW blocks of
//     32 positions (the last block may be partly empty),
//   - a group of images, walked in batches of EB = 4 IW,
//   - a tile of 64 filters.
// Wave w takes IW images of the batch at once and all NB blocks of the region: 4 slots of 32 positions x 2 blocks
// of 32 filters = 8 accumulator tiles (v_mfma_i32_32x32x32_i8, filters = A operand, so a lane holds one position
// and 16 filters per tile and stores 16 contiguous bytes of NPQK int32 per register quad).
//
// Reuse of the input.  For a chunk of 64 channels the (RH + 2) x (RW + 2) input positions under the region are
// staged once per image and all nine taps read them from there; a sub-step is one filter row (3 taps x 64
// channels = 6 steps of 32 along the reduction axis, 48 matrix instructions a wave).
//
// Pipeline.  Filters: a ring of four sub-stages, requested three sub-steps ahead.  Activations: two stages,
// the next step's requested during filter row 0.  One barrier per sub-step, placed behind the first two matrix
// instructions of the sub-step; the first fragments of sub-step u + 1 are read at the end of sub-step u (the
// barrier of sub-step u has already shown that they landed; for a new activation stage a second barrier in the
// middle of filter row 2 does), so no wave waits for LDS behind a barrier.  Every matrix instruction is followed
// by at most one fragment read or a few loads / stores (sched_barrier fences keep that order).  Two accumulator
// sets: a batch's outputs are stored from the idle set during the next batch's first chunk.
// Vector-memory instructions complete in issue order and every sub-step issues a fixed number of them (loads
// that have nothing to fetch are issued masked), so the s_waitcnt immediates are compile-time counts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include "conv_box_kernel.h"

namespace abed {

typedef int i32x16 __attribute__((ext_vector_type(16)));

struct ImgParams {
    const int8_t *x, *w;
    void *y;                     // int32 [N][P][Q][K], or int8 after the epilog
    const float *scale, *bias;   // epilog (Sec. 4.3): K floats each, or null (OUT8 = false)
    int relu;
    int N, H, W, C, K, P, Q, ph, pw;
    int RW, RH, rx, ry;          // region size (output positions), regions per row / column of the image plane
    int PW;                      // pitch of the position numbering inside a region (>= RW; lanes with column >= RW idle)
    int swz;                     // LDS swizzle constant c: channel group g of input position (hy, hx) sits in part g ^ ((hx >> 1) + c hy)
    int nch, nft;                // C / 64, K / 64
    int ngroups, group_len;      // image groups; group_len is a multiple of the batch size
    // builds with ABED_ENABLE_DBG only.  dbg_clk: workgroup 0 leaves the main loop's length in shader-clock ticks and in
    // ticks of the 100 MHz real-time counter there (their ratio is the shader clock under this kernel's load);
    // dbg bit 0: the loop's activation loads fetch nothing, bit 1: its filter loads (timing experiments, wrong outputs)
    long long *dbg_clk;
    int dbg;
};

constexpr int kImgPlane = 832;                   // 64-byte slots (images of a batch x input positions of a region) of an activation stage at most
constexpr int kImgAStage = kImgPlane * 64;       // 53248 bytes
constexpr int kImgA1 = 65536;                    // where the second activation stage starts
constexpr int kImgBSub = 64 * 192;               // one filter sub-stage: 64 filters x 3 taps x 64 channels
constexpr int kImgLds = 118784 + 3 * kImgBSub + 1024;
constexpr int kImgOOB = 0x7ffffff0;

// IW: images a wave holds at once; OUT8: the epilog of Sec. 4.3 is applied and int8 is stored
template <int IW, bool OUT8>
__global__ __launch_bounds__(256, 1) void img_conv_kernel(const ImgParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int MB = 4, MA = 2, NB = MB / IW, EB = 4 * IW, LA = 13, LB = 3;
    __shared__ __attribute__((aligned(1024))) int8_t lds[kImgLds];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lh = lane >> 5, lj = lane & 31;

    const int nreg = p.rx * p.ry;
    const int ntiles = nreg * p.ngroups * p.nft;
    const int per_xcd = (ntiles + 7) >> 3;
    int bid = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (bid >= ntiles) return;
    const int ft = bid % p.nft; bid /= p.nft;
    const int group = bid % p.ngroups;
    const int region = bid / p.ngroups;
    const int ryi = region / p.rx, rxi = region - ryi * p.rx;
    const int y0 = ryi * p.RH, x0 = rxi * p.RW;
    const int rh = min(p.RH, p.P - y0), rw = min(p.RW, p.Q - x0);
    const int HP = p.RW + 2;
    const int slots = (p.RH + 2) * HP;
    const int n0 = group * p.group_len;
    const int n_end = min(p.N, n0 + p.group_len);
    const int nbatch = (n_end - n0 + EB - 1) / EB;
    const int HWC = p.H * p.W * p.C;
    constexpr int OB = OUT8 ? 1 : 4;                 // bytes of an output element
    const int PQK4 = p.P * p.Q * p.K * OB;           // bytes of one image's output
    const int crsb = 9 * p.C;

    constexpr int kMasked = 0x40000000;
    const __amdgpu_buffer_rsrc_t rs_x = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, n_end * HWC, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_w = __builtin_amdgcn_make_buffer_rsrc((void *)p.w, 0, p.K * crsb, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.N * PQK4, 0x00020000);

    // ---- filter sub-stage: piece q = f * 12 + sx * 4 + part'; fetched group = part' ^ ((f >> 1) & 3)
    int b_off[LB];
#pragma unroll
    for (int jj = 0; jj < LB; ++jj) {
        const int q = (jj * 4 + wave) * 64 + lane;
        const int f = (q * 0x5556) >> 18 /* q / 12 for q < 768 */, rem = q - f * 12;
        const int sx = rem >> 2, part = rem & 3;
        b_off[jj] = (ft * 64 + f) * crsb + sx * p.C + ((part ^ ((f >> 1) & 3)) << 4);
    }
    // ---- activation stage: piece q = (e * slots + slot) * 4 + part'; the channel group fetched into part' is part' ^ (((hx >> 1) + c hy) & 3)
    // (small non-negative integers divided in floating point: exact, the quotient's distance to an integer is at least 1/(2d))
    const float r_slots = 1.0f / (float)slots, r_hp = 1.0f / (float)HP, r_pw = 1.0f / (float)p.PW;
    auto fdiv = [](int a, float rd) { return (int)(((float)a + 0.5f) * rd); };
    int a_off[LA];
#pragma unroll
    for (int jj = 0; jj < LA; ++jj) {
        const int q = (jj * 4 + wave) * 64 + lane;
        const int idx = q >> 2, part = q & 3;
        const int e = fdiv(idx, r_slots), slot = idx - e * slots;
        const int hy = fdiv(slot, r_hp), hx = slot - hy * HP;
        const int iy = y0 - p.ph + hy, ix = x0 - p.pw + hx;
        a_off[jj] = kMasked;
        if (e < EB && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W)
            a_off[jj] = ((e * p.H + iy) * p.W + ix) * p.C + ((part ^ (((hx >> 1) + p.swz * hy) & 3)) << 4);
    }
    auto b_slot_off = [](int s) { return s == 0 ? kImgAStage : 118784 + (s - 1) * kImgBSub; };

    i32x16 acc[2][MB][MA];
    i32x4 fa[2][MA], fb[2][MB];
    // the epilog's scale and bias of this tile's 64 filters (the prologue's barrier publishes them)
    float *e_scale = reinterpret_cast<float *>(lds + kImgLds - 1024), *e_bias = e_scale + 64;
    if constexpr (OUT8) {
        if (tid < 128) e_scale[tid] = (tid < 64 ? p.scale : p.bias)[ft * 64 + (tid & 63)];
    }
    int st_off[MB];     // previous batch's output offsets (its stores are issued during this batch)
#pragma unroll
    for (int m = 0; m < MB; ++m) st_off[m] = kImgOOB;
    // store number q (0..31) of accumulator set PAR: slot m = q / 8, filter block a = (q / 4) & 1, register group g = q & 3:
    // this lane's filters a * 32 + 8 g + 4 h .. + 3 of its position: 16 bytes of int32, or 4 bytes after the epilog
    auto store_item = [&](auto par_tag, auto q_tag) {
        constexpr int PAR = decltype(par_tag)::value, Q = decltype(q_tag)::value;
        constexpr int SM = Q / 8, SA = (Q / 4) & 1, SG = Q & 3;
        if constexpr (!OUT8) {
            const u32x4 v = {(unsigned)acc[PAR][SM][SA][4 * SG], (unsigned)acc[PAR][SM][SA][4 * SG + 1], (unsigned)acc[PAR][SM][SA][4 * SG + 2], (unsigned)acc[PAR][SM][SA][4 * SG + 3]};
            __builtin_amdgcn_raw_buffer_store_b128(v, rs_y, st_off[SM], SA * 128 + SG * 32, 0);
        } else {
            const int k = SA * 32 + SG * 8 + lh * 4;
            const f32x4 s4 = *reinterpret_cast<const f32x4 *>(e_scale + k), b4 = *reinterpret_cast<const f32x4 *>(e_bias + k);
            const int a4[4] = {acc[PAR][SM][SA][4 * SG], acc[PAR][SM][SA][4 * SG + 1], acc[PAR][SM][SA][4 * SG + 2], acc[PAR][SM][SA][4 * SG + 3]};
            const float sc[4] = {s4[0], s4[1], s4[2], s4[3]}, bi[4] = {b4[0], b4[1], b4[2], b4[3]};
            __builtin_amdgcn_raw_buffer_store_b32(requant_pack4(a4, sc, bi, p.relu), rs_y, st_off[SM], SA * 32 + SG * 8, 0);
        }
    };

    const int nsteps = nbatch * p.nch;
    const int nsub = nsteps * 3;


    int pf_r = 0, pf_chunk = 1 % p.nch;       // (row, chunk) of sub-step u + 3
    int u = 0, step = 0, chunk = 0, batch = 0;

    auto dma_b = [&](auto jt, int slot, int soff) {
        constexpr int JJ = decltype(jt)::value;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_w, (__attribute__((address_space(3))) void *)(lds + b_slot_off(slot) + (JJ * 4 + wave) * 1024), 16, b_off[JJ], soff, 0, 0);
    };
    auto dma_a = [&](auto jt, int buf, int voff_base, int soff) {
        constexpr int JJ = decltype(jt)::value;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_x, (__attribute__((address_space(3))) void *)(lds + buf * kImgA1 + (JJ * 4 + wave) * 1024), 16, a_off[JJ] + voff_base, soff, 0, 0);
    };

    // prologue: activations of step 0, filters of sub-steps 0..2
    static_for<0, LA>([&](auto jt) { dma_a(jt, 0, n0 * HWC, 0); });
    static_for<0, LB>([&](auto jt) { dma_b(jt, 0, 0); });
    static_for<0, LB>([&](auto jt) { dma_b(jt, 1, nsub > 1 ? 3 * p.C : kMasked); });
    static_for<0, LB>([&](auto jt) { dma_b(jt, 2, nsub > 2 ? 6 * p.C : kMasked); });
    // ---- fragment addresses (k32-step t = 0; t = 1 is the same address with bit 5 flipped)
    const int zf = (lj >> 1) & 3;
    const int bfr0 = lj * 192 + (((lh ^ (zf & 1)) | (zf & 2)) << 4);
    int afr[MB][3][3], out_off[MB];      // [slot][tap column][filter row]
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const int iw = m / NB, b = m % NB;
        const int e = wave * IW + iw;
        const int pos = b * 32 + lj;
        int yy = fdiv(pos, r_pw), xx = pos - yy * p.PW;
        const bool valid = yy < rh && xx < rw;
        // idle lanes read what a neighbour reads (the same address is served once): nothing of theirs is stored
        yy = min(yy, rh - 1); xx = min(xx, rw - 1);
#pragma unroll
        for (int sx = 0; sx < 3; ++sx)
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const int hx = xx + sx, hy = yy + r, z = ((hx >> 1) + p.swz * hy) & 3;
                afr[m][sx][r] = (e * slots + hy * HP + hx) * 64 + (((lh ^ (z & 1)) | (z & 2)) << 4);
            }
        out_off[m] = valid ? (((e * p.P + y0 + yy) * p.Q + x0 + xx) * p.K + ft * 64 + lh * 4) * OB : kImgOOB;
    }

    ABED_WAIT_VMCNT(0);
    __builtin_amdgcn_s_waitcnt(0xc07f);          // this wave's LDS writes (scale and bias) are done: lgkmcnt(0)
    __builtin_amdgcn_s_barrier();

    // one fragment read; order 0..5: fa0, fb0, fa1, fb1, fb2, fb3 (the order the matrix instructions need them)
    auto fetch_one = [&](auto it, int set, int bbase, int abase, auto r_tag, int sx, int t) {
        constexpr int I = decltype(it)::value, FR = decltype(r_tag)::value;
        if constexpr (I == 0) fa[set][0] = *reinterpret_cast<const i32x4 *>(lds + ((bfr0 + bbase + sx * 64) ^ (t * 32)));
        else if constexpr (I == 2) fa[set][1] = *reinterpret_cast<const i32x4 *>(lds + ((bfr0 + bbase + sx * 64) ^ (t * 32)) + 32 * 192);
        else {
            constexpr int M = I == 1 ? 0 : I - 2;
            fb[set][M] = *reinterpret_cast<const i32x4 *>(lds + ((afr[M][sx][FR] + abase) ^ (t * 32)));
        }
    };
    static_for<0, 6>([&](auto it) { fetch_one(it, 0, b_slot_off(0), 0, std::integral_constant<int, 0>{}, 0, 0); });

    int prev_all = 0, prev_after = 0, prev2_after = 0;   // vector-memory operations issued in sub-step u - 1 (all; after its last filter load) and in sub-step u - 2 after its last filter load

    auto wait_upto = [&](int n) {
        if (n >= 35) ABED_WAIT_VMCNT(35); else if (n >= 32) ABED_WAIT_VMCNT(32); else if (n >= 24) ABED_WAIT_VMCNT(24); else if (n >= 23) ABED_WAIT_VMCNT(23);
        else if (n >= 20) ABED_WAIT_VMCNT(20); else if (n >= 16) ABED_WAIT_VMCNT(16);
        else if (n >= 12) ABED_WAIT_VMCNT(12); else if (n >= 3) ABED_WAIT_VMCNT(3); else ABED_WAIT_VMCNT(0);
    };

    // R: filter row; PAR: accumulator set; FIRSTK: first sub-step of a batch; ST: this chunk carries the previous batch's stores
    auto substep = [&](auto r_tag, auto par_tag, auto first_tag, auto st_tag) {
        constexpr int R = decltype(r_tag)::value, PAR = decltype(par_tag)::value;
        constexpr bool FIRSTK = decltype(first_tag)::value, ST = decltype(st_tag)::value;
        // addresses of this sub-step's refill loads and of the next sub-step's first fragments (scalar work; it runs while the
        // first matrix instructions execute)
        const int bslot_new = (u + 3) & 3;
#ifdef ABED_ENABLE_DBG
        const int b_soff = (u + 3 < nsub && !(p.dbg & 2)) ? pf_r * 3 * p.C + pf_chunk * 64 : kMasked;
#else
        const int b_soff = (u + 3 < nsub) ? pf_r * 3 * p.C + pf_chunk * 64 : kMasked;
#endif
#ifdef ABED_ENABLE_DBG
        const bool more_a = step + 1 < nsteps && !(p.dbg & 1);
#else
        const bool more_a = step + 1 < nsteps;
#endif
        const int nc = chunk + 1 == p.nch ? 0 : chunk + 1;
        const int a_vbase = more_a ? (n0 + (nc == 0 ? batch + 1 : batch) * EB) * HWC : kMasked;
        const int a_soff = nc * 64;
        const int a_buf = (step + 1) & 1;
        const int cur_b = b_slot_off(u & 3), nxt_b = b_slot_off((u + 1) & 3);
        const int cur_a = (step & 1) * kImgA1;
        const int nxt_a = R == 2 ? ((step + 1) & 1) * kImgA1 : cur_a;
        const int wait_n = prev2_after + prev_all;
        // (3) multiply: 6 k32-steps of 8 matrix instructions; behind instruction i < 6 of a k32-step comes one fragment read of the
        // next k32-step, behind instructions 6 and 7 the refill loads and the stores
        static_for<0, 6>([&](auto kt) {
            constexpr int KS = decltype(kt)::value;
            constexpr int cur = KS & 1;
            if constexpr (R == 2 && KS == 3) {
                // the next step's activations (last load: R == 1, k32-step 3) have landed for everybody before anyone reads them
                // (vector-memory operations issued since the last activation load, R == 0, k32-step 5)
                if constexpr (ST && OUT8) ABED_WAIT_VMCNT(25); else if constexpr (ST) ABED_WAIT_VMCNT(26); else ABED_WAIT_VMCNT(6);
                __builtin_amdgcn_s_barrier();
            }
            static_for<0, 8>([&](auto it) {
                constexpr int I = decltype(it)::value;
                constexpr int M = I >> 1, A = I & 1;
                if constexpr (FIRSTK && KS == 0) {
                    const i32x16 z = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                    acc[PAR][M][A] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[cur][A], fb[cur][M], z, 0, 0, 0);
                } else {
                    acc[PAR][M][A] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[cur][A], fb[cur][M], acc[PAR][M][A], 0, 0, 0);
                }
                if constexpr (I < 6) {
                    if constexpr (KS < 5) fetch_one(it, cur ^ 1, cur_b, cur_a, r_tag, (KS + 1) >> 1, (KS + 1) & 1);
                    else fetch_one(it, cur ^ 1, nxt_b, nxt_a, std::integral_constant<int, (R + 1) % 3>{}, 0, 0);
                    if constexpr (KS == 0 && I == 1) {
                        // the filters of sub-step u + 1 have landed (issued in sub-step u - 2), and everybody is done with sub-step
                        // u - 1: its filter slot and, at R == 0, the activation buffer of the step before can be refilled
                        wait_upto(wait_n);
                        __builtin_amdgcn_s_barrier();
                    }
                }
                if constexpr (I >= 6) {
                    constexpr int SL = I & 1;
                    // filters of sub-step u + 3: k32-steps 0..2, first side slot
                    if constexpr (SL == 0 && KS < 3) dma_b(std::integral_constant<int, KS>{}, bslot_new, b_soff);
                    // activations of the next step, all in R == 0: second side slot of every k32-step (loads 0..5, and 9..12 behind
                    // them in k32-steps 0..3), first side slot of k32-steps 3..5 (loads 6..8)
                    if constexpr (R == 0 && SL == 1) dma_a(std::integral_constant<int, KS>{}, a_buf, a_vbase, a_soff);
                    if constexpr (R == 0 && SL == 1 && KS < 4) dma_a(std::integral_constant<int, (KS < 4 ? 9 + KS : 0)>{}, a_buf, a_vbase, a_soff);
                    if constexpr (R == 0 && SL == 0 && KS >= 3) dma_a(std::integral_constant<int, (KS >= 3 ? 3 + KS : 0)>{}, a_buf, a_vbase, a_soff);
                    // stores of the previous batch.  int32: R == 1: k32-steps 4, 5 (stores 0..7); R == 2: every k32-step (stores 8..31),
                    // two per side slot.  int8 (each store comes with its epilog arithmetic): one per side slot, from the
                    // fifth side slot of R == 0 to the tenth of R == 2
                    if constexpr (ST && !OUT8 && ((R == 1 && KS >= 4) || R == 2)) {
                        static_for<0, 2>([&](auto qt) {
                            constexpr int Q = R == 1 ? (KS - 4) * 4 + SL * 2 + decltype(qt)::value : 8 + KS * 4 + SL * 2 + decltype(qt)::value;
                            store_item(std::integral_constant<int, PAR ^ 1>{}, std::integral_constant<int, Q>{});
                        });
                    }
                    if constexpr (ST && OUT8) {
                        constexpr int Q = R * 12 + KS * 2 + SL - 4;
                        if constexpr (Q >= 0 && Q < 32) store_item(std::integral_constant<int, PAR ^ 1>{}, std::integral_constant<int, Q>{});
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        });
        // vector-memory operations of this sub-step: in all / after its last filter load
        prev2_after = prev_after;
        if constexpr (ST && OUT8) {
            prev_all = R == 0 ? 24 : 15;
            prev_after = R == 0 ? 17 : 8;
        } else {
            prev_all = R == 0 ? 16 : R == 1 ? (ST ? 11 : 3) : (ST ? 27 : 3);
            prev_after = R == 0 ? 9 : R == 1 ? (ST ? 8 : 0) : (ST ? 16 : 0);
        }
        ++u;
        if (++pf_r == 3) { pf_r = 0; if (++pf_chunk == p.nch) pf_chunk = 0; }
        if (R == 2) { ++step; if (++chunk == p.nch) chunk = 0; }
    };

    using I0 = std::integral_constant<int, 0>; using I1 = std::integral_constant<int, 1>; using I2 = std::integral_constant<int, 2>;
    using T = std::true_type; using F = std::false_type;
    auto one_batch = [&](auto par_tag) {
        substep(I0{}, par_tag, T{}, T{});
        substep(I1{}, par_tag, F{}, T{});
        substep(I2{}, par_tag, F{}, T{});
#pragma unroll 1
        for (int c = 1; c < p.nch; ++c) {
            substep(I0{}, par_tag, F{}, F{});
            substep(I1{}, par_tag, F{}, F{});
            substep(I2{}, par_tag, F{}, F{});
        }
        // this batch's outputs: stored during the next batch (or after the loop)
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            const int e = n0 + batch * EB + wave * IW + m / NB;
            st_off[m] = (e < n_end && out_off[m] != kImgOOB) ? out_off[m] + (n0 + batch * EB) * PQK4 : kImgOOB;
        }
        ++batch;
    };
#ifdef ABED_ENABLE_DBG
    const long long ck0 = (long long)__builtin_amdgcn_s_memtime(), rt0 = (long long)__builtin_amdgcn_s_memrealtime();
#endif
#pragma unroll 1
    for (int b2 = 0; b2 < nbatch; b2 += 2) {
        one_batch(I0{});
        if (b2 + 1 < nbatch) one_batch(I1{});
    }
#ifdef ABED_ENABLE_DBG
    if (p.dbg_clk && blockIdx.x == 0 && tid == 0) {
        p.dbg_clk[0] = (long long)__builtin_amdgcn_s_memtime() - ck0;
        p.dbg_clk[1] = (long long)__builtin_amdgcn_s_memrealtime() - rt0;
    }
#endif
    // stores of the last batch
    auto store_all = [&](auto par_tag) {
        static_for<0, 32>([&](auto q_tag) { store_item(par_tag, q_tag); });
    };
    if (((nbatch - 1) & 1) == 0) store_all(I0{}); else store_all(I1{});
#endif
}

}  // namespace abed
