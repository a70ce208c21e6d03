// Host side of libabed: argument checks, tile plan, workspace carving and kernel
// launches for the variants of Sec. 4.3.  See include/abed.h for the contract.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <mutex>

#include "../../include/abed.h"
#include "aux_kernels.h"
#include "fic_kernels.h"
#include "ic2_kernels.h"
#include "abft_gemm_kernels.h"
#include "conv_launch.h"
#include "conv_box_launch.h"
#include "conv_img_kernel.h"
#include "conv_img_launch.h"

using namespace abed;

// Scratch of the entry point that allocates nothing (abed_conv_int8_static): one array per GPU, held
// until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the device
// address it yields (kept per device in g_scratch_ptr) is what kernels and fills get.
static __device__ __align__(256) unsigned char scratch[ABED_STATIC_SCRATCH_BYTES];

namespace {

const int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];       // device address of `scratch` on each GPU, or null until first use there
std::mutex g_scratch_mutex;

thread_local char g_hip_error[256] = "";

abed_status_t hip_fail(hipError_t e, const char *what)
{
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
    return ABED_EHIP;
}

#define HIP_TRY(expr)                                            \
    do {                                                         \
        hipError_t e_ = (expr);                                  \
        if (e_ != hipSuccess) return hip_fail(e_, #expr);        \
    } while (0)

#define LAUNCH_CHECK(name)                                       \
    do {                                                         \
        hipError_t e_ = hipGetLastError();                       \
        if (e_ != hipSuccess) return hip_fail(e_, name);         \
    } while (0)

int digits_for_count(long long count)
{
    // a sum of `count` int8 values lies in [-128 count, 127 count]; d balanced base-256
    // digits cover [-128 (256^d - 1)/255, 127 (256^d - 1)/255]  (Sec. 4.1)
    int d = 1;
    long long reach = 1;   // (256^d - 1) / 255
    while (count > reach) { reach = reach * 256 + 1; ++d; }
    return d;
}

struct Plan {
    int P, Q, PQ, crs;
    int esize;                            // bytes per element: 1 (int8) or 2 (fp16)
    int d_f, d_i;
    int n_entries, kblk, n_fblk;          // batch entries, real filter blocks, filter blocks incl. the digit block
    int wm, wk, mb;                       // entries per wave, filter blocks per tile, entries per tile
    int kg;                               // groups of 4 waves along the reduction axis
    int variant;                          // the variant without the scheme selection bits
    int l1;                               // fp16: threshold relative to the sum of magnitudes
    int packed;                           // digit filters in the free rows of the last real filter block
    int grid_m, grid_b, grid_n;
    // workspace offsets in bytes (-1 = unused)
    long long off_cnt_fc, off_cnt_ic, off_convout, off_yf, off_yi, off_yfi, off_fc, off_ic, off_nx, ws_bytes;
};

long long align256(long long v) { return (v + 255) & ~255LL; }

int env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

// Tile shape: WK filter blocks x 4*WM batch entries x 16 pixels per workgroup.  The layers this
// library targets are small next to 256 compute units, so tiles are kept small (measured on
// ResNet-50-shaped layers: 64 filters x 8..12 entries was best or within a few percent of it):
// more workgroups in flight hide memory latency better than larger tiles save traffic.
// Tile shape from the problem's extents.  The rules come from timing sweeps over the ResNet-style
// layers: the kernel is bound by how fast a CU can fill LDS, so bigger tiles (more matrix
// instructions per byte loaded) win as long as the grid still gives every CU work; below that,
// smaller tiles and wave groups along the reduction axis keep the chip busy.
void choose_tile(Plan &pl)
{
    int wk;
    if (pl.n_fblk <= 1) wk = 1;
    else {
        const int pad4 = (pl.n_fblk + 3) / 4 * 4, pad5 = (pl.n_fblk + 4) / 5 * 5;
        // 5 where it pads less: 64 filters + the digit block in one tile (FC stays local); on grids of 256 tiles or
        // more also where it saves a single block, 33 blocks in 7 tiles instead of 9 (512 filters + the digit block
        // at N = 128: the same or up to 15 % faster on every such layer; at N = 32 the 4-wide plan is 3 % faster)
        const long long tiles5 = (long long)((pl.PQ + 15) / 16) * ((pl.n_entries + 7) / 8) * (pad5 / 5);
        wk = (pad5 + 2 <= pad4 || pl.n_fblk == 5 || (pad5 < pad4 && tiles5 >= 256)) ? 5 : 4;
    }
    // tiles 8 blocks wide and 8 entries deep read the activations half as often; they pay when the filter
    // blocks fill them exactly and the grid stays large (measured: 64->256 1x1 at 56x56, 256->256 3x3 at
    // 14x14 with 128 images), and lose on small grids; with a long reduction axis one workgroup per CU is
    // enough (512 -> 512 3x3 at 7x7 with 128 images: 39 -> 31 us)
    bool wide = false;
    {
        const long long tiles8 = (long long)((pl.PQ + 15) / 16) * ((pl.n_entries + 7) / 8) * (pl.n_fblk / 8);
        const int steps = (pl.crs * pl.esize + 63) / 64;
        const bool plain_problem = pl.variant == ABED_NONE || pl.variant == ABED_DUPLICATE;   // (measured there only)
        if (pl.n_fblk % 8 == 0 && (tiles8 >= 384 || (plain_problem && tiles8 >= 256 && steps >= 64))) { wk = 8; wide = true; }
    }
    // Tiles 9 blocks wide (and 8 entries deep) for the filter checksum alone, whose digit block makes the
    // filter blocks 8 m + 1:
    //  - 128 filters + digit block = 9: one filter tile, so the FC residual stays inside the tile and the
    //    activations are read once (128 -> 128 3x3 at 28x28: -20 / -13 / -8 % at N = 64 / 128 / 256, 512 -> 128 1x1 at
    //    28x28 and N = 64: +26 % -> +4 % over the unchecked layer; slower at N = 32, and no gain with both schemes
    //    on the ResNet-50 layers);
    //  - 256 or 512 filters (17 or 33 blocks, which 4- and 5-wide tiles split 5 or 7 ways and 9-wide tiles 2 or
    //    4 ways): -10 ... -27 % on the ResNet-50 layers at N = 64 and 128 where the reduction axis is long and at
    //    least 200 tiles remain, slower on short axes and smaller grids.
    const int pad9 = (pl.n_fblk + 8) / 9 * 9;
    if (!wide && pl.esize == 1 && pl.n_fblk > pl.kblk && !pl.packed) {
        const long long tiles9 = (long long)((pl.PQ + 15) / 16) * ((pl.n_entries + 7) / 8) * (pad9 / 9);
        const bool fc_alone = pl.d_i == 0;
        bool nine = false;
        if (fc_alone && pl.n_fblk == 9) nine = tiles9 >= 384;
        else if (fc_alone && pl.n_fblk >= 17 && pad9 - pl.n_fblk <= 3 && pl.crs >= 1024) nine = tiles9 >= 200;
        if (nine) { wk = 9; wide = true; }
    }
    const int grid_m = (pl.PQ + 15) / 16, grid_n = (pl.n_fblk + wk - 1) / wk;
    auto tiles = [&](int wm) { return (long long)grid_m * ((pl.n_entries + 4 * wm - 1) / (4 * wm)) * grid_n; };
    auto waste = [&](int wm) { const int mb = 4 * wm; return (pl.n_entries + mb - 1) / mb * mb - pl.n_entries; };
    static const int cand[] = {5, 3, 2};
    int wm = 0;
    // among the tiles that leave at least 1.5 workgroups per CU and pad the batch by at most a fifth,
    // the one that pads least (the larger one on a tie); failing that, the largest that still gives
    // most CUs a workgroup; failing that, the smallest
    for (int c : cand)
        if (tiles(c) >= 384 && 5 * waste(c) <= pl.n_entries && (!wm || waste(c) < waste(wm))) wm = c;
    // (the plain problem, with no exchange between tiles, rather fills every CU with a smaller tile than three
    // quarters of them with a larger one: 2048 -> 512 1x1 at 7x7 with 64 images, 14.2 -> 12.5 us)
    const bool plain = pl.variant == ABED_NONE || pl.variant == ABED_DUPLICATE;
    if (!wm && plain)
        for (int c : cand)
            if (!wm && tiles(c) >= 256 && 5 * waste(c) <= pl.n_entries) wm = c;
    if (!wm)
        for (int c : cand)
            if (!wm && tiles(c) >= 160 && 5 * waste(c) <= pl.n_entries) wm = c;
    if (!wm) wm = 1;
    if (wide) wm = 2;
    if (pl.n_entries <= 4) wm = 1;
    wm = env_int("ABED_TILE_WM", wm);
    wk = env_int("ABED_TILE_WK", wk);
    pl.wm = wm; pl.wk = wk; pl.mb = 4 * wm;
    pl.grid_m = grid_m;
    pl.grid_b = (pl.n_entries + pl.mb - 1) / pl.mb;
    pl.grid_n = (pl.n_fblk + wk - 1) / wk;
    // wave groups along the reduction axis when the grid alone cannot put two waves on every SIMD
    const long long t = (long long)pl.grid_m * pl.grid_b * pl.grid_n;
    const int nsteps = (pl.crs * pl.esize + 63) / 64;
    int kg = 1;
    if (t < 384 && nsteps >= 16) kg = (t <= 256 && nsteps >= 64) ? 4 : 2;
    else if (t < 512 && nsteps >= 64) kg = 2;       // long loops still gain with 1.5-2 workgroups per CU (fp16 3x3, 256 channels: 30.8 -> 26.2 us)
    kg = env_int("ABED_TILE_KG", kg);
    while (kg > 1 && !tile_ok(wm, wk, kg)) kg /= 2;
    pl.kg = kg;
}

abed_status_t make_plan(const abed_conv_desc_t *d, int dtype, int variant, bool int8_out, Plan &pl)
{
    if (!d) return ABED_EINVAL;
    if (d->N < 1 || d->H < 1 || d->W < 1 || d->C < 1 || d->K < 1 || d->R < 1 || d->S < 1 ||
        d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0)
        return ABED_EINVAL;
    if (d->H + 2 * d->pad_h < d->R || d->W + 2 * d->pad_w < d->S) return ABED_EINVAL;
    // scheme selection bits: one of FC alone / IC alone, with a checked variant only
    const int packed = variant & ABED_PACKED_FC;
    const int l1 = variant & ABED_L1_THRESHOLD;
    const int only = variant & ~0xff & ~ABED_PACKED_FC & ~ABED_L1_THRESHOLD;
    variant &= 0xff;
    if (variant < ABED_NONE || variant > ABED_DUPLICATE) return ABED_EINVAL;
    if (only != 0 && only != ABED_ONLY_FC && only != ABED_ONLY_IC) return ABED_EINVAL;
    if (only != 0 && !(variant >= ABED_UNFUSED && variant <= ABED_FUSED_IOCG)) return ABED_EINVAL;
    if (only == ABED_ONLY_FC && variant == ABED_FUSED_IOCG) return ABED_EINVAL;
    if (packed && (only == ABED_ONLY_IC || dtype != ABED_INT8 || !(variant == ABED_FUSED_OCG || variant == ABED_FUSED_IOCG))) return ABED_EINVAL;
    if (l1 && (dtype != ABED_FP16 || !(variant >= ABED_UNFUSED && variant <= ABED_FUSED_IOCG))) return ABED_EINVAL;
    pl.variant = variant;
    pl.l1 = l1 ? 1 : 0;
    pl.packed = 0;
    if (dtype != ABED_INT8 && dtype != ABED_FP16) return ABED_EINVAL;
    const bool f16 = dtype == ABED_FP16;
    pl.esize = f16 ? 2 : 1;
    if ((d->C * pl.esize) % 16 != 0) return ABED_EUNSUPPORTED;   // 16-byte chunks of one filter tap
    const long long crs = (long long)d->C * d->R * d->S;
    if (crs > 65536) return ABED_EUNSUPPORTED;             // int32 accumulators are exact up to C*R*S = 64K (Sec. 4.1)
    // byte offsets inside a tensor are 32-bit (buffer descriptors); the largest offset marks "out of range"
    const long long kMaxBytes = 0x7ffffff0LL;
    if ((long long)d->N * d->H * d->W * d->C * pl.esize >= kMaxBytes) return ABED_EUNSUPPORTED;
    if ((long long)d->K * crs * pl.esize >= kMaxBytes) return ABED_EUNSUPPORTED;
    pl.P = (d->H + 2 * d->pad_h - d->R) / d->stride_h + 1;
    pl.Q = (d->W + 2 * d->pad_w - d->S) / d->stride_w + 1;
    pl.PQ = pl.P * pl.Q;
    pl.crs = (int)crs;
    if ((long long)d->N * pl.PQ * d->K >= (1LL << 31)) return ABED_EUNSUPPORTED;
    pl.d_f = f16 ? 2 : digits_for_count(d->K);             // fp16: the hi/lo pair (Sec. 7)
    pl.d_i = f16 ? 2 : digits_for_count(d->N);
    if (pl.d_f > 4 || pl.d_i > 4) return ABED_ERANGE;

    // Variants 1..5 report flags on the tile grid of the augmented problem (N + d_i batch
    // entries, one extra filter block); the unchecked kernels get the plain problem's grid.
    const bool checked = variant >= ABED_UNFUSED && variant <= ABED_FUSED_IOCG;
    if (only == ABED_ONLY_FC) pl.d_i = 0;
    if (only == ABED_ONLY_IC) pl.d_f = 0;
    pl.kblk = (d->K + 15) / 16;
    pl.n_entries = d->N + (checked ? pl.d_i : 0);
    if (packed) {
        // room for the digit filters behind the last real filter of its block?
        if (d->K % 16 == 0 || d->K % 16 + pl.d_f > 16) return ABED_EUNSUPPORTED;
        pl.packed = 1;
    }
    pl.n_fblk = pl.kblk + (checked && pl.d_f && !pl.packed ? 1 : 0);
    choose_tile(pl);

    // workspace: the two counter arrays come first and must be zero before the first call
    long long off = 0;
    auto take = [&](long long bytes) { long long o = off; off = align256(off + bytes); return o; };
    pl.off_cnt_fc = take((long long)pl.grid_m * pl.grid_b * 4);
    pl.off_cnt_ic = take((long long)pl.grid_m * pl.grid_n * 4);
    pl.off_convout = pl.off_yf = pl.off_yi = pl.off_yfi = pl.off_fc = pl.off_ic = pl.off_nx = -1;
    const long long npqk = (long long)d->N * pl.PQ * d->K;
    if (variant == ABED_UNFUSED || variant == ABED_FUSED_WRITE) {
        if (int8_out) pl.off_convout = take(npqk * 4);
        pl.off_yf = take((long long)d->N * pl.PQ * pl.d_f * 4);
        pl.off_yi = take((long long)pl.d_i * pl.PQ * d->K * 4);
        pl.off_yfi = take((long long)pl.d_i * pl.PQ * pl.d_f * 4);
    } else if (variant == ABED_FUSED_PARTIAL_REDUCTION || variant == ABED_FUSED_OCG || variant == ABED_FUSED_IOCG) {
        const long long tiles = (long long)pl.grid_m * pl.grid_b * pl.grid_n;
        pl.off_fc = take(tiles * pl.mb * 16 * 4 * (f16 ? 3 : 1));     // fp16 keeps sum, checksum value and sum of magnitudes apart
        pl.off_ic = take(tiles * pl.wk * 256 * 4 * (f16 ? 3 : 1));
        if (variant == ABED_FUSED_IOCG) pl.off_nx = take(tiles * pl.wk * 256 * 4);
    }
    pl.ws_bytes = off;
    return ABED_OK;
}

void fill_params(ConvParams &cp, const abed_conv_desc_t *d, const Plan &pl)
{
    memset(&cp, 0, sizeof(cp));
    cp.N = d->N; cp.H = d->H; cp.W = d->W; cp.C = d->C; cp.K = d->K; cp.R = d->R; cp.S = d->S;
    cp.sh = d->stride_h; cp.sw = d->stride_w; cp.ph = d->pad_h; cp.pw = d->pad_w;
    cp.P = pl.P; cp.Q = pl.Q;
    cp.cb = d->C * pl.esize; cp.crsb = pl.crs * pl.esize; cp.nsteps = (cp.crsb + 63) / 64;
    cp.n_entries = pl.n_entries; cp.n_fblk = pl.n_fblk; cp.kblk = pl.kblk;
    cp.d_f = pl.d_f; cp.d_i = pl.d_i;
    cp.packed_df = pl.packed ? pl.d_f : 0;
    cp.grid_m = pl.grid_m; cp.grid_b = pl.grid_b; cp.grid_n = pl.grid_n;
    cp.kt_slowest = env_int("ABED_KT_SLOWEST", (long long)d->K * pl.crs > (long long)d->N * d->H * d->W * d->C ? 1 : 0);
#ifdef ABED_ENABLE_DBG
    cp.dbg = env_int("ABED_DBG", 0);
#endif
}

void set_injection(ConvParams &cp, const abed_conv_desc_t *d, const Plan &pl, const abed_inject_t *inject)
{
    if (!inject || inject->site != 1) return;
    const long long k = inject->index % d->K, row = inject->index / d->K;   // row = n * PQ + pix
    const long long n = row / pl.PQ, pix = row % pl.PQ;
    const int fb = (int)(k / 16), i = (int)(k % 16);
    cp.inj_on = 1;
    cp.inj_pg = (int)(pix / 16); cp.inj_nt = (int)(n / pl.mb); cp.inj_mb = (int)(n % pl.mb);
    cp.inj_kt = fb / pl.wk; cp.inj_kb = fb % pl.wk;
    cp.inj_lane = (i / 4) * 16 + (int)(pix % 16); cp.inj_v = i % 4;
    cp.inj_mask = 1u << inject->bit;
}

// ---------------------------------------------------------------------------
// The box kernel (conv_box_kernel.h): 3x3 stride-1 layers, checksums local to a workgroup
// ---------------------------------------------------------------------------
struct BoxPlan {
    int P, Q, crs;
    int fb, fbr, xch;          // filter blocks per tile incl. the digit block, real ones, chunks of the batch checksum (0 = none)
    bool fc, ic;
    int boxes_x, boxes_y, grid_n, nranges, range_len;
    int eh;                    // 2: workgroups of 8 waves, batches of 8 entries; 1: of 4 waves and 4 entries, two per CU
};

// Shapes the box kernel takes: 3x3, stride 1, padding below 3, channels in chunks of 64, filters in tiles of 64.
bool box_shape_ok(const abed_conv_desc_t *d)
{
    if (d->R != 3 || d->S != 3 || d->stride_h != 1 || d->stride_w != 1 || d->pad_h > 2 || d->pad_w > 2) return false;
    if (d->C % 64 != 0 || d->K % 64 != 0) return false;
    const long long P = d->H + 2 * d->pad_h - 2, Q = d->W + 2 * d->pad_w - 2;
    if (P < 1 || Q < 1) return false;
    // 32-bit byte offsets, with room for a batch that runs up to 7 entries past N
    if ((long long)(d->N + 8) * d->H * d->W * d->C >= 0x40000000LL) return false;    // (the kernel's mask offset is 2^30)
    if ((long long)d->N * P * Q * d->K * 4 >= 0x7ffffff0LL) return false;
    if ((long long)d->K * 9 * d->C >= 0x7ffffff0LL) return false;
    return true;
}

// want_fc / want_ic: which checksums ride along (both false: the unchecked kernel)
abed_status_t make_box_plan(const abed_conv_desc_t *d, bool want_fc, bool want_ic, BoxPlan &bp)
{
    if (!box_shape_ok(d)) return ABED_EUNSUPPORTED;
    bp.P = d->H + 2 * d->pad_h - 2; bp.Q = d->W + 2 * d->pad_w - 2; bp.crs = 9 * d->C;
    bp.fc = want_fc; bp.ic = want_ic;
    const int nch = d->C / 64;
    bp.xch = want_ic ? nch : 0;
    bp.boxes_x = (bp.Q + 7) / 8; bp.boxes_y = (bp.P + 7) / 8;
    const int nboxes = bp.boxes_x * bp.boxes_y;
    // 64 filters per tile, or 128 (without the batch checksum, whose registers it would take) where that still
    // leaves every CU a workgroup: twice the matrix instructions per barrier and a quarter less LDS traffic per
    // matrix instruction (measured -9 ... -17 % on the 128- and 256-filter layers at 256 images, slower below)
    bp.fbr = 4;
    if (!want_ic && d->K % 128 == 0 && (long long)nboxes * (d->K / 128) * ((d->N + 7) / 8) >= 256) bp.fbr = 8;
    bp.fbr = env_int("ABED_BOX_FBR", bp.fbr);
    if (bp.fbr != 4 && bp.fbr != 8) return ABED_EUNSUPPORTED;
    bp.eh = env_int("ABED_BOX_EH", 2);
    if (bp.eh != 1 && bp.eh != 2) return ABED_EUNSUPPORTED;
    const int eb = 4 * bp.eh;                                  // entries per batch
    if (d->K % (16 * bp.fbr) != 0) return ABED_EUNSUPPORTED;
    bp.fb = bp.fbr + (want_fc ? 1 : 0);
    bp.grid_n = d->K / (16 * bp.fbr);
    if (!box_compiled(bp.fb, want_fc, bp.xch, bp.eh)) return ABED_EUNSUPPORTED;
    // Entry ranges: a range is a whole number of batches of 8 (at most 256 entries: the checksum's 16-bit
    // fields and two digits).  Longer ranges make the digit batch cheaper (it costs about half a batch),
    // shorter ones fill the chip; pick the best product of the two.
    const long long base = (long long)nboxes * bp.grid_n;
    int best_len = eb; double best = -1.0;
    const double slots = 256.0 * (3 - bp.eh);                  // workgroups the chip holds at once
    for (int len = eb; len <= 256; len += eb) {
        const int nr = (d->N + len - 1) / len;
        const long long tiles = base * nr;
        const double fill = (double)tiles / (slots * (double)((tiles + (long long)slots - 1) / (long long)slots));
        const double nb = len / (double)eb;
        const double score = fill * (want_ic ? nb / (nb + 0.5) : 1.0) * (1.0 - 0.02 / nb);
        if (score > best + 1e-9) { best = score; best_len = len; }
        if (len >= d->N) break;
    }
    bp.range_len = env_int("ABED_BOX_RANGE", best_len);
    if (bp.range_len < eb || bp.range_len > 256 || bp.range_len % eb != 0) return ABED_EUNSUPPORTED;
    bp.nranges = (d->N + bp.range_len - 1) / bp.range_len;
    return ABED_OK;
}

abed_status_t launch_box_conv(const abed_conv_desc_t *d, const BoxPlan &bp, const int8_t *x, const int8_t *w, const int8_t *wchk,
                              void *y, const abed_epilogue_t *epi, uint32_t *flags, const abed_inject_t *inject, hipStream_t st)
{
    BoxParams p;
    memset(&p, 0, sizeof(p));
    p.x = x; p.w = w; p.wchk = wchk; p.y = y; p.flags = flags;
    if (epi) { p.scale = epi->scale; p.bias = epi->bias; p.relu = epi->relu; p.out_int8 = 1; }
    p.N = d->N; p.H = d->H; p.W = d->W; p.C = d->C; p.K = d->K; p.P = bp.P; p.Q = bp.Q; p.ph = d->pad_h; p.pw = d->pad_w;
    p.crsb = bp.crs; p.nch = d->C / 64;
    p.boxes_x = bp.boxes_x; p.boxes_y = bp.boxes_y; p.grid_n = bp.grid_n; p.nranges = bp.nranges; p.range_len = bp.range_len;
    if (inject && inject->site == 1) {
        const long long k = inject->index % d->K, row = inject->index / d->K;
        const int n = (int)(row / (bp.P * bp.Q)), pix = (int)(row % (bp.P * bp.Q));
        const int oy = pix / bp.Q, ox = pix % bp.Q;
        const int tile_n = 16 * bp.fbr, rel = n % bp.range_len;
        p.inj_on = 1;
        p.inj_box = (oy / 8) * bp.boxes_x + ox / 8; p.inj_range = n / bp.range_len; p.inj_kt = (int)(k / tile_n);
        const int eb = 4 * bp.eh;
        p.inj_batch = rel / eb;
        const int pgrp = ((oy % 8) / 4) * 2 + (ox % 8) / 4, eh = (rel % eb) / 4;
        p.inj_wave = pgrp * bp.eh + eh; p.inj_i = rel % 4;
        p.inj_fb = (int)((k % tile_n) / 16);
        p.inj_lane = (int)((k % 16) / 4) * 16 + (oy % 4) * 4 + ox % 4; p.inj_v = (int)(k % 4);
        p.inj_mask = 1u << inject->bit;
    }
#ifdef ABED_ENABLE_DBG
    p.dbg = env_int("ABED_DBG", 0);
    { const char *v = getenv("ABED_DBG_PTR"); p.dbg_ts = (v && *v) ? (long long *)strtoull(v, nullptr, 0) : nullptr; }
#endif
    const int tiles = bp.boxes_x * bp.boxes_y * bp.nranges * bp.grid_n;
    if (!launch_box(bp.fb, bp.fc, bp.xch, bp.eh, p, (tiles + 7) / 8 * 8, st)) return ABED_EUNSUPPORTED;
    LAUNCH_CHECK("box_conv_kernel");
    return ABED_OK;
}

// Whether the unchecked convolution should take the box kernel: shapes it covers, with enough boxes to
// give most CUs a workgroup (ABED_BOX=0/1 overrides, for tests and sweeps).
bool box_preferred_plain(const abed_conv_desc_t *d)
{
    const int forced = env_int("ABED_BOX", -1);
    if (forced == 0 || !box_shape_ok(d)) return false;
    if (forced == 1) return true;
    const long long P = d->H + 2 * d->pad_h - 2, Q = d->W + 2 * d->pad_w - 2;
    // measured on the configured 3x3 layers at 32 and 256 images: faster than the pixel-group kernel from about
    // three quarters of a workgroup per CU on, slower below (few, long-running workgroups)
    const long long tiles = ((P + 7) / 8) * ((Q + 7) / 8) * (d->K / 64) * ((d->N + 7) / 8);
    return tiles >= 192;
}

// ---------------------------------------------------------------------------
// The one-wave-per-SIMD kernel (conv_img_kernel.h): 3x3 stride-1 layers, unchecked, int32 ConvOut; opt-in (ABED_IMG=1)
// ---------------------------------------------------------------------------
struct ImgPlan {
    int iw, RW, RH, PW, swz, rx, ry, ngroups, group_len, tiles;
};

// LDS cycles per fragment read of the kernel's activation operand, relative to a conflict-free read: a 16-byte-per-lane
// read serves 8 consecutive lanes per cycle out of one 128-byte bank window, so the 8 lanes (8 consecutive positions
// of the region's numbering, possibly wrapping into the next row) should fall into 8 different 16-byte columns;
// lanes on the same address count once.  Averaged over blocks, taps and lane groups; the same function of
// (row, column) as the kernel's loader and fragment addresses use.
double img_read_conflicts(int rh, int rw, int pw, int c, int hp)
{
    const int nb = (rh * pw + 31) / 32;
    long long tot = 0, n = 0;
    for (int b = 0; b < nb; ++b)
        for (int r = 0; r < 3; ++r)
            for (int sx = 0; sx < 3; ++sx)
                for (int g = 0; g < 4; ++g) {
                    int slot_of[8], col_of[8], worst = 1;
                    for (int j = 0; j < 8; ++j) {
                        const int pos = b * 32 + g * 8 + j;
                        int yy = pos / pw, xx = pos % pw;
                        if (yy >= rh) yy = rh - 1;
                        if (xx >= rw) xx = rw - 1;
                        const int hy = yy + r, hx = xx + sx;
                        slot_of[j] = hy * hp + hx;
                        col_of[j] = (slot_of[j] & 1) * 4 + (((hx >> 1) + c * hy) & 3);
                    }
                    for (int j = 0; j < 8; ++j) {
                        int cnt = 0;
                        for (int k = 0; k < 8; ++k) {
                            if (col_of[k] != col_of[j]) continue;
                            bool seen = false;
                            for (int q = 0; q < k; ++q) seen = seen || (col_of[q] == col_of[j] && slot_of[q] == slot_of[k]);
                            if (!seen) ++cnt;
                        }
                        if (cnt > worst) worst = cnt;
                    }
                    tot += worst; ++n;
                }
    return (double)tot / (double)n;
}

// Region shape: among the rectangles whose positions (numbered with pitch PW = the width, or the width rounded up to a
// multiple of 8) fit the wave's 4 / iw blocks of 32 and whose input positions, times the images of a batch, fit an
// activation stage, the one that leaves the fewest block lanes empty over the image plane; ties: the fewest LDS
// cycles per fragment read (with the best of the four swizzle constants), then the least input staged per output
// position.  Image groups: the split with the fewest rounds of 256 workgroups times (batches per group + 2) (ties:
// the shorter groups).  The last plan is kept: a layer is planned once, not per call.
abed_status_t make_img_plan(const abed_conv_desc_t *d, ImgPlan &ip)
{
    static thread_local abed_conv_desc_t last_d;
    static thread_local ImgPlan last_ip;
    static thread_local bool have_last = false;
    if (have_last && memcmp(&last_d, d, sizeof(*d)) == 0) { ip = last_ip; return ABED_OK; }
    if (!box_shape_ok(d)) return ABED_EUNSUPPORTED;
    const int P = d->H + 2 * d->pad_h - 2, Q = d->W + 2 * d->pad_w - 2;
    double best_eff = -1.0;
    for (int pass = 0; pass < 2; ++pass) {
        double best_conf = 1e9, best_halo = 1e9;
        ip.iw = 0;
        for (int iw = 1; iw <= 2; ++iw) {
            const int maxpos = 32 * (4 / iw), maxslots = kImgPlane / (4 * iw);
            for (int rw = 1; rw <= Q && rw <= maxpos; ++rw)
                for (int rh = 1; rh <= P && rh * rw <= maxpos; ++rh) {
                    if ((rh + 2) * (rw + 2) > maxslots) continue;
                    const int rx = (Q + rw - 1) / rw, ry = (P + rh - 1) / rh;
                    const double eff = (double)P * Q / ((double)rx * ry * maxpos);
                    if (pass == 0) { if (eff > best_eff) best_eff = eff; continue; }
                    if (eff < best_eff - 1e-9) continue;
                    const double halo = (double)(rh + 2) * (rw + 2) / (rh * rw);
                    for (int pw = rw; pw <= (rw + 7) / 8 * 8; pw += ((rw + 7) / 8 * 8 - rw ? (rw + 7) / 8 * 8 - rw : 8)) {
                        if (rh * pw > maxpos) break;
                        for (int c = 0; c < 4; ++c) {
                            const double conf = img_read_conflicts(rh, rw, pw, c, rw + 2);
                            if (conf < best_conf - 1e-9 || (conf < best_conf + 1e-9 && halo < best_halo - 1e-9)) {
                                best_conf = conf; best_halo = halo;
                                ip.iw = iw; ip.RW = rw; ip.RH = rh; ip.PW = pw; ip.swz = c; ip.rx = rx; ip.ry = ry;
                            }
                        }
                    }
                }
        }
    }
    if (!ip.iw || !img_compiled(ip.iw)) return ABED_EUNSUPPORTED;
    const int eb = 4 * ip.iw;
    const long long base = (long long)ip.rx * ip.ry * (d->K / 64);
    long long best_cost = -1;
    for (int len = eb; ; len += eb) {
        const int ng = (d->N + len - 1) / len;
        const long long tiles = base * ng;
        // a round of workgroups costs its batches plus a start and an end worth about two more
        const long long cost = ((tiles + 255) / 256) * (len / eb + 2);
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; ip.group_len = len; ip.ngroups = ng; }
        if (len >= d->N) break;
    }
    ip.tiles = (int)(base * ip.ngroups);
    last_d = *d; last_ip = ip; have_last = true;
    return ABED_OK;
}

abed_status_t launch_img_conv(const abed_conv_desc_t *d, const ImgPlan &ip, const int8_t *x, const int8_t *w, void *y, const abed_epilogue_t *epi,
                              hipStream_t st)
{
    ImgParams p;
    memset(&p, 0, sizeof(p));
    p.x = x; p.w = w; p.y = y;
    if (epi) { p.scale = epi->scale; p.bias = epi->bias; p.relu = epi->relu; }
    p.N = d->N; p.H = d->H; p.W = d->W; p.C = d->C; p.K = d->K; p.ph = d->pad_h; p.pw = d->pad_w;
    p.P = d->H + 2 * d->pad_h - 2; p.Q = d->W + 2 * d->pad_w - 2;
    p.RW = ip.RW; p.RH = ip.RH; p.PW = ip.PW; p.swz = ip.swz; p.rx = ip.rx; p.ry = ip.ry; p.nch = d->C / 64; p.nft = d->K / 64;
    p.ngroups = ip.ngroups; p.group_len = ip.group_len;
#ifdef ABED_ENABLE_DBG
    p.dbg = env_int("ABED_DBG", 0);
    { const char *v = getenv("ABED_DBG_PTR"); p.dbg_clk = (v && *v) ? (long long *)strtoull(v, nullptr, 0) : nullptr; }
#endif
    if (!launch_img(ip.iw, p, (ip.tiles + 7) / 8 * 8, st)) return ABED_EUNSUPPORTED;
    LAUNCH_CHECK("img_conv_kernel");
    return ABED_OK;
}

// An unchecked convolution with its own tile plan (the baseline, and the checksum
// convolutions of the unfused variant).
abed_status_t plain_conv(const abed_conv_desc_t *d, const int8_t *x, const int8_t *w, void *y,
                         const abed_epilogue_t *epi, const abed_inject_t *inject, hipStream_t st)
{
    Plan pl;
    abed_status_t s = make_plan(d, ABED_INT8, ABED_NONE, false, pl);
    if (s != ABED_OK) return s;
    if (!(inject && inject->site) && env_int("ABED_IMG", 0) == 1) {
        ImgPlan ip;
        if (make_img_plan(d, ip) == ABED_OK) return launch_img_conv(d, ip, x, w, y, epi, st);
    }
    if (box_preferred_plain(d)) {
        BoxPlan bp;
        if (make_box_plan(d, false, false, bp) == ABED_OK) return launch_box_conv(d, bp, x, w, nullptr, y, epi, nullptr, inject, st);
    }
    ConvParams cp;
    fill_params(cp, d, pl);
    cp.x = x; cp.w = w; cp.y = y; cp.mode = MODE_PLAIN;
    if (epi) { cp.scale = epi->scale; cp.bias = epi->bias; cp.relu = epi->relu; cp.out_int8 = 1; }
    set_injection(cp, d, pl, inject);
    if (!launch_conv(false, pl.wm, pl.wk, pl.kg, cp, (pl.grid_m * pl.grid_b * pl.grid_n + 7) / 8 * 8, st)) return ABED_EUNSUPPORTED;
    LAUNCH_CHECK("conv_kernel (unchecked)");
    return ABED_OK;
}

}  // namespace

extern "C" {

const char *abed_status_string(abed_status_t s)
{
    switch (s) {
    case ABED_OK: return "ok";
    case ABED_EINVAL: return "invalid argument";
    case ABED_EUNSUPPORTED: return "unsupported shape or option";
    case ABED_EWORKSPACE: return "workspace too small";
    case ABED_EHIP: return "HIP error";
    case ABED_ERANGE: return "checksum needs more than four digits";
    }
    return "unknown status";
}

// ---------------------------------------------------------------------------
// FIC scheme (Sec. 3.3)
// ---------------------------------------------------------------------------
namespace {

abed_status_t fic_plan(const abed_conv_desc_t *desc, int variant, Plan &pl, bool int8_out)
{
    if (variant != ABED_UNFUSED && variant != ABED_FUSED_OCG && variant != ABED_FUSED_IOCG) return desc ? ABED_EUNSUPPORTED : ABED_EINVAL;
    abed_status_t s = make_plan(desc, ABED_INT8, ABED_NONE, int8_out, pl);
    if (s != ABED_OK) return s;
    if (128LL * desc->N * pl.PQ >= (1LL << 31)) return ABED_ERANGE;     // input checksum entries are int32 (Sec. 4.1)
    if (pl.crs >= 32768) return ABED_ERANGE;                            // four accumulators are added in 32 bits before widening
    if (desc->S > 7) return ABED_EUNSUPPORTED;
    return ABED_OK;
}

// Parts of the batch the input checksum workgroups take side by side.  With a launch of their own
// (unfused option): enough workgroups for the chip.  Riding in the convolution's launch (fused option):
// as few as keep one workgroup short, about 16 loads per lane.
int fic_parts(const abed_conv_desc_t *d, int variant)
{
    int parts;
    if (variant == ABED_UNFUSED) {
        const int per_part = d->H * ((d->C + 63) / 64);
        parts = (512 + per_part - 1) / per_part;
        if (parts > 8) parts = 8;
    } else {
        const int nsub = d->W >= 64 ? 1 : 64 / d->W;      // image subsets a workgroup takes side by side
        parts = (d->N + 16 * nsub - 1) / (16 * nsub);
    }
    if (parts < (d->N + 255) / 256) parts = (d->N + 255) / 256;   // a lane sums at most 256 images in its 16-bit fields
    if (parts > d->N) parts = d->N;
    return parts < 1 ? 1 : parts;
}

int fic_rows_blocks(const abed_conv_desc_t *d, int variant) { return fic_parts(d, variant) * d->H * ((d->C + 63) / 64); }

// Input checksum kernel.  wsum/dotpart null: only xrows is made.  from_rows: xrows is given and only
// the partial dot products are formed from it.
abed_status_t fic_input_rows(const abed_conv_desc_t *d, const Plan &pl, int variant, const int8_t *x, const int32_t *wsum,
                             int32_t *xrows, long long *dotpart, bool from_rows, hipStream_t st)
{
    FicRowsParams rp;
    rp.x = x; rp.wsum = wsum; rp.xrows = xrows; rp.dotpart = dotpart; rp.parts = fic_parts(d, variant); rp.from_rows = from_rows ? 1 : 0;
    rp.xsum = nullptr;
    rp.N = d->N; rp.H = d->H; rp.W = d->W; rp.C = d->C; rp.R = wsum ? d->R : 0; rp.S = d->S; rp.P = pl.P; rp.Q = pl.Q;
    rp.sh = d->stride_h; rp.sw = d->stride_w; rp.ph = d->pad_h; rp.pw = d->pad_w;
    const dim3 grid((unsigned)((fic_rows_blocks(d, variant) + 7) / 8 * 8));   // whole rounds over the 8 XCDs
    if (d->S <= 1) fic_input_rows_i8_kernel<1><<<grid, dim3(256), 0, st>>>(rp);
    else if (d->S <= 3) fic_input_rows_i8_kernel<3><<<grid, dim3(256), 0, st>>>(rp);
    else fic_input_rows_i8_kernel<7><<<grid, dim3(256), 0, st>>>(rp);
    LAUNCH_CHECK("fic_input_rows_i8_kernel");
    return ABED_OK;
}

const int kFicSumBlocks = 1024;   // workgroups (= partial sums) of the separate output checksum pass

}  // namespace

abed_status_t abed_fic_get_layout(const abed_conv_desc_t *desc, int32_t variant, abed_fic_layout_t *out)
{
    if (!out) return ABED_EINVAL;
    Plan pl;
    abed_status_t s = fic_plan(desc, variant, pl, false);
    if (s != ABED_OK) return s;
    out->wsum_bytes = 4LL * pl.crs;
    out->xrows_parts = fic_parts(desc, variant);
    out->xrows_bytes = 4LL * out->xrows_parts * desc->H * desc->S * desc->C;
    // partial output checksums (one per tile / per workgroup of the separate pass); the unfused
    // option keeps the int32 ConvOut behind them when the output is int8
    const long long partials = align256(8LL * (variant == ABED_UNFUSED ? kFicSumBlocks : (long long)pl.grid_m * pl.grid_b * pl.grid_n));
    const long long dotparts = align256(8LL * fic_rows_blocks(desc, variant));
    out->workspace_bytes = 256 + partials + dotparts + (variant == ABED_UNFUSED ? align256(4LL * desc->N * pl.PQ * desc->K) : 0);
    out->xsum_bytes = 4LL * desc->H * desc->W * desc->C;
    out->xsum_next_bytes = 4LL * pl.PQ * desc->K;
    return ABED_OK;
}

abed_status_t abed_fic_filter_prepare_int8(const abed_conv_desc_t *desc, const int8_t *w, int32_t *wsum, void *stream)
{
    Plan pl;
    abed_status_t s = make_plan(desc, ABED_INT8, ABED_NONE, false, pl);
    if (s != ABED_OK) return s;
    if (!w || !wsum) return ABED_EINVAL;
    fic_filter_checksum_i8_kernel<<<dim3((pl.crs + 63) / 64), dim3(1024), 0, (hipStream_t)stream>>>(w, wsum, desc->K, pl.crs);
    LAUNCH_CHECK("fic_filter_checksum_i8_kernel");
    return ABED_OK;
}

abed_status_t abed_fic_input_checksum_int8(const abed_conv_desc_t *desc, int32_t variant, const int8_t *x, int32_t *xrows, void *stream)
{
    Plan pl;
    abed_status_t s = fic_plan(desc, variant, pl, false);
    if (s != ABED_OK) return s;
    if (!x || !xrows) return ABED_EINVAL;
    return fic_input_rows(desc, pl, variant, x, nullptr, xrows, nullptr, false, (hipStream_t)stream);
}

abed_status_t abed_fic_conv_int8(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w,
                                 const int32_t *wsum, int32_t *xrows, int32_t compute_xrows,
                                 void *y, const abed_epilogue_t *epi, int32_t variant,
                                 int64_t *result, uint32_t *flag,
                                 int32_t *xsum_in, int32_t *xsum_next,
                                 void *workspace, size_t workspace_bytes,
                                 const abed_inject_t *inject, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const bool int8_out = epi != nullptr;
    Plan pl;
    abed_status_t s = fic_plan(desc, variant, pl, int8_out);
    if (s != ABED_OK) return s;
    if (!x || !w || !wsum || !xrows || !y) return ABED_EINVAL;
    if ((result == nullptr) != (flag == nullptr)) return ABED_EINVAL;
    const bool deferred = result == nullptr;          // the partial sums stay in the workspace for abed_fic_verify
    if (epi && (!epi->scale || !epi->bias)) return ABED_EINVAL;
    // handing the batch sum from layer to layer belongs to the input-and-output-fused option only,
    // and the sum handed on is that of the epilog's int8 output
    if (variant != ABED_FUSED_IOCG && (xsum_in || xsum_next)) return ABED_EINVAL;
    if (xsum_next && !int8_out) return ABED_EINVAL;
    if (xsum_in && xsum_in == xsum_next) return ABED_EINVAL;
    const long long npqk = (long long)desc->N * pl.PQ * desc->K;
    if (inject && inject->site != 0) {
        if (inject->site != 1 && inject->site != 2) return ABED_EINVAL;
        if (inject->index < 0 || inject->index >= npqk || inject->bit < 0 || inject->bit > 31) return ABED_EINVAL;
        if (inject->site == 2 && variant != ABED_UNFUSED) return ABED_EUNSUPPORTED;
    }
    abed_fic_layout_t lay;
    if ((s = abed_fic_get_layout(desc, variant, &lay)) != ABED_OK) return s;
    if (!workspace || (long long)workspace_bytes < lay.workspace_bytes) return ABED_EWORKSPACE;
    const int ntiles = pl.grid_m * pl.grid_b * pl.grid_n;
    // workspace: 256 bytes kept free, partial output checksums, partial dot products, ConvOut
    long long *partial = (long long *)((char *)workspace + 256);
    const long long npart_bytes = align256(8LL * (variant == ABED_UNFUSED ? kFicSumBlocks : ntiles));
    long long *dotpart = (long long *)((char *)workspace + 256 + npart_bytes);
    const int rows_blocks = fic_rows_blocks(desc, variant);
    const long long convout_off = 256 + npart_bytes + align256(8LL * rows_blocks);

    ConvParams cp;
    fill_params(cp, desc, pl);
    cp.x = x; cp.w = w; cp.mode = MODE_PLAIN;
    set_injection(cp, desc, pl, inject);
    const int grid = (ntiles + 7) / 8 * 8;
    if (variant == ABED_FUSED_OCG || variant == ABED_FUSED_IOCG) {
        // Two launches (tasks 2 to 7 of Sec. 4.3).  First: the leading workgroups make the input checksum
        // and its partial dot products while the tile workgroups convolve, apply the epilog and reduce
        // their accumulators.  Second: a one-workgroup kernel adds up the partial sums and compares.
        const int lead = (rows_blocks + 7) / 8 * 8;      // keeps the tiles' block index aligned to the 8 XCDs
        cp.y = y; cp.fic_ocs = partial; cp.fic_sum32 = !cp.inj_on && (long long)pl.crs * 4 * pl.wm * pl.wk * 16384 < (1LL << 31);
        cp.fic_wsum = wsum; cp.fic_xrows = xrows; cp.fic_dotpart = dotpart;
        cp.fic_parts = lay.xrows_parts; cp.fic_rows_lead = lead; cp.fic_from_rows = xsum_in ? 2 : (compute_xrows ? 0 : 1);
        cp.fic_xsum_in = xsum_in; cp.fic_xsum_next = xsum_next;
        if (epi) { cp.scale = epi->scale; cp.bias = epi->bias; cp.relu = epi->relu; cp.out_int8 = 1; }
        // 1024-thread workgroups take a CU each, so every input checksum workgroup in front of them would push
        // a tile into a second round (measured +6.5 us on 512 filters at 7x7): two wave groups there instead of four
        const int kg = (pl.kg == 4 && lead > 0) ? 2 : pl.kg;
        if (!launch_conv(false, pl.wm, pl.wk, kg, cp, lead + grid, st)) return ABED_EUNSUPPORTED;
        LAUNCH_CHECK("conv_kernel (FIC, fused)");
        if (deferred) return ABED_OK;
        FicVerifyParams vp;
        vp.dotpart = dotpart; vp.partial = partial; vp.result = (long long *)result; vp.flag = flag;
        vp.ndot = rows_blocks; vp.npartial = ntiles;
        fic_verify_kernel<<<1, 1024, 0, st>>>(vp);
        LAUNCH_CHECK("fic_verify_kernel");
        return ABED_OK;
    }

    // unfused option: one kernel per task
    if ((s = fic_input_rows(desc, pl, variant, x, wsum, xrows, dotpart, !compute_xrows, st)) != ABED_OK) return s;
    int32_t *convout = int8_out ? (int32_t *)((char *)workspace + convout_off) : (int32_t *)y;
    cp.y = convout;
    if (!launch_conv(false, pl.wm, pl.wk, pl.kg, cp, grid, st)) return ABED_EUNSUPPORTED;
    LAUNCH_CHECK("conv_kernel (unchecked)");
    if (inject && inject->site == 2) flip_bit_u32_kernel<<<1, 1, 0, st>>>((uint32_t *)convout, inject->index, 1u << inject->bit);
    fic_output_sum_kernel<<<dim3(kFicSumBlocks), dim3(256), 0, st>>>(convout, npqk, partial);
    LAUNCH_CHECK("fic_output_sum_kernel");
    if (int8_out) {
        epilog_i8_kernel<<<dim3((unsigned)((npqk / 4 + 256) / 256)), dim3(256), 0, st>>>(convout, (int8_t *)y, epi->scale, epi->bias, epi->relu, npqk, desc->K);
        LAUNCH_CHECK("epilog_i8_kernel");
    }
    if (deferred) return ABED_OK;
    FicVerifyParams vp;
    vp.dotpart = dotpart; vp.partial = partial; vp.result = (long long *)result; vp.flag = flag;
    vp.ndot = rows_blocks; vp.npartial = kFicSumBlocks;
    fic_verify_kernel<<<1, 1024, 0, st>>>(vp);
    LAUNCH_CHECK("fic_verify_kernel");
    return ABED_OK;
}

// FIC with the input side formed in the convolution's main loop: what a layer's call and the deferred
// comparison both need
namespace {

struct InloopPlan {
    Plan pl;
    int nstages, gpad;
    unsigned dyn_lds;
    long long partial_bytes, dot_bytes;
};

abed_status_t inloop_plan(const abed_conv_desc_t *desc, bool int8_out, InloopPlan &ip)
{
    abed_status_t s = make_plan(desc, ABED_INT8, ABED_NONE, int8_out, ip.pl);
    if (s != ABED_OK) return s;
    const Plan &pl = ip.pl;
    const int nsteps = (pl.crs + 63) / 64;
    ip.nstages = (nsteps + pl.kg - 1) / pl.kg;
    ip.gpad = nsteps * 64;
    // three digits hold |filter checksum| <= 128 K below 2^23; a lane's 32-bit sums take at most
    // 16 * wm products of magnitude <= 2^14 per step
    if (desc->K > 32768 || pl.crs >= 32768) return ABED_ERANGE;
    if ((long long)pl.wm * ip.nstages >= 8192) return ABED_ERANGE;
    const long long dyn = 3LL * ip.nstages * pl.kg * 64;
    if (dyn > 24 * 1024) return ABED_EUNSUPPORTED;         // beside the kernel's own LDS (at most 128 KB of 160 KB)
    ip.dyn_lds = (unsigned)(dyn < 128 ? 128 : dyn);
    ip.partial_bytes = align256(8LL * pl.grid_m * pl.grid_b * pl.grid_n);
    ip.dot_bytes = align256(8LL * pl.grid_m * pl.grid_b);
    return ABED_OK;
}

}  // namespace

abed_status_t abed_fic_verify(int32_t n_layers, const abed_conv_desc_t *descs, const int32_t *variants,
                              void *const *workspaces, int64_t *results, uint32_t *flags, void *stream)
{
    if (n_layers < 0 || (n_layers > 0 && (!descs || !variants || !workspaces || !results || !flags))) return ABED_EINVAL;
    // check everything before the first launch
    for (int i = 0; i < n_layers; ++i) {
        Plan pl;
        InloopPlan ip;
        abed_status_t s = variants[i] == ABED_FIC_INLOOP ? inloop_plan(&descs[i], false, ip) : fic_plan(&descs[i], variants[i], pl, false);
        if (s != ABED_OK) return s;
        if (!workspaces[i]) return ABED_EINVAL;
    }
    for (int base = 0; base < n_layers; base += kFicVerifyBatch) {
        FicVerifyBatchParams bp;
        const int n = n_layers - base < kFicVerifyBatch ? n_layers - base : kFicVerifyBatch;
        for (int j = 0; j < n; ++j) {
            const int i = base + j;
            Plan pl;
            const bool inloop = variants[i] == ABED_FIC_INLOOP;
            if (inloop) make_plan(&descs[i], ABED_INT8, ABED_NONE, false, pl);
            else fic_plan(&descs[i], variants[i], pl, false);
            // the same carving as in the call that ran the layer: 256 bytes kept free, partial output checksums, partial dot products
            const int npartial = variants[i] == ABED_UNFUSED ? kFicSumBlocks : pl.grid_m * pl.grid_b * pl.grid_n;
            FicVerifyParams &vp = bp.layer[j];
            vp.partial = (const long long *)((const char *)workspaces[i] + 256);
            vp.dotpart = (const long long *)((const char *)workspaces[i] + 256 + align256(8LL * npartial));
            vp.ndot = inloop ? pl.grid_m * pl.grid_b : fic_rows_blocks(&descs[i], variants[i]);
            vp.npartial = npartial;
            vp.result = (long long *)results + 2 * i;
            vp.flag = flags + i;
        }
        fic_verify_batch_kernel<<<dim3(n), dim3(1024), 0, (hipStream_t)stream>>>(bp);
        LAUNCH_CHECK("fic_verify_batch_kernel");
    }
    return ABED_OK;
}

// ---------------------------------------------------------------------------
// FIC with the input side formed in the convolution's main loop
// ---------------------------------------------------------------------------
abed_status_t abed_fic_inloop_get_layout(const abed_conv_desc_t *desc, abed_fic_inloop_layout_t *out)
{
    if (!out) return ABED_EINVAL;
    InloopPlan ip;
    abed_status_t s = inloop_plan(desc, false, ip);
    if (s != ABED_OK) return s;
    out->workspace_bytes = 256 + ip.partial_bytes + ip.dot_bytes;
    out->wdig_bytes = 3LL * ip.gpad;
    return ABED_OK;
}

abed_status_t abed_fic_inloop_filter_prepare_int8(const abed_conv_desc_t *desc, const int8_t *w, int8_t *wdig, void *stream)
{
    InloopPlan ip;
    abed_status_t s = inloop_plan(desc, false, ip);
    if (s != ABED_OK) return s;
    if (!w || !wdig) return ABED_EINVAL;
    fic_filter_digits_i8_kernel<<<dim3(ip.gpad / 64), dim3(1024), 0, (hipStream_t)stream>>>(w, wdig, desc->K, ip.pl.crs, ip.gpad);
    LAUNCH_CHECK("fic_filter_digits_i8_kernel");
    return ABED_OK;
}

abed_status_t abed_fic_inloop_conv_int8(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w, const int8_t *wdig,
                                        void *y, const abed_epilogue_t *epi, int64_t *result, uint32_t *flag,
                                        void *workspace, size_t workspace_bytes, const abed_inject_t *inject, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    InloopPlan ip;
    abed_status_t s = inloop_plan(desc, epi != nullptr, ip);
    if (s != ABED_OK) return s;
    const Plan &pl = ip.pl;
    if (!x || !w || !wdig || !y) return ABED_EINVAL;
    if ((result == nullptr) != (flag == nullptr)) return ABED_EINVAL;
    if (epi && (!epi->scale || !epi->bias)) return ABED_EINVAL;
    if (inject && inject->site != 0) {
        if (inject->site != 1) return inject->site == 2 ? ABED_EUNSUPPORTED : ABED_EINVAL;
        if (inject->index < 0 || inject->index >= (long long)desc->N * pl.PQ * desc->K || inject->bit < 0 || inject->bit > 31) return ABED_EINVAL;
    }
    if (!workspace || (long long)workspace_bytes < 256 + ip.partial_bytes + ip.dot_bytes) return ABED_EWORKSPACE;
    long long *partial = (long long *)((char *)workspace + 256);
    long long *dotpart = (long long *)((char *)workspace + 256 + ip.partial_bytes);
    const int ntiles = pl.grid_m * pl.grid_b * pl.grid_n;
    ConvParams cp;
    fill_params(cp, desc, pl);
    cp.x = x; cp.w = w; cp.y = y; cp.mode = MODE_PLAIN;
    set_injection(cp, desc, pl, inject);
    cp.fic_ocs = partial; cp.fic_sum32 = !cp.inj_on && (long long)pl.crs * 4 * pl.wm * pl.wk * 16384 < (1LL << 31); cp.fic_dotpart = dotpart; cp.fic_wdig = wdig;
    cp.fic_ndig = 128LL * desc->K < 32768 ? 2 : 3;          // |filter checksum| <= 128 K; two digits reach 32767 + 128
    if (epi) { cp.scale = epi->scale; cp.bias = epi->bias; cp.relu = epi->relu; cp.out_int8 = 1; }
    if (!launch_conv(false, pl.wm, pl.wk, pl.kg, cp, (ntiles + 7) / 8 * 8, st, ip.dyn_lds)) return ABED_EUNSUPPORTED;
    LAUNCH_CHECK("conv_kernel (FIC, input side in the main loop)");
    if (!result) return ABED_OK;
    FicVerifyParams vp;
    vp.dotpart = dotpart; vp.partial = partial; vp.result = (long long *)result; vp.flag = flag;
    vp.ndot = pl.grid_m * pl.grid_b; vp.npartial = ntiles;
    fic_verify_kernel<<<1, 1024, 0, st>>>(vp);
    LAUNCH_CHECK("fic_verify_kernel");
    return ABED_OK;
}

// ---------------------------------------------------------------------------
// IC option 2 (Sec. 3.2): K values
// ---------------------------------------------------------------------------
namespace {

const int kIc2SumBlocks = 512;    // workgroups (= partial sums per filter) of the separate output checksum pass

abed_status_t ic2_plan(const abed_conv_desc_t *desc, int variant, Plan &pl, bool int8_out)
{
    if (variant != ABED_UNFUSED && variant != ABED_FUSED_OCG) return desc ? ABED_EUNSUPPORTED : ABED_EINVAL;
    return fic_plan(desc, variant, pl, int8_out);      // same input checksum, same limits
}

}  // namespace

abed_status_t abed_ic2_get_layout(const abed_conv_desc_t *desc, int32_t variant, abed_ic2_layout_t *out)
{
    if (!out) return ABED_EINVAL;
    Plan pl;
    abed_status_t s = ic2_plan(desc, variant, pl, false);
    if (s != ABED_OK) return s;
    out->xrows_parts = fic_parts(desc, variant);
    out->xrows_bytes = 4LL * out->xrows_parts * desc->H * desc->S * desc->C;
    out->n_values = desc->K;
    const long long partials = variant == ABED_UNFUSED ? 8LL * kIc2SumBlocks * desc->K
                                                       : 8LL * pl.grid_m * pl.grid_b * pl.grid_n * pl.wk * 16;
    // 256 bytes kept free, the filter-sized input checksum, the partial output sums, ConvOut of the unfused option
    out->workspace_bytes = 256 + align256(4LL * pl.crs) + align256(partials) + (variant == ABED_UNFUSED ? align256(4LL * desc->N * pl.PQ * desc->K) : 0);
    return ABED_OK;
}

abed_status_t abed_ic2_conv_int8(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w,
                                 int32_t *xrows, int32_t compute_xrows,
                                 void *y, const abed_epilogue_t *epi, int32_t variant,
                                 int64_t *result, uint32_t *flags,
                                 void *workspace, size_t workspace_bytes,
                                 const abed_inject_t *inject, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    const bool int8_out = epi != nullptr;
    Plan pl;
    abed_status_t s = ic2_plan(desc, variant, pl, int8_out);
    if (s != ABED_OK) return s;
    if (!x || !w || !xrows || !y || !result || !flags) return ABED_EINVAL;
    if (epi && (!epi->scale || !epi->bias)) return ABED_EINVAL;
    const long long npqk = (long long)desc->N * pl.PQ * desc->K;
    if (inject && inject->site != 0) {
        if (inject->site != 1 && inject->site != 2) return ABED_EINVAL;
        if (inject->index < 0 || inject->index >= npqk || inject->bit < 0 || inject->bit > 31) return ABED_EINVAL;
        if (inject->site == 2 && variant != ABED_UNFUSED) return ABED_EUNSUPPORTED;
    }
    abed_ic2_layout_t lay;
    if ((s = abed_ic2_get_layout(desc, variant, &lay)) != ABED_OK) return s;
    if (!workspace || (long long)workspace_bytes < lay.workspace_bytes) return ABED_EWORKSPACE;
    const int ntiles = pl.grid_m * pl.grid_b * pl.grid_n;
    int32_t *X = (int32_t *)((char *)workspace + 256);
    long long *part = (long long *)((char *)workspace + 256 + align256(4LL * pl.crs));
    const int rows_blocks = fic_rows_blocks(desc, variant);

    ConvParams cp;
    fill_params(cp, desc, pl);
    cp.x = x; cp.w = w; cp.mode = MODE_PLAIN;
    set_injection(cp, desc, pl, inject);
    const int grid = (ntiles + 7) / 8 * 8;
    Ic2FoldParams fp;
    fp.xrows = xrows; fp.X = X; fp.H = desc->H; fp.C = desc->C; fp.R = desc->R; fp.S = desc->S; fp.P = pl.P;
    fp.sh = desc->stride_h; fp.ph = desc->pad_h; fp.parts = lay.xrows_parts;
    Ic2VerifyParams vp;
    vp.w = w; vp.X = X; vp.part = part; vp.result = (long long *)result; vp.flags = flags;
    vp.K = desc->K; vp.crs = pl.crs;
    if (variant == ABED_FUSED_OCG) {
        // Three launches: the input checksum workgroups lead the convolution's launch, whose tiles reduce
        // their accumulators per filter; a small kernel folds the row-wise checksum to the filter's
        // size; then one workgroup per filter convolves the checksum tensor with its filter, adds up
        // the partial output sums and compares.
        const int lead = compute_xrows ? (rows_blocks + 7) / 8 * 8 : 0;
        cp.y = y; cp.ic2_part = part;
        cp.fic_xrows = xrows; cp.fic_parts = lay.xrows_parts; cp.fic_rows_lead = lead;
        if (epi) { cp.scale = epi->scale; cp.bias = epi->bias; cp.relu = epi->relu; cp.out_int8 = 1; }
        const int kg = (pl.kg == 4 && lead > 0) ? 2 : pl.kg;     // as in abed_fic_conv_int8
        if (!launch_conv(false, pl.wm, pl.wk, kg, cp, lead + grid, st)) return ABED_EUNSUPPORTED;
        LAUNCH_CHECK("conv_kernel (IC option 2, fused)");
        vp.nrows = pl.grid_m * pl.grid_b; vp.kstride = pl.grid_n * pl.wk * 16;
        ic2_fold_kernel<<<dim3((pl.crs + 63) / 64), dim3(1024), 0, st>>>(fp);
        LAUNCH_CHECK("ic2_fold_kernel");
        ic2_verify_kernel<<<dim3(desc->K), dim3(256), 0, st>>>(vp);
        LAUNCH_CHECK("ic2_verify_kernel");
        return ABED_OK;
    }
    // unfused option: one kernel per task
    if ((size_t)desc->K * 8 > 64 * 1024) return ABED_EUNSUPPORTED;   // the output sum kernel's LDS
    if (compute_xrows && (s = fic_input_rows(desc, pl, variant, x, nullptr, xrows, nullptr, false, st)) != ABED_OK) return s;
    int32_t *convout = int8_out ? (int32_t *)((char *)workspace + 256 + align256(4LL * pl.crs) + align256(8LL * kIc2SumBlocks * desc->K)) : (int32_t *)y;
    cp.y = convout;
    if (!launch_conv(false, pl.wm, pl.wk, pl.kg, cp, grid, st)) return ABED_EUNSUPPORTED;
    LAUNCH_CHECK("conv_kernel (unchecked)");
    if (inject && inject->site == 2) flip_bit_u32_kernel<<<1, 1, 0, st>>>((uint32_t *)convout, inject->index, 1u << inject->bit);
    ic2_output_sums_kernel<<<dim3(kIc2SumBlocks), dim3(256), (size_t)desc->K * 8, st>>>(convout, (long long)desc->N * pl.PQ, desc->K, part);
    LAUNCH_CHECK("ic2_output_sums_kernel");
    if (int8_out) {
        epilog_i8_kernel<<<dim3((unsigned)((npqk / 4 + 256) / 256)), dim3(256), 0, st>>>(convout, (int8_t *)y, epi->scale, epi->bias, epi->relu, npqk, desc->K);
        LAUNCH_CHECK("epilog_i8_kernel");
    }
    vp.nrows = kIc2SumBlocks; vp.kstride = desc->K;
    ic2_fold_kernel<<<dim3((pl.crs + 63) / 64), dim3(1024), 0, st>>>(fp);
    LAUNCH_CHECK("ic2_fold_kernel");
    ic2_verify_kernel<<<dim3(desc->K), dim3(256), 0, st>>>(vp);
    LAUNCH_CHECK("ic2_verify_kernel");
    return ABED_OK;
}

const char *abed_last_hip_error(void) { return g_hip_error; }

abed_status_t abed_get_layout(const abed_conv_desc_t *desc, int32_t dtype, int32_t variant, abed_layout_t *out)
{
    if (!out) return ABED_EINVAL;
    Plan pl;
    // the workspace is sized for the int8-output case, which needs the most
    abed_status_t s = make_plan(desc, dtype, variant & ~ABED_LOCAL, true, pl);
    if (s != ABED_OK) return s;
    memset(out, 0, sizeof(*out));
    if (variant & ABED_LOCAL) {
        if (dtype != ABED_INT8 || pl.variant != ABED_FUSED_OCG) return ABED_EUNSUPPORTED;
        BoxPlan bp;
        if ((s = make_box_plan(desc, pl.d_f > 0, pl.d_i > 0, bp)) != ABED_OK) return s;
        out->tile_pixels = 64; out->tile_box = 8;
        out->tile_batch = bp.range_len; out->tile_n = 16 * bp.fbr;
        out->grid_m = bp.boxes_x * bp.boxes_y; out->grid_b = bp.nranges; out->grid_n = bp.grid_n;
        out->d_f = bp.fc ? 2 : 0; out->d_i = bp.ic ? 2 : 0;
        out->n_flag_words = (long long)out->grid_m * out->grid_b * out->grid_n;
        out->workspace_bytes = 0;
        out->wchk_bytes = (long long)out->d_f * bp.grid_n * bp.crs;
        out->xchk_bytes = 0; out->xchk_next_bytes = 0;
        out->local_checksums = 1;
        // Measured on the configured 3x3 layers at 32 and 256 images: this form beats the layer-wide checksums
        // (input checksum kernel + augmented convolution with its exchange between tiles) where the tiles give
        // at least three quarters of the CUs a workgroup and the digit batch is a small part of a workgroup's
        // life: one chunk of channels (the filters then stay in LDS), or batch tiles of at least 32 images.  The
        // filter checksum alone has no digit batch (+2 ... 14 % over the unchecked box kernel at 256 images).
        out->local_preferred = (out->n_flag_words >= 192 && (!bp.ic || desc->C == 64 || bp.range_len >= 32)) ? 1 : 0;
        return ABED_OK;
    }
    out->tile_pixels = 16;
    out->tile_batch = pl.mb;
    out->tile_n = 16 * pl.wk;
    out->grid_m = pl.grid_m;
    out->grid_b = pl.grid_b;
    out->grid_n = pl.grid_n;
    out->d_f = pl.d_f;
    out->d_i = pl.d_i;
    out->n_flag_words = (long long)pl.grid_m * pl.grid_b * pl.grid_n;
    out->workspace_bytes = pl.ws_bytes;
    out->wchk_bytes = (long long)pl.d_f * pl.crs * pl.esize;
    out->xchk_bytes = (long long)pl.d_i * desc->H * desc->W * desc->C * pl.esize;
    out->xchk_next_bytes = (long long)pl.d_i * pl.PQ * desc->K;
    return ABED_OK;
}

abed_status_t abed_probe(int32_t kind, void *a, void *b, size_t bytes, int32_t iters, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    if (!a || iters < 1) return ABED_EINVAL;
    if (kind == 0) {
        if (bytes < 256u * 512u * 4u) return ABED_EINVAL;
        probe_mfma_i8_kernel<<<dim3(256), dim3(512), 0, st>>>((int *)a, iters);
    } else if (kind == 1 || kind == 2) {
        if (bytes < 16 || (kind == 2 && !b)) return ABED_EINVAL;
        for (int i = 0; i < iters; ++i)
            probe_stream_kernel<<<dim3(256 * 8), dim3(256), 0, st>>>(kind == 2 ? (const i32x4p *)a : nullptr, (i32x4p *)(kind == 2 ? b : a), (long long)(bytes / 16));
    } else {
        return ABED_EINVAL;
    }
    LAUNCH_CHECK("probe kernel");
    return ABED_OK;
}

abed_status_t abed_workspace_init(void *workspace, size_t workspace_bytes, void *stream)
{
    if (!workspace) return workspace_bytes == 0 ? ABED_OK : ABED_EINVAL;
    const long long words = (long long)(workspace_bytes / 4);
    if (words == 0) return ABED_OK;
    fill_u32_kernel<<<dim3((unsigned)((words + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>((uint32_t *)workspace, words, 0u);
    LAUNCH_CHECK("fill_u32_kernel");
    return ABED_OK;
}

abed_status_t abed_filter_prepare_int8(const abed_conv_desc_t *desc, const int8_t *w, int8_t *wchk, void *stream)
{
    Plan pl;
    abed_status_t s = make_plan(desc, ABED_INT8, ABED_NONE, false, pl);
    if (s != ABED_OK) return s;
    if (!w || !wchk) return ABED_EINVAL;
    filter_checksum_i8_kernel<<<dim3((pl.crs + 63) / 64), dim3(1024), 0, (hipStream_t)stream>>>(w, wchk, desc->K, pl.crs, pl.d_f);
    LAUNCH_CHECK("filter_checksum_i8_kernel");
    return ABED_OK;
}

abed_status_t abed_filter_prepare_local_int8(const abed_conv_desc_t *desc, int32_t variant, const int8_t *w, int8_t *wchk, void *stream)
{
    abed_layout_t lay;
    abed_status_t s = abed_get_layout(desc, ABED_INT8, variant, &lay);
    if (s != ABED_OK) return s;
    if (!lay.local_checksums) return abed_filter_prepare_int8(desc, w, wchk, stream);
    if (lay.d_f == 0) return ABED_OK;
    if (!w || !wchk) return ABED_EINVAL;
    const int crs = 9 * desc->C;
    for (int g = 0; g < lay.grid_n; ++g) {
        filter_checksum_i8_kernel<<<dim3((crs + 63) / 64), dim3(1024), 0, (hipStream_t)stream>>>(
            w + (long long)g * lay.tile_n * crs, wchk + (long long)g * lay.d_f * crs, lay.tile_n, crs, lay.d_f);
        LAUNCH_CHECK("filter_checksum_i8_kernel (per filter tile)");
    }
    return ABED_OK;
}

abed_status_t abed_input_checksum_int8(const abed_conv_desc_t *desc, const int8_t *x, int8_t *xchk, void *stream)
{
    Plan pl;
    abed_status_t s = make_plan(desc, ABED_INT8, ABED_NONE, false, pl);
    if (s != ABED_OK) return s;
    if (!x || !xchk) return ABED_EINVAL;
    const long long hwc = (long long)desc->H * desc->W * desc->C;
    const long long chunks = hwc / 16;
    batch_checksum_i8_kernel<<<dim3((unsigned)((chunks + 31) / 32)), dim3(256), 0, (hipStream_t)stream>>>(x, xchk, desc->N, hwc, pl.d_i);
    LAUNCH_CHECK("batch_checksum_i8_kernel");
    return ABED_OK;
}

abed_status_t abed_filter_prepare_fp16(const abed_conv_desc_t *desc, const void *w, void *wchk, void *stream)
{
    Plan pl;
    abed_status_t s = make_plan(desc, ABED_FP16, ABED_NONE, false, pl);
    if (s != ABED_OK) return s;
    if (!w || !wchk) return ABED_EINVAL;
    filter_checksum_f16_kernel<<<dim3((pl.crs + 255) / 256), dim3(256), 0, (hipStream_t)stream>>>((const _Float16 *)w, (_Float16 *)wchk, desc->K, pl.crs);
    LAUNCH_CHECK("filter_checksum_f16_kernel");
    return ABED_OK;
}

abed_status_t abed_input_checksum_fp16(const abed_conv_desc_t *desc, const void *x, void *xchk, void *stream)
{
    Plan pl;
    abed_status_t s = make_plan(desc, ABED_FP16, ABED_NONE, false, pl);
    if (s != ABED_OK) return s;
    if (!x || !xchk) return ABED_EINVAL;
    const long long hwc = (long long)desc->H * desc->W * desc->C;
    const long long chunks = hwc / 8;
    batch_checksum_f16_kernel<<<dim3((unsigned)((chunks + 63) / 64)), dim3(256), 0, (hipStream_t)stream>>>((const _Float16 *)x, (_Float16 *)xchk, desc->N, hwc);
    LAUNCH_CHECK("batch_checksum_f16_kernel");
    return ABED_OK;
}

}  // extern "C"

namespace {

// abed_conv_int8; with validate_only every check is made and nothing is enqueued
abed_status_t conv_int8_impl(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w,
                             const int8_t *wchk, int8_t *xchk, int32_t compute_xchk,
                             void *y, const abed_epilogue_t *epi, int32_t variant,
                             uint32_t *flags, int8_t *xchk_next,
                             void *workspace, size_t workspace_bytes,
                             const abed_inject_t *inject, void *y2, void *stream, bool validate_only)
{
    hipStream_t st = (hipStream_t)stream;
    const bool int8_out = epi != nullptr;
    const bool local = (variant & ABED_LOCAL) != 0;
    Plan pl;
    abed_status_t s = make_plan(desc, ABED_INT8, variant & ~ABED_LOCAL, int8_out, pl);
    if (s != ABED_OK) return s;
    variant = pl.variant;                       // scheme selection is in pl.d_f / pl.d_i from here on
    if (!x || !w || !y) return ABED_EINVAL;
    if (int8_out && (!epi->scale || !epi->bias)) return ABED_EINVAL;
    if (local) {
        // checksums local to a workgroup: one launch, no workspace, no checksum images in memory
        if (variant != ABED_FUSED_OCG) return ABED_EUNSUPPORTED;
        BoxPlan bp;
        if ((s = make_box_plan(desc, pl.d_f > 0, pl.d_i > 0, bp)) != ABED_OK) return s;
        if ((bp.fc && !wchk) || !flags) return ABED_EINVAL;
        if (inject && inject->site != 0) {
            if (inject->site != 1) return inject->site == 2 ? ABED_EUNSUPPORTED : ABED_EINVAL;
            if (inject->index < 0 || inject->index >= (long long)desc->N * bp.P * bp.Q * desc->K || inject->bit < 0 || inject->bit > 31) return ABED_EINVAL;
        }
        if (validate_only) return ABED_OK;
        return launch_box_conv(desc, bp, x, w, wchk, y, epi, flags, inject, st);
    }
    const bool checked = variant >= ABED_UNFUSED && variant <= ABED_FUSED_IOCG;
    if (checked && ((pl.d_f && !wchk) || (pl.d_i && !xchk) || !flags)) return ABED_EINVAL;
    if (pl.packed && wchk != w + (long long)desc->K * pl.crs) return ABED_EINVAL;   // the digit filters must follow w in memory
    if (variant == ABED_DUPLICATE && (!y2 || !flags)) return ABED_EINVAL;
    if (variant == ABED_FUSED_IOCG && int8_out && !xchk_next) return ABED_EINVAL;
    if (checked && (!workspace || (long long)workspace_bytes < pl.ws_bytes)) return ABED_EWORKSPACE;
    if (inject && inject->site != 0) {
        if (inject->site != 1 && inject->site != 2) return ABED_EINVAL;
        if (inject->index < 0 || inject->index >= (long long)desc->N * pl.PQ * desc->K || inject->bit < 0 || inject->bit > 31)
            return ABED_EINVAL;
        if (inject->site == 2 && int8_out && !(variant == ABED_UNFUSED || variant == ABED_FUSED_WRITE)) return ABED_EUNSUPPORTED;
    }
    char *ws = (char *)workspace;
    auto wsp = [&](long long off) { return off < 0 ? (int32_t *)nullptr : (int32_t *)(ws + off); };
    const long long npqk = (long long)desc->N * pl.PQ * desc->K;
    const bool stored_flip = inject && inject->site == 2;

    if ((variant == ABED_UNFUSED || variant == ABED_FUSED_WRITE) && ((size_t)desc->N + desc->K + 2) * 4 > 64 * 1024)
        return ABED_EUNSUPPORTED;                                     // the verify kernel keeps N + K sums in LDS
    if (!tile_compiled(pl.wm, pl.wk, pl.kg)) return ABED_EUNSUPPORTED;   // before anything is enqueued
    if (validate_only) return ABED_OK;
    if (checked && compute_xchk && pl.d_i) {
        s = abed_input_checksum_int8(desc, x, xchk, stream);
        if (s != ABED_OK) return s;
    }

    if (variant == ABED_NONE) {
        if ((s = plain_conv(desc, x, w, y, epi, inject, st)) != ABED_OK) return s;
        if (stored_flip) flip_bit_u32_kernel<<<1, 1, 0, st>>>((uint32_t *)y, inject->index, 1u << inject->bit);
        return ABED_OK;
    }
    if (variant == ABED_DUPLICATE) {
        fill_u32_kernel<<<1, 64, 0, st>>>(flags, 1, 0u);
        if ((s = plain_conv(desc, x, w, y, epi, inject, st)) != ABED_OK) return s;
        if ((s = plain_conv(desc, x, w, y2, epi, nullptr, st)) != ABED_OK) return s;
        if (stored_flip) flip_bit_u32_kernel<<<1, 1, 0, st>>>((uint32_t *)y, inject->index, 1u << inject->bit);
        const long long bytes = npqk * (int8_out ? 1 : 4);
        compare_kernel<<<dim3((unsigned)((bytes / 16 + 256) / 256)), dim3(256), 0, st>>>(y, y2, bytes, flags);
        LAUNCH_CHECK("compare_kernel");
        return ABED_OK;
    }

    ConvParams cp;
    fill_params(cp, desc, pl);
    cp.x = x; cp.w = w; cp.wchk = wchk; cp.xchk = xchk; cp.y = y;
    cp.flags = flags; cp.xchk_next = xchk_next;
    if (int8_out) { cp.scale = epi->scale; cp.bias = epi->bias; cp.relu = epi->relu; cp.out_int8 = 1; }
    set_injection(cp, desc, pl, inject);
    const int grid = (pl.grid_m * pl.grid_b * pl.grid_n + 7) / 8 * 8;   // whole rounds over the 8 XCDs

    if (variant == ABED_UNFUSED || variant == ABED_FUSED_WRITE) {
        const size_t shm = ((size_t)desc->N + desc->K + 2) * 4;      // the verify kernel's LDS (checked above)
        int32_t *convout = int8_out ? wsp(pl.off_convout) : (int32_t *)y;
        int32_t *yf = wsp(pl.off_yf), *yi = wsp(pl.off_yi), *yfi = wsp(pl.off_yfi);
        if (variant == ABED_UNFUSED) {
            // one kernel per task (Sec. 4.3): the convolution, then the three checksum convolutions
            if ((s = plain_conv(desc, x, w, convout, nullptr, inject, st)) != ABED_OK) return s;
            abed_conv_desc_t df = *desc; df.K = pl.d_f;               // x * checksum filters
            if (pl.d_f && (s = plain_conv(&df, x, wchk, yf, nullptr, nullptr, st)) != ABED_OK) return s;
            abed_conv_desc_t di = *desc; di.N = pl.d_i;               // checksum images * w
            if (pl.d_i && (s = plain_conv(&di, xchk, w, yi, nullptr, nullptr, st)) != ABED_OK) return s;
            abed_conv_desc_t dfi = di; dfi.K = pl.d_f;                // checksum images * checksum filters
            if (pl.d_f && pl.d_i && (s = plain_conv(&dfi, xchk, wchk, yfi, nullptr, nullptr, st)) != ABED_OK) return s;
        } else {
            cp.y = convout;
            cp.out_int8 = 0;
            cp.mode = MODE_WRITE;
            cp.ws_yf = yf; cp.ws_yi = yi; cp.ws_yfi = yfi;
            if (!launch_conv(false, pl.wm, pl.wk, pl.kg, cp, grid, st)) return ABED_EUNSUPPORTED;
            LAUNCH_CHECK("conv_i8_kernel (augmented, write)");
        }
        if (stored_flip) flip_bit_u32_kernel<<<1, 1, 0, st>>>((uint32_t *)convout, inject->index, 1u << inject->bit);
        VerifyParams vp;
        vp.y = convout; vp.yf = yf; vp.yi = yi; vp.yfi = yfi; vp.flags = flags;
        vp.N = desc->N; vp.PQ = pl.PQ; vp.K = desc->K; vp.d_f = pl.d_f; vp.d_i = pl.d_i;
        vp.tile_batch = pl.mb; vp.tile_n = 16 * pl.wk; vp.grid_b = pl.grid_b; vp.grid_n = pl.grid_n;
        const long long words = (long long)pl.grid_m * pl.grid_b * pl.grid_n;
        fill_u32_kernel<<<dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st>>>(flags, words, 0u);
        LAUNCH_CHECK("fill_u32_kernel");
        verify_i8_kernel<<<dim3(pl.PQ), dim3(256), shm, st>>>(vp);
        LAUNCH_CHECK("verify_i8_kernel");
        if (int8_out) {
            epilog_i8_kernel<<<dim3((unsigned)((npqk / 4 + 256) / 256)), dim3(256), 0, st>>>(convout, (int8_t *)y, epi->scale, epi->bias, epi->relu, npqk, desc->K);
            LAUNCH_CHECK("epilog_i8_kernel");
        }
        return ABED_OK;
    }

    // variants 3, 4, 5
    cp.mode = variant == ABED_FUSED_PARTIAL_REDUCTION ? MODE_PARTIAL : (variant == ABED_FUSED_OCG ? MODE_CHECK : MODE_CHECK_NEXT);
    cp.cnt_fc = (uint32_t *)wsp(pl.off_cnt_fc);
    cp.cnt_ic = (uint32_t *)wsp(pl.off_cnt_ic);
    cp.ws_fc = wsp(pl.off_fc); cp.ws_ic = wsp(pl.off_ic); cp.ws_nx = wsp(pl.off_nx);
    if (!launch_conv(false, pl.wm, pl.wk, pl.kg, cp, grid, st)) return ABED_EUNSUPPORTED;
    LAUNCH_CHECK("conv_i8_kernel (augmented)");
    if (stored_flip) flip_bit_u32_kernel<<<1, 1, 0, st>>>((uint32_t *)y, inject->index, 1u << inject->bit);
    if (variant == ABED_FUSED_PARTIAL_REDUCTION) {
        FinishParams fp;
        fp.fc = pl.d_f ? cp.ws_fc : nullptr; fp.ic = pl.d_i ? cp.ws_ic : nullptr; fp.flags = flags;
        fp.N = desc->N; fp.kblk = pl.kblk; fp.tile_batch = pl.mb; fp.wk = pl.wk; fp.grid_b = pl.grid_b; fp.grid_n = pl.grid_n;
        finish_i8_kernel<<<dim3(pl.grid_m * (pl.grid_b + pl.grid_n)), dim3(256), 0, st>>>(fp);
        LAUNCH_CHECK("finish_i8_kernel");
    }
    return ABED_OK;
}

}  // namespace

extern "C" {

abed_status_t abed_conv_int8(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w,
                             const int8_t *wchk, int8_t *xchk, int32_t compute_xchk,
                             void *y, const abed_epilogue_t *epi, int32_t variant,
                             uint32_t *flags, int8_t *xchk_next,
                             void *workspace, size_t workspace_bytes,
                             const abed_inject_t *inject, void *y2, void *stream)
{
    return conv_int8_impl(desc, x, w, wchk, xchk, compute_xchk, y, epi, variant, flags, xchk_next,
                          workspace, workspace_bytes, inject, y2, stream, false);
}

abed_status_t abed_conv_int8_static(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w,
                                    const int8_t *wchk, int8_t *xchk, int32_t compute_xchk,
                                    void *y, const abed_epilogue_t *epi, int32_t variant,
                                    uint32_t *flags, int8_t *xchk_next,
                                    const abed_inject_t *inject, void *y2, void *stream)
{
    // the variants with checksums local to a workgroup use no scratch memory at all
    if (variant & ABED_LOCAL)
        return conv_int8_impl(desc, x, w, wchk, xchk, compute_xchk, y, epi, variant, flags, xchk_next, nullptr, 0, inject, y2, stream, false);
    // sized as abed_get_layout reports it (the int8-output case, which needs the most)
    Plan pl;
    abed_status_t s = make_plan(desc, ABED_INT8, variant, true, pl);
    if (s != ABED_OK) return s;
    if (pl.ws_bytes > (long long)ABED_STATIC_SCRATCH_BYTES) return ABED_EWORKSPACE;
    // this GPU's copy of the scratch array: looked up once per device, with that device current
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ABED_EUNSUPPORTED;
    void *ptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void *sym = nullptr;
            HIP_TRY(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
            if (!sym) return hip_fail(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
            g_scratch_ptr[dev] = sym;
        }
        ptr = g_scratch_ptr[dev];
    }
    // every argument check before the first launch
    s = conv_int8_impl(desc, x, w, wchk, xchk, compute_xchk, y, epi, variant, flags, xchk_next,
                       ptr, (size_t)ABED_STATIC_SCRATCH_BYTES, inject, y2, stream, true);
    if (s != ABED_OK) return s;
    // The array keeps the previous call's contents; only the arrival counters at its start must be
    // zero.  A fill kernel clears them (a memset node would not survive graph replays).
    const long long cnt_bytes = pl.off_cnt_ic + align256((long long)pl.grid_m * pl.grid_n * 4);
    const long long words = cnt_bytes / 4;
    fill_u32_kernel<<<dim3((unsigned)((words + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>((uint32_t *)ptr, words, 0u);
    LAUNCH_CHECK("fill_u32_kernel (static scratch)");
    return abed_conv_int8(desc, x, w, wchk, xchk, compute_xchk, y, epi, variant, flags, xchk_next,
                          ptr, (size_t)ABED_STATIC_SCRATCH_BYTES, inject, y2, stream);
}

// ---- traditional ABFT at the GEMM level (Sec. 5.3): the comparison system
namespace {
constexpr int kAbftParts = 2048;      // blocks of the row pass (each leaves one partial sum)
struct AbftPlan {
    long long M, m_pad;          // data rows; rows of the larger A' and C' (a multiple of 256: the GEMM runs as a 1x1 convolution over 16x16 planes)
    int Ng, Kg, d_a, d_b, ld;    // ld: columns of C' and rows of B' = Ng + d_b rounded up to a multiple of 4 (16-byte rows)
    long long off_a, off_b, off_c, off_sums, bytes;
};
abed_status_t make_abft_plan(int64_t M, int32_t Ng, int32_t Kg, AbftPlan &ap)
{
    if (M < 1 || Ng < 1 || Kg < 1) return ABED_EINVAL;
    if (Kg % 16 != 0 || Kg > 65536) return ABED_EUNSUPPORTED;            // 16-byte pieces; exact int32 accumulation (Sec. 4.1)
    ap.M = M; ap.Ng = Ng; ap.Kg = Kg;
    ap.d_a = digits_for_count(M); ap.d_b = digits_for_count(Ng);
    if (ap.d_a > 4 || ap.d_b > 4) return ABED_ERANGE;
    ap.m_pad = (M + ap.d_a + 255) / 256 * 256;
    ap.ld = (Ng + ap.d_b + 3) / 4 * 4;
    if (ap.m_pad * (long long)Kg >= 0x7ffffff0LL || ap.m_pad * (long long)ap.ld >= (1LL << 29) || (long long)ap.ld * Kg >= 0x7ffffff0LL) return ABED_EUNSUPPORTED;
    long long off = 0;
    auto take = [&](long long bytes) { long long o = off; off = align256(off + bytes); return o; };
    ap.off_a = take(ap.m_pad * (long long)Kg);
    ap.off_b = take((long long)ap.ld * Kg);
    ap.off_c = take(ap.m_pad * (long long)ap.ld * 4);
    ap.off_sums = take(((long long)Kg * 2 + ap.ld + kAbftParts + (Ng + 255) / 256 + 8) * 4);   // column sums of A, of B's rows, of C'; partial sums for the corner
    ap.bytes = off;
    return ABED_OK;
}
}  // namespace

abed_status_t abed_abft_gemm_get_layout(int64_t M, int32_t Ng, int32_t Kg, abed_abft_layout_t *out)
{
    if (!out) return ABED_EINVAL;
    AbftPlan ap;
    abed_status_t s = make_abft_plan(M, Ng, Kg, ap);
    if (s != ABED_OK) return s;
    memset(out, 0, sizeof(*out));
    out->d_a = ap.d_a; out->d_b = ap.d_b; out->rows_padded = ap.m_pad; out->ld_c = ap.ld;
    out->workspace_bytes = (uint64_t)ap.bytes; out->c_offset = (uint64_t)ap.off_c;
    return ABED_OK;
}

abed_status_t abed_abft_gemm_int8(int64_t M, int32_t Ng, int32_t Kg, const int8_t *A, const int8_t *B, int32_t *C,
                                  uint32_t *flags, void *workspace, size_t workspace_bytes, int32_t tasks,
                                  const abed_inject_t *inject, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    AbftPlan ap;
    abed_status_t s = make_abft_plan(M, Ng, Kg, ap);
    if (s != ABED_OK) return s;
    if (!A || !B || !C || !flags) return ABED_EINVAL;
    if (!workspace || (long long)workspace_bytes < ap.bytes) return ABED_EWORKSPACE;
    if (tasks == 0) tasks = ABED_ABFT_ALL_TASKS;
    if (inject && inject->site != 0) {
        if (inject->site != 2) return ABED_EUNSUPPORTED;                  // a bit of the stored larger output, between tasks 4 and 5
        if (inject->index < 0 || inject->index >= (M + ap.d_a) * (long long)ap.ld || inject->bit < 0 || inject->bit > 31) return ABED_EINVAL;
    }
    char *ws = (char *)workspace;
    int8_t *Ap = (int8_t *)(ws + ap.off_a), *Bp = (int8_t *)(ws + ap.off_b);
    int *Cp = (int *)(ws + ap.off_c), *sums = (int *)(ws + ap.off_sums);
    int *sumA = sums, *sumB = sums + Kg, *sumC = sums + 2 * Kg, *row_part = sumC + ap.ld, *col_part = row_part + kAbftParts;
    // about 512 blocks per launch: each ends with one global atomic per column, and atomics on one address are served one after the other
    auto chunk_rows = [](long long rows, int col_blocks) { long long r = (rows * col_blocks + 511) / 512; return (int)(r < 32 ? 32 : r); };
    const long long a_bytes = M * (long long)Kg, b_bytes = (long long)Ng * Kg;
    // the larger GEMM as a 1x1 convolution: m_pad / 256 images of 16x16 pixels, Kg channels, Ng + d_b filters
    abed_conv_desc_t gd;
    gd.N = (int32_t)(ap.m_pad / 256); gd.H = 16; gd.W = 16; gd.C = Kg; gd.K = ap.ld; gd.R = gd.S = 1;
    gd.stride_h = gd.stride_w = 1; gd.pad_h = gd.pad_w = 0;
    {
        Plan pl;
        if ((s = make_plan(&gd, ABED_INT8, ABED_NONE, false, pl)) != ABED_OK) return s;
        if (!tile_compiled(pl.wm, pl.wk, pl.kg)) return ABED_EUNSUPPORTED;
    }
    if (tasks & ABED_ABFT_TASK_COPY_IN) {
        // task 2: the operands into their larger buffers; the rows behind the checksum rows are zeros
        abft_copy_rows_kernel<<<dim3((unsigned)((a_bytes / 16 + 255) / 256)), dim3(256), 0, st>>>((const unsigned char *)A, (unsigned char *)Ap, 1, a_bytes, a_bytes, a_bytes);
        abft_copy_rows_kernel<<<dim3((unsigned)((b_bytes / 16 + 255) / 256)), dim3(256), 0, st>>>((const unsigned char *)B, (unsigned char *)Bp, 1, b_bytes, b_bytes, b_bytes);
        const long long tail = (ap.m_pad - M) * (long long)Kg / 4, tail_b = (ap.ld - Ng) * (long long)Kg / 4;
        fill_u32_kernel<<<dim3((unsigned)((tail + 255) / 256)), dim3(256), 0, st>>>((uint32_t *)(Ap + a_bytes), tail, 0u);
        fill_u32_kernel<<<dim3((unsigned)((tail_b + 255) / 256)), dim3(256), 0, st>>>((uint32_t *)(Bp + b_bytes), tail_b, 0u);
        LAUNCH_CHECK("abft copy in");
    }
    if (tasks & ABED_ABFT_TASK_CHECKSUMS) {
        // task 3: column checksum of A, checksum over the rows of B, as int8 digit rows behind the data
        const long long nsum = (long long)Kg * 2;
        fill_u32_kernel<<<dim3((unsigned)((nsum + 255) / 256)), dim3(256), 0, st>>>((uint32_t *)sums, nsum, 0u);
        const int units = Kg / 16, cb = (units + 255) / 256;
        const int rpb_a = chunk_rows(M, cb), rpb_b = chunk_rows(Ng, cb);
        abft_colsum_kernel<1><<<dim3(cb, (unsigned)((M + rpb_a - 1) / rpb_a)), dim3(256), 0, st>>>((const unsigned char *)Ap, M, units, Kg, rpb_a, sumA);
        abft_colsum_kernel<1><<<dim3(cb, (unsigned)((Ng + rpb_b - 1) / rpb_b)), dim3(256), 0, st>>>((const unsigned char *)Bp, Ng, units, Kg, rpb_b, sumB);
        abft_digits_kernel<<<dim3((Kg + 255) / 256), dim3(256), 0, st>>>(sumA, Kg, ap.d_a, Ap + a_bytes);
        abft_digits_kernel<<<dim3((Kg + 255) / 256), dim3(256), 0, st>>>(sumB, Kg, ap.d_b, Bp + b_bytes);
        LAUNCH_CHECK("abft checksums");
    }
    if (tasks & ABED_ABFT_TASK_GEMM) {
        if ((s = plain_conv(&gd, Ap, Bp, Cp, nullptr, nullptr, st)) != ABED_OK) return s;       // task 4
    }
    if (inject && inject->site == 2) flip_bit_u32_kernel<<<1, 1, 0, st>>>((uint32_t *)Cp, inject->index, 1u << inject->bit);
    if (tasks & ABED_ABFT_TASK_VERIFY) {
        // task 5: the output read once along its rows and once along its columns
        fill_u32_kernel<<<1, 64, 0, st>>>(flags, 8, 0u);
        fill_u32_kernel<<<dim3((unsigned)((ap.ld + 255) / 256)), dim3(256), 0, st>>>((uint32_t *)sumC, ap.ld, 0u);
        long long row_blocks = (M + 3) / 4; if (row_blocks > kAbftParts) row_blocks = kAbftParts;
        abft_row_check_kernel<<<dim3((unsigned)row_blocks), dim3(256), 0, st>>>(Cp, M, Ng, ap.d_b, ap.ld, flags, row_part);
        const int units = ap.ld / 4, cb = (units + 255) / 256, rpb = chunk_rows(M, cb);
        abft_colsum_kernel<4><<<dim3(cb, (unsigned)((M + rpb - 1) / rpb)), dim3(256), 0, st>>>((const unsigned char *)Cp, M, units, (long long)ap.ld * 4, rpb, sumC);
        const int col_blocks = (Ng + 255) / 256;
        abft_col_check_kernel<<<dim3(col_blocks), dim3(256), 0, st>>>(Cp, M, Ng, ap.d_a, ap.ld, sumC, flags, col_part);
        abft_corner_kernel<<<1, 256, 0, st>>>(Cp, M, Ng, ap.d_a, ap.d_b, ap.ld, row_part, (int)row_blocks, col_part, col_blocks, flags);
        LAUNCH_CHECK("abft verify");
    }
    if (tasks & ABED_ABFT_TASK_COPY_OUT) {
        // task 6: the result without its checksum rows and columns, in 16-byte pieces where the widths allow
        if (Ng % 4 == 0)
            abft_copy_rows_kernel<<<dim3((unsigned)((M * (Ng / 4) + 255) / 256)), dim3(256), 0, st>>>((const unsigned char *)Cp, (unsigned char *)C, M, (long long)ap.ld * 4, (long long)Ng * 4, (long long)Ng * 4);
        else
            abft_copy_words_kernel<<<dim3((unsigned)((M * Ng + 255) / 256)), dim3(256), 0, st>>>(Cp, C, M, ap.ld, Ng);
        LAUNCH_CHECK("abft copy out");
    }
    return ABED_OK;
}

abed_status_t abed_pad_channels(const void *src, void *dst, int64_t rows, int32_t c, int32_t c_pad, int32_t elem_bytes,
                                void *stream)
{
    if (!src || !dst || rows < 1 || c < 1 || c_pad < c || (elem_bytes != 1 && elem_bytes != 2)) return ABED_EINVAL;
    if (rows * (long long)c_pad >= (1LL << 40)) return ABED_EUNSUPPORTED;
    const long long total = rows * c_pad;
    pad_channels_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream>>>(
        (const unsigned char *)src, (unsigned char *)dst, rows, c, c_pad, elem_bytes);
    LAUNCH_CHECK("pad_channels_kernel");
    return ABED_OK;
}

abed_status_t abed_conv_fp16(const abed_conv_desc_t *desc, const void *x, const void *w,
                             const void *wchk, void *xchk, int32_t compute_xchk,
                             void *y, int32_t out_fp32, int32_t variant, float rtol, float atol,
                             uint32_t *flags, void *workspace, size_t workspace_bytes,
                             const abed_inject_t *inject, void *y2, void *stream)
{
    hipStream_t st = (hipStream_t)stream;
    Plan pl;
    // the variants that verify from memory keep an fp32 ConvOut in the workspace when the caller's output is fp16
    abed_status_t s = make_plan(desc, ABED_FP16, variant, !out_fp32, pl);
    if (s != ABED_OK) return s;
    variant = pl.variant;
    if (!x || !w || !y) return ABED_EINVAL;
    const bool checked = variant >= ABED_UNFUSED && variant <= ABED_FUSED_IOCG;
    if (checked && ((pl.d_f && !wchk) || (pl.d_i && !xchk) || !flags)) return ABED_EINVAL;
    if (checked && !(rtol >= 0.f && atol >= 0.f)) return ABED_EINVAL;
    if (variant == ABED_FUSED_IOCG && !y2) return ABED_EINVAL;        // y2 takes the next layer's checksum images
    if (variant == ABED_DUPLICATE && (!y2 || !flags)) return ABED_EINVAL;
    if (checked && (!workspace || (long long)workspace_bytes < pl.ws_bytes)) return ABED_EWORKSPACE;
    if (inject && inject->site != 0) {
        if (inject->site != 1) return ABED_EUNSUPPORTED;
        if (inject->index < 0 || inject->index >= (long long)desc->N * pl.PQ * desc->K || inject->bit < 0 || inject->bit > 15)
            return ABED_EINVAL;
    }
    if (!tile_compiled(pl.wm, pl.wk, pl.kg)) return ABED_EUNSUPPORTED;   // before anything is enqueued
    char *ws = (char *)workspace;
    auto wsp = [&](long long off) { return off < 0 ? (int32_t *)nullptr : (int32_t *)(ws + off); };
    // an unchecked fp16 convolution of its own plan (the unfused variant's four convolutions)
    auto plain16 = [&](const abed_conv_desc_t *d, const void *xin, const void *win, void *out, int fp32_out,
                       const abed_inject_t *inj) -> abed_status_t {
        Plan pp;
        abed_status_t r = make_plan(d, ABED_FP16, ABED_NONE, false, pp);
        if (r != ABED_OK) return r;
        ConvParams c;
        fill_params(c, d, pp);
        c.x = (const int8_t *)xin; c.w = (const int8_t *)win; c.y = out; c.out_fp32 = fp32_out; c.mode = MODE_PLAIN;
        set_injection(c, d, pp, inj);
        const int g = (pp.grid_m * pp.grid_b * pp.grid_n + 7) / 8 * 8;
        if (!launch_conv(true, pp.wm, pp.wk, pp.kg, c, g, st)) return ABED_EUNSUPPORTED;
        LAUNCH_CHECK("conv_kernel (fp16, unchecked)");
        return ABED_OK;
    };
    if (checked && compute_xchk && pl.d_i) {
        s = abed_input_checksum_fp16(desc, x, xchk, stream);
        if (s != ABED_OK) return s;
    }
    ConvParams cp;
    fill_params(cp, desc, pl);
    cp.x = (const int8_t *)x; cp.w = (const int8_t *)w; cp.wchk = (const int8_t *)wchk; cp.xchk = (const int8_t *)xchk;
    cp.y = y; cp.flags = flags; cp.out_fp32 = out_fp32 ? 1 : 0; cp.rtol = rtol; cp.atol = atol; cp.l1 = pl.l1;
    set_injection(cp, desc, pl, inject);
    const int grid = (pl.grid_m * pl.grid_b * pl.grid_n + 7) / 8 * 8;   // whole rounds over the 8 XCDs
    const long long words = (long long)pl.grid_m * pl.grid_b * pl.grid_n;
    if (variant == ABED_NONE || variant == ABED_DUPLICATE) {
        cp.mode = MODE_PLAIN;
        if (variant == ABED_DUPLICATE) fill_u32_kernel<<<1, 64, 0, st>>>(flags, 1, 0u);
        if (!launch_conv(true, pl.wm, pl.wk, pl.kg, cp, grid, st)) return ABED_EUNSUPPORTED;
        if (variant == ABED_DUPLICATE) {
            cp.y = y2; cp.inj_on = 0;
            launch_conv(true, pl.wm, pl.wk, pl.kg, cp, grid, st);
            const long long bytes = (long long)desc->N * pl.PQ * desc->K * (out_fp32 ? 4 : 2);
            compare_kernel<<<dim3((unsigned)((bytes / 16 + 256) / 256)), dim3(256), 0, st>>>(y, y2, bytes, flags);
        }
        LAUNCH_CHECK("conv_kernel (fp16, unchecked)");
        return ABED_OK;
    }
    if (variant == ABED_UNFUSED || variant == ABED_FUSED_WRITE) {
        // Sec. 4.3 applied to fp16 (Sec. 7): ConvOut and the checksum fmaps go to memory as fp32, a verify kernel
        // reads them back, reduces and compares; the caller's fp16 output is rounded from the fp32 ConvOut last
        const long long npqk = (long long)desc->N * pl.PQ * desc->K;
        float *convout = out_fp32 ? (float *)y : (float *)wsp(pl.off_convout);
        float *yf = (float *)wsp(pl.off_yf), *yi = (float *)wsp(pl.off_yi), *yfi = (float *)wsp(pl.off_yfi);
        if (variant == ABED_UNFUSED) {
            if ((s = plain16(desc, x, w, convout, 1, inject)) != ABED_OK) return s;
            abed_conv_desc_t df = *desc; df.K = pl.d_f;               // x * checksum filters
            if (pl.d_f && (s = plain16(&df, x, wchk, yf, 1, nullptr)) != ABED_OK) return s;
            abed_conv_desc_t di = *desc; di.N = pl.d_i;               // checksum images * w
            if (pl.d_i && (s = plain16(&di, xchk, w, yi, 1, nullptr)) != ABED_OK) return s;
            abed_conv_desc_t dfi = di; dfi.K = pl.d_f;                // checksum images * checksum filters
            if (pl.d_f && pl.d_i && (s = plain16(&dfi, xchk, wchk, yfi, 1, nullptr)) != ABED_OK) return s;
        } else {
            cp.y = convout; cp.out_fp32 = 1; cp.mode = MODE_WRITE;
            cp.ws_yf = (int32_t *)yf; cp.ws_yi = (int32_t *)yi; cp.ws_yfi = (int32_t *)yfi;
            if (!launch_conv(true, pl.wm, pl.wk, pl.kg, cp, grid, st)) return ABED_EUNSUPPORTED;
            LAUNCH_CHECK("conv_kernel (fp16, augmented, write)");
        }
        VerifyF16Params vp;
        vp.y = convout; vp.yf = yf; vp.yi = yi; vp.yfi = yfi; vp.flags = flags;
        vp.N = desc->N; vp.PQ = pl.PQ; vp.K = desc->K; vp.d_f = pl.d_f; vp.d_i = pl.d_i;
        vp.tile_batch = pl.mb; vp.tile_n = 16 * pl.wk; vp.grid_b = pl.grid_b; vp.grid_n = pl.grid_n;
        vp.l1 = pl.l1; vp.rtol = rtol; vp.atol = atol;
        fill_u32_kernel<<<dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st>>>(flags, words, 0u);
        LAUNCH_CHECK("fill_u32_kernel");
        verify_f16_kernel<<<dim3(pl.PQ), dim3(256), 0, st>>>(vp);
        LAUNCH_CHECK("verify_f16_kernel");
        if (!out_fp32) {
            cast_f32_f16_kernel<<<dim3((unsigned)((npqk + 255) / 256)), dim3(256), 0, st>>>(convout, (_Float16 *)y, npqk);
            LAUNCH_CHECK("cast_f32_f16_kernel");
        }
        return ABED_OK;
    }
    cp.mode = variant == ABED_FUSED_PARTIAL_REDUCTION ? MODE_PARTIAL : (variant == ABED_FUSED_IOCG ? MODE_CHECK_NEXT : MODE_CHECK);
    cp.cnt_fc = (uint32_t *)wsp(pl.off_cnt_fc);
    cp.cnt_ic = (uint32_t *)wsp(pl.off_cnt_ic);
    cp.ws_fc = wsp(pl.off_fc); cp.ws_ic = wsp(pl.off_ic); cp.ws_nx = wsp(pl.off_nx);
    if (variant == ABED_FUSED_IOCG) cp.xchk_next = (int8_t *)y2;
    if (variant == ABED_FUSED_PARTIAL_REDUCTION) {
        fill_u32_kernel<<<dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st>>>(flags, words, 0u);
        LAUNCH_CHECK("fill_u32_kernel");
    }
    if (!launch_conv(true, pl.wm, pl.wk, pl.kg, cp, grid, st)) return ABED_EUNSUPPORTED;
    LAUNCH_CHECK("conv_kernel (fp16, augmented)");
    if (variant == ABED_FUSED_PARTIAL_REDUCTION) {
        FinishF16Params fp;
        fp.fc = pl.d_f ? (const float *)cp.ws_fc : nullptr; fp.ic = pl.d_i ? (const float *)cp.ws_ic : nullptr; fp.flags = flags;
        fp.N = desc->N; fp.kblk = pl.kblk; fp.tile_batch = pl.mb; fp.wk = pl.wk; fp.grid_b = pl.grid_b; fp.grid_n = pl.grid_n;
        fp.l1 = pl.l1; fp.rtol = rtol; fp.atol = atol;
        finish_f16_kernel<<<dim3(pl.grid_m * (pl.grid_b + pl.grid_n)), dim3(256), 0, st>>>(fp);
        LAUNCH_CHECK("finish_f16_kernel");
    }
    return ABED_OK;
}

}  // extern "C"
