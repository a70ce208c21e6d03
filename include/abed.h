/*
 * libabed: 2-D convolution with algorithm-based error detection (ABED) fused
 * in, for AMD gfx950.  C ABI, no C++ or framework types in any signature.
 *
 * The method (Hari, Sullivan, Tsai, Keckler, "Making Convolutions Resilient via
 * Algorithm-Based Error Detection Techniques"):
 *   FC, filter checksum (Sec. 3.1): a checksum filter wsum = sum_k w[k] is
 *     convolved with the input; the extra output fmap must equal sum_k y[.,k].
 *   IC option 1, batch checksum (Sec. 3.2): a checksum image xsum = sum_n x[n]
 *     is convolved with the filters; the extra batch entry must equal sum_n y[n].
 *   Both meet in a corner value conv(xsum, wsum) (row+column checksums, Sec. 2.1).
 *   int8 (Sec. 4.1): checksums are generated in int32 and stored as int8 digit
 *     tensors (balanced base 256); digit fmaps are recombined by shifts of
 *     8 bits per digit; all reductions and comparisons are made mod 2^32
 *     (the modular fallback named at the end of Sec. 4.1), equality is exact.
 *   fp16 (Sec. 7): checksums are stored as a hi/lo pair of fp16 tensors,
 *     accumulation is fp32, comparison is against a threshold.
 *   Variants (Sec. 4.3): how much of the checking is fused into the
 *     convolution kernel; the check is always made on the accumulators
 *     (ConvOut) before the epilog.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library
 *     never allocates, frees or synchronises.  Descriptor/epilogue/injection
 *     structs and the layout struct are HOST pointers, read during the call.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and the call returns without waiting.
 *   - Layouts: x[N][H][W][C], w[K][R][S][C] (R = filter height, S = width),
 *     y[N][P][Q][K]; P = (H + 2 pad_h - R)/stride_h + 1, Q likewise.
 *     Cross-correlation, dilation 1, one group, zero padding.
 *   - Every call returns an abed_status_t; nothing is thrown.
 *   - A workspace belongs to one call at a time: calls that may overlap on the device (different
 *     streams) need workspaces of their own; calls on one stream may share one, unless a call says
 *     that it leaves results in its workspace for a later call.  A status other than ABED_OK means
 *     that nothing was enqueued, except for ABED_EHIP, which reports a failed launch.
 */
#ifndef ABED_H
#define ABED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ABED_OK = 0,
    ABED_EINVAL = 1,        /* null / negative / inconsistent argument               */
    ABED_EUNSUPPORTED = 2,  /* valid convolution outside the implemented shape set    */
    ABED_EWORKSPACE = 3,    /* workspace smaller than abed_get_layout() reports        */
    ABED_EHIP = 4,          /* a HIP call failed (see abed_last_hip_error)             */
    ABED_ERANGE = 5         /* a checksum would need more than four digits (Sec. 4.1), or a
                               scheme's exact-arithmetic bound is exceeded (see its entry point) */
} abed_status_t;

/* Implementation options (Sec. 4.3).  All checked variants give the same
 * outputs and the same flags on a fault-free run. */
typedef enum {
    ABED_NONE = 0,                     /* unchecked convolution (the baseline)                         */
    ABED_UNFUSED = 1,                  /* one kernel per task: ICG, conv, checksum convs, verify, epilog */
    ABED_FUSED_WRITE = 2,              /* one augmented conv kernel writes ConvOut and the checksum fmaps;
                                          a verify kernel reads them back                              */
    ABED_FUSED_PARTIAL_REDUCTION = 3,  /* the conv kernel reduces inside each tile and writes partial
                                          sums; a small finish kernel compares                         */
    ABED_FUSED_OCG = 4,                /* the conv kernel reduces, compares and sets the flags itself  */
    ABED_FUSED_IOCG = 5,               /* as 4, and also emits the next layer's batch checksum from
                                          the epilog's output                                          */
    ABED_DUPLICATE = 6                 /* unchecked convolution twice + element-wise compare           */
} abed_variant_t;

/* Which checksums a checked variant (1..5) carries.  By default both: the filter checksum (FC,
 * Sec. 3.1) and the batch checksum image (IC option 1, Sec. 3.2), which also check each other.
 * OR one of these into the `variant` argument of abed_get_layout / abed_conv_int8 / abed_conv_fp16 to
 * run one scheme alone, with the protection Table 1 (Sec. 3.4) lists for it:
 *   ABED_ONLY_FC  the K filters and the block of checksum filters, no checksum images: d_i = 0, xchk is
 *                 not read and no input checksum kernel runs; only flag bit 0 can be set.  Not with
 *                 ABED_FUSED_IOCG (there is no batch checksum to hand on).
 *   ABED_ONLY_IC  the N images and the d_i checksum images, no checksum filters: d_f = 0, wchk is not
 *                 read; only flag bit 1 can be set.
 * Both at once, or either with ABED_NONE / ABED_DUPLICATE, is ABED_EINVAL. */
#define ABED_ONLY_FC 0x100
#define ABED_ONLY_IC 0x200
/* Space reserved for the checksum filters (Sec. 6.2: a layer whose filter count leaves room, as pruned
 * networks do, pays nothing for the larger convolution).  OR into ABED_FUSED_OCG / ABED_FUSED_IOCG (int8,
 * with or without ABED_ONLY_FC): the d_f checksum filters ride in the free rows of the last block of 16
 * filters instead of a block of their own.  Needs K % 16 != 0 and K % 16 + d_f <= 16 (else
 * ABED_EUNSUPPORTED), and the caller must keep filters and checksum filters in ONE buffer, wchk ==
 * w + K*R*S*C (else ABED_EINVAL).  Outputs and flags are those of the plain layout. */
#define ABED_PACKED_FC 0x400

/* Checksums local to a workgroup.  OR into ABED_FUSED_OCG (int8; with or without ABED_ONLY_FC / ABED_ONLY_IC):
 * the schemes of Sec. 3.1 and Sec. 3.2 option 1 are applied per tile instead of per layer, so that no tile
 * waits for another and no checksum tensor is made at run time:
 *   - FC per filter tile: every tile of tile_n filters carries the d_f = 2 digit filters of ITS OWN filters'
 *     sum; wchk is [grid_n][d_f][R][S][C], made offline by abed_filter_prepare_local_int8;
 *   - IC per batch tile: every range of tile_batch images carries the d_i = 2 digit images of ITS OWN images'
 *     sum, formed inside the convolution kernel from the inputs it stages (no input checksum kernel,
 *     xchk and compute_xchk are ignored, no workspace).
 * A tile is a box of 8x8 output pixels x tile_batch images x tile_n filters; flag word (box, batch tile,
 * filter tile) = flags[(box * grid_b + tb) * grid_n + tn] with box = (p / 8) * ceil(Q / 8) + q / 8, and every
 * bit is reported on the tile it was found in.  What is protected is what Table 1 (Sec. 3.4) lists for the
 * schemes; outputs are those of every other variant.  Shapes: 3x3 filters, stride 1, C and K multiples of 64,
 * C/64 in {1, 2, 4, 8} with the batch checksum; else ABED_EUNSUPPORTED. */
#define ABED_LOCAL 0x800

/* fp16 only (Sec. 7: the reduced values are compared "using a threshold", chosen by heuristics).  OR into
 * ABED_FUSED_OCG of abed_conv_fp16: the threshold is taken relative to the sum of magnitudes of the elements that
 * were reduced, tol = rtol * sum|y| + atol (sum over the real filters of the row for FC, over the real images for
 * IC, of the fp32 accumulators), instead of relative to the compared values.  Rounding error of a sum grows with
 * that norm, so sums that cancel to near zero no longer fail at atol = 0.  With int8 data or another variant:
 * ABED_EINVAL. */
#define ABED_L1_THRESHOLD 0x1000

typedef enum { ABED_INT8 = 0, ABED_FP16 = 1 } abed_dtype_t;

typedef struct {
    int32_t N, H, W, C, K, R, S;
    int32_t stride_h, stride_w, pad_h, pad_w;
} abed_conv_desc_t;

/* Epilog of Sec. 4.3 for the int8 path: ConvOut -> fp32, * scale[k], + bias[k]
 * (two separately rounded fp32 operations), ReLU if relu != 0, round to
 * nearest even, clamp to [-128,127].  scale and bias are device pointers to K
 * floats.  With a NULL epilogue the raw int32 ConvOut is the output. */
typedef struct {
    const float *scale;
    const float *bias;
    int32_t relu;
} abed_epilogue_t;

/* Fault injection for tests (Sec. 5.4 "Resilience Evaluation").  One bit of one
 * element is flipped:
 *   site 1 (ACC): accumulator of output element `index` (flat index into
 *     y[N][P][Q][K]) after the convolution loop, before the reductions and the store;
 *   site 2 (STORED): the stored ConvOut element `index`, after the convolution
 *     kernel and before any kernel that reads ConvOut back (only the variants that
 *     verify from memory, 1 and 2, can see it; int32 ConvOut only).
 * Flips in x, w, wchk or xchk need no library support: the caller owns those buffers. */
typedef struct {
    int32_t site;
    int64_t index;
    int32_t bit;
} abed_inject_t;

/* What abed_get_layout reports for one (convolution, dtype, variant).
 * A tile is tile_pixels consecutive output pixels (pixel index p*Q + q) x tile_batch
 * batch entries x tile_n filters.  For the checked variants the batch entries are
 * the N images followed by the d_i checksum images, and the filters are the K
 * filters (padded to a multiple of 16) followed by one block of 16 checksum filters. */
typedef struct {
    int32_t tile_pixels;   /* 16                                                             */
    int32_t tile_batch;    /* batch entries per tile                                         */
    int32_t tile_n;        /* filters per tile (a multiple of 16)                            */
    int32_t grid_m;        /* ceil(P*Q / tile_pixels)                                        */
    int32_t grid_b;        /* ceil(batch entries / tile_batch)                               */
    int32_t grid_n;        /* ceil(filter blocks * 16 / tile_n)                              */
    int32_t d_f, d_i;      /* checksum tensors per filter / batch checksum (0: scheme not selected) */
    int64_t n_flag_words;  /* grid_m * grid_b * grid_n uint32 words                          */
    int64_t workspace_bytes;
    int64_t wchk_bytes;    /* d_f * R*S*C elements                                           */
    int64_t xchk_bytes;    /* d_i * H*W*C elements                                           */
    int64_t xchk_next_bytes; /* d_i * P*Q*K elements (variant 5)                             */
    int32_t tile_box;      /* 0: a tile's pixels are consecutive in p*Q + q; 8: a box of 8x8 pixels (ABED_LOCAL) */
    int32_t local_checksums; /* 1: FC per filter tile, IC per batch tile, wchk is [grid_n][d_f][R][S][C]   */
    int32_t local_preferred; /* ABED_LOCAL layouts: 1 where the library's timing rule expects this form to be
                                faster than the layer-wide checksums for this shape, else 0                   */
    int32_t reserved_;
} abed_layout_t;

/* Flag word of tile (tm, tb, tn) is flags[(tm * grid_b + tb) * grid_n + tn].
 *   bit 0: FC mismatch (Sec. 3.1) in an output row (n,p,q): pixel in group tm, image n in
 *          batch tile tb = n / tile_batch; reported on tn = 0;
 *   bit 1: IC mismatch (Sec. 3.2 option 1) at a (p,q,k): pixel in group tm, channel k in
 *          filter tile tn = k / tile_n; reported on tb = 0;
 *   bit 2: the checksums disagree with each other at a pixel of group tm (the corner of
 *          the row+column scheme: the filter-sum of a checksum-image fmap or the batch-sum
 *          of a checksum-filter fmap differs from the fmap of checksum image x checksum
 *          filter); reported on some word of group tm.
 *   bit 3: not a checksum mismatch: an arrival counter of the workspace was not zero when the call started
 *          (abed_workspace_init not called on this workspace, or two calls used it at once), so some comparison
 *          that spans tiles was made early or not at all; the call's other flag bits cannot be trusted.
 *          Only variants 3..5 whose sums span tiles use the counters.
 * Every word is written on every checked call. */
#define ABED_FLAG_FC 1u
#define ABED_FLAG_IC 2u
#define ABED_FLAG_CORNER 4u
#define ABED_FLAG_WORKSPACE 8u

/* Host only.  Fills *out; ABED_EINVAL / ABED_EUNSUPPORTED / ABED_ERANGE as above. */
abed_status_t abed_get_layout(const abed_conv_desc_t *desc, int32_t dtype, int32_t variant,
                              abed_layout_t *out);

/* Offline step (Sec. 3.1, Sec. 4.1, Sec. 4.2): wsum = sum_k w[k] in int32, split
 * into d_f int8 digit filters wchk[d_f][R][S][C].  fp16: wsum in fp32, stored as
 * hi = fp16(wsum), lo = fp16(wsum - hi): wchk[2][R][S][C]. */
abed_status_t abed_filter_prepare_int8(const abed_conv_desc_t *desc, const int8_t *w, int8_t *wchk,
                                       void *stream);
abed_status_t abed_filter_prepare_fp16(const abed_conv_desc_t *desc, const void *w, void *wchk,
                                       void *stream);
/* The offline step for a given variant: with ABED_LOCAL the checksum filters of every filter tile
 * (wchk[grid_n][d_f][R][S][C], tile g = sum of filters g*tile_n .. (g+1)*tile_n - 1, split into digits as
 * above; Sec. 3.1, 4.1, 4.2), else exactly abed_filter_prepare_int8. */
abed_status_t abed_filter_prepare_local_int8(const abed_conv_desc_t *desc, int32_t variant, const int8_t *w,
                                             int8_t *wchk, void *stream);

/* Online input checksum generation, ICG (Sec. 3.2 option 1, Sec. 4.3): xsum =
 * sum_n x[n] in int32 (fp32), split into d_i digit images xchk[d_i][H][W][C]. */
abed_status_t abed_input_checksum_int8(const abed_conv_desc_t *desc, const int8_t *x, int8_t *xchk,
                                       void *stream);
abed_status_t abed_input_checksum_fp16(const abed_conv_desc_t *desc, const void *x, void *xchk,
                                       void *stream);

/* ------------------------------------------------------------------------------------------
 * The traditional ABFT technique at the GEMM level: the comparison system of Sec. 5.3 (results: Sec. 6.3), with
 * the row + column checksums that Sec. 2.1 recalls.  C[M][Ng] = A[M][Kg] . B[Ng][Kg]^T, int8 operands, int32
 * result (a convolution lowered to a GEMM has M = N*P*Q, Kg = C*R*S, Ng = K).  The call performs the paper's tasks
 * (2)-(6): copy A and B into larger buffers in the workspace, generate the column checksum of A and the checksum
 * over the rows of B as int8 digit rows (Sec. 4.1), run the larger GEMM (the library's unchecked 1x1 convolution),
 * verify the larger output by reading it once along its rows and once along its columns, copy the result to C.
 * `tasks` selects which of them run (0 = all; for timing them one by one, as the paper's breakdown does).
 * flags (8 words, device): [0] bit 0 a row sum disagrees, bit 1 a column sum, bit 2 the corner; [1], [2] numbers of
 * bad rows and columns; [3], [4] the largest bad row and column index (one bad row and one bad column locate a
 * single wrong element, the correction capability of the classical scheme).  inject: site 2 only, index =
 * row * ld_c + column of the larger output, flipped between tasks 4 and 5.  Kg must be a multiple of 16.
 * ------------------------------------------------------------------------------------------ */
#define ABED_ABFT_TASK_COPY_IN 1
#define ABED_ABFT_TASK_CHECKSUMS 2
#define ABED_ABFT_TASK_GEMM 4
#define ABED_ABFT_TASK_VERIFY 8
#define ABED_ABFT_TASK_COPY_OUT 16
#define ABED_ABFT_ALL_TASKS 31
typedef struct {
    int32_t d_a, d_b;            /* digit rows of A's column checksum, of the checksum over B's rows */
    int32_t ld_c, reserved_;     /* columns of the larger output (Ng + d_b rounded up to a multiple of 4) */
    int64_t rows_padded;         /* rows of the larger A and of the larger output (M + d_a rounded up to a multiple of 256) */
    uint64_t workspace_bytes;    /* the larger A, B and output, and the sums */
    uint64_t c_offset;           /* byte offset of the larger output inside the workspace (for tests) */
} abed_abft_layout_t;
/* Host only. */
abed_status_t abed_abft_gemm_get_layout(int64_t M, int32_t Ng, int32_t Kg, abed_abft_layout_t *out);
abed_status_t abed_abft_gemm_int8(int64_t M, int32_t Ng, int32_t Kg, const int8_t *A, const int8_t *B, int32_t *C,
                                  uint32_t *flags, void *workspace, size_t workspace_bytes, int32_t tasks,
                                  const abed_inject_t *inject, void *stream);

/* Channel padding for layers whose channel count the kernels do not take (C must be a multiple of 16 for int8,
 * 8 for fp16; the 3-channel first layer of a network, which the paper's own evaluation leaves out, Sec. 5.2):
 * dst[row][0..c_pad) = src[row][0..c) followed by zeros, for `rows` rows of elements of elem_bytes (1 or 2) bytes.
 * Use it once offline on the filters (rows = K*R*S) and per call on the activations (rows = N*H*W), then describe
 * the layer with C = c_pad: zero channels add nothing to the convolution or to any checksum, so outputs and checks
 * are those of the unpadded layer.  src and dst are device pointers and must not overlap. */
abed_status_t abed_pad_channels(const void *src, void *dst, int64_t rows, int32_t c, int32_t c_pad, int32_t elem_bytes,
                                void *stream);

/* Zero the part of a workspace that the library expects to be zero on first
 * use (arrival counters).  Call once after allocating a workspace. */
abed_status_t abed_workspace_init(void *workspace, size_t workspace_bytes, void *stream);

/* Checked int8 convolution (int32 accumulation; Sec. 3.1, 3.2, 4.1, 4.3).
 *   x, w        inputs, int8.
 *   wchk        from abed_filter_prepare_int8 (ignored for variants 0 and 6; may be NULL then).
 *   xchk        digit images of the batch checksum.  For checked variants the caller
 *               provides the buffer (xchk_bytes); if compute_xchk != 0 the call first
 *               runs the ICG kernel into it (counted as part of the variant), else it
 *               uses the contents as given (a previous layer's xchk_next, or a test's).
 *   y           int32[N][P][Q][K] if epilogue == NULL, else int8[N][P][Q][K].
 *   flags       n_flag_words words (checked variants), else may be NULL.
 *   xchk_next   variant 5 with an epilogue: int8[d_i][P][Q][K], the batch checksum
 *               digits of the int8 output; else NULL.
 *   workspace   workspace_bytes of scratch, 256-byte aligned.
 *   y2          variant 6 only: second output buffer of the same size as y; flags[0]
 *               is set to 1 if the two runs differ.
 * Errors: ABED_EINVAL (null pointer that is needed, bad descriptor),
 * ABED_EUNSUPPORTED (C not a multiple of 16, C*R*S > 65536, tensors of 2^31 elements or more),
 * ABED_EWORKSPACE, ABED_EHIP. */
abed_status_t abed_conv_int8(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w,
                             const int8_t *wchk, int8_t *xchk, int32_t compute_xchk,
                             void *y, const abed_epilogue_t *epilogue, int32_t variant,
                             uint32_t *flags, int8_t *xchk_next,
                             void *workspace, size_t workspace_bytes,
                             const abed_inject_t *inject, void *y2, void *stream);

/* abed_conv_int8 for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results, flags
 * and errors as abed_conv_int8, without `workspace`: the scratch memory is an array of
 * ABED_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the process ends.  The call
 * allocates and frees nothing.  A convolution whose layout reports workspace_bytes above
 * ABED_STATIC_SCRATCH_BYTES (the variants that keep ConvOut in the workspace, very large grids) is
 * refused with ABED_EWORKSPACE and nothing is enqueued.  All calls on one GPU share that GPU's array: the
 * call clears what must start at zero itself (no abed_workspace_init), and calls that may overlap on
 * one GPU (different streams, different threads) race - serialise them. */
#define ABED_STATIC_SCRATCH_BYTES (16u << 20)
abed_status_t abed_conv_int8_static(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w,
                                    const int8_t *wchk, int8_t *xchk, int32_t compute_xchk,
                                    void *y, const abed_epilogue_t *epilogue, int32_t variant,
                                    uint32_t *flags, int8_t *xchk_next,
                                    const abed_inject_t *inject, void *y2, void *stream);

/* Checked fp16 convolution (fp32 accumulation; Sec. 7).  As above with fp16
 * data; y is fp16 (out_fp32 == 0) or fp32.  All variants; with ABED_FUSED_IOCG y2 takes the next layer's
 * checksum images, fp16 [2][P][Q][K]: the hi/lo pair of the batch sum of the outputs rounded to fp16 (with
 * ABED_DUPLICATE y2 is the second output); the variants that verify from memory keep ConvOut and the checksum
 * fmaps as fp32 in the workspace and round the fp16 output from there.  inject: site 1 only, bit 0..15 of the
 * value rounded to fp16.  A check fails unless
 * |s - c| <= rtol * max(|s|, |c|) + atol, s the reduction of the real
 * accumulators and c the checksum-path value (with ABED_L1_THRESHOLD: rtol * sum|y| + atol);
 * a NaN or an infinity on either side is a failure. */
abed_status_t abed_conv_fp16(const abed_conv_desc_t *desc, const void *x, const void *w,
                             const void *wchk, void *xchk, int32_t compute_xchk,
                             void *y, int32_t out_fp32, int32_t variant, float rtol, float atol,
                             uint32_t *flags, void *workspace, size_t workspace_bytes,
                             const abed_inject_t *inject, void *y2, void *stream);

/* ------------------------------------------------------------------------------------------
 * FIC, the filter and input fmap checksum scheme (Sec. 3.3): one scalar check per convolution.
 *   wsum[r,s,c]  = sum_k w[k,r,s,c]                                   (filter checksum, offline, int32)
 *   X[r,s,c]     = sum over n and over all output positions (p,q) of the input element that
 *                  filter element (r,s,c) meets there                 (input fmap checksum, int32)
 *   dot          = sum_{r,s,c} X[r,s,c] * wsum[r,s,c]                 (int64)
 *   ocs          = sum of all ConvOut accumulators                    (output fmap checksum, int64)
 * and ocs must equal dot (bit widths: Sec. 4.1; tasks and their fusion: Sec. 4.3).  The convolution
 * runs with its original parameters: nothing is appended to it.  int8 only.
 *
 * The input checksum is kept in its row-wise form xrows[j,h,s,c] = sum over the images n of part j of
 * the batch and over the input columns that filter column s meets of x[n,h,w,c] (int32
 * [xrows_parts][H][S][C]; the kernel splits the batch into parts to have enough workgroups).
 * X[r,s,c] is the sum of xrows over the parts and over the input rows that filter row r meets;
 * that sum is formed together with the dot product.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    int64_t workspace_bytes;
    int64_t wsum_bytes;    /* R*S*C int32 */
    int64_t xrows_bytes;   /* xrows_parts*H*S*C int32 */
    int32_t xrows_parts;   /* parts of the batch summed separately */
    int64_t xsum_bytes;      /* H*W*C int32: batch sum of the input, handed over by the previous layer */
    int64_t xsum_next_bytes; /* P*Q*K int32: batch sum of this layer's int8 output, for the next layer */
} abed_fic_layout_t;

/* Host only.  variant: ABED_UNFUSED (one kernel per task), ABED_FUSED_OCG (output fmap checksum
 * generation fused into the convolution + epilog kernel) or ABED_FUSED_IOCG (as FUSED_OCG, and the
 * kernel also prepares the next layer's input checksum from its own epilog output, Sec. 4.3);
 * ABED_EUNSUPPORTED otherwise. */
abed_status_t abed_fic_get_layout(const abed_conv_desc_t *desc, int32_t variant, abed_fic_layout_t *out);

/* Offline (task 1 of Sec. 4.3): the filter checksum. */
abed_status_t abed_fic_filter_prepare_int8(const abed_conv_desc_t *desc, const int8_t *w, int32_t *wsum,
                                           void *stream);

/* Online input fmap checksum generation (task 2), row-wise form; one pass over x.  xrows has the
 * layout abed_fic_get_layout reports for the same variant. */
abed_status_t abed_fic_input_checksum_int8(const abed_conv_desc_t *desc, int32_t variant, const int8_t *x,
                                           int32_t *xrows, void *stream);

/* Convolution checked by FIC (tasks 2 to 7 of Sec. 4.3).
 *   wsum          from abed_fic_filter_prepare_int8.
 *   xrows         xrows_bytes, caller-provided; if compute_xrows != 0 the call first runs the input
 *                 checksum kernel into it, else it uses the contents as given (a test's).
 *   y, epilogue   as for abed_conv_int8.
 *   result        two int64 on the device: [0] = ocs, [1] = dot.
 *   flag          one word on the device: 1 if ocs != dot, else 0 (written on every call).
 *                 result and flag may both be NULL: the call then leaves its partial sums in the workspace
 *                 and makes no comparison; abed_fic_verify makes it later, for several layers in one launch
 *                 (each layer needs a workspace of its own until then).
 *   xsum_in       ABED_FUSED_IOCG only, else NULL: int32 [H][W][C], the batch sum of this layer's input that
 *                 the previous layer's call produced as its xsum_next.  If non-NULL the input checksum is
 *                 made from it instead of a pass over x (compute_xrows is ignored), and the call leaves the
 *                 buffer zero again.
 *   xsum_next     ABED_FUSED_IOCG with an epilogue, else NULL: int32 [P][Q][K]; the call ADDS the batch sum of
 *                 its int8 output to it.  The buffer must be zero on entry: zero it once when it is
 *                 allocated; the consuming call (its xsum_in) restores the zeros.
 *   workspace     workspace_bytes of scratch, 256-byte aligned (partial sums, ConvOut of the unfused option).
 * ABED_FUSED_OCG is two launches: the input checksum workgroups ride in front of the convolution's
 * tiles in one launch (they do not depend on each other), then a one-workgroup kernel adds up the
 * partial sums and compares.
 *   inject        site 1 (accumulator) for both variants; site 2 (stored ConvOut) for ABED_UNFUSED.
 * Errors as for abed_conv_int8; ABED_ERANGE if an input checksum entry could exceed int32
 * (128 * N*P*Q >= 2^31) or if R*S*C >= 32768 (the kernel adds four accumulators in 32 bits before it widens). */
abed_status_t abed_fic_conv_int8(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w,
                                 const int32_t *wsum, int32_t *xrows, int32_t compute_xrows,
                                 void *y, const abed_epilogue_t *epilogue, int32_t variant,
                                 int64_t *result, uint32_t *flag,
                                 int32_t *xsum_in, int32_t *xsum_next,
                                 void *workspace, size_t workspace_bytes,
                                 const abed_inject_t *inject, void *stream);

/* Probes of the machine's own ceilings, for roofline reports (no part of the method; for benchmark
 * programs that may not allocate or launch kernels of their own).  Enqueues on `stream`:
 *   kind 0: a register-resident loop of `iters` x 16 int8 matrix instructions (16x16x64) per wave on 256
 *           workgroups of 8 waves = 256 * 8 * iters * 16 * 32768 operations; a: device scratch, bytes >= 512 KiB;
 *   kind 1: `iters` fills of the `bytes` at a (16 bytes per lane);
 *   kind 2: `iters` copies of `bytes` from a to b.
 * ABED_EINVAL for other kinds, null pointers or too small a buffer. */
abed_status_t abed_probe(int32_t kind, void *a, void *b, size_t bytes, int32_t iters, void *stream);

const char *abed_status_string(abed_status_t status);
/* Text of the last HIP error seen by this thread's most recent failing call. */
const char *abed_last_hip_error(void);

/* The final sums and comparisons (last step of tasks 3 and 7 of Sec. 4.3; the paper leaves the comparison
 * to the host) of n_layers convolutions that were run by abed_fic_conv_int8 with result == flag == NULL, in
 * one launch per 32 layers.  descs, variants and workspaces are HOST arrays of n_layers entries (the
 * descriptor, variant and workspace pointer each layer's call was given); results (device, 2 * n_layers
 * int64: ocs, dot per layer) and flags (device, n_layers words) are written for every layer. */
abed_status_t abed_fic_verify(int32_t n_layers, const abed_conv_desc_t *descs, const int32_t *variants,
                              void *const *workspaces, int64_t *results, uint32_t *flags, void *stream);

/* ------------------------------------------------------------------------------------------
 * FIC with the input side formed inside the convolution's main loop (a fusion beyond those of Sec. 4.3).
 * The dot product of the scheme (Sec. 3.3) is also the sum, over all rows of the input patch matrix, of
 * row . filter checksum:  dot = sum_{n,p,q} sum_{r,s,c} x[n, p*stride_h - pad_h + r, q*stride_w - pad_w + s, c]
 * * wsum[r,s,c].  The tiles of the first filter tile hold exactly those rows in their operand fragments, so
 * they multiply them with the filter checksum as well (vector dot instructions against three base-256 digits
 * of wsum, exact) while the matrix units do the convolution: there is no second pass over x, no input checksum
 * tensor, and one launch (plus the one-workgroup comparison).  ocs, dot, the comparison and the flag are those
 * of abed_fic_conv_int8, bit for bit.
 * What it protects: the filters (against their offline checksum), the convolution arithmetic and the
 * accumulators, as FIC does.  A fault in x is seen only where the tiles of the other filter tiles read x
 * differently from the first; where a layer has a single filter tile the input is not protected (FC alone
 * has the same coverage, Table 1 of Sec. 3.4).  int8 only.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    int64_t workspace_bytes;
    int64_t wdig_bytes;    /* 3 * 64 * ceil(R*S*C / 64) int8 */
} abed_fic_inloop_layout_t;

/* Value for abed_fic_verify's variants[] that names a layer run by abed_fic_inloop_conv_int8. */
#define ABED_FIC_INLOOP 0x1000

/* Host only.  ABED_ERANGE if the three digits or a lane's 32-bit sums could overflow (K > 32768, R*S*C >=
 * 32768); ABED_EUNSUPPORTED if R*S*C exceeds about 8000 (the digits must fit the LDS left beside the tile:
 * 3 * 64 * ceil(R*S*C / 64) bytes, rounded up to the tile's wave groups, at most 24 KB). */
abed_status_t abed_fic_inloop_get_layout(const abed_conv_desc_t *desc, abed_fic_inloop_layout_t *out);

/* Offline: the filter checksum wsum[r,s,c] = sum_k w[k,r,s,c] as three balanced base-256 digits,
 * wdig[d][e] int8, e along (r,s,c), rows of 64 * ceil(R*S*C / 64) bytes, zero from R*S*C on. */
abed_status_t abed_fic_inloop_filter_prepare_int8(const abed_conv_desc_t *desc, const int8_t *w, int8_t *wdig,
                                                  void *stream);

/* The checked convolution.  x, w, y, epilogue, result, flag, workspace, inject (site 1 only), errors: as for
 * abed_fic_conv_int8; result == flag == NULL defers the comparison to abed_fic_verify (variant
 * ABED_FIC_INLOOP).  All pointers are device pointers except desc, epilogue and inject. */
abed_status_t abed_fic_inloop_conv_int8(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w,
                                        const int8_t *wdig, void *y, const abed_epilogue_t *epilogue,
                                        int64_t *result, uint32_t *flag,
                                        void *workspace, size_t workspace_bytes,
                                        const abed_inject_t *inject, void *stream);

/* ------------------------------------------------------------------------------------------
 * IC option 2 (Sec. 3.2): the input fmaps are reduced to a checksum tensor of the size of one filter
 * (the same X[r,s,c] as in the FIC scheme above, in the same row-wise form xrows), that tensor is
 * convolved with the K filters, which gives K values chk[k] = sum_{r,s,c} X[r,s,c] * w[k,r,s,c], and
 * the output fmaps reduced over batch, height and width, osum[k] = sum_{n,p,q} y[n,p,q,k], must equal
 * them element by element.  All sums int64 (Sec. 4.1).  Protects the computation and the input and
 * output fmaps, not the filters (Table 1 of Sec. 3.4).  int8 only.
 * ------------------------------------------------------------------------------------------ */
typedef struct {
    int64_t workspace_bytes;
    int64_t xrows_bytes;   /* xrows_parts*H*S*C int32 */
    int32_t xrows_parts;
    int32_t n_values;      /* K: flag words; result holds 2*K int64 */
} abed_ic2_layout_t;

/* Host only.  variant: ABED_UNFUSED (one kernel per task) or ABED_FUSED_OCG (the output sums are formed
 * in the convolution + epilog kernel); ABED_EUNSUPPORTED otherwise. */
abed_status_t abed_ic2_get_layout(const abed_conv_desc_t *desc, int32_t variant, abed_ic2_layout_t *out);

/* Convolution checked by IC option 2.
 *   xrows       xrows_bytes, caller-provided, in the layout abed_fic_input_checksum_int8 writes for the
 *               same variant; if compute_xrows != 0 the call makes it first (ABED_FUSED_OCG: by workgroups
 *               that ride in front of the convolution's tiles), else it uses the contents as given.
 *   y, epilogue as for abed_conv_int8.
 *   result      2*K int64 on the device: [0..K) = osum, [K..2K) = chk.
 *   flags       K words on the device: 1 where osum[k] != chk[k], else 0 (all written on every call).
 *   workspace   workspace_bytes of scratch, 256-byte aligned.
 *   inject      site 1 for both variants; site 2 (stored ConvOut) for ABED_UNFUSED.
 * Errors as for abed_fic_conv_int8. */
abed_status_t abed_ic2_conv_int8(const abed_conv_desc_t *desc, const int8_t *x, const int8_t *w,
                                 int32_t *xrows, int32_t compute_xrows,
                                 void *y, const abed_epilogue_t *epilogue, int32_t variant,
                                 int64_t *result, uint32_t *flags,
                                 void *workspace, size_t workspace_bytes,
                                 const abed_inject_t *inject, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ABED_H */
