/*
 * CPU oracle (test infrastructure only): the plain definition of a 2-D
 * convolution as the paper states it in Sec. 2.2 ("each output feature map
 * value is a dot-product between a filter and a same-sized portion of the input
 * fmaps"), written as seven nested loops.  Nothing here is blocked, fused or
 * reordered.  Only tests, the smoke check and the benchmark's cpu_baseline leg
 * may use this file; the product path never does.
 *
 * Layouts: x[N][H][W][C], w[K][R][S][C], y[N][P][Q][K]; R is the filter height,
 * S the filter width; cross-correlation (no flip), dilation 1, one group;
 * positions outside the image read as zero.
 *   P = floor((H + 2*pad_h - R) / stride_h) + 1, Q likewise.
 *
 * The integer routine takes int32 operands so that the same loops serve the
 * int8 tensors and their int32 checksums (filter checksum, Sec. 3.1; batch
 * checksum, Sec. 3.2 option 1).  It accumulates in int64, which cannot
 * overflow for |x| < 2^31, |w| < 2^31 only if C*R*S is small; callers keep
 * |x|*|w|*C*R*S < 2^62 (true for int8 data and for the checksums of Sec. 4.1).
 * The caller reduces the int64 result mod 2^32 where the wrapped value is
 * wanted.
 */
#include <stdint.h>

void oracle_conv_i32(const int32_t *x, const int32_t *w, int64_t *y,
                     int N, int H, int W, int C, int K, int R, int S,
                     int stride_h, int stride_w, int pad_h, int pad_w)
{
    const int P = (H + 2 * pad_h - R) / stride_h + 1;
    const int Q = (W + 2 * pad_w - S) / stride_w + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int k = 0; k < K; ++k) {
                    int64_t acc = 0;
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < S; ++s) {
                            const int h = p * stride_h - pad_h + r;
                            const int v = q * stride_w - pad_w + s;
                            if (h < 0 || h >= H || v < 0 || v >= W)
                                continue;
                            for (int c = 0; c < C; ++c)
                                acc += (int64_t)x[(((int64_t)n * H + h) * W + v) * C + c] *
                                       (int64_t)w[(((int64_t)k * R + r) * S + s) * C + c];
                        }
                    y[(((int64_t)n * P + p) * Q + q) * K + k] = acc;
                }
}

/* Same loops in double precision: the reference for the fp16 path (Sec. 7:
 * fp16 inputs, exact products, a high-precision accumulator). */
void oracle_conv_f64(const double *x, const double *w, double *y,
                     int N, int H, int W, int C, int K, int R, int S,
                     int stride_h, int stride_w, int pad_h, int pad_w)
{
    const int P = (H + 2 * pad_h - R) / stride_h + 1;
    const int Q = (W + 2 * pad_w - S) / stride_w + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int p = 0; p < P; ++p)
            for (int q = 0; q < Q; ++q)
                for (int k = 0; k < K; ++k) {
                    double acc = 0.0;
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < S; ++s) {
                            const int h = p * stride_h - pad_h + r;
                            const int v = q * stride_w - pad_w + s;
                            if (h < 0 || h >= H || v < 0 || v >= W)
                                continue;
                            for (int c = 0; c < C; ++c)
                                acc += x[(((int64_t)n * H + h) * W + v) * C + c] *
                                       w[(((int64_t)k * R + r) * S + s) * C + c];
                        }
                    y[(((int64_t)n * P + p) * Q + q) * K + k] = acc;
                }
}

/* A few output elements only (sampled parity at full layer sizes): element e is
 * (n[e], p[e], q[e], k[e]); same arithmetic as oracle_conv_i32. */
void oracle_conv_i32_points(const int32_t *x, const int32_t *w, int64_t *y, int n_points,
                            const int32_t *pn, const int32_t *pp, const int32_t *pq, const int32_t *pk,
                            int N, int H, int W, int C, int K, int R, int S,
                            int stride_h, int stride_w, int pad_h, int pad_w)
{
    (void)N; (void)K;
#pragma omp parallel for schedule(static)
    for (int e = 0; e < n_points; ++e) {
        const int n = pn[e], p = pp[e], q = pq[e], k = pk[e];
        int64_t acc = 0;
        for (int r = 0; r < R; ++r)
            for (int s = 0; s < S; ++s) {
                const int h = p * stride_h - pad_h + r;
                const int v = q * stride_w - pad_w + s;
                if (h < 0 || h >= H || v < 0 || v >= W)
                    continue;
                for (int c = 0; c < C; ++c)
                    acc += (int64_t)x[(((int64_t)n * H + h) * W + v) * C + c] *
                           (int64_t)w[(((int64_t)k * R + r) * S + s) * C + c];
            }
        y[e] = acc;
    }
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
