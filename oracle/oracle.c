/*
 * CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain nested-loop definitions of the unfused operators whose composition a fused
 * primitive function computes (paper: Section 4.1, operator fusion -- a fused group is
 * the same expression factored into a function -- and Section 4.2, quantization, the
 * realized operator Q = cast(clip(round(x * 2^-s)))).  Floating point is carried in
 * double, the integer path in int64.  Tensors are NCHW, weights OIHW.  No blocking, no
 * fusion, no reordering: one loop nest per operator, sums taken in (c, r, s) order.
 *
 * Nothing in the product path may link or call this file; it shares no code with the
 * GPU kernels.  OpenMP only spreads independent (image, channel) pairs over cores.
 */
#include <stdint.h>
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* threads the loop nests below spread over */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* conv2d (cross-correlation, dilation 1, zero padding):
 *   y[n,k,p,q] = sum_{c,r,s} x[n,c,p*sh-ph+r,q*sw-pw+s] * w[k,c,r,s],  out-of-range x = 0
 *   Ho = floor((H + 2ph - R)/sh) + 1 (caller passes Ho, Wo).                              */
void oracle_conv2d_f64(const double *x, const double *w, double *y,
                       int N, int C, int H, int W, int K, int R, int S,
                       int sh, int sw, int ph, int pw, int Ho, int Wo)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int ih = p * sh - ph + r;
                                int iw = q * sw - pw + s;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                acc += x[(((size_t)n * C + c) * H + ih) * W + iw] *
                                       w[(((size_t)k * C + c) * R + r) * S + s];
                            }
                    y[(((size_t)n * K + k) * Ho + p) * Wo + q] = acc;
                }
}

/* Same contraction on int8 operands with an exact int64 sum. */
void oracle_conv2d_i8(const int8_t *x, const int8_t *w, int64_t *y,
                      int N, int C, int H, int W, int K, int R, int S,
                      int sh, int sw, int ph, int pw, int Ho, int Wo)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    int64_t acc = 0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                int ih = p * sh - ph + r;
                                int iw = q * sw - pw + s;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                acc += (int64_t)x[(((size_t)n * C + c) * H + ih) * W + iw] *
                                       (int64_t)w[(((size_t)k * C + c) * R + r) * S + s];
                            }
                    y[(((size_t)n * K + k) * Ho + p) * Wo + q] = acc;
                }
}

/* depthwise conv2d: one filter per channel, y[n,c,p,q] = sum_{r,s} x[n,c,..]*w[c,r,s]. */
void oracle_dwconv2d_f64(const double *x, const double *w, double *y,
                         int N, int C, int H, int W, int R, int S,
                         int sh, int sw, int ph, int pw, int Ho, int Wo)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    double acc = 0.0;
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < S; ++s) {
                            int ih = p * sh - ph + r;
                            int iw = q * sw - pw + s;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            acc += x[(((size_t)n * C + c) * H + ih) * W + iw] *
                                   w[((size_t)c * R + r) * S + s];
                        }
                    y[(((size_t)n * C + c) * Ho + p) * Wo + q] = acc;
                }
}

/* dense: y[m,j] = sum_i x[m,i] * w[j,i]  (one weight row per output unit). */
void oracle_dense_f64(const double *x, const double *w, double *y, int M, int Nout, int Kin)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int m = 0; m < M; ++m)
        for (int j = 0; j < Nout; ++j) {
            double acc = 0.0;
            for (int i = 0; i < Kin; ++i)
                acc += x[(size_t)m * Kin + i] * w[(size_t)j * Kin + i];
            y[(size_t)m * Nout + j] = acc;
        }
}

/* Elementwise operators on [N, K, HW] (HW = 1 for dense outputs), in place. */
void oracle_bias_add_f64(double *y, const double *b, int N, int K, int HW)
{
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int i = 0; i < HW; ++i)
                y[((size_t)n * K + k) * HW + i] += b[k];
}

/* folded batch norm: y = y*scale[k] + shift[k] (built with -ffp-contract=off: a rounded
 * product, then a rounded sum). */
void oracle_scale_shift_f64(double *y, const double *scale, const double *shift, int N, int K, int HW)
{
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int i = 0; i < HW; ++i) {
                size_t o = ((size_t)n * K + k) * HW + i;
                double prod = y[o] * scale[k];
                y[o] = prod + shift[k];
            }
}

void oracle_add_f64(double *y, const double *other, size_t count)
{
    for (size_t i = 0; i < count; ++i) y[i] += other[i];
}

void oracle_relu_f64(double *y, size_t count)
{
    for (size_t i = 0; i < count; ++i) y[i] = y[i] > 0.0 ? y[i] : 0.0;
}

/* Integer elementwise operators of the realized quantization (Section 4.2, "Realize"). */
void oracle_bias_add_i64(int64_t *y, const int64_t *b, int N, int K, int HW)
{
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int i = 0; i < HW; ++i)
                y[((size_t)n * K + k) * HW + i] += b[k];
}

/* residual brought to the accumulator's scale: y += res * 2^l, l >= 0 */
void oracle_add_lshift_i64(int64_t *y, const int8_t *res, int lshift, size_t count)
{
    for (size_t i = 0; i < count; ++i) y[i] += (int64_t)res[i] * ((int64_t)1 << lshift);
}

/* round(x * 2^-s), nearest with ties toward +inf: floor((x + 2^(s-1)) / 2^s); s = 0 is identity.
 * Floor division is written out with the remainder so that no shift of a negative is needed. */
void oracle_rshift_round_i64(int64_t *y, int s, size_t count)
{
    if (s == 0) return;
    const int64_t d = (int64_t)1 << s, half = (int64_t)1 << (s - 1);
    for (size_t i = 0; i < count; ++i) {
        int64_t t = y[i] + half;
        int64_t qt = t / d, rm = t % d;       /* C division truncates toward zero */
        if (rm < 0) qt -= 1;                  /* -> floor */
        y[i] = qt;
    }
}

void oracle_clip_i64(int64_t *y, int64_t lo, int64_t hi, size_t count)
{
    for (size_t i = 0; i < count; ++i) y[i] = y[i] < lo ? lo : (y[i] > hi ? hi : y[i]);
}

void oracle_relu_i64(int64_t *y, size_t count)
{
    for (size_t i = 0; i < count; ++i) y[i] = y[i] > 0 ? y[i] : 0;
}

/* cast to int8; returns the number of elements that did not fit (must be 0 after clip). */
size_t oracle_cast_i8(const int64_t *y, int8_t *out, size_t count)
{
    size_t bad = 0;
    for (size_t i = 0; i < count; ++i) {
        if (y[i] < -128 || y[i] > 127) ++bad;
        out[i] = (int8_t)y[i];
    }
    return bad;
}

/* number of elements outside int32 (the accumulator type the quantized path states) */
size_t oracle_count_outside_i32(const int64_t *y, size_t count)
{
    size_t bad = 0;
    for (size_t i = 0; i < count; ++i)
        if (y[i] < INT32_MIN || y[i] > INT32_MAX) ++bad;
    return bad;
}

/* Pools that chain the real layer shapes (standard architecture, not from the paper). */
void oracle_maxpool2d_f64(const double *x, double *y, int N, int C, int H, int W,
                          int R, int stride, int pad, int Ho, int Wo)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int p = 0; p < Ho; ++p)
                for (int q = 0; q < Wo; ++q) {
                    int have = 0;
                    double best = 0.0;
                    for (int r = 0; r < R; ++r)
                        for (int s = 0; s < R; ++s) {
                            int ih = p * stride - pad + r, iw = q * stride - pad + s;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            double v = x[(((size_t)n * C + c) * H + ih) * W + iw];
                            if (!have || v > best) { best = v; have = 1; }
                        }
                    y[(((size_t)n * C + c) * Ho + p) * Wo + q] = best;
                }
}

void oracle_global_avgpool_f64(const double *x, double *y, int N, int C, int HW)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            double acc = 0.0;
            for (int i = 0; i < HW; ++i) acc += x[((size_t)n * C + c) * HW + i];
            y[(size_t)n * C + c] = acc / (double)HW;
        }
}
