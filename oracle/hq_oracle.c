/*
 * CPU oracle for the Hadamard-quantised layer of HQ-DM (arxiv 2512.05746).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a deliberately plain, slow, fp64 / int64
 * statement of what the layer computes.  It shares no code, header, table or
 * helper with the HIP library; the product never calls it.
 *
 * Variant implemented (the paper leaves these open or the task fixes them):
 *   - H is the Sylvester matrix of the Background section ("Hadamard
 *     Transformation": H_0 = [1], H_k = 2^{-1/2} [[H,H],[H,-H]]), embedded
 *     block-diagonally over the contracted (input-channel) axis
 *     (Method, "Matrix Multiplication": H = BlockDiag(H_k x m), C_i = m 2^k).
 *     The transform is an explicit dense matrix product, not a butterfly.
 *   - The quantiser is the symmetric one of Background, "Model Quantization":
 *     X_int = clamp(round(X_fp / S), min, max), X_hat = S X_int, with
 *     round = round-half-to-even, [min, max] = [-2^(b-1), 2^(b-1)-1], and a
 *     dynamic abs-max scale S = max|row| / (2^(b-1)-1) (S = 1 for an all-zero
 *     row): one scale per token (pixel) for activations and one per output
 *     channel for weights.  (The paper trains S; the dynamic scale is the
 *     task's reading.)
 *   - The weights carry the same transform along their input-channel axis,
 *     applied offline before they are quantised, so the integer stage is
 *     (XH)_int (WH)_int^T.  In the paper's vocabulary (Method, "Single
 *     Hadamard Transformation") this is the arithmetic of the scheme that
 *     quantises H^T W offline; the un-rotated-weight form
 *     (XH)_int H W_int is not what this file computes.
 *   - Convolution transforms over input channels at every pixel (the paper
 *     transforms along the width axis instead), NHWC, taps [Cout,R,S,Cin].
 *     Because every input pixel has its own scale, the integer sum is kept
 *     per kernel tap and the taps are combined in floating point:
 *     y = s_w[co] * sum_t s_x[pixel_t] * acc_t  (+ bias).
 *   - Dequantisation is the product of scales of the Method section
 *     (Y ~ S_XH S_W (integer product)), in fp64, plus an optional bias.
 *   - Static mode (the *_static functions): the activation scale is one
 *     caller-supplied number for the whole tensor, as in the paper, where S
 *     is a learned parameter kept per timestep (Background, "Model
 *     Quantization"; Method, timestep-indexed quantisation parameters).  The
 *     clamp is then active (codes reach -2^(b-1)), and a convolution is the
 *     paper's form: ONE integer sum over all taps and input channels followed
 *     by one product of scales, y = S_x s_w[co] * sum + bias.
 *   - Single scheme (the *_single functions): the paper's own linear layer
 *     (Method, linear-layer equation and "Single Hadamard Transformation"):
 *     the weights are quantised WITHOUT the transform, W_int = Q(W), one
 *     abs-max scale per output channel, and the transform of the contracted
 *     axis stays in the integer domain between the two quantised operands:
 *         Y ~ S_XH S_W 2^(-k/2) ( (XH)_int  H_raw  W_int^T ),
 *     H_raw the +-1 matrix, block-diagonal over the input channels.  The steps
 *     are taken in that order: the activation codes times H_raw first
 *     (integers up to 8 * block in magnitude), then times the weight codes.
 *   - Width-axis convolution (the *_width functions): the paper's own
 *     convolution (Method, "Convolution"): the activation tensor is reshaped to
 *     rows of one image line each, (B C_in h) x w, and transformed along the
 *     WIDTH axis, X~ H_c with H_c = BlockDiag(H_k) of size w x w; it is quantised
 *     with one scale for the tensor; the weights are quantised without any
 *     transform; and
 *         Y ~ S S_W 2^(-k/2) Conv( (X~ H_c)_int H_c,raw , W_int ),
 *     i.e. the integer codes are taken back along the width axis with the +-1
 *     matrix (integers up to 8 * block in magnitude) and convolved with the
 *     integer weights, one integer sum over all taps and input channels.
 *
 * All arrays are row-major and owned by the caller.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the row loops below run on (for reporting next to timings). */
int hqo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Sylvester recursion without the 1/sqrt(2): h is n x n with entries +-1,
 * n a power of two.  (Background, "Hadamard Transformation".) */
void hqo_hadamard_raw(int n, double *h)
{
    h[0] = 1.0;
    for (int size = 1; size < n; size *= 2) {
        /* [[H, H], [H, -H]] built in place from the size x size top-left corner */
        for (int i = 0; i < size; ++i)
            for (int j = 0; j < size; ++j) {
                double v = h[(size_t)i * n + j];
                h[(size_t)i * n + (j + size)] = v;
                h[(size_t)(i + size) * n + j] = v;
                h[(size_t)(i + size) * n + (j + size)] = -v;
            }
    }
}

/* xt = x * BlockDiag(Hn), Hn = 2^{-k/2} Hraw of order `block`
 * (H_k = 2^{-k/2} H_k^raw).  x, xt: [m, k].  k must be a multiple of block.
 * block == 1 is the identity (the paper's bypass H = I).  Returns 0, or -1 on
 * a bad shape. */
int hqo_block_hadamard(const double *x, int64_t m, int k, int block, double *xt)
{
    if (block < 1 || (block & (block - 1)) != 0 || k % block != 0) return -1;
    double *hn = (double *)malloc(sizeof(double) * (size_t)block * block);
    if (!hn) return -1;
    hqo_hadamard_raw(block, hn);
    double norm = 1.0 / sqrt((double)block);
    for (int i = 0; i < block * block; ++i) hn[i] *= norm;

#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < m; ++r) {
        const double *xr = x + (size_t)r * k;
        double *yr = xt + (size_t)r * k;
        for (int b0 = 0; b0 < k; b0 += block)
            for (int j = 0; j < block; ++j) {
                double s = 0.0;
                for (int i = 0; i < block; ++i) s += xr[b0 + i] * hn[(size_t)i * block + j];
                yr[b0 + j] = s;
            }
    }
    free(hn);
    return 0;
}

/* Symmetric quantiser with one dynamic abs-max scale per row.
 * xt: [m, k] -> q: [m, k] codes, scale: [m], t: [m, k] pre-rounding values
 * xt / scale (t may be NULL). */
int hqo_quantize_rows(const double *xt, int64_t m, int k, int bits,
                      int8_t *q, double *scale, double *t)
{
    if (bits < 2 || bits > 8) return -1;
    const double qmax = (double)((1 << (bits - 1)) - 1);
    const double qmin = -(double)(1 << (bits - 1));
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < m; ++r) {
        const double *xr = xt + (size_t)r * k;
        double amax = 0.0;
        for (int j = 0; j < k; ++j) {
            double a = fabs(xr[j]);
            if (a > amax) amax = a;
        }
        double s = (amax > 0.0) ? amax / qmax : 1.0;
        scale[r] = s;
        for (int j = 0; j < k; ++j) {
            double v = xr[j] / s;
            if (t) t[(size_t)r * k + j] = v;
            double c = nearbyint(v); /* default rounding mode: ties to even */
            if (c < qmin) c = qmin;
            if (c > qmax) c = qmax;
            q[(size_t)r * k + j] = (int8_t)c;
        }
    }
    return 0;
}

/* acc[i, j] = sum_k xq[i, k] * wq[j, k], int64.  xq: [m, k], wq: [n, k]. */
void hqo_int_gemm(const int8_t *xq, const int8_t *wq, int64_t m, int n, int k, int64_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int j = 0; j < n; ++j) {
            int64_t s = 0;
            for (int c = 0; c < k; ++c)
                s += (int64_t)xq[(size_t)i * k + c] * (int64_t)wq[(size_t)j * k + c];
            acc[(size_t)i * n + j] = s;
        }
}

/* y[i, j] = acc[i, j] * sx[i] * sw[j] (+ bias[j]).  bias may be NULL. */
void hqo_dequant_linear(const int64_t *acc, const double *sx, const double *sw,
                        const double *bias, int64_t m, int n, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int j = 0; j < n; ++j) {
            double v = (double)acc[(size_t)i * n + j] * sx[i] * sw[j];
            if (bias) v += bias[j];
            y[(size_t)i * n + j] = v;
        }
}

/* Integer convolution with one accumulator per kernel tap, and its
 * dequantisation.
 *   xq: [nb, h, w, cin] codes, sx: [nb, h, w] scales,
 *   wq: [cout, r, s, cin] codes, sw: [cout], bias: [cout] or NULL.
 *   ho = (h + 2 pad - r) / stride + 1, wo likewise.
 *   acc_t: [nb, ho, wo, r*s, cout] int64, or NULL if not wanted.
 *   y:     [nb, ho, wo, cout] fp64, or NULL if not wanted.
 * A tap that falls outside the image contributes code 0 (zero padding commutes
 * with H because 0 H = 0).  Taps are combined in the order t = 0 .. r*s-1. */
int hqo_int_conv2d(const int8_t *xq, const double *sx, const int8_t *wq, const double *sw,
                   const double *bias, int nb, int h, int w, int cin, int cout,
                   int r, int s, int stride, int pad, int64_t *acc_t, double *y)
{
    if (stride < 1 || pad < 0 || h + 2 * pad < r || w + 2 * pad < s) return -1;
    const int ho = (h + 2 * pad - r) / stride + 1;
    const int wo = (w + 2 * pad - s) / stride + 1;
    const int taps = r * s;
#pragma omp parallel for schedule(static)
    for (int64_t pix = 0; pix < (int64_t)nb * ho * wo; ++pix) {
        const int b = (int)(pix / ((int64_t)ho * wo));
        const int p = (int)((pix / wo) % ho);
        const int q = (int)(pix % wo);
        for (int co = 0; co < cout; ++co) {
            double sum = 0.0;
            for (int t = 0; t < taps; ++t) {
                const int ih = p * stride + t / s - pad;
                const int iw = q * stride + t % s - pad;
                int64_t a = 0;
                double sxt = 0.0;
                if (ih >= 0 && ih < h && iw >= 0 && iw < w) {
                    const size_t ipix = ((size_t)b * h + ih) * w + iw;
                    const int8_t *xr = xq + ipix * cin;
                    const int8_t *wr = wq + ((size_t)co * taps + t) * cin;
                    for (int c = 0; c < cin; ++c) a += (int64_t)xr[c] * (int64_t)wr[c];
                    sxt = sx[ipix];
                }
                if (acc_t) acc_t[((size_t)pix * taps + t) * cout + co] = a;
                sum += sxt * (double)a;
            }
            if (y) {
                double v = sw[co] * sum;
                if (bias) v += bias[co];
                y[(size_t)pix * cout + co] = v;
            }
        }
    }
    return 0;
}

/* Symmetric quantiser with one caller-supplied scale for the whole tensor
 * (Background, "Model Quantization": X_int = clamp(round(X_fp / S), min, max)).
 * xt: [count] -> q: [count] codes, t: [count] pre-rounding values xt / scale
 * (t may be NULL).  scale must be positive and finite. */
int hqo_quantize_static(const double *xt, int64_t count, int bits, double scale, int8_t *q, double *t)
{
    if (bits < 2 || bits > 8 || !(scale > 0.0) || isinf(scale)) return -1;
    const double qmax = (double)((1 << (bits - 1)) - 1);
    const double qmin = -(double)(1 << (bits - 1));
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        double v = xt[i] / scale;
        if (t) t[i] = v;
        double c = nearbyint(v); /* default rounding mode: ties to even */
        if (c < qmin) c = qmin;
        if (c > qmax) c = qmax;
        q[i] = (int8_t)c;
    }
    return 0;
}

/* NHWC convolution with ONE activation scale for the tensor (Method,
 * "Convolution": integer convolution of the codes, then the product of scales).
 *   xq: [nb, h, w, cin], wq: [cout, r, s, cin], sw: [cout], bias: [cout] or NULL.
 *   acc: [nb, ho, wo, cout] int64 = sum over taps and input channels, or NULL.
 *   y:   [nb, ho, wo, cout] fp64 = sx * sw[co] * acc + bias, or NULL.
 * A tap outside the image contributes code 0. */
int hqo_int_conv2d_static(const int8_t *xq, double sx, const int8_t *wq, const double *sw,
                          const double *bias, int nb, int h, int w, int cin, int cout,
                          int r, int s, int stride, int pad, int64_t *acc, double *y)
{
    if (stride < 1 || pad < 0 || h + 2 * pad < r || w + 2 * pad < s) return -1;
    const int ho = (h + 2 * pad - r) / stride + 1;
    const int wo = (w + 2 * pad - s) / stride + 1;
#pragma omp parallel for schedule(static)
    for (int64_t pix = 0; pix < (int64_t)nb * ho * wo; ++pix) {
        const int b = (int)(pix / ((int64_t)ho * wo));
        const int p = (int)((pix / wo) % ho);
        const int q = (int)(pix % wo);
        for (int co = 0; co < cout; ++co) {
            int64_t a = 0;
            for (int kr = 0; kr < r; ++kr)
                for (int ks = 0; ks < s; ++ks) {
                    const int ih = p * stride + kr - pad;
                    const int iw = q * stride + ks - pad;
                    if (ih < 0 || ih >= h || iw < 0 || iw >= w) continue;
                    const int8_t *xr = xq + (((size_t)b * h + ih) * w + iw) * cin;
                    const int8_t *wr = wq + (((size_t)co * r + kr) * s + ks) * cin;
                    for (int c = 0; c < cin; ++c) a += (int64_t)xr[c] * (int64_t)wr[c];
                }
            if (acc) acc[(size_t)pix * cout + co] = a;
            if (y) {
                double v = sx * sw[co] * (double)a;
                if (bias) v += bias[co];
                y[(size_t)pix * cout + co] = v;
            }
        }
    }
    return 0;
}

/* Single scheme, integer stage (Method, linear-layer equation):
 * acc[i, j] = sum_c u[i, c] * wq[j, c]  with  u[i, :] = xq[i, :] * BlockDiag(H_raw),
 * H_raw the +-1 Sylvester matrix of size `block` (block = 1: u = xq).  All int64.
 * xq: [m, k] activation codes (of the transformed activations), wq: [n, k] codes of the
 * un-transformed weights.  Returns -1 if block does not divide k or is not a power of two. */
int hqo_int_gemm_single(const int8_t *xq, const int8_t *wq, int64_t m, int n, int k, int block,
                        int64_t *acc)
{
    if (block < 1 || (block & (block - 1)) || k % block) return -1;
    double *h = (double *)malloc(sizeof(double) * (size_t)block * block);
    if (!h) return -2;
    hqo_hadamard_raw(block, h);
    int failed = 0;
#pragma omp parallel
    {
        int64_t *u = (int64_t *)malloc(sizeof(int64_t) * (size_t)k);
        if (!u) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t i = 0; i < m; ++i) {
            if (!u) continue;
            const int8_t *xr = xq + (size_t)i * k;
            for (int b0 = 0; b0 < k; b0 += block)
                for (int c = 0; c < block; ++c) {
                    int64_t v = 0;
                    for (int e = 0; e < block; ++e)
                        v += (int64_t)xr[b0 + e] * (int64_t)h[(size_t)e * block + c];
                    u[b0 + c] = v;
                }
            for (int j = 0; j < n; ++j) {
                int64_t a = 0;
                for (int c = 0; c < k; ++c) a += u[c] * (int64_t)wq[(size_t)j * k + c];
                acc[(size_t)i * n + j] = a;
            }
        }
        free(u);
    }
    free(h);
    return failed ? -2 : 0;
}

/* Width-axis convolution, integer stage and dequantisation (Method, "Convolution"):
 *   u[b, i, :, c] = q[b, i, :, c] * BlockDiag(H_raw)   along the width axis (block | w),
 *   acc[b, p, q, co] = sum_{r, s, ci} u[b, p*st + r - pad, q*st + s - pad, ci] * wq[co, r, s, ci],
 *   y = sx * sw[co] * acc / sqrt(block) + bias[co].
 * xq: [nb, h, w, cin] codes of the width-transformed activations, wq: [cout, r, s, cin] codes
 * of the un-transformed weights.  acc / y: [nb, ho, wo, cout] or NULL.  Taps outside the image
 * contribute 0. */
int hqo_int_conv2d_width(const int8_t *xq, double sx, const int8_t *wq, const double *sw,
                         const double *bias, int nb, int h, int w, int cin, int cout, int r, int s,
                         int stride, int pad, int block, int64_t *acc, double *y)
{
    if (stride < 1 || pad < 0 || h + 2 * pad < r || w + 2 * pad < s) return -1;
    if (block < 1 || (block & (block - 1)) || w % block) return -1;
    const int ho = (h + 2 * pad - r) / stride + 1;
    const int wo = (w + 2 * pad - s) / stride + 1;
    double *hm = (double *)malloc(sizeof(double) * (size_t)block * block);
    int32_t *u = (int32_t *)malloc(sizeof(int32_t) * (size_t)nb * h * w * cin);
    if (!hm || !u) { free(hm); free(u); return -2; }
    hqo_hadamard_raw(block, hm);
    /* the codes times the +-1 matrix along the width axis */
#pragma omp parallel for schedule(static)
    for (int64_t line = 0; line < (int64_t)nb * h; ++line)
        for (int c = 0; c < cin; ++c)
            for (int b0 = 0; b0 < w; b0 += block)
                for (int j = 0; j < block; ++j) {
                    int32_t v = 0;
                    for (int e = 0; e < block; ++e)
                        v += (int32_t)xq[((size_t)line * w + b0 + e) * cin + c] * (int32_t)hm[(size_t)e * block + j];
                    u[((size_t)line * w + b0 + j) * cin + c] = v;
                }
    const double norm = 1.0 / sqrt((double)block);
#pragma omp parallel for schedule(static)
    for (int64_t pix = 0; pix < (int64_t)nb * ho * wo; ++pix) {
        const int b = (int)(pix / ((int64_t)ho * wo));
        const int p = (int)((pix / wo) % ho);
        const int q = (int)(pix % wo);
        for (int co = 0; co < cout; ++co) {
            int64_t a = 0;
            for (int kr = 0; kr < r; ++kr)
                for (int ks = 0; ks < s; ++ks) {
                    const int ih = p * stride + kr - pad;
                    const int iw = q * stride + ks - pad;
                    if (ih < 0 || ih >= h || iw < 0 || iw >= w) continue;
                    const int32_t *ur = u + (((size_t)b * h + ih) * w + iw) * cin;
                    const int8_t *wr = wq + (((size_t)co * r + kr) * s + ks) * cin;
                    for (int c = 0; c < cin; ++c) a += (int64_t)ur[c] * (int64_t)wr[c];
                }
            if (acc) acc[(size_t)pix * cout + co] = a;
            if (y) {
                double v = sx * sw[co] * (double)a * norm;
                if (bias) v += bias[co];
                y[(size_t)pix * cout + co] = v;
            }
        }
    }
    free(hm);
    free(u);
    return 0;
}
