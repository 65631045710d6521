/* Driver for the host-side sanitizer run of the CPU oracle: calls every function of
 * oracle/hq_oracle.c on small ragged inputs (block sizes 1..64, strides 1 and 2, pads 0 and 1,
 * optional outputs left NULL) and checks a few facts that need no second implementation
 * (H H^T = n I; codes in range; a one-hot row becomes a flat +-qmax pattern).  Built and run
 * with -fsanitize=address,undefined by tests/test_oracle_sanitizers.py: any out-of-bounds
 * access, use of uninitialised padding, signed overflow or misaligned access aborts the run. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int hqo_max_threads(void);
void hqo_hadamard_raw(int n, double *h);
int hqo_block_hadamard(const double *x, int64_t m, int k, int block, double *xt);
int hqo_quantize_rows(const double *xt, int64_t m, int k, int bits, int8_t *q, double *scale, double *t);
void hqo_int_gemm(const int8_t *xq, const int8_t *wq, int64_t m, int n, int k, int64_t *acc);
void hqo_dequant_linear(const int64_t *acc, const double *sx, const double *sw, const double *bias,
                        int64_t m, int n, double *y);
int hqo_int_conv2d(const int8_t *xq, const double *sx, const int8_t *wq, const double *sw,
                   const double *bias, int nb, int h, int w, int cin, int cout, int r, int s, int stride,
                   int pad, int64_t *acc_t, double *y);
int hqo_quantize_static(const double *xt, int64_t count, int bits, double scale, int8_t *q, double *t);
int hqo_int_conv2d_static(const int8_t *xq, double sx, const int8_t *wq, const double *sw,
                          const double *bias, int nb, int h, int w, int cin, int cout, int r, int s,
                          int stride, int pad, int64_t *acc, double *y);
int hqo_int_gemm_single(const int8_t *xq, const int8_t *wq, int64_t m, int n, int k, int block, int64_t *acc);
int hqo_int_conv2d_width(const int8_t *xq, double sx, const int8_t *wq, const double *sw,
                         const double *bias, int nb, int h, int w, int cin, int cout, int r, int s,
                         int stride, int pad, int block, int64_t *acc, double *y);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform(void) {   /* xorshift64*, in (-1, 1) */
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return (double)((rng_state * 0x2545F4914F6CDD1Dull) >> 11) / 4503599627370496.0 - 1.0;
}
static int fails = 0;
#define CHECK(c) do { if (!(c)) { printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #c); ++fails; } } while (0)

int main(void) {
    CHECK(hqo_max_threads() >= 1);
    for (int n = 1; n <= 64; n *= 2) {
        double *h = malloc(sizeof(double) * n * n);
        hqo_hadamard_raw(n, h);
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                double d = 0;
                for (int k = 0; k < n; ++k) d += h[i * n + k] * h[j * n + k];
                CHECK(d == (i == j ? n : 0));
            }
        free(h);
    }
    const int blocks[] = {1, 2, 8, 64};
    for (int bi = 0; bi < 4; ++bi) {
        const int block = blocks[bi], k = block * 3, m = 7, n = 5;
        double *x = malloc(sizeof(double) * m * k), *xt = malloc(sizeof(double) * m * k), *t = malloc(sizeof(double) * m * k);
        double *w = malloc(sizeof(double) * n * k), *wt = malloc(sizeof(double) * n * k);
        for (int i = 0; i < m * k; ++i) x[i] = uniform();
        for (int i = 0; i < n * k; ++i) w[i] = 0.02 * uniform();
        memset(x + 2 * k, 0, sizeof(double) * k);                 /* an all-zero row */
        memset(x + 3 * k, 0, sizeof(double) * k); x[3 * k] = -2.5;       /* a one-hot row */
        CHECK(hqo_block_hadamard(x, m, k, block, xt) == 0);
        CHECK(hqo_block_hadamard(w, n, k, block, wt) == 0);
        CHECK(hqo_block_hadamard(x, m, k, 3, xt) != 0);          /* not a power of two: refused */
        int8_t *xq = malloc(m * k), *wq = malloc(n * k);
        double *sx = malloc(sizeof(double) * m), *sw = malloc(sizeof(double) * n);
        for (int bits = 2; bits <= 8; ++bits) {
            CHECK(hqo_quantize_rows(xt, m, k, bits, xq, sx, t) == 0);
            CHECK(hqo_quantize_rows(wt, n, k, bits, wq, sw, NULL) == 0);
            const int qmax = (1 << (bits - 1)) - 1;
            for (int i = 0; i < m * k; ++i) CHECK(xq[i] >= -qmax - 1 && xq[i] <= qmax);
            CHECK(sx[2] == 1.0);
            for (int j = 0; j < block; ++j) CHECK(abs(xq[3 * k + j]) == qmax);   /* flat pattern of row 0 of H */
            int64_t *acc = malloc(sizeof(int64_t) * m * n);
            double *y = malloc(sizeof(double) * m * n);
            hqo_int_gemm(xq, wq, m, n, k, acc);
            hqo_dequant_linear(acc, sx, sw, NULL, m, n, y);
            hqo_dequant_linear(acc, sx, sw, sw, m, n, y);
            CHECK(hqo_int_gemm_single(xq, wq, m, n, k, block, acc) == 0);
            CHECK(hqo_quantize_static(xt, (int64_t)m * k, bits, 0.05, xq, t) == 0);
            CHECK(hqo_quantize_static(xt, (int64_t)m * k, bits, 0.05, xq, NULL) == 0);
            free(acc); free(y);
        }
        free(x); free(xt); free(t); free(w); free(wt); free(xq); free(wq); free(sx); free(sw);
    }
    /* convolutions: NHWC [nb, h, w, cin], weights [cout, r, s, cin]; strides 1, 2; pads 0, 1; 1x1 and 3x3 */
    const int nb = 2, h = 5, w = 8, cin = 8, cout = 3;
    int8_t *xq = malloc(nb * h * w * cin), *wq = malloc(cout * 9 * cin);
    double *sx = malloc(sizeof(double) * nb * h * w), sw[3] = {0.01, 0.02, 0.03}, bias[3] = {0.5, -0.5, 0.0};
    for (int i = 0; i < nb * h * w * cin; ++i) xq[i] = (int8_t)lrint(7.9 * uniform());
    for (int i = 0; i < cout * 9 * cin; ++i) wq[i] = (int8_t)lrint(7.9 * uniform());
    for (int i = 0; i < nb * h * w; ++i) sx[i] = 0.1 + fabs(uniform());
    for (int ks = 1; ks <= 3; ks += 2)
        for (int stride = 1; stride <= 2; ++stride)
            for (int pad = 0; pad <= 1; ++pad) {
                const int ho = (h + 2 * pad - ks) / stride + 1, wo = (w + 2 * pad - ks) / stride + 1;
                int64_t *acc_t = malloc(sizeof(int64_t) * nb * ho * wo * ks * ks * cout);
                int64_t *acc = malloc(sizeof(int64_t) * nb * ho * wo * cout);
                double *y = malloc(sizeof(double) * nb * ho * wo * cout);
                CHECK(hqo_int_conv2d(xq, sx, wq, sw, bias, nb, h, w, cin, cout, ks, ks, stride, pad, acc_t, y) == 0);
                CHECK(hqo_int_conv2d(xq, sx, wq, sw, NULL, nb, h, w, cin, cout, ks, ks, stride, pad, NULL, y) == 0);
                CHECK(hqo_int_conv2d(xq, sx, wq, sw, NULL, nb, h, w, cin, cout, ks, ks, stride, pad, acc_t, NULL) == 0);
                CHECK(hqo_int_conv2d_static(xq, 0.3, wq, sw, bias, nb, h, w, cin, cout, ks, ks, stride, pad, acc, y) == 0);
                CHECK(hqo_int_conv2d_static(xq, 0.3, wq, sw, NULL, nb, h, w, cin, cout, ks, ks, stride, pad, NULL, y) == 0);
                /* the per-tap sums add up to the one sum of the static form */
                for (int i = 0; i < nb * ho * wo; ++i)
                    for (int co = 0; co < cout; ++co) {
                        int64_t sum = 0;
                        for (int t = 0; t < ks * ks; ++t) sum += acc_t[((size_t)i * ks * ks + t) * cout + co];
                        CHECK(sum == acc[(size_t)i * cout + co]);
                    }
                for (int block = 1; block <= 8; block *= 2) {
                    CHECK(hqo_int_conv2d_width(xq, 0.3, wq, sw, bias, nb, h, w, cin, cout, ks, ks, stride, pad, block, acc, y) == 0);
                    CHECK(hqo_int_conv2d_width(xq, 0.3, wq, sw, NULL, nb, h, w, cin, cout, ks, ks, stride, pad, block, NULL, y) == 0);
                }
                free(acc_t); free(acc); free(y);
            }
    free(xq); free(wq); free(sx);
    printf(fails ? "oracle sanitizer driver: %d checks failed\n" : "oracle sanitizer driver: ok\n", fails);
    return fails ? 1 : 0;
}
