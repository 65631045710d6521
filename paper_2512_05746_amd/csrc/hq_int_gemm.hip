// Entry points of the integer GEMM / convolution: argument checks and the choice of the
// workgroup tile.  The kernels live in hq_int_gemm_kernel.h.
#include <math.h>

#include "hq_int_gemm_kernel.h"

namespace {

// Tile choice (measured on MI355X; all configurations share one kernel template):
//   - with at least two 64 x 128 tiles per CU, 64-channel tiles at three workgroups per CU win
//     even where 128-channel tiles waste nothing: three waves per SIMD hide the latencies of
//     the chunk loop better than two, which outweighs the extra nibble expansion;
//   - otherwise 128 x 128 tiles if there is at least one per CU;
//   - a layer with fewer tiles takes 64 x 64 tiles at four workgroups per CU.
hq_status launch_gemm(const GemmArgs &a, int taps, hq_dtype y_dtype, hipStream_t stream) {
    if ((a.bits == 8 ? a.k : a.k / 2) % 96 != 0) return hq_gemm_launch_128x128(a, taps, y_dtype, stream);
    const int64_t cus = hq::compute_units();
    const int64_t pix128 = (static_cast<int64_t>(a.pixels) + 127) / 128;
    if (a.n % 64 == 0 && pix128 * (a.n / 64) >= 2 * cus) return hq_gemm_launch_64x128(a, taps, y_dtype, stream);
    if (pix128 * ((a.n + 127) / 128) >= cus) return hq_gemm_launch_128x128(a, taps, y_dtype, stream);
    return hq_gemm_launch_64x64(a, taps, y_dtype, stream);
}

// The kernels index pixels with 32 bits and address the packed operands with
// 32-bit byte offsets; a 3x3 tap shifts an activation offset by up to w + 1 pixels
// before it is clamped, which must not wrap past 2^32 either.
bool fits_32bit(int64_t pixels, int w, int n, int taps, int k) {
    const int64_t lim = 0xFFFFFFFFLL;
    return pixels < 0x7FFFFFFFLL && (pixels + w + 2) * (k / 2) <= lim &&
           static_cast<int64_t>(n) * taps * (k / 2) <= lim;
}

// k_unit: what k must be a multiple of (64 for the kernels that fetch whole 64-code chunks; 8 where the
// kernel for other channel counts can take over)
hq_status check_common(const uint8_t *xq, const float *x_scale, const uint8_t *wq, const float *w_scale,
                       const void *bias, int64_t pixels, int n, int k, const void *y, hq_dtype y_dtype,
                       int k_unit = 64) {
    if (y_dtype != HQ_F16 && y_dtype != HQ_F32 && y_dtype != HQ_I32) return HQ_ERR_DTYPE;
    if (!xq || !wq || !y) return HQ_ERR_NULL;
    if (y_dtype != HQ_I32 && (!x_scale || !w_scale)) return HQ_ERR_NULL;
    if (pixels <= 0 || n <= 0 || k <= 0 || k % k_unit != 0 || k >= 131072) return HQ_ERR_SHAPE;
    if (!hq::aligned16(xq) || !hq::aligned16(wq) || !hq::aligned16(y)) return HQ_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(x_scale) & 3u) || (reinterpret_cast<uintptr_t>(w_scale) & 3u) ||
        (reinterpret_cast<uintptr_t>(bias) & 1u))
        return HQ_ERR_ALIGN;
    return HQ_OK;
}

// Which kernel serves a stride-1 convolution.  The choice depends on the shape only, never on the
// output type: the integer output (the raw sums) comes from the same kernel as the fp output.
enum ConvKernel { kConvKernelTile = 0, kConvKernelWave = 1, kConvKernelHalo = 2, kConvKernelRes = 3 };

ConvKernel choose_conv_kernel(int64_t pixels, int w, int c_in, int c_out, int r, int sx_static, int bits) {
    if (bits == 8 || r != 3) return kConvKernelTile;   // the other kernels expand nibbles, 3x3 only
    const int64_t cus = hq::compute_units();
    // At least one 64 x 256 tile per CU and image rows short enough for the packed activation tile of
    // the four-wave kernel that keeps it in LDS for all nine taps.
    const int64_t tiles256 = ((pixels + 255) / 256) * ((c_out + 63) / 64);
    GemmArgs probe{};
    probe.k = c_in;
    probe.w = w;
    probe.pixels = static_cast<uint32_t>(pixels);
    const bool halo_ok = tiles256 >= cus && hq_conv3x3_halo_fits(probe, HQ_F16);
    // Per-pixel scales and ONE 192-channel slice: that kernel is still the fastest (measured 30.4 against
    // 31.9 us on 64 x 64 x 192 at batch 16, buffers rotating through HBM).
    if (!sx_static && c_in == 192 && halo_ok) return kConvKernelHalo;
    // Per-pixel scales, 192-channel slices, an activation tile that fits the LDS as int8 and at least
    // half a tile per CU: the kernel with the expanded activation tile resident, whose workgroup
    // splits the K range over its waves so that one round of tiles fills the machine.
    if (!sx_static && hq_conv3x3_res_fits(pixels, w, c_in, c_out)) return kConvKernelRes;
    // A 3x3 layer with about one 64x64 output tile per CU or fewer cannot fill the machine with
    // whole tiles: it takes the kernel that also splits a tile's K range over waves.  (With one
    // scale for the tensor that kernel still combines per-tap sums in fp32, which equals the one
    // integer sum times one product of scales up to fp32 rounding.)
    const int64_t tiles64 = ((pixels + 63) / 64) * ((c_out + 63) / 64);
    if (c_in % 192 == 0 && tiles64 * 4 <= 5 * cus) return kConvKernelWave;
    // One scale for the tensor: no per-tap fold at all, the kernel with the packed activation tile in
    // LDS at three workgroups per CU.
    if (sx_static && halo_ok) return kConvKernelHalo;
    return kConvKernelTile;
}

}  // namespace

namespace {

// bits: 4 (packed pairs of codes) or 8 (int8 codes, one per byte)
hq_status int_linear(const uint8_t *xq, const float *x_scale, const uint8_t *wq, const float *w_scale,
                     const void *bias, int64_t m, int n, int k, void *y, hq_dtype y_dtype, int sx_static,
                     int bits, void *stream) {
    hq_status st = check_common(xq, x_scale, wq, w_scale, bias, m, n, k, y, y_dtype, bits == 4 ? 8 : 64);
    if (st != HQ_OK) return st;
    if (!fits_32bit(m, 1, n, 1, bits == 8 ? 2 * k : k)) return HQ_ERR_UNSUPPORTED;
    GemmArgs a{xq, x_scale, wq, w_scale, bias, y, static_cast<uint32_t>(m), n, k, 1, 1, 0, 0, 0, 1, sx_static,
               1.0f, bits};
    if (k % 64 != 0) return hq_gemm_launch_anyk(a, 1, y_dtype, static_cast<hipStream_t>(stream));
    return launch_gemm(a, 1, y_dtype, static_cast<hipStream_t>(stream));
}

// Linear layer of the Single scheme: the weights are three digit planes, the kernel keeps one
// integer sum per plane and weighs plane p by 16^p when it folds the sums into the fp32 result.
hq_status int_linear_single(const uint8_t *xq, const float *x_scale, const uint8_t *wq3, const float *w_scale,
                            const void *bias, int64_t m, int n, int k, int had_block, void *y, hq_dtype y_dtype,
                            void *stream) {
    hq_status st = check_common(xq, x_scale, wq3, w_scale, bias, m, n, k, y, y_dtype);
    if (st != HQ_OK) return st;
    if (!hq::pow2_upto_128(had_block) || k % had_block != 0) return HQ_ERR_SHAPE;
    if (!fits_32bit(m, 1, n, 3, k)) return HQ_ERR_UNSUPPORTED;
    const float norm = static_cast<float>(1.0 / sqrt(static_cast<double>(had_block)));
    GemmArgs a{xq, x_scale, wq3, w_scale, bias, y, static_cast<uint32_t>(m), n, k, 1, 1, 0, 0, 0, 1, 0, norm, 4};
    // |W_int H_raw| <= 8 x block: up to block 8 that is two signed base-16 digits ([-136, 119]) and the third
    // plane is zero, so its pass is skipped (the integer output keeps all three sums)
    const int planes = had_block <= 8 && y_dtype != HQ_I32 ? 2 : 3;
    return launch_gemm(a, planes, y_dtype, static_cast<hipStream_t>(stream));
}

hq_status int_conv2d(const uint8_t *xq, const float *x_scale, const uint8_t *wq, const float *w_scale,
                     const void *bias, int nb, int h, int w, int c_in, int c_out, int r, int s, int stride,
                     int pad, void *y, hq_dtype y_dtype, int sx_static, int bits, void *stream) {
    if (nb <= 0 || h <= 0 || w <= 0 || r <= 0 || s <= 0 || stride <= 0 || pad < 0) {
        if (!xq || !wq || !y) return HQ_ERR_NULL;
        return HQ_ERR_SHAPE;
    }
    const int64_t pixels = static_cast<int64_t>(nb) * h * w;
    hq_status st = check_common(xq, x_scale, wq, w_scale, bias, pixels, c_out, c_in, y, y_dtype,
                                bits == 4 && stride == 1 ? 8 : 64);   // (8-bit codes and stride 2: whole 64-code chunks)
    if (st != HQ_OK) return st;
    const bool down = r == 3 && s == 3 && stride == 2 && pad == 1 && !(bits == 8 && sx_static);   // the downsampling convolution
    if (!down && (r != s || (r != 1 && r != 3) || stride != 1 || pad != (r - 1) / 2)) return HQ_ERR_UNSUPPORTED;
    if (!fits_32bit(pixels, w, c_out, r * s, bits == 8 ? 2 * c_in : c_in)) return HQ_ERR_UNSUPPORTED;
    // one sum over all taps: 256 * (64 per product) * (codes per sum) must stay below 2^31
    if (sx_static && static_cast<int64_t>(c_in) * r * s >= 131072) return HQ_ERR_SHAPE;
    GemmArgs a{xq, x_scale, wq, w_scale, bias, y, static_cast<uint32_t>(pixels), c_out, c_in, h, w, 0, 0, 0, 1,
               sx_static, 1.0f, bits};
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    if (down) {   // output [nb, (h - 1) / 2 + 1, (w - 1) / 2 + 1, c_out]: the tile kernel's stride-2 form
        a.stride = 2;
        a.h_out = (h - 1) / 2 + 1;
        a.w_out = (w - 1) / 2 + 1;
        a.in_pixels = static_cast<uint32_t>(pixels);
        a.pixels = static_cast<uint32_t>(static_cast<int64_t>(nb) * a.h_out * a.w_out);
        return hq_gemm_launch_64x64(a, 9, y_dtype, st_);
    }
    if (c_in % 64 != 0) return hq_gemm_launch_anyk(a, r * s, y_dtype, st_);
    switch (choose_conv_kernel(pixels, w, c_in, c_out, r, sx_static, bits)) {
        case kConvKernelWave: return hq_conv3x3_wave_launch(a, y_dtype, st_);
        case kConvKernelHalo: return hq_conv3x3_halo_launch(a, y_dtype, st_);
        case kConvKernelRes: return hq_conv3x3_res_launch(a, y_dtype, st_);
        default: break;
    }
    return launch_gemm(a, r * s, y_dtype, st_);
}

// The paper's width-axis convolution: the activations arrive as three digit planes of the integers
// (X~ H_c)_int H_c,raw; the kernel walks 27 steps (plane-major), keeps one integer sum per plane
// over its nine taps (taps outside the image load zeros) and weighs plane p by 16^p.
hq_status int_conv2d_width(const uint8_t *xu3, const float *x_scale, const uint8_t *wq, const float *w_scale,
                           const void *bias, int nb, int h, int w, int c_in, int c_out, int r, int s, int stride,
                           int pad, int had_block, void *y, hq_dtype y_dtype, void *stream) {
    if (nb <= 0 || h <= 0 || w <= 0 || r <= 0 || s <= 0 || stride <= 0 || pad < 0) {
        if (!xu3 || !wq || !y) return HQ_ERR_NULL;
        return HQ_ERR_SHAPE;
    }
    const int64_t pixels = static_cast<int64_t>(nb) * h * w;
    hq_status st = check_common(xu3, x_scale, wq, w_scale, bias, pixels, c_out, c_in, y, y_dtype);
    if (st != HQ_OK) return st;
    if (!hq::pow2_upto_128(had_block) || had_block > 64 || w % had_block != 0) return HQ_ERR_SHAPE;
    if (r != 3 || s != 3 || (stride != 1 && stride != 2) || pad != 1) return HQ_ERR_UNSUPPORTED;
    // three planes of activations behind one 32-bit offset; 256 * 64 * (codes per plane sum) below 2^31
    if (!fits_32bit(3 * pixels, w, c_out, 9, c_in)) return HQ_ERR_UNSUPPORTED;
    if (static_cast<int64_t>(c_in) * 9 >= 131072) return HQ_ERR_SHAPE;
    const float norm = static_cast<float>(1.0 / sqrt(static_cast<double>(had_block)));
    GemmArgs a{xu3, x_scale, wq, w_scale, bias, y, static_cast<uint32_t>(pixels), c_out, c_in, h, w, 0, 0, 0, 1,
               1, norm, 4};
    if (stride == 2) {   // output [nb, (h - 1) / 2 + 1, (w - 1) / 2 + 1, c_out]: the tile kernel's stride-2 form
        a.stride = 2;
        a.h_out = (h - 1) / 2 + 1;
        a.w_out = (w - 1) / 2 + 1;
        a.in_pixels = static_cast<uint32_t>(pixels);
        a.pixels = static_cast<uint32_t>(static_cast<int64_t>(nb) * a.h_out * a.w_out);
        return hq_gemm_launch_64x64(a, had_block <= 8 ? 18 : 27, y_dtype, static_cast<hipStream_t>(stream));
    }
    // |q H_raw| <= 8 x block: up to block 8 the third digit plane is zero and its nine steps are skipped
    return launch_gemm(a, had_block <= 8 ? 18 : 27, y_dtype, static_cast<hipStream_t>(stream));
}

}  // namespace

extern "C" hq_status hq_int_linear(const uint8_t *xq, const float *x_scale, const uint8_t *wq,
                                   const float *w_scale, const void *bias, int64_t m, int n, int k,
                                   void *y, hq_dtype y_dtype, void *stream) {
    return int_linear(xq, x_scale, wq, w_scale, bias, m, n, k, y, y_dtype, 0, 4, stream);
}

extern "C" hq_status hq_int_linear_static(const uint8_t *xq, const float *x_scale, const uint8_t *wq,
                                          const float *w_scale, const void *bias, int64_t m, int n, int k,
                                          void *y, hq_dtype y_dtype, void *stream) {
    return int_linear(xq, x_scale, wq, w_scale, bias, m, n, k, y, y_dtype, 1, 4, stream);
}

extern "C" hq_status hq_int_conv2d(const uint8_t *xq, const float *x_scale, const uint8_t *wq,
                                   const float *w_scale, const void *bias, int nb, int h, int w, int c_in,
                                   int c_out, int r, int s, int stride, int pad, void *y, hq_dtype y_dtype,
                                   void *stream) {
    return int_conv2d(xq, x_scale, wq, w_scale, bias, nb, h, w, c_in, c_out, r, s, stride, pad, y, y_dtype, 0,
                      4, stream);
}

extern "C" hq_status hq_int_conv2d_static(const uint8_t *xq, const float *x_scale, const uint8_t *wq,
                                          const float *w_scale, const void *bias, int nb, int h, int w,
                                          int c_in, int c_out, int r, int s, int stride, int pad, void *y,
                                          hq_dtype y_dtype, void *stream) {
    return int_conv2d(xq, x_scale, wq, w_scale, bias, nb, h, w, c_in, c_out, r, s, stride, pad, y, y_dtype, 1,
                      4, stream);
}

extern "C" hq_status hq_int_linear_single(const uint8_t *xq, const float *x_scale, const uint8_t *wq3,
                                          const float *w_scale, const void *bias, int64_t m, int n, int k,
                                          int had_block, void *y, hq_dtype y_dtype, void *stream) {
    return int_linear_single(xq, x_scale, wq3, w_scale, bias, m, n, k, had_block, y, y_dtype, stream);
}

extern "C" hq_status hq_int_conv2d_width(const uint8_t *xu3, const float *x_scale, const uint8_t *wq,
                                         const float *w_scale, const void *bias, int nb, int h, int w,
                                         int c_in, int c_out, int r, int s, int stride, int pad,
                                         int had_block, void *y, hq_dtype y_dtype, void *stream) {
    return int_conv2d_width(xu3, x_scale, wq, w_scale, bias, nb, h, w, c_in, c_out, r, s, stride, pad, had_block,
                            y, y_dtype, stream);
}

extern "C" hq_status hq_int_linear_i8(const int8_t *xq, const float *x_scale, const int8_t *wq,
                                      const float *w_scale, const void *bias, int64_t m, int n, int k,
                                      void *y, hq_dtype y_dtype, void *stream) {
    return int_linear(reinterpret_cast<const uint8_t *>(xq), x_scale, reinterpret_cast<const uint8_t *>(wq), w_scale,
                      bias, m, n, k, y, y_dtype, 0, 8, stream);
}

extern "C" hq_status hq_int_conv2d_i8(const int8_t *xq, const float *x_scale, const int8_t *wq,
                                      const float *w_scale, const void *bias, int nb, int h, int w, int c_in,
                                      int c_out, int r, int s, int stride, int pad, void *y, hq_dtype y_dtype,
                                      void *stream) {
    return int_conv2d(reinterpret_cast<const uint8_t *>(xq), x_scale, reinterpret_cast<const uint8_t *>(wq), w_scale,
                      bias, nb, h, w, c_in, c_out, r, s, stride, pad, y, y_dtype, 0, 8, stream);
}

extern "C" const char *hq_int_conv2d_kernel_name(int nb, int h, int w, int c_in, int c_out, int r, int s, int stride,
                                                 int pad, int static_scale, int bits) {
    if (nb <= 0 || h <= 0 || w <= 0 || c_in <= 0 || c_out <= 0 || (bits != 4 && bits != 8)) return "unsupported";
    if (r == 3 && s == 3 && stride == 2 && pad == 1) return c_in % 64 == 0 ? "tile (stride 2)" : "unsupported";
    if (r != s || (r != 1 && r != 3) || stride != 1 || pad != (r - 1) / 2) return "unsupported";
    if (c_in % 8 != 0 || (bits == 8 && c_in % 64 != 0)) return "unsupported";
    if (c_in % 64 != 0) return "small-channel-count";
    switch (choose_conv_kernel(static_cast<int64_t>(nb) * h * w, w, c_in, c_out, r, static_scale, bits)) {
        case kConvKernelWave: return "wave-split";
        case kConvKernelHalo: return "activation-resident";
        case kConvKernelRes:
            switch (hq_conv3x3_res_tile_pixels(static_cast<int64_t>(nb) * h * w, w, c_in, c_out)) {
                case 256: return "activation-resident-int8 (256 pixels)";
                case 129: return "activation-resident-int8 (128 pixels, 4 waves)";
                case 128: return "activation-resident-int8 (128 pixels)";
                default: return "activation-resident-int8 (64 pixels)";
            }
        default: return "tile";
    }
}
