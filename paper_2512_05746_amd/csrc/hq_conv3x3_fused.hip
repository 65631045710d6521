// hq_act_quant_int_conv2d: the whole layer in one launch for a 3x3 convolution.  The fp16
// activations are transformed (block-64 Hadamard over the channels of every pixel), quantised with
// one abs-max scale per pixel, multiplied with the prepared weight codes and dequantised by the
// kernel of hq_conv3x3_res_kernel.h; the activation codes exist only in LDS.  (Method, "Matrix
// Multiplication": the transformed activations X H are only ever an operand of the integer
// product; Method, "Convolution".)
#include "hq_conv3x3_res_kernel.h"

extern "C" hq_status hq_act_quant_int_conv2d(const void *x, hq_dtype x_dtype, const uint8_t *wq, const float *w_scale,
                                             const void *bias, int nb, int h, int w, int c_in, int c_out, int r,
                                             int s, int stride, int pad, int had_block, int a_bits, void *y,
                                             hq_dtype y_dtype, uint8_t *xq_out, float *x_scale_out, void *stream) {
    if (!x || !wq || !y) return HQ_ERR_NULL;
    if (y_dtype != HQ_F16 && y_dtype != HQ_F32 && y_dtype != HQ_I32) return HQ_ERR_DTYPE;
    if (y_dtype != HQ_I32 && !w_scale) return HQ_ERR_NULL;
    if (x_dtype != HQ_F16 && x_dtype != HQ_F32) return HQ_ERR_DTYPE;
    if (nb <= 0 || h <= 0 || w <= 0 || c_in <= 0 || c_out <= 0 || r <= 0 || s <= 0 || stride <= 0 || pad < 0)
        return HQ_ERR_SHAPE;
    if (a_bits < 2 || a_bits > 4) return HQ_ERR_BITS;
    if (!hq::pow2_upto_128(had_block) || c_in % had_block != 0 || (c_in & 7) != 0 || c_in >= 131072) return HQ_ERR_SHAPE;
    if (!hq::aligned16(x) || !hq::aligned16(wq) || !hq::aligned16(y) || (xq_out && !hq::aligned16(xq_out)))
        return HQ_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(w_scale) & 3u) || (reinterpret_cast<uintptr_t>(x_scale_out) & 3u) ||
        (reinterpret_cast<uintptr_t>(bias) & 1u))
        return HQ_ERR_ALIGN;
    // built: fp16 activations, block 64, 3x3 / stride 1 / pad 1, channel slices of 192 and a tile that fits the LDS
    if (x_dtype != HQ_F16 || had_block != 64 || r != 3 || s != 3 || stride != 1 || pad != 1 || c_in % 192 != 0 ||
        c_in > 576)   // (the kernel keeps the fp16 pieces of up to three 192-channel slices of a row in registers)
        return HQ_ERR_UNSUPPORTED;
    const int64_t pixels = static_cast<int64_t>(nb) * h * w;
    // 32-bit pixel indices and weight offsets; the fp16 rows are addressed with 64 bits
    if (pixels >= 0x7FFFFFFFLL || static_cast<int64_t>(c_out) * 9 * (c_in / 2) > 0xFFFFFFFFLL) return HQ_ERR_UNSUPPORTED;
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    ResPlan p;
    if (!res_choose(pixels, w, c_in, c_out, hq::compute_units(), true, p)) return HQ_ERR_UNSUPPORTED;
    if (p.tiles > 0x7fffffffLL) return HQ_ERR_SHAPE;
    GemmArgs g{};
    g.wq = wq; g.sw = w_scale; g.bias = bias; g.y = y;
    g.pixels = static_cast<uint32_t>(pixels); g.n = c_out; g.k = c_in; g.h = h; g.w = w;
    ResArgs a{};
    res_fill_args(a, g, p);
    a.x = static_cast<const __half *>(x);
    a.qmax = static_cast<float>((1 << (a_bits - 1)) - 1);
    a.xq_out = xq_out;
    a.sx_out = x_scale_out;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (y_dtype == HQ_I32) {
        const hq_status zs = hq_fill_zero_launch(y, static_cast<uint64_t>(pixels) * 9 * c_out, st);
        if (zs != HQ_OK) return zs;
    }
    res_launch_plan<true>(a, p, y_dtype, st);
    return check.status();
}
