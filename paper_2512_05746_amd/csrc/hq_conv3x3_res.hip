// Launcher of the 3x3 convolution with the int8 activation tile resident in LDS (the kernel and the
// choice of its configuration are in hq_conv3x3_res_kernel.h), for activations that arrive as codes.
#include "hq_conv3x3_res_kernel.h"


// True if the layer is one for this kernel: per-pixel scales, channel slices of 192, a pixel tile
// whose activations fit the LDS, and enough tiles to occupy at least half of the CUs.
bool hq_conv3x3_res_fits(int64_t pixels, int w, int c_in, int c_out) {
    ResPlan p;
    const int cus = hq::compute_units();
    return res_choose(pixels, w, c_in, c_out, cus, false, p) && 2 * p.tiles >= cus;
}

// Pixels per workgroup tile (256, 128 or 64) the kernel takes for this layer, plus 1 if the workgroup
// has four waves instead of eight; 0 if it does not serve the layer.
int hq_conv3x3_res_tile_pixels(int64_t pixels, int w, int c_in, int c_out) {
    ResPlan p;
    const int cus = hq::compute_units();
    if (!res_choose(pixels, w, c_in, c_out, cus, false, p) || 2 * p.tiles < cus) return 0;
    return (64 << p.pg_log2) + (p.nw_log2 == 2 ? 1 : 0);
}

hq_status hq_conv3x3_res_launch(const GemmArgs &g, hq_dtype y_dtype, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    ResPlan p;
    if (g.sx_static || !res_choose(g.pixels, g.w, g.k, g.n, hq::compute_units(), false, p)) return HQ_ERR_UNSUPPORTED;
    if (p.tiles > 0x7fffffffLL) return HQ_ERR_SHAPE;
    if (y_dtype != HQ_I32 && y_dtype != HQ_F16 && y_dtype != HQ_F32) return HQ_ERR_DTYPE;
    ResArgs a{};
    res_fill_args(a, g, p);
    if (y_dtype == HQ_I32) {
        const hq_status st = hq_fill_zero_launch(g.y, static_cast<uint64_t>(g.pixels) * 9 * g.n, stream);
        if (st != HQ_OK) return st;
    }
    res_launch_plan<false>(a, p, y_dtype, stream);
    return check.status();
}
