// Integer GEMM / 3x3 and 1x1 convolution for channel counts that are a multiple of 8 but not of
// 64 (Method, "Matrix Multiplication": a layer with fewer input channels than the transform's
// order keeps H = I, e.g. the convolution on a 4- or 8-channel latent; such layers are small).
//
// The large kernels fetch 64-code chunks with 16-byte direct-to-LDS loads and so need rows that
// are whole chunks.  Here a workgroup of four waves owns a 64-pixel x 64-channel tile (one 32 x 32
// MFMA tile per wave) and walks K in chunks of 32 codes: 128 threads fetch one row's chunk each
// with four guarded dword loads (a dword past the end of the row is taken as zero codes, which
// is what pads K up to a multiple of 32; K is a multiple of 8, so validity is per dword), expand
// the nibbles to int8 (16 x code) and store 32 bytes to LDS; every wave then multiplies one
// 32 x 32 x 32 step.  A tap outside the image fetches zeros.  Per-pixel scales: one integer sum per
// tap, folded into the fp32 result with the scale of the input pixel under the tap; one scale for
// the tensor: one integer sum over all taps.
#include "hq_int_gemm_kernel.h"

namespace {

struct AnyKArgs {
    const uint8_t *xq;   // [pixels, k/2]
    const float *sx;     // [pixels], or one value (sx_static)
    const uint8_t *wq;   // [n, taps, k/2]
    const float *sw;     // [n]
    const void *bias;    // [n] of the output dtype, or null
    void *y;             // [pixels, n]; integer output: [pixels, taps, n] (per-pixel scales) or [pixels, n]
    uint32_t pixels;
    int n, k, h, w, taps;   // taps 1 (linear / 1x1) or 9 (3x3, stride 1, pad 1)
    int sx_static;
    uint32_t n_co_tiles;
};

template <int OUT>
__global__ __launch_bounds__(256) void int_gemm_anyk_kernel(AnyKArgs a) {
    constexpr bool INT_OUT = OUT == kOutI32;
    using Out = typename OutT<OUT>::type;
    __shared__ __attribute__((aligned(16))) uint8_t s_a[64 * 32];   // weight rows: [row][first 16 | second 16] int8
    __shared__ __attribute__((aligned(16))) uint8_t s_b[64 * 32];   // activation rows

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;          // channel half, pixel half of the tile
    const int kbytes = a.k >> 1;
    const int chunks = (kbytes + 15) / 16;            // 32-code chunks, the last one possibly short
    const uint32_t tile = blockIdx.x;
    const int co0 = static_cast<int>(tile % a.n_co_tiles) * 64;
    const uint32_t p0 = (tile / a.n_co_tiles) * 64;

    // the row this thread fetches: threads 0..63 weight rows, 64..127 activation rows
    const bool loads_a = tid < 64, loads_b = tid >= 64 && tid < 128;
    const int lr = tid & 63;
    const int my_co = co0 + lr;
    const uint32_t my_pix = p0 + lr;
    int my_oh = 0, my_ow = 0;
    if (a.taps == 9) {
        const uint32_t q = my_pix / static_cast<uint32_t>(a.w);
        my_ow = static_cast<int>(my_pix - q * a.w);
        my_oh = static_cast<int>(q % static_cast<uint32_t>(a.h));
    }

    // this lane's output pixel (column lrow of the wave's MFMA tile) and its tap masks
    const uint32_t out_pix = p0 + wn * 32 + lrow;
    int out_mask = a.taps == 9 ? tap_mask<9>(out_pix < a.pixels ? out_pix : 0, a.h, a.w) : 1;
    if (out_pix >= a.pixels) out_mask = 0;

    float facc[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) facc[r] = 0.f;
    v16i acc;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0;

    for (int tap = 0; tap < a.taps; ++tap) {
        const int dr = a.taps == 9 ? tap / 3 - 1 : 0, ds = a.taps == 9 ? tap % 3 - 1 : 0;
        if (!a.sx_static || tap == 0) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0;
        }
        for (int ch = 0; ch < chunks; ++ch) {
            // ---- fetch and expand one row's chunk ------------------------------------------------
            if (loads_a || loads_b) {
                const uint8_t *src = nullptr;
                if (loads_a) {
                    if (my_co < a.n) src = a.wq + (static_cast<uint64_t>(my_co) * a.taps + tap) * kbytes;
                } else if (my_pix < a.pixels) {
                    const int ih = my_oh + dr, iw = my_ow + ds;
                    if (a.taps == 1 || (ih >= 0 && ih < a.h && iw >= 0 && iw < a.w))
                        src = a.xq + (static_cast<uint64_t>(my_pix) + static_cast<int64_t>(dr) * a.w + ds) * kbytes;
                }
                v4i p = {0, 0, 0, 0};
                if (src) {
                    const uint32_t *s32 = reinterpret_cast<const uint32_t *>(src + ch * 16);
                    const int left = kbytes - ch * 16;   // bytes of the row from this chunk on (a multiple of 4)
                    if (left > 0) p.x = static_cast<int>(s32[0]);
                    if (left > 4) p.y = static_cast<int>(s32[1]);
                    if (left > 8) p.z = static_cast<int>(s32[2]);
                    if (left > 12) p.w = static_cast<int>(s32[3]);
                }
                v4i first, second;
                expand(p, first, second);
                v4i *dst = reinterpret_cast<v4i *>((loads_a ? s_a : s_b) + lr * 32);
                dst[0] = first;
                dst[1] = second;
            }
            __syncthreads();
            // ---- one 32 x 32 x 32 step per wave ------------------------------------------------------
            const v4i av = *reinterpret_cast<const v4i *>(s_a + (wm * 32 + lrow) * 32 + lhalf * 16);
            const v4i bv = *reinterpret_cast<const v4i *>(s_b + (wn * 32 + lrow) * 32 + lhalf * 16);
            acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(av, bv, acc, 0, 0, 0);
            __syncthreads();
        }
        // ---- end of a tap ------------------------------------------------------------------------------
        if (a.sx_static) continue;   // one sum over all taps
        if constexpr (INT_OUT) {
            int *yi = static_cast<int *>(a.y);
            if (out_pix < a.pixels) {
                const bool inside = (out_mask >> tap) & 1;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int c = co0 + wm * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                    if (c < a.n) yi[(static_cast<int64_t>(out_pix) * a.taps + tap) * a.n + c] = inside ? acc[r] >> 8 : 0;
                }
            }
        } else {
            float s = 0.f;
            if ((out_mask >> tap) & 1)
                s = a.sx[static_cast<int64_t>(out_pix) + static_cast<int64_t>(dr) * a.w + ds] * (1.0f / 256.0f);
#pragma unroll
            for (int r = 0; r < 16; ++r) facc[r] += s * static_cast<float>(acc[r]);
        }
    }

    if (out_pix >= a.pixels) return;
    if constexpr (INT_OUT) {
        if (a.sx_static) {
            int *yi = static_cast<int *>(a.y);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int c = co0 + wm * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                if (c < a.n) yi[static_cast<int64_t>(out_pix) * a.n + c] = acc[r] >> 8;
            }
        }
    } else {
        Out *y = static_cast<Out *>(a.y);
        const Out *bias = static_cast<const Out *>(a.bias);
        const float s1 = a.sx_static ? a.sx[0] * (1.0f / 256.0f) : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int c = co0 + wm * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
            if (c >= a.n) continue;
            const float v = a.sx_static ? s1 * static_cast<float>(acc[r]) : facc[r];
            y[static_cast<int64_t>(out_pix) * a.n + c] =
                static_cast<Out>(v * a.sw[c] + (bias ? to_float(bias[c]) : 0.f));
        }
    }
}

}  // namespace

// Linear / 1x1 (taps = 1) or 3x3, stride 1, pad 1 (taps = 9) for any k that is a multiple of 8.
hq_status hq_gemm_launch_anyk(const GemmArgs &g, int taps, hq_dtype y_dtype, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    if ((taps != 1 && taps != 9) || g.bits != 4 || (g.k & 7) != 0) return HQ_ERR_UNSUPPORTED;
    AnyKArgs a{};
    a.xq = g.xq; a.sx = g.sx; a.wq = g.wq; a.sw = g.sw; a.bias = g.bias; a.y = g.y;
    a.pixels = g.pixels; a.n = g.n; a.k = g.k; a.h = g.h; a.w = g.w; a.taps = taps; a.sx_static = g.sx_static;
    a.n_co_tiles = static_cast<uint32_t>((g.n + 63) / 64);
    const int64_t tiles = ((static_cast<int64_t>(g.pixels) + 63) / 64) * a.n_co_tiles;
    if (tiles > 0x7fffffffLL) return HQ_ERR_SHAPE;
    const dim3 grid(static_cast<unsigned>(tiles)), block(256);
    if (y_dtype == HQ_F16) hipLaunchKernelGGL((int_gemm_anyk_kernel<kOutF16>), grid, block, 0, stream, a);
    else if (y_dtype == HQ_F32) hipLaunchKernelGGL((int_gemm_anyk_kernel<kOutF32>), grid, block, 0, stream, a);
    else if (y_dtype == HQ_I32) hipLaunchKernelGGL((int_gemm_anyk_kernel<kOutI32>), grid, block, 0, stream, a);
    else return HQ_ERR_DTYPE;
    return check.status();
}
