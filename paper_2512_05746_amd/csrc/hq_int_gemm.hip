// Integer GEMM / implicit-GEMM NHWC convolution on int8 MFMA with a dequantising
// epilogue (gfx950).  Method, linear-layer and "Convolution" equations: an
// integer product of the quantised operands, then the product of scales.
//
// Orientation.  The MFMA "A" operand (rows of the result tile) is the weight
// tile, the "B" operand (columns) is the activation tile.  In the 32x32 result
// layout a lane then owns ONE pixel (column lane%32) and 16 output channels, so
// the per-pixel activation scale of a tap is a single per-lane register and the
// 16 channels of a lane are contiguous in the NHWC output.
//
// Nibble handling.  Codes stay packed (two per byte) in HBM and in LDS.  A
// packed dword w is split in registers into two int8x4 vectors
//     lo = (w << 4) & 0xF0F0F0F0,   hi = w & 0xF0F0F0F0,
// each byte holding 16 * code exactly (two's complement).  Both operands are
// fed that way, so the MFMA accumulates 256 * sum(xq * wq); the factor is exact
// and is removed by an arithmetic shift (int32 output) or folded into the
// activation scale (floating-point output).  The order in which the codes of a
// 64-wide K step reach the MFMA lanes is a permutation applied identically to
// both operands, which leaves the sum unchanged.
#include <hip/hip_fp16.h>

#include "hq_common.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kOutF16 = 0, kOutF32 = 1, kOutI32 = 2;

struct GemmArgs {
    const uint8_t *xq;   // [pixels, k/2]
    const float *sx;     // [pixels]
    const uint8_t *wq;   // [n, taps, k/2]
    const float *sw;     // [n]
    const void *bias;    // [n] of the output dtype, or null
    void *y;
    int64_t pixels;      // rows of the activation matrix (= nb*h*w for a convolution)
    int n;               // output channels
    int k;               // input channels (codes per tap)
    int h, w;            // image size (convolution only)
    int n_co_tiles;
};

// Output channel handled by row i of a 32-row MFMA tile.  Chosen so that the
// 16 results of a lane (rows 8*(r/4) + 4*(lane/32) + r%4, r = 0..15) are the
// consecutive channels 16*(lane/32) + r.
__device__ __forceinline__ int tile_row_to_channel(int i) {
    return 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3);
}

__device__ __forceinline__ void unpack16(const v4i &p, v4i &first, v4i &second) {
    const int m = static_cast<int>(0xF0F0F0F0u);
    first = v4i{(p.x << 4) & m, p.x & m, (p.y << 4) & m, p.y & m};
    second = v4i{(p.z << 4) & m, p.z & m, (p.w << 4) & m, p.w & m};
}

template <int OUT> struct OutT;
template <> struct OutT<kOutF16> { using type = __half; };
template <> struct OutT<kOutF32> { using type = float; };
template <> struct OutT<kOutI32> { using type = int; };

__device__ __forceinline__ float to_float(__half v) { return __half2float(v); }
__device__ __forceinline__ float to_float(float v) { return v; }

__device__ __forceinline__ void store16(__half *dst, const float (&v)[16]) {
    uint4 lo, hi;
    __half2 *pl = reinterpret_cast<__half2 *>(&lo);
    __half2 *ph = reinterpret_cast<__half2 *>(&hi);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        pl[i] = __floats2half2_rn(v[2 * i], v[2 * i + 1]);
        ph[i] = __floats2half2_rn(v[8 + 2 * i], v[8 + 2 * i + 1]);
    }
    reinterpret_cast<uint4 *>(dst)[0] = lo;
    reinterpret_cast<uint4 *>(dst)[1] = hi;
}

__device__ __forceinline__ void store16(float *dst, const float (&v)[16]) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
        reinterpret_cast<float4 *>(dst)[i] = float4{v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]};
}

// TM x TN MFMA tiles of 32x32 per wave, WAVES_M x WAVES_N waves per workgroup.
// TAPS = 1 (linear / 1x1) or 9 (3x3, stride 1, pad 1).
template <int TM, int TN, int WAVES_M, int WAVES_N, int TAPS, int OUT>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void int_gemm_kernel(GemmArgs a) {
    constexpr int kThreadsWg = 64 * WAVES_M * WAVES_N;
    constexpr int BCO = 32 * TM * WAVES_M;   // output channels per workgroup
    constexpr int BP = 32 * TN * WAVES_N;    // pixels per workgroup
    constexpr int A_PIECES = 2 * BCO, B_PIECES = 2 * BP;   // 16-byte pieces per K step
    constexpr int A_PER_T = (A_PIECES + kThreadsWg - 1) / kThreadsWg;
    constexpr int B_PER_T = (B_PIECES + kThreadsWg - 1) / kThreadsWg;
    constexpr int STAGE_BYTES = (BCO + BP) * 32;
    using Out = typename OutT<OUT>::type;

    // [stage][operand][half][row][16 bytes]
    __shared__ __attribute__((aligned(16))) uint8_t lds[2 * STAGE_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
    const int lrow = lane & 31, lhalf = lane >> 5;

    const int tile_co = blockIdx.x % a.n_co_tiles;
    const int64_t tile_p = blockIdx.x / a.n_co_tiles;
    const int co0 = tile_co * BCO;
    const int64_t p0 = tile_p * BP;
    const int kbytes = a.k >> 1;      // packed bytes per (row, tap)
    const int kc_steps = a.k >> 6;    // 64-code steps per tap

    // ---- per-thread global->LDS pieces ---------------------------------------------------
    const uint8_t *a_src[A_PER_T];
    int a_dst[A_PER_T];
    bool a_ok[A_PER_T];
#pragma unroll
    for (int j = 0; j < A_PER_T; ++j) {
        const int piece = tid + j * kThreadsWg;
        const int row = piece >> 1, half = piece & 1;
        const int co = co0 + (row & ~31) + tile_row_to_channel(row & 31);
        a_ok[j] = piece < A_PIECES && co < a.n;
        a_src[j] = a.wq + (static_cast<int64_t>(co) * TAPS) * kbytes + half * 16;
        a_dst[j] = half * (BCO * 16) + row * 16;
    }
    int64_t b_pix[B_PER_T];   // linear index of the output pixel of this piece
    int b_oh[B_PER_T], b_ow[B_PER_T];
    int b_dst[B_PER_T];
    bool b_ok[B_PER_T];
    int b_half[B_PER_T];
#pragma unroll
    for (int j = 0; j < B_PER_T; ++j) {
        const int piece = tid + j * kThreadsWg;
        const int row = piece >> 1;
        b_half[j] = piece & 1;
        b_pix[j] = p0 + row;
        b_ok[j] = piece < B_PIECES && b_pix[j] < a.pixels;
        b_dst[j] = BCO * 32 + b_half[j] * (BP * 16) + row * 16;
        if (TAPS > 1) {
            const int64_t q = b_pix[j] / a.w;
            b_ow[j] = static_cast<int>(b_pix[j] - q * a.w);
            b_oh[j] = static_cast<int>(q % a.h);
        } else {
            b_oh[j] = b_ow[j] = 0;
        }
    }

    // ---- pixels this lane owns in the result tiles ----------------------------------------
    int64_t c_pix[TN];
    int c_oh[TN], c_ow[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        c_pix[tn] = p0 + (wave_n * TN + tn) * 32 + lrow;
        if (TAPS > 1) {
            const int64_t q = c_pix[tn] / a.w;
            c_ow[tn] = static_cast<int>(c_pix[tn] - q * a.w);
            c_oh[tn] = static_cast<int>(q % a.h);
        } else {
            c_oh[tn] = c_ow[tn] = 0;
        }
    }

    v16i acc[TM][TN];
    float facc[TAPS > 1 ? TM : 1][TAPS > 1 ? TN : 1][16];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0;
            if constexpr (TAPS > 1) {
#pragma unroll
                for (int r = 0; r < 16; ++r) facc[tm][tn][r] = 0.f;
            }
        }

    v4i ga[A_PER_T], gb[B_PER_T];

    auto global_load = [&](int tap, int kc) {
        const int koff = kc * 32;
#pragma unroll
        for (int j = 0; j < A_PER_T; ++j) {
            ga[j] = v4i{0, 0, 0, 0};
            if (a_ok[j])
                ga[j] = *reinterpret_cast<const v4i *>(a_src[j] + static_cast<int64_t>(tap) * kbytes + koff);
        }
#pragma unroll
        for (int j = 0; j < B_PER_T; ++j) {
            gb[j] = v4i{0, 0, 0, 0};
            bool ok = b_ok[j];
            int64_t src_pix = b_pix[j];
            if (TAPS > 1) {
                const int dr = tap / 3 - 1, ds = tap % 3 - 1;
                const int ih = b_oh[j] + dr, iw = b_ow[j] + ds;
                ok = ok && ih >= 0 && ih < a.h && iw >= 0 && iw < a.w;
                src_pix += dr * a.w + ds;
            }
            if (ok) gb[j] = *reinterpret_cast<const v4i *>(a.xq + src_pix * kbytes + koff + b_half[j] * 16);
        }
    };
    auto lds_store = [&](int stage) {
        uint8_t *base = lds + stage * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < A_PER_T; ++j)
            if (tid + j * kThreadsWg < A_PIECES) *reinterpret_cast<v4i *>(base + a_dst[j]) = ga[j];
#pragma unroll
        for (int j = 0; j < B_PER_T; ++j)
            if (tid + j * kThreadsWg < B_PIECES) *reinterpret_cast<v4i *>(base + b_dst[j]) = gb[j];
    };

    // scale of the input pixel under tap `tap` for each owned output pixel (0 outside the image)
    float sx_tap[TN];
    auto load_tap_scales = [&](int tap) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            bool ok = c_pix[tn] < a.pixels;
            int64_t src_pix = c_pix[tn];
            if (TAPS > 1) {
                const int dr = tap / 3 - 1, ds = tap % 3 - 1;
                const int ih = c_oh[tn] + dr, iw = c_ow[tn] + ds;
                ok = ok && ih >= 0 && ih < a.h && iw >= 0 && iw < a.w;
                src_pix += dr * a.w + ds;
            }
            sx_tap[tn] = ok ? a.sx[src_pix] * (1.0f / 256.0f) : 0.f;
        }
    };

    const int total_steps = TAPS * kc_steps;
    int tap = 0, kc = 0;         // step being computed
    int ntap = 0, nkc = 0;       // step being fetched
    global_load(0, 0);
    lds_store(0);
    if (OUT != kOutI32) load_tap_scales(0);
    __syncthreads();

    for (int step = 0; step < total_steps; ++step) {
        const int stage = step & 1;
        if (++nkc == kc_steps) { nkc = 0; ++ntap; }
        const bool more = step + 1 < total_steps;
        if (more) global_load(ntap, nkc);

        const uint8_t *sa = lds + stage * STAGE_BYTES + lhalf * (BCO * 16) + (wave_m * TM * 32 + lrow) * 16;
        const uint8_t *sb = lds + stage * STAGE_BYTES + BCO * 32 + lhalf * (BP * 16) + (wave_n * TN * 32 + lrow) * 16;
        v4i a0[TM], a1[TM], b0[TN], b1[TN];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) unpack16(*reinterpret_cast<const v4i *>(sa + tm * 512), a0[tm], a1[tm]);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) unpack16(*reinterpret_cast<const v4i *>(sb + tn * 512), b0[tn], b1[tn]);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[tm], b0[tn], acc[tm][tn], 0, 0, 0);
                acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[tm], b1[tn], acc[tm][tn], 0, 0, 0);
            }

        if (++kc == kc_steps) {
            kc = 0;
            // ---- end of a tap: fold the integer sums into the result ----------------------
            if constexpr (OUT == kOutI32) {
                int *yi = static_cast<int *>(a.y);
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const int cbase = co0 + (wave_m * TM + tm) * 32 + 16 * lhalf;
                        if (c_pix[tn] < a.pixels) {
                            int *dst = yi + (c_pix[tn] * TAPS + tap) * a.n + cbase;
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (cbase + r < a.n) dst[r] = acc[tm][tn][r] >> 8;
                        }
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0;
                    }
            } else if constexpr (TAPS > 1) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            facc[tm][tn][r] += sx_tap[tn] * static_cast<float>(acc[tm][tn][r]);
                            acc[tm][tn][r] = 0;
                        }
                if (tap + 1 < TAPS) load_tap_scales(tap + 1);
            }
            ++tap;
        }

        if (more) lds_store(stage ^ 1);
        __syncthreads();
    }

    // ---- dequantising epilogue -------------------------------------------------------------
    if constexpr (OUT != kOutI32) {
        Out *y = static_cast<Out *>(a.y);
        const Out *bias = static_cast<const Out *>(a.bias);
        const bool vec_ok = (a.n & 15) == 0;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int cbase = co0 + (wave_m * TM + tm) * 32 + 16 * lhalf;
            float swv[16], bv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const bool ok = cbase + r < a.n;
                swv[r] = ok ? a.sw[cbase + r] : 0.f;
                bv[r] = (ok && bias) ? to_float(bias[cbase + r]) : 0.f;
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                if (c_pix[tn] >= a.pixels) continue;
                float out[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float s;
                    if constexpr (TAPS > 1) s = facc[tm][tn][r];
                    else s = sx_tap[tn] * static_cast<float>(acc[tm][tn][r]);
                    out[r] = s * swv[r] + bv[r];
                }
                Out *dst = y + c_pix[tn] * a.n + cbase;
                if (vec_ok && cbase + 16 <= a.n) {
                    store16(dst, out);
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (cbase + r < a.n) dst[r] = static_cast<Out>(out[r]);
                }
            }
        }
    }
}

template <int TM, int TN, int WAVES_M, int WAVES_N, int TAPS, int OUT>
hq_status launch_tile(GemmArgs a, hipStream_t stream) {
    constexpr int BCO = 32 * TM * WAVES_M, BP = 32 * TN * WAVES_N;
    a.n_co_tiles = (a.n + BCO - 1) / BCO;
    const int64_t p_tiles = (a.pixels + BP - 1) / BP;
    const int64_t grid = p_tiles * a.n_co_tiles;
    if (grid > 0x7fffffffLL) return HQ_ERR_SHAPE;
    hipLaunchKernelGGL((int_gemm_kernel<TM, TN, WAVES_M, WAVES_N, TAPS, OUT>),
                       dim3(static_cast<unsigned>(grid)), dim3(64 * WAVES_M * WAVES_N), 0, stream, a);
    return hq::launch_status();
}

template <int TAPS, int OUT>
hq_status launch_shape(const GemmArgs &a, hipStream_t stream) {
    return launch_tile<2, 2, 2, 2, TAPS, OUT>(a, stream);
}

template <int TAPS>
hq_status launch_out(const GemmArgs &a, hq_dtype y_dtype, hipStream_t stream) {
    switch (y_dtype) {
        case HQ_F16: return launch_shape<TAPS, kOutF16>(a, stream);
        case HQ_F32: return launch_shape<TAPS, kOutF32>(a, stream);
        case HQ_I32: return launch_shape<TAPS, kOutI32>(a, stream);
    }
    return HQ_ERR_DTYPE;
}

hq_status check_common(const uint8_t *xq, const float *x_scale, const uint8_t *wq, const float *w_scale,
                       const void *bias, int64_t pixels, int n, int k, const void *y, hq_dtype y_dtype) {
    if (y_dtype != HQ_F16 && y_dtype != HQ_F32 && y_dtype != HQ_I32) return HQ_ERR_DTYPE;
    if (!xq || !wq || !y) return HQ_ERR_NULL;
    if (y_dtype != HQ_I32 && (!x_scale || !w_scale)) return HQ_ERR_NULL;
    if (pixels <= 0 || n <= 0 || k <= 0 || (k & 63) != 0 || k >= 131072) return HQ_ERR_SHAPE;
    if (!hq::aligned16(xq) || !hq::aligned16(wq) || !hq::aligned16(y)) return HQ_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(x_scale) & 3u) || (reinterpret_cast<uintptr_t>(w_scale) & 3u) ||
        (reinterpret_cast<uintptr_t>(bias) & 1u))
        return HQ_ERR_ALIGN;
    return HQ_OK;
}

}  // namespace

extern "C" hq_status hq_int_linear(const uint8_t *xq, const float *x_scale, const uint8_t *wq,
                                   const float *w_scale, const void *bias, int64_t m, int n, int k,
                                   void *y, hq_dtype y_dtype, void *stream) {
    hq_status st = check_common(xq, x_scale, wq, w_scale, bias, m, n, k, y, y_dtype);
    if (st != HQ_OK) return st;
    GemmArgs a{xq, x_scale, wq, w_scale, bias, y, m, n, k, 1, 1, 0};
    return launch_out<1>(a, y_dtype, static_cast<hipStream_t>(stream));
}

extern "C" hq_status hq_int_conv2d(const uint8_t *xq, const float *x_scale, const uint8_t *wq,
                                   const float *w_scale, const void *bias, int nb, int h, int w, int c_in,
                                   int c_out, int r, int s, int stride, int pad, void *y, hq_dtype y_dtype,
                                   void *stream) {
    if (nb <= 0 || h <= 0 || w <= 0 || r <= 0 || s <= 0 || stride <= 0 || pad < 0) {
        if (!xq || !wq || !y) return HQ_ERR_NULL;
        return HQ_ERR_SHAPE;
    }
    const int64_t pixels = static_cast<int64_t>(nb) * h * w;
    hq_status st = check_common(xq, x_scale, wq, w_scale, bias, pixels, c_out, c_in, y, y_dtype);
    if (st != HQ_OK) return st;
    if (r != s || (r != 1 && r != 3) || stride != 1 || pad != (r - 1) / 2) return HQ_ERR_UNSUPPORTED;
    GemmArgs a{xq, x_scale, wq, w_scale, bias, y, pixels, c_out, c_in, h, w, 0};
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    return r == 1 ? launch_out<1>(a, y_dtype, st_) : launch_out<9>(a, y_dtype, st_);
}
