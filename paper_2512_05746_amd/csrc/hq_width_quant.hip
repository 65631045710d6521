// Activation side of the paper's own convolution (Method, "Convolution"): the NHWC tensor is
// read as rows of one image line each, X~ of shape (B C_in h) x w, transformed along the WIDTH
// axis with H_c = BlockDiag(H_k) and quantised with one scale for the whole tensor,
//     q = clamp(rne((X~ H_c) / S)).
// The integer convolution of that scheme runs on (X~ H_c)_int H_c,raw, i.e. on the codes taken
// back along the width axis with the +-1 matrix.  That integer product is formed here, in the
// same pass, exactly: u = q * BlockDiag(H_raw), |u| <= 2^(a_bits-1) * had_block <= 512, and stored
// as three signed base-16 digit planes, u = d0 + 16 d1 + 256 d2 with every digit in [-8, 7], each
// plane an NHWC tensor of packed nibbles.  The convolution then runs once per plane on the
// 4-bit path.
//
// One thread owns two neighbouring channels (one byte of packed digits per pixel and plane) of
// one transform block of one image line: it loads the 2 x had_block values, transforms them in
// registers (Sylvester order: the in-place butterfly with strides 1, 2, 4, ...), quantises,
// transforms the codes back in integers and writes the digits.  Neighbouring threads own
// neighbouring channel pairs, so loads and stores of a pixel are contiguous.
#include <hip/hip_fp16.h>

#include "hq_common.h"

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ void load_pair(const __half *p, float &a, float &b) {
    const __half2 v = *reinterpret_cast<const __half2 *>(p);
    a = __low2float(v);
    b = __high2float(v);
}
__device__ __forceinline__ void load_pair(const float *p, float &a, float &b) {
    const float2 v = *reinterpret_cast<const float2 *>(p);
    a = v.x;
    b = v.y;
}

template <int B, typename V>
__device__ __forceinline__ void butterfly(V (&v)[B]) {
#pragma unroll
    for (int h = 1; h < B; h <<= 1)
#pragma unroll
        for (int i = 0; i < B; ++i)
            if ((i & h) == 0) {
                const V x = v[i], y = v[i + h];
                v[i] = x + y;
                v[i + h] = x - y;
            }
}

template <typename T, int LOGB>
__global__ __launch_bounds__(kThreads) void width_quant_kernel(const T *__restrict__ x, int w, int c, float qmax,
                                                               const float *__restrict__ given,
                                                               uint8_t *__restrict__ xu3, uint32_t plane_bytes) {
    constexpr int B = 1 << LOGB;
    const int blocks_per_line = w >> LOGB;
    const uint32_t line = blockIdx.x / blocks_per_line;                     // image * h + row
    const uint32_t pix0 = line * w + (blockIdx.x % blocks_per_line) * B;   // first pixel of the block
    const int half_c = c >> 1;
    // the butterfly yields sqrt(B) x the orthonormal transform
    const float inv = 1.0f / (given[0] * sqrtf(static_cast<float>(B)));
    for (int j = threadIdx.x; j < half_c; j += kThreads) {
        float v0[B], v1[B];
#pragma unroll
        for (int e = 0; e < B; ++e) load_pair(x + (static_cast<int64_t>(pix0 + e) * c + 2 * j), v0[e], v1[e]);
        butterfly<B>(v0);
        butterfly<B>(v1);
        int q0[B], q1[B];
#pragma unroll
        for (int e = 0; e < B; ++e) {
            q0[e] = static_cast<int>(fminf(fmaxf(rintf(v0[e] * inv), -qmax - 1.0f), qmax));   // rint: ties to even
            q1[e] = static_cast<int>(fminf(fmaxf(rintf(v1[e] * inv), -qmax - 1.0f), qmax));
        }
        butterfly<B>(q0);
        butterfly<B>(q1);
#pragma unroll
        for (int e = 0; e < B; ++e) {
            int lo[3], hi[3];
            hq::digits16(q0[e], lo);
            hq::digits16(q1[e], hi);
            uint8_t *dst = xu3 + (static_cast<int64_t>(pix0 + e) * half_c + j);
#pragma unroll
            for (int p = 0; p < 3; ++p)
                dst[static_cast<int64_t>(p) * plane_bytes] = static_cast<uint8_t>((lo[p] & 15) | ((hi[p] & 15) << 4));
        }
    }
}

template <typename T>
hq_status launch_width_quant(const T *x, int64_t lines, int w, int c, int had_block, int bits, const float *given,
                             uint8_t *xu3, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    const float qmax = static_cast<float>((1 << (bits - 1)) - 1);
    const int64_t grid = lines * (w / had_block);
    const int64_t plane = lines * w * (c / 2);
    if (grid > 0x7fffffffLL || lines * w > 0x7fffffffLL || plane > 0xffffffffLL) return HQ_ERR_SHAPE;
    const dim3 g(static_cast<unsigned>(grid)), b(kThreads);
    const uint32_t pb = static_cast<uint32_t>(plane);
    switch (hq::ilog2(had_block)) {
#define HQ_WIDTH_CASE(L) \
    case L: hipLaunchKernelGGL((width_quant_kernel<T, L>), g, b, 0, stream, x, w, c, qmax, given, xu3, pb); break;
        HQ_WIDTH_CASE(0) HQ_WIDTH_CASE(1) HQ_WIDTH_CASE(2) HQ_WIDTH_CASE(3)
        HQ_WIDTH_CASE(4) HQ_WIDTH_CASE(5) HQ_WIDTH_CASE(6)
#undef HQ_WIDTH_CASE
        default: return HQ_ERR_SHAPE;
    }
    return check.status();
}

}  // namespace

extern "C" hq_status hq_act_hadamard_quant_width(const void *x, hq_dtype x_dtype, int nb, int h, int w, int c,
                                                 int had_block, int a_bits, const float *x_scale,
                                                 uint8_t *xu3, void *stream) {
    if (!x || !x_scale || !xu3) return HQ_ERR_NULL;
    if (x_dtype != HQ_F16 && x_dtype != HQ_F32) return HQ_ERR_DTYPE;
    if (a_bits < 2 || a_bits > 4) return HQ_ERR_BITS;
    if (nb <= 0 || h <= 0 || w <= 0 || c <= 0 || (c & 1)) return HQ_ERR_SHAPE;
    if (!hq::pow2_upto_128(had_block) || had_block > 64 || w % had_block != 0) return HQ_ERR_SHAPE;
    if (!hq::aligned16(x) || !hq::aligned16(xu3) || (reinterpret_cast<uintptr_t>(x_scale) & 3u)) return HQ_ERR_ALIGN;
    const int64_t lines = static_cast<int64_t>(nb) * h;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (x_dtype == HQ_F16)
        return launch_width_quant(static_cast<const __half *>(x), lines, w, c, had_block, a_bits, x_scale, xu3, s);
    return launch_width_quant(static_cast<const float *>(x), lines, w, c, had_block, a_bits, x_scale, xu3, s);
}
