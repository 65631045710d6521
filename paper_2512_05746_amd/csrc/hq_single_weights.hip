// Offline weight preparation of the Single scheme (Method, linear-layer equation and "Single
// Hadamard Transformation"): the weights are quantised as they are, W_int = clamp(rne(W / s_w)),
// one abs-max scale per output channel, and the integer transform that the scheme keeps
// between the two quantised operands is folded into them here, exactly:
//     B = W_int * BlockDiag(H_raw)        (integers, |B| <= 2^(w_bits-1) * had_block <= 1024),
// so that (XH)_int H_raw W_int^T = (XH)_int B^T.  B does not fit a 4-bit code; it is stored as
// three signed base-16 digits, B = d0 + 16 d1 + 256 d2 with every digit in [-8, 7] (which covers
// [-2184, 1911]), each digit plane in the packed-nibble format of the other operands.  The
// integer GEMM then runs once per plane on the 4-bit path and combines the three sums.
//
// One workgroup per output channel: pass 1 finds max |w| of the row, pass 2 quantises one
// transform block per thread, transforms the codes in registers (Sylvester order: the in-place
// butterfly with strides 1, 2, 4, ...) and writes the digits.  Offline, not tuned.
#include <hip/hip_fp16.h>

#include "hq_common.h"

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float as_float(__half v) { return __half2float(v); }
__device__ __forceinline__ float as_float(float v) { return v; }

template <typename T, int LOGB>
__global__ __launch_bounds__(kThreads) void single_weights_kernel(const T *__restrict__ w, int k_in, float qmax,
                                                                  uint8_t *__restrict__ wq3,
                                                                  float *__restrict__ w_scale) {
    constexpr int B = 1 << LOGB;
    constexpr int U = B < 2 ? 2 : B;   // elements per thread and step: whole bytes of packed codes
    __shared__ unsigned s_max;
    const int tid = threadIdx.x;
    const T *row = w + static_cast<int64_t>(blockIdx.x) * k_in;
    if (tid == 0) s_max = 0u;
    __syncthreads();
    float amax = 0.f;
    for (int c = tid; c < k_in; c += kThreads) amax = fmaxf(amax, fabsf(as_float(row[c])));
    atomicMax(&s_max, __float_as_uint(amax));   // non-negative floats order like their bit patterns
    __syncthreads();
    amax = __uint_as_float(s_max);
    const float inv = amax > 0.f ? qmax / amax : 0.f;
    if (tid == 0) w_scale[blockIdx.x] = amax > 0.f ? amax / qmax : 1.0f;

    const int kbytes = k_in >> 1;
    uint8_t *out = wq3 + static_cast<int64_t>(blockIdx.x) * 3 * kbytes;
    for (int u0 = tid * U; u0 < k_in; u0 += kThreads * U) {
        int c[U];
#pragma unroll
        for (int e = 0; e < U; ++e) {
            const float t = rintf(as_float(row[u0 + e]) * inv);   // ties to even
            c[e] = static_cast<int>(fminf(fmaxf(t, -qmax - 1.0f), qmax));
        }
        if constexpr (B >= 2) {
#pragma unroll
            for (int h = 1; h < B; h <<= 1)
#pragma unroll
                for (int i = 0; i < B; ++i)
                    if ((i & h) == 0) {
                        const int x = c[i], y = c[i + h];
                        c[i] = x + y;
                        c[i + h] = x - y;
                    }
        }
#pragma unroll
        for (int e = 0; e < U; e += 2) {
            int lo[3], hi[3];
            hq::digits16(c[e], lo);
            hq::digits16(c[e + 1], hi);
#pragma unroll
            for (int p = 0; p < 3; ++p)
                out[p * kbytes + ((u0 + e) >> 1)] = static_cast<uint8_t>((lo[p] & 15) | ((hi[p] & 15) << 4));
        }
    }
}

template <typename T>
hq_status launch_single_weights(const T *w, int n_out, int k_in, int had_block, int bits, uint8_t *wq3,
                                float *w_scale, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    const float qmax = static_cast<float>((1 << (bits - 1)) - 1);
    const dim3 grid(static_cast<unsigned>(n_out)), block(kThreads);
    switch (hq::ilog2(had_block)) {
#define HQ_SINGLE_CASE(L) \
    case L: hipLaunchKernelGGL((single_weights_kernel<T, L>), grid, block, 0, stream, w, k_in, qmax, wq3, w_scale); break;
        HQ_SINGLE_CASE(0) HQ_SINGLE_CASE(1) HQ_SINGLE_CASE(2) HQ_SINGLE_CASE(3)
        HQ_SINGLE_CASE(4) HQ_SINGLE_CASE(5) HQ_SINGLE_CASE(6) HQ_SINGLE_CASE(7)
#undef HQ_SINGLE_CASE
        default: return HQ_ERR_SHAPE;
    }
    return check.status();
}

}  // namespace

extern "C" hq_status hq_quantize_weights_single(const void *w, hq_dtype w_dtype, int n_out, int k_in,
                                                int had_block, int w_bits, uint8_t *wq3, float *w_scale,
                                                void *stream) {
    if (!w || !wq3 || !w_scale) return HQ_ERR_NULL;
    if (w_dtype != HQ_F16 && w_dtype != HQ_F32) return HQ_ERR_DTYPE;
    if (w_bits < 2 || w_bits > 4) return HQ_ERR_BITS;
    if (n_out <= 0 || k_in <= 0 || (k_in & 1)) return HQ_ERR_SHAPE;
    if (!hq::pow2_upto_128(had_block) || k_in % had_block != 0) return HQ_ERR_SHAPE;
    if (!hq::aligned16(w) || !hq::aligned16(wq3) || (reinterpret_cast<uintptr_t>(w_scale) & 3u)) return HQ_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (w_dtype == HQ_F16)
        return launch_single_weights(static_cast<const __half *>(w), n_out, k_in, had_block, w_bits, wq3, w_scale, s);
    return launch_single_weights(static_cast<const float *>(w), n_out, k_in, had_block, w_bits, wq3, w_scale, s);
}
