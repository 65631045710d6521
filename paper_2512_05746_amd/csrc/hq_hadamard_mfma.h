// The 64-point Hadamard transform of 16 tokens on the matrix cores, and the packing of eight
// quantised values into one dword; shared by the transform-quantise kernels and the convolution
// that transforms and quantises its own activation tile.  (Background, "Hadamard Transformation":
// Sylvester order, entry (i, j) = (-1)^popcount(i & j); Background, "Model Quantization".)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr float kMagic = 12582920.0f;                                 // 1.5 * 2^23 + 8
constexpr uint32_t kMagicSum = 0x4B400000u * 0x11111111u;             // sum_i 0x4B400000 << 4i (mod 2^32)
constexpr int kMaxBlocks = 16;                                        // 64-channel blocks per row

__device__ __forceinline__ uint32_t pack8_magic(const float *v, float inv) {
    uint32_t w = __float_as_uint(__builtin_fmaf(v[7], inv, kMagic));
#pragma unroll
    for (int i = 6; i >= 0; --i) w = (w << 4) + __float_as_uint(__builtin_fmaf(v[i], inv, kMagic));
    return (w - kMagicSum) ^ 0x88888888u;
}

// The same with the clamp of a given scale: v is limited to [lo, hi] = [qmin / inv, qmax / inv]
// first (rounding is monotonic and the limits are integers, so clamp and round commute).
__device__ __forceinline__ uint32_t pack8_magic_clamped(const float *v, float inv, float lo, float hi) {
    float c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = fminf(fmaxf(v[i], lo), hi);
    return pack8_magic(c, inv);
}


// "A" operands of v_mfma_f32_16x16x32_f16 for out^T = H^T x^T: tile ct (4 tiles of 16 rows) x K
// half h.  Lane l supplies row l % 16 and K slice q = l / 16 of a tile.  Row i of tile ct is
// channel c = 16 (i / 4) + 4 ct + i % 4, so that the lane that owns (token, q) of the "B" operand
// ends up with channels 16 q + 4 ct + r of the block.  Sign of H[c][kk] = parity of
// popcount(c & kk), kk = 32 h + 8 q + e: the bits of e (0..2) and of 32 h + 8 q (3..5) do not
// overlap, so the sign is (pattern over e from c & 7) xor (one bit from c & (32 h + 8 q)).
__device__ __forceinline__ void hadamard64_operands(int lane, v8h (&hmat)[4][2]) {
    const int i = lane & 15, q = lane >> 4;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
        const int c = 16 * (i >> 2) + 4 * ct + (i & 3);
        uint32_t pat[4];
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) {
            const uint32_t s0 = __popc(c & (2 * e2)) & 1, s1 = __popc(c & (2 * e2 + 1)) & 1;
            pat[e2] = 0x3C003C00u ^ (s0 << 15) ^ (s1 << 31);   // +-1.0 in fp16
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t flip = (__popc(c & (32 * h + 8 * q)) & 1) ? 0x80008000u : 0u;
            const uint4 w = uint4{pat[0] ^ flip, pat[1] ^ flip, pat[2] ^ flip, pat[3] ^ flip};
            hmat[ct][h] = __builtin_bit_cast(v8h, w);
        }
    }
}

// The 16 sums of this lane for one block (8 x the orthonormal transform): b[h] is the lane's
// 16-byte piece at channels 32 h + 8 q of the block of its token.
__device__ __forceinline__ void hadamard64_transform(const v8h (&hmat)[4][2], const v8h (&b)[2], float (&v)[16]) {
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
        v4f acc = {0.f, 0.f, 0.f, 0.f};
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(hmat[ct][0], b[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(hmat[ct][1], b[1], acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) v[4 * ct + r] = acc[r];
    }
}
