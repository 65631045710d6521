// Block Hadamard transform fused with per-row symmetric quantisation (gfx950).
//
// One kernel family serves both the online activation path (one row per token,
// Method "Matrix Multiplication" + Background "Model Quantization") and the
// offline weight path (one row per output channel, all taps of it).
//
// Work decomposition: a lane owns a "chunk" of 8 consecutive elements (one
// 16-byte load of fp16).  The Sylvester transform of order 2^LOGB is a
// butterfly over the LOGB index bits: bits 0..2 live inside the lane's
// registers, bits 3.. live across 2^(LOGB-3) neighbouring lanes and are done
// with DPP lane permutes.  The normalisation 2^{-LOGB/2} is never applied to
// the data: it only enters the reported scale (the paper absorbs it into the
// scales as well).
#include <hip/hip_fp16.h>

#include "hq_common.h"
#include "hq_hadamard_mfma.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxRowsPerWg = 1024;

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Value held by lane (lane ^ (1 << J)), J = 0..3; partners stay inside a row of 16 lanes.
template <int J>
__device__ __forceinline__ float lane_xor(float v) {
    static_assert(J >= 0 && J <= 3, "partner must be inside a DPP row");
    if constexpr (J == 0) return dpp_mov<0xB1>(v);                       // quad_perm [1,0,3,2]
    else if constexpr (J == 1) return dpp_mov<0x4E>(v);                  // quad_perm [2,3,0,1]
    else if constexpr (J == 2) return dpp_mov<0x1B>(dpp_mov<0x141>(v));  // half-row mirror, then quad reverse
    else return dpp_mov<0x128>(v);                                       // row rotate by 8
}

__device__ __forceinline__ void load8(const __half *p, float (&v)[8]) {
    uint4 raw = *reinterpret_cast<const uint4 *>(p);
    const __half2 *h = reinterpret_cast<const __half2 *>(&raw);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float2 f = __half22float2(h[i]);
        v[2 * i] = f.x;
        v[2 * i + 1] = f.y;
    }
}

__device__ __forceinline__ void load8(const float *p, float (&v)[8]) {
    float4 a = reinterpret_cast<const float4 *>(p)[0];
    float4 b = reinterpret_cast<const float4 *>(p)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

template <int S>
__device__ __forceinline__ void stage_in_lane(float (&v)[8]) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if ((i & S) == 0) {
            float a = v[i], b = v[i + S];
            v[i] = a + b;
            v[i + S] = a - b;
        }
}

template <int J>
__device__ __forceinline__ void stage_cross_lane(float (&v)[8], int lane) {
    const bool upper = (lane >> J) & 1;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float p = lane_xor<J>(v[i]);
        v[i] = upper ? (p - v[i]) : (v[i] + p);
    }
}

// Unnormalised Sylvester transform of order 2^LOGB over element index bits 0..LOGB-1.
template <int LOGB>
__device__ __forceinline__ void hadamard_raw(float (&v)[8], int lane) {
    if constexpr (LOGB >= 1) stage_in_lane<1>(v);
    if constexpr (LOGB >= 2) stage_in_lane<2>(v);
    if constexpr (LOGB >= 3) stage_in_lane<4>(v);
    if constexpr (LOGB >= 4) stage_cross_lane<0>(v, lane);
    if constexpr (LOGB >= 5) stage_cross_lane<1>(v, lane);
    if constexpr (LOGB >= 6) stage_cross_lane<2>(v, lane);
    if constexpr (LOGB >= 7) stage_cross_lane<3>(v, lane);
}

__device__ __forceinline__ float absmax8(const float (&v)[8]) {
    float a = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(v[i]));
    return a;
}

// max over an aligned group of `group` lanes (group = 1, 2, 4, 8 or 16; wave-uniform)
__device__ __forceinline__ float group_max(float a, int group) {
    if (group > 1) a = fmaxf(a, lane_xor<0>(a));
    if (group > 2) a = fmaxf(a, lane_xor<1>(a));
    if (group > 4) a = fmaxf(a, lane_xor<2>(a));
    if (group > 8) a = fmaxf(a, lane_xor<3>(a));
    return a;
}

// codes = clamp(rne(v * inv), qmin, qmax), eight of them packed into one dword,
// element i in bits 4i..4i+3 (two's complement).
__device__ __forceinline__ uint32_t quant_pack8(const float (&v)[8], float inv, float qmin, float qmax) {
    uint32_t w = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float r = fminf(fmaxf(rintf(v[i] * inv), qmin), qmax);
        w |= (static_cast<uint32_t>(static_cast<int>(r)) & 0xFu) << (4 * i);
    }
    return w;
}

// The same codes one per byte (8-bit codes), element i in byte i.
__device__ __forceinline__ uint2 quant_bytes8(const float (&v)[8], float inv, float qmin, float qmax) {
    uint32_t w[2] = {0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float r = fminf(fmaxf(rintf(v[i] * inv), qmin), qmax);
        w[i >> 2] |= (static_cast<uint32_t>(static_cast<int>(r)) & 0xFFu) << (8 * (i & 3));
    }
    return uint2{w[0], w[1]};
}

// Stores the eight codes of chunk `chunk`: half a byte each, or one byte each for 8-bit codes.
__device__ __forceinline__ void store_codes8(uint32_t *xq, int64_t chunk, const float (&v)[8], float inv,
                                             float qmin, float qmax, bool bytes) {
    if (bytes) reinterpret_cast<uint2 *>(xq)[chunk] = quant_bytes8(v, inv, qmin, qmax);
    else xq[chunk] = quant_pack8(v, inv, qmin, qmax);
}

struct RowQuantArgs {
    int64_t m;          // rows
    int chunks;         // 8-element chunks per row
    uint32_t inv_chunks;  // ceil(2^32 / chunks) for chunks >= 2 (exact quotient for slot < 65536)
    int rows_per_wg;
    int max_group;      // power of two <= 16 dividing `chunks`
    float qmin, qmax;
    float norm;         // 2^{-LOGB/2}
    const float *given;   // static mode: one scale for the whole tensor (device); NULL = per-row abs-max
    int bytes;            // 8-bit codes: one byte per code instead of half a byte
};

// Rows short enough that a workgroup keeps several whole rows in registers.
template <typename T, int LOGB, int U>
__global__ __launch_bounds__(kThreads) void rowquant_small(const T *__restrict__ x, RowQuantArgs a,
                                                           uint32_t *__restrict__ xq,
                                                           float *__restrict__ scale) {
    __shared__ unsigned s_max[kMaxRowsPerWg];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int64_t row0 = static_cast<int64_t>(blockIdx.x) * a.rows_per_wg;
    const int64_t left = a.m - row0;
    const int nrows = left < a.rows_per_wg ? static_cast<int>(left) : a.rows_per_wg;
    const int nslots = nrows * a.chunks;
    const int64_t chunk0 = row0 * a.chunks;

    for (int i = tid; i < a.rows_per_wg; i += kThreads) s_max[i] = 0u;

    float v[U][8];
    int rl[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int slot = tid + kThreads * u;
        if (slot < nslots) {
            load8(x + (chunk0 + slot) * 8, v[u]);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[u][i] = 0.f;
        }
        rl[u] = a.chunks == 1 ? slot : static_cast<int>(__umulhi(static_cast<uint32_t>(slot), a.inv_chunks));
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) {
        hadamard_raw<LOGB>(v[u], lane);
        const float amax = group_max(absmax8(v[u]), a.max_group);
        const int slot = tid + kThreads * u;
        if (slot < nslots && (lane & (a.max_group - 1)) == 0)
            atomicMax(&s_max[rl[u]], __float_as_uint(amax));  // non-negative floats order like uints
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int slot = tid + kThreads * u;
        if (slot < nslots) {
            const float amax = __uint_as_float(s_max[rl[u]]);
            const float inv = a.given ? a.norm / a.given[0] : (amax > 0.f ? a.qmax / amax : 0.f);
            store_codes8(xq, chunk0 + slot, v[u], inv, a.qmin, a.qmax, a.bytes != 0);
            if (!a.given && slot == rl[u] * a.chunks)
                scale[row0 + rl[u]] = amax > 0.f ? (amax * a.norm) / a.qmax : 1.0f;
        }
    }
}

// Arbitrarily long rows: one workgroup per row, the row is read twice.
template <typename T, int LOGB>
__global__ __launch_bounds__(kThreads) void rowquant_large(const T *__restrict__ x, RowQuantArgs a,
                                                           uint32_t *__restrict__ xq,
                                                           float *__restrict__ scale) {
    __shared__ unsigned s_max;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int64_t chunk0 = static_cast<int64_t>(blockIdx.x) * a.chunks;
    const int rounded = (a.chunks + kThreads - 1) / kThreads * kThreads;
    if (tid == 0) s_max = 0u;
    __syncthreads();

    float amax = 0.f;
    for (int c = tid; c < rounded; c += kThreads) {
        float v[8];
        if (c < a.chunks) {
            load8(x + (chunk0 + c) * 8, v);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = 0.f;
        }
        hadamard_raw<LOGB>(v, lane);
        amax = fmaxf(amax, absmax8(v));
    }
    atomicMax(&s_max, __float_as_uint(amax));
    __syncthreads();
    amax = __uint_as_float(s_max);
    const float inv = a.given ? a.norm / a.given[0] : (amax > 0.f ? a.qmax / amax : 0.f);

    for (int c = tid; c < rounded; c += kThreads) {
        float v[8];
        if (c < a.chunks) {
            load8(x + (chunk0 + c) * 8, v);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = 0.f;
        }
        hadamard_raw<LOGB>(v, lane);
        if (c < a.chunks) store_codes8(xq, chunk0 + c, v, inv, a.qmin, a.qmax, a.bytes != 0);
    }
    if (tid == 0 && !a.given) scale[blockIdx.x] = amax > 0.f ? (amax * a.norm) / a.qmax : 1.0f;
}

// ---- fp16 input, block 64, rows of up to 1024 channels: the transform on the matrix cores ------
//
// For the streaming activation path the butterfly above is bound by vector-ALU work
// (about 14 instructions per element), not by HBM.  Here the same product x * H64 is
// evaluated as an MFMA: out^T = H^T x^T with H (entries +-1, exact in fp16) as the "A"
// operand and 16 tokens as the columns of "B" of v_mfma_f32_16x16x32_f16, accumulated in
// fp32; the products are exact, so only the summation order differs from the butterfly.
//
// Decomposition.  One wave transforms and quantises 16 whole tokens: lane l owns token l % 16
// and K slice q = l / 16; its B operands of block b are the two 16-byte pieces at channels
// 64 b + 32 h + 8 q (h = 0, 1), so activations go from HBM straight into the matrix core.  All
// loads of the wave are issued first.  The rows of H are permuted so that the 16 results of a
// lane per block are the 16 consecutive channels 16 q .. 16 q + 15 of the block: 8 packed
// bytes, and the four lanes of a token write 32 contiguous bytes.  The abs-max of a token is
// a maximum over the lane's values and over the four lanes of the token (two lane exchanges):
// no LDS, no barrier, waves are independent.  Rows of up to four blocks keep the transformed
// values in registers; longer rows keep the fp16 inputs instead and run the (cheap) MFMAs a
// second time once the scale is known.
//
// Only pairing matters for the K index: element e of K slice q of operand h is channel
// 32 h + 8 q + e for both operands, whatever order the hardware sums them in.
//
// Quantisation: m = fma(v, qmax / amax, 1.5 * 2^23 + 8) rounds v * inv to the nearest
// integer (ties to even, one rounding) and leaves code + 8 (1..15) in the low nibble of the
// float's bit pattern.  Eight such patterns are merged by w = (w << 4) + m; the known
// constant contributed by the upper bits is subtracted and the offset removed by
// xor 0x88888888, which yields the eight two's-complement nibbles.
// STATIC: the scale is given (one for the tensor): no abs-max, clamp active, no scale output;
// `given` points to it.  NBLK: 64-channel blocks per row.  Four waves (token groups) per workgroup.
template <int NBLK, bool STATIC>
__global__ __launch_bounds__(256) void hadamard64_quant_f16(const __half *__restrict__ x, int64_t m, float qmax,
                                                           uint8_t *__restrict__ xq, float *__restrict__ scale,
                                                           const float *__restrict__ given) {
    constexpr int K = 64 * NBLK;
    constexpr bool KEEP = STATIC || NBLK <= 4;   // transformed values stay in registers
    const int lane = threadIdx.x & 63;
    const int tok = lane & 15, q = lane >> 4;
    const int64_t grp = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    if (grp * 16 >= m) return;   // no barrier below: a wave without tokens just leaves
    const int64_t token = grp * 16 + tok;
    const bool live = token < m;

    v8h b[NBLK][2];
    {
        const __half *src = x + (live ? token : m - 1) * K + 8 * q;
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            b[blk][0] = *reinterpret_cast<const v8h *>(src + 64 * blk);
            b[blk][1] = *reinterpret_cast<const v8h *>(src + 64 * blk + 32);
        }
    }

    // "A" operands: tile ct (4 tiles of 16 rows) x K half h.  Row i of tile ct is channel
    // c = 16 (i / 4) + 4 ct + i % 4, so lane (token, q) ends up with channels 16 q + 4 ct + r.
    // Sign of H[c][kk] = parity of popcount(c & kk), kk = 32 h + 8 q' + e with q' = this lane's
    // K slice: the bits of e (0..2) and of 32 h + 8 q' (3..5) do not overlap, so the sign is
    // (pattern over e from c & 7) xor (one bit from c & (32 h + 8 q')).
    v8h hmat[4][2];
    hadamard64_operands(lane, hmat);
    // the 16 sums of this lane for one block: 8 x the orthonormal transform
    auto transform = [&](int blk, float (&v)[16]) {
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
            v4f acc = {0.f, 0.f, 0.f, 0.f};
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(hmat[ct][0], b[blk][0], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(hmat[ct][1], b[blk][1], acc, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) v[4 * ct + r] = acc[r];
        }
    };
    uint8_t *dst = xq + token * (K / 2) + 8 * q;

    if constexpr (STATIC) {
        const float inv = 0.125f / given[0];
        const float lo = (-qmax - 1.0f) / inv, hi = qmax / inv;
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            float v[16];
            transform(blk, v);
            uint2 w;
            w.x = pack8_magic_clamped(v, inv, lo, hi);
            w.y = pack8_magic_clamped(v + 8, inv, lo, hi);
            if (live) *reinterpret_cast<uint2 *>(dst + 32 * blk) = w;
        }
    } else {
        float v[KEEP ? NBLK : 1][16];
        float amax = 0.f;
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            float (&vb)[16] = v[KEEP ? blk : 0];
            transform(blk, vb);
#pragma unroll
            for (int r = 0; r < 16; ++r) amax = fmaxf(amax, fabsf(vb[r]));
        }
        amax = fmaxf(amax, __shfl_xor(amax, 16));   // the token's other three K slices
        amax = fmaxf(amax, __shfl_xor(amax, 32));
        const float inv = amax > 0.f ? qmax / amax : 0.f;
        if (live && q == 0) scale[token] = amax > 0.f ? (amax * 0.125f) / qmax : 1.0f;
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            float (&vb)[16] = v[KEEP ? blk : 0];
            if constexpr (!KEEP) transform(blk, vb);
            uint2 w;
            w.x = pack8_magic(vb, inv);
            w.y = pack8_magic(vb + 8, inv);
            if (live) *reinterpret_cast<uint2 *>(dst + 32 * blk) = w;
        }
    }
}

// The same for tensors with too few tokens to fill the chip with one wave per 16 tokens: a
// workgroup has one wave per 64-channel block of the row and handles groups of 16 tokens; wave b
// transforms block b.  The abs-max of a token then needs every wave: they exchange their maxima
// through LDS (one barrier per group, two sets of slots).  Workgroups are persistent and fetch
// the next group's pieces before they work on the current one.
template <bool STATIC>
__global__ __launch_bounds__(64 * kMaxBlocks) void hadamard64_quant_split_f16(const __half *__restrict__ x, int64_t m,
                                                                        int k, float qmax,
                                                                        uint8_t *__restrict__ xq,
                                                                        float *__restrict__ scale,
                                                                        const float *__restrict__ given) {
    __shared__ float s_amax[2][kMaxBlocks][16];
    const int lane = threadIdx.x & 63;
    const int blk = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // 64-channel block of this wave
    const int nblk = k >> 6;
    const int tok = lane & 15, q = lane >> 4;

    // "A" operands: tile ct (4 tiles of 16 rows) x K half h.  Row i of tile ct is channel
    // c = 16 (i / 4) + 4 ct + i % 4, so lane (token, q) ends up with channels 16 q + 4 ct + r.
    // Sign of H[c][kk] = parity of popcount(c & kk), kk = 32 h + 8 q' + e with q' = this lane's
    // K slice: the bits of e (0..2) and of 32 h + 8 q' (3..5) do not overlap, so the sign is
    // (pattern over e from c & 7) xor (one bit from c & (32 h + 8 q')).
    v8h hmat[4][2];
    hadamard64_operands(lane, hmat);

    const int64_t groups = (m + 15) >> 4;
    auto fetch = [&](int64_t grp, v8h (&b)[2]) {
        int64_t token = grp * 16 + tok;
        token = token < m ? token : m - 1;
        const __half *src = x + token * k + 64 * blk + 8 * q;
        b[0] = *reinterpret_cast<const v8h *>(src);
        b[1] = *reinterpret_cast<const v8h *>(src + 32);
    };

    v8h b[2], bn[2];
    int64_t grp = blockIdx.x;
    if (grp < groups) fetch(grp, b);
    int set = 0;
    for (; grp < groups; grp += gridDim.x, set ^= 1) {
        const int64_t next = grp + gridDim.x;
        if (next < groups) fetch(next, bn);

        float v[16];
        float amax = 0.f;
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) {
            v4f acc = {0.f, 0.f, 0.f, 0.f};
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(hmat[ct][0], b[0], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(hmat[ct][1], b[1], acc, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                v[4 * ct + r] = acc[r];
                amax = fmaxf(amax, fabsf(acc[r]));
            }
        }
        const int64_t token = grp * 16 + tok;
        if constexpr (STATIC) {
            if (token < m) {
                const float inv = 0.125f / given[0];   // the sums are 8 x the orthonormal transform
                const float lo = (-qmax - 1.0f) / inv, hi = qmax / inv;
                uint2 w;
                w.x = pack8_magic_clamped(v, inv, lo, hi);
                w.y = pack8_magic_clamped(v + 8, inv, lo, hi);
                *reinterpret_cast<uint2 *>(xq + token * (k >> 1) + 32 * blk + 8 * q) = w;
            }
        } else {
            // the token's other three K slices of this block, then its other blocks
            amax = fmaxf(amax, __shfl_xor(amax, 16));
            amax = fmaxf(amax, __shfl_xor(amax, 32));
            if (nblk > 1) {
                if (q == 0) s_amax[set][blk][tok] = amax;
                __syncthreads();
                for (int w = 0; w < nblk; ++w) amax = fmaxf(amax, s_amax[set][w][tok]);
            }
            if (token < m) {
                const float inv = amax > 0.f ? qmax / amax : 0.f;
                if (blk == 0 && q == 0) scale[token] = amax > 0.f ? (amax * 0.125f) / qmax : 1.0f;
                uint2 w;
                w.x = pack8_magic(v, inv);
                w.y = pack8_magic(v + 8, inv);
                *reinterpret_cast<uint2 *>(xq + token * (k >> 1) + 32 * blk + 8 * q) = w;
            }
        }
        b[0] = bn[0];
        b[1] = bn[1];
    }
}

hq_status launch_hadamard64_split(const __half *x, int64_t m, int k, int bits, uint8_t *xq, float *scale,
                            const float *given, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    const float qmax = static_cast<float>((1 << (bits - 1)) - 1);
    const int nblk = k / 64;
    const int64_t groups = (m + 15) / 16;
    // resident workgroups: 32 waves per CU at the register use of this kernel
    const int64_t cap = static_cast<int64_t>(hq::compute_units()) * (32 / nblk > 0 ? 32 / nblk : 1);
    const int64_t rounds = (groups + cap - 1) / cap;          // groups per workgroup
    const int64_t grid = (groups + rounds - 1) / rounds;      // the same number for (almost) all of them
    if (given)
        hipLaunchKernelGGL(hadamard64_quant_split_f16<true>, dim3(static_cast<unsigned>(grid)), dim3(64 * nblk), 0,
                           stream, x, m, k, qmax, xq, scale, given);
    else
        hipLaunchKernelGGL(hadamard64_quant_split_f16<false>, dim3(static_cast<unsigned>(grid)), dim3(64 * nblk), 0,
                           stream, x, m, k, qmax, xq, scale, given);
    return check.status();
}

template <int NBLK>
void launch_hadamard64_blocks(const __half *x, int64_t m, float qmax, uint8_t *xq, float *scale,
                              const float *given, unsigned grid, hipStream_t stream) {
    if (given)
        hipLaunchKernelGGL((hadamard64_quant_f16<NBLK, true>), dim3(grid), dim3(256), 0, stream, x, m, qmax, xq,
                           scale, given);
    else
        hipLaunchKernelGGL((hadamard64_quant_f16<NBLK, false>), dim3(grid), dim3(256), 0, stream, x, m, qmax, xq,
                           scale, given);
}

hq_status launch_hadamard64(const __half *x, int64_t m, int k, int bits, uint8_t *xq, float *scale,
                            const float *given, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    // one wave per 16 tokens needs about two waves per SIMD to hide the latency of its loads
    if ((m + 15) / 16 < 8 * static_cast<int64_t>(hq::compute_units()))
        return launch_hadamard64_split(x, m, k, bits, xq, scale, given, stream);
    const float qmax = static_cast<float>((1 << (bits - 1)) - 1);
    const int64_t wgs = ((m + 15) / 16 + 3) / 4;   // 16 tokens per wave, four waves per workgroup
    if (wgs > 0x7fffffffLL) return HQ_ERR_SHAPE;
    const unsigned grid = static_cast<unsigned>(wgs);
    switch (k / 64) {
#define HQ_BLOCKS_CASE(N) \
    case N: launch_hadamard64_blocks<N>(x, m, qmax, xq, scale, given, grid, stream); break;
        HQ_BLOCKS_CASE(1) HQ_BLOCKS_CASE(2) HQ_BLOCKS_CASE(3) HQ_BLOCKS_CASE(4)
        HQ_BLOCKS_CASE(5) HQ_BLOCKS_CASE(6) HQ_BLOCKS_CASE(7) HQ_BLOCKS_CASE(8)
        HQ_BLOCKS_CASE(9) HQ_BLOCKS_CASE(10) HQ_BLOCKS_CASE(11) HQ_BLOCKS_CASE(12)
        HQ_BLOCKS_CASE(13) HQ_BLOCKS_CASE(14) HQ_BLOCKS_CASE(15) HQ_BLOCKS_CASE(16)
#undef HQ_BLOCKS_CASE
        default: return HQ_ERR_SHAPE;
    }
    return check.status();
}

template <typename T, int LOGB>
hq_status launch_rowquant(const T *x, int64_t m, int row_len, int bits, bool bytes, uint32_t *xq, float *scale,
                          const float *given, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    RowQuantArgs a;
    a.given = given;
    a.m = m;
    a.chunks = row_len / 8;
    a.inv_chunks = a.chunks >= 2 ? static_cast<uint32_t>(((1ull << 32) + a.chunks - 1) / a.chunks) : 0u;
    a.max_group = 1;
    while (a.max_group < 16 && a.chunks % (a.max_group * 2) == 0) a.max_group *= 2;
    a.qmax = static_cast<float>((1 << (bits - 1)) - 1);
    a.qmin = -static_cast<float>(1 << (bits - 1));
    a.bytes = bytes ? 1 : 0;
    a.norm = static_cast<float>(1.0 / sqrt(static_cast<double>(1 << LOGB)));

    if (a.chunks <= kThreads * 4) {
        // several loads in flight per lane once the tensor is big enough to fill the chip anyway
        const bool deep = a.chunks > kThreads || m * static_cast<int64_t>(a.chunks) >= (1 << 21);
        const int cap = kThreads * (deep ? 4 : 1);
        a.rows_per_wg = cap / a.chunks;
        const int64_t grid = (m + a.rows_per_wg - 1) / a.rows_per_wg;
        if (grid > 0x7fffffffLL) return HQ_ERR_SHAPE;
        if (deep)
            hipLaunchKernelGGL((rowquant_small<T, LOGB, 4>), dim3(static_cast<unsigned>(grid)),
                               dim3(kThreads), 0, stream, x, a, xq, scale);
        else
            hipLaunchKernelGGL((rowquant_small<T, LOGB, 1>), dim3(static_cast<unsigned>(grid)),
                               dim3(kThreads), 0, stream, x, a, xq, scale);
    } else {
        if (m > 0x7fffffffLL) return HQ_ERR_SHAPE;
        a.rows_per_wg = 1;
        hipLaunchKernelGGL((rowquant_large<T, LOGB>), dim3(static_cast<unsigned>(m)), dim3(kThreads), 0,
                           stream, x, a, xq, scale);
    }
    return check.status();
}

template <typename T>
// bytes: one code per byte (always so for 8-bit codes) instead of two
hq_status dispatch_block(const T *x, int64_t m, int row_len, int had_block, int bits, bool bytes, uint32_t *xq,
                         float *scale, const float *given, hipStream_t stream) {
    switch (hq::ilog2(had_block)) {
        case 0: return launch_rowquant<T, 0>(x, m, row_len, bits, bytes || bits == 8, xq, scale, given, stream);
        case 1: return launch_rowquant<T, 1>(x, m, row_len, bits, bytes || bits == 8, xq, scale, given, stream);
        case 2: return launch_rowquant<T, 2>(x, m, row_len, bits, bytes || bits == 8, xq, scale, given, stream);
        case 3: return launch_rowquant<T, 3>(x, m, row_len, bits, bytes || bits == 8, xq, scale, given, stream);
        case 4: return launch_rowquant<T, 4>(x, m, row_len, bits, bytes || bits == 8, xq, scale, given, stream);
        case 5: return launch_rowquant<T, 5>(x, m, row_len, bits, bytes || bits == 8, xq, scale, given, stream);
        case 6: return launch_rowquant<T, 6>(x, m, row_len, bits, bytes || bits == 8, xq, scale, given, stream);
        case 7: return launch_rowquant<T, 7>(x, m, row_len, bits, bytes || bits == 8, xq, scale, given, stream);
        default: return HQ_ERR_SHAPE;
    }
}

// Shared argument checks.  `k` is the length the transform blocks must divide,
// `row_len` the length one scale covers.
hq_status check_rowquant(const void *x, hq_dtype dt, int64_t m, int k, int64_t row_len, int had_block,
                         int bits, const void *xq, const void *scale) {
    if (!x || !xq || !scale) return HQ_ERR_NULL;
    if (dt != HQ_F16 && dt != HQ_F32) return HQ_ERR_DTYPE;
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return HQ_ERR_BITS;
    if (m <= 0 || k <= 0 || row_len <= 0 || row_len > 0x7fffffffLL) return HQ_ERR_SHAPE;
    if (!hq::pow2_upto_128(had_block) || k % had_block != 0 || k % 8 != 0) return HQ_ERR_SHAPE;
    if (!hq::aligned16(x) || !hq::aligned16(xq) || (reinterpret_cast<uintptr_t>(scale) & 3u))
        return HQ_ERR_ALIGN;
    return HQ_OK;
}

}  // namespace

namespace {

// Activation path; given == NULL: per-token abs-max scales written to x_scale, else one static scale.
hq_status act_hadamard_quant(const void *x, hq_dtype x_dtype, int64_t m, int k, int had_block, int a_bits,
                             bool bytes, uint8_t *xq, float *x_scale, const float *given, void *stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t *out = reinterpret_cast<uint32_t *>(xq);
    if (x_dtype == HQ_F16 && had_block == 64 && k <= 64 * kMaxBlocks && a_bits != 8 && !bytes)
        return launch_hadamard64(static_cast<const __half *>(x), m, k, a_bits, xq, x_scale, given, s);
    if (x_dtype == HQ_F16)
        return dispatch_block(static_cast<const __half *>(x), m, k, had_block, a_bits, bytes, out, x_scale, given, s);
    return dispatch_block(static_cast<const float *>(x), m, k, had_block, a_bits, bytes, out, x_scale, given, s);
}

}  // namespace

extern "C" hq_status hq_act_hadamard_quant(const void *x, hq_dtype x_dtype, int64_t m, int k,
                                           int had_block, int a_bits, uint8_t *xq, float *x_scale,
                                           void *stream) {
    hq_status st = check_rowquant(x, x_dtype, m, k, k, had_block, a_bits, xq, x_scale);
    if (st != HQ_OK) return st;
    return act_hadamard_quant(x, x_dtype, m, k, had_block, a_bits, false, xq, x_scale, nullptr, stream);
}

extern "C" hq_status hq_act_hadamard_quant_i8(const void *x, hq_dtype x_dtype, int64_t m, int k, int had_block,
                                              int a_bits, int8_t *xq, float *x_scale, void *stream) {
    hq_status st = check_rowquant(x, x_dtype, m, k, k, had_block, a_bits, xq, x_scale);
    if (st != HQ_OK) return st;
    return act_hadamard_quant(x, x_dtype, m, k, had_block, a_bits, true, reinterpret_cast<uint8_t *>(xq), x_scale,
                              nullptr, stream);
}

extern "C" hq_status hq_act_hadamard_quant_static(const void *x, hq_dtype x_dtype, int64_t m, int k,
                                                  int had_block, int a_bits, const float *x_scale,
                                                  uint8_t *xq, void *stream) {
    hq_status st = check_rowquant(x, x_dtype, m, k, k, had_block, a_bits, xq, x_scale);
    if (st != HQ_OK) return st;
    return act_hadamard_quant(x, x_dtype, m, k, had_block, a_bits, false, xq, nullptr, x_scale, stream);
}

extern "C" hq_status hq_quantize_weights(const void *w, hq_dtype w_dtype, int n_out, int taps, int k_in,
                                         int had_block, int w_bits, uint8_t *wq, float *w_scale,
                                         void *stream) {
    if (taps <= 0) return (!w || !wq || !w_scale) ? HQ_ERR_NULL : HQ_ERR_SHAPE;
    const int64_t row_len = static_cast<int64_t>(taps) * k_in;
    hq_status st = check_rowquant(w, w_dtype, n_out, k_in, row_len, had_block, w_bits, wq, w_scale);
    if (st != HQ_OK) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t *out = reinterpret_cast<uint32_t *>(wq);
    const int len = static_cast<int>(row_len);
    if (w_dtype == HQ_F16)
        return dispatch_block(static_cast<const __half *>(w), n_out, len, had_block, w_bits, false, out, w_scale, nullptr, s);
    return dispatch_block(static_cast<const float *>(w), n_out, len, had_block, w_bits, false, out, w_scale, nullptr, s);
}

extern "C" const char *hq_status_string(hq_status s) {
    switch (s) {
        case HQ_OK: return "ok";
        case HQ_ERR_NULL: return "a required pointer is NULL";
        case HQ_ERR_SHAPE: return "bad shape";
        case HQ_ERR_DTYPE: return "bad dtype";
        case HQ_ERR_BITS: return "unsupported bit width";
        case HQ_ERR_ALIGN: return "pointer not 16-byte aligned";
        case HQ_ERR_UNSUPPORTED: return "configuration not supported";
        case HQ_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}
