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

#include <utility>

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

// Waits until at most N of this wave's vector-memory operations are outstanding
// (LDS / scalar counters untouched).
template <int N>
__device__ __forceinline__ void wait_vmem() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

__device__ __forceinline__ void load_to_lds16(const uint8_t *src, uint8_t *lds_wave_base) {
    // each lane's 16 bytes land at lds_wave_base + 16 * lane (the LDS base is wave-uniform)
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void *)src,
        (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

// LDS reads of the DMA-filled stages are written as inline asm: the compiler's
// wait-count pass cannot tell which stage a direct-to-LDS load targets and would
// otherwise drain every outstanding load (vmcnt(0)) before each LDS read, which
// serialises the pipeline.  The waits these reads need are placed by hand.
__device__ __forceinline__ uint32_t lds_address(const void *p) {
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((const __attribute__((address_space(3))) void *)p));
}

template <int OFFSET>
__device__ __forceinline__ v4i lds_read16(uint32_t addr) {
    v4i r;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFFSET) : "memory");
    return r;
}

__device__ __forceinline__ float lds_read_f32_now(uint32_t addr) {
    float r;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(r) : "v"(addr) : "memory");
    return r;
}

// dst[i] = 16 bytes at addr + STRIDE * i (one 32-row tile apart)
template <int STRIDE, int... I>
__device__ __forceinline__ void read_tiles(v4i *dst, uint32_t addr, std::integer_sequence<int, I...>) {
    ((dst[I] = lds_read16<I * STRIDE>(addr)), ...);
}

__device__ __forceinline__ void lds_wait_all() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// Ties a register to the point after the preceding hand-placed wait.
__device__ __forceinline__ void pin(v4i &v) { asm volatile("" : "+v"(v)); }

// TM x TN MFMA tiles of 32x32 per wave, WAVES_M x WAVES_N waves per workgroup.
// TAPS = 1 (linear / 1x1) or 9 (3x3, stride 1, pad 1).
//
// K is consumed in chunks of KCH 16-byte pieces per row (KCH * 32 codes); NSTAGE
// chunks of both operands live in LDS, filled by direct-to-LDS loads issued
// NSTAGE-1 chunks ahead of the MFMAs.  Inside a wave-wide load, KCH consecutive
// lanes fetch one row's contiguous KCH*16 bytes and consecutive lane groups
// fetch consecutive rows, so a load of activation rows reads one contiguous
// KiB; the LDS image of a stage is therefore row-major [row][KCH*16 bytes].
//
// Rows that do not exist (channels >= n, pixels >= pixels, taps outside the
// image) are loaded from a clamped in-bounds address instead of being zeroed:
// their sums are never stored, and a tap outside the image has scale 0.
template <int TM, int TN, int WAVES_M, int WAVES_N, int TAPS, int OUT, int KCH, int NSTAGE, int OCC>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, OCC) void int_gemm_kernel(GemmArgs a) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int kThreadsWg = 64 * NW;
    constexpr int BCO = 32 * TM * WAVES_M;   // output channels per workgroup
    constexpr int BP = 32 * TN * WAVES_N;    // pixels per workgroup
    constexpr int ROWB = KCH * 16;           // bytes per row per chunk
    static_assert(KCH % 2 == 0, "a 64-code K step is two pieces");
    static_assert((BCO * KCH) % 64 == 0 && (BP * KCH) % 64 == 0, "whole wave-wide loads only");
    constexpr int A_INSTR = BCO * KCH / 64, B_INSTR = BP * KCH / 64;   // 1 KiB loads per chunk
    static_assert((A_INSTR + B_INSTR) % NW == 0, "loads must split evenly over the waves");
    constexpr int LPW = (A_INSTR + B_INSTR) / NW;
    static_assert((NSTAGE - 2) * LPW < 64, "vmcnt range");
    constexpr int STAGE_BYTES = (BCO + BP) * ROWB;
    using Out = typename OutT<OUT>::type;

    // [stage][operand][row][ROWB bytes]
    __shared__ __attribute__((aligned(16))) uint8_t lds[NSTAGE * STAGE_BYTES];
    __shared__ float s_sx[TAPS][BP];   // x_scale / 256 of the input pixel under tap t; 0 outside
    __shared__ int s_mask[BP];         // bit t: tap t of this output pixel is inside the image

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
    const int lrow = lane & 31, lhalf = lane >> 5;

    const int tile_co = blockIdx.x % a.n_co_tiles;
    const int64_t tile_p = blockIdx.x / a.n_co_tiles;
    const int co0 = tile_co * BCO;
    const int64_t p0 = tile_p * BP;
    const int kbytes = a.k >> 1;                 // packed bytes per (row, tap)
    const int chunks_per_tap = kbytes / ROWB;    // host guarantees divisibility
    const int total_chunks = TAPS * chunks_per_tap;

    // ---- per-pixel tables ------------------------------------------------------------------
    for (int p = tid; p < BP; p += kThreadsWg) {
        const int64_t pix = p0 + p;
        const bool valid = pix < a.pixels;
        int mask = 0;
        if constexpr (TAPS > 1) {
            const int64_t q = pix / a.w;
            const int ow = static_cast<int>(pix - q * a.w);
            const int oh = static_cast<int>(q % a.h);
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                const int dr = t / 3 - 1, ds = t % 3 - 1;
                const bool ok = valid && oh + dr >= 0 && oh + dr < a.h && ow + ds >= 0 && ow + ds < a.w;
                mask |= ok ? (1 << t) : 0;
                if constexpr (OUT != kOutI32)
                    s_sx[t][p] = ok ? a.sx[pix + dr * a.w + ds] * (1.0f / 256.0f) : 0.f;
            }
        } else {
            mask = valid ? 1 : 0;
            if constexpr (OUT != kOutI32) s_sx[0][p] = valid ? a.sx[pix] * (1.0f / 256.0f) : 0.f;
        }
        s_mask[p] = mask;
    }
    __syncthreads();

    // ---- this wave's share of the direct-to-LDS loads -------------------------------------------
    uint32_t ld_off[LPW];     // byte offset of this lane's piece at tap 0, chunk 0
    int ld_mask[LPW];         // activation rows: taps inside the image
#pragma unroll
    for (int j = 0; j < LPW; ++j) {
        const int ii = j * NW + wave;          // wave-uniform
        if (ii < A_INSTR) {
            const int q = ii * 64 + lane;
            const int row = q / KCH, piece = q % KCH;
            int co = co0 + (row & ~31) + tile_row_to_channel(row & 31);
            co = co < a.n ? co : a.n - 1;
            ld_off[j] = static_cast<uint32_t>(co) * TAPS * kbytes + piece * 16;
            ld_mask[j] = 0;
        } else {
            const int q = (ii - A_INSTR) * 64 + lane;
            const int row = q / KCH, piece = q % KCH;
            int64_t pix = p0 + row;
            pix = pix < a.pixels ? pix : a.pixels - 1;
            ld_off[j] = static_cast<uint32_t>(pix) * kbytes + piece * 16;
            ld_mask[j] = s_mask[row];
        }
    }
    uint32_t ld_cur[LPW];     // ld_off + the term of the tap being fetched
    auto set_fetch_tap = [&](int t) {
        const int shift = TAPS > 1 ? ((t / 3 - 1) * a.w + (t % 3 - 1)) * kbytes : 0;
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            if (j * NW + wave < A_INSTR) ld_cur[j] = ld_off[j] + t * kbytes;
            else ld_cur[j] = ld_off[j] + (((ld_mask[j] >> t) & 1) ? shift : 0);
        }
    };
    auto issue_loads = [&](int stage, int chunk_in_tap) {
#pragma unroll
        for (int j = 0; j < LPW; ++j) {
            const int ii = j * NW + wave;
            const uint8_t *base = (ii < A_INSTR ? a.wq : a.xq) + chunk_in_tap * ROWB;
            // stage image: A rows then B rows, each wave-wide load fills the next 1 KiB
            load_to_lds16(base + ld_cur[j], lds + stage * STAGE_BYTES + ii * 1024);
        }
    };

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

    const uint32_t lds_a = lds_address(lds) + (wave_m * TM * 32 + lrow) * ROWB + lhalf * 16;
    const uint32_t lds_b = lds_address(lds) + BCO * ROWB + (wave_n * TN * 32 + lrow) * ROWB + lhalf * 16;
    const uint32_t lds_sx = lds_address(&s_sx[0][0]) + (wave_n * TN * 32 + lrow) * 4;

    // ---- prologue: fill NSTAGE-1 stages ------------------------------------------------------
    int ftap = 0, fch = 0, fetched = 0;   // chunk being fetched
    set_fetch_tap(0);
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) {
        if (fetched < total_chunks) {
            issue_loads(s, fch);
            ++fetched;
            if (++fch == chunks_per_tap) { fch = 0; ++ftap; if (ftap < TAPS) set_fetch_tap(ftap); }
        }
    }

    int tap = 0, ch = 0;
    for (int chunk = 0; chunk < total_chunks; ++chunk) {
        const int stage = chunk % NSTAGE;
        // this chunk has landed once at most the later (NSTAGE-2) chunks' loads are pending
        if (chunk + NSTAGE - 2 < total_chunks) wait_vmem<(NSTAGE - 2) * LPW>();
        else wait_vmem<0>();
        __builtin_amdgcn_s_barrier();   // every wave's share has landed; the previous stage is free
        if (fetched < total_chunks) {
            issue_loads((chunk + NSTAGE - 1) % NSTAGE, fch);
            ++fetched;
            if (++fch == chunks_per_tap) { fch = 0; ++ftap; if (ftap < TAPS) set_fetch_tap(ftap); }
        }

        const uint32_t sa = lds_a + stage * STAGE_BYTES, sb = lds_b + stage * STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < KCH / 2; ++ks) {
            v4i pa[TM], pb[TN];
            read_tiles<32 * ROWB>(pa, sa + ks * 32, std::make_integer_sequence<int, TM>{});
            read_tiles<32 * ROWB>(pb, sb + ks * 32, std::make_integer_sequence<int, TN>{});
            lds_wait_all();
            v4i a0[TM], a1[TM], b0[TN], b1[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) { pin(pa[tm]); unpack16(pa[tm], a0[tm], a1[tm]); }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) { pin(pb[tn]); unpack16(pb[tn], b0[tn], b1[tn]); }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[tm], b0[tn], acc[tm][tn], 0, 0, 0);
                    acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[tm], b1[tn], acc[tm][tn], 0, 0, 0);
                }
        }

        if (++ch == chunks_per_tap) {
            ch = 0;
            // ---- end of a tap: fold the integer sums into the result ----------------------
            if constexpr (OUT == kOutI32) {
                int *yi = static_cast<int *>(a.y);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const int prow = (wave_n * TN + tn) * 32 + lrow;
                    const int64_t pix = p0 + prow;
                    const bool inside = (s_mask[prow] >> tap) & 1;   // also false for pixels >= pixels
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
                        const int cbase = co0 + (wave_m * TM + tm) * 32 + 16 * lhalf;
                        if (pix < a.pixels) {
                            int *dst = yi + (pix * TAPS + tap) * a.n + cbase;
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (cbase + r < a.n) dst[r] = inside ? (acc[tm][tn][r] >> 8) : 0;
                        }
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[tm][tn][r] = 0;
                    }
                }
            } else if constexpr (TAPS > 1) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const float s = lds_read_f32_now(lds_sx + (tap * BP + tn * 32) * 4);
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            facc[tm][tn][r] += s * static_cast<float>(acc[tm][tn][r]);
                            acc[tm][tn][r] = 0;
                        }
                }
            }
            ++tap;
        }
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
                const int prow = (wave_n * TN + tn) * 32 + lrow;
                const int64_t pix = p0 + prow;
                if (pix >= a.pixels) continue;
                float out[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float s;
                    if constexpr (TAPS > 1) s = facc[tm][tn][r];
                    else s = s_sx[0][prow] * static_cast<float>(acc[tm][tn][r]);
                    out[r] = s * swv[r] + bv[r];
                }
                Out *dst = y + pix * a.n + cbase;
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

template <int TM, int TN, int WAVES_M, int WAVES_N, int TAPS, int OUT, int KCH, int NSTAGE, int OCC>
hq_status launch_tile(GemmArgs a, hipStream_t stream) {
    constexpr int BCO = 32 * TM * WAVES_M, BP = 32 * TN * WAVES_N;
    a.n_co_tiles = (a.n + BCO - 1) / BCO;
    const int64_t p_tiles = (a.pixels + BP - 1) / BP;
    const int64_t grid = p_tiles * a.n_co_tiles;
    if (grid > 0x7fffffffLL) return HQ_ERR_SHAPE;
    hipLaunchKernelGGL((int_gemm_kernel<TM, TN, WAVES_M, WAVES_N, TAPS, OUT, KCH, NSTAGE, OCC>),
                       dim3(static_cast<unsigned>(grid)), dim3(64 * WAVES_M * WAVES_N), 0, stream, a);
    return hq::launch_status();
}

template <int TAPS, int OUT>
hq_status launch_shape(const GemmArgs &a, hipStream_t stream) {
    // chunks of 192 codes (96 contiguous bytes per row) whenever the channel count allows
    if (a.k % 192 == 0) return launch_tile<2, 2, 2, 2, TAPS, OUT, 6, 3, 2>(a, stream);
    return launch_tile<2, 2, 2, 2, TAPS, OUT, 2, 4, 2>(a, stream);
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

// The kernels address the packed operands with 32-bit byte offsets.
bool fits_32bit_offsets(int64_t pixels, int n, int taps, int k) {
    const int64_t lim = 0xFFFFFFFFLL;
    return pixels * (k / 2) <= lim && static_cast<int64_t>(n) * taps * (k / 2) <= lim;
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
    if (!fits_32bit_offsets(m, n, 1, k)) return HQ_ERR_UNSUPPORTED;
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
    if (!fits_32bit_offsets(pixels, c_out, r * s, c_in)) return HQ_ERR_UNSUPPORTED;
    GemmArgs a{xq, x_scale, wq, w_scale, bias, y, pixels, c_out, c_in, h, w, 0};
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    return r == 1 ? launch_out<1>(a, y_dtype, st_) : launch_out<9>(a, y_dtype, st_);
}
