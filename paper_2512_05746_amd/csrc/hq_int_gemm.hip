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
// Nibble handling.  Codes are packed (two per byte) in HBM.  They are expanded
// to int8 once per workgroup, on the way from global memory to LDS: a packed
// dword w becomes the two int8x4 vectors
//     lo = (w << 4) & 0xF0F0F0F0,   hi = w & 0xF0F0F0F0,
// each byte holding 16 * code exactly (two's complement).  Both operands are
// stored that way, so the MFMA accumulates 256 * sum(xq * wq); the factor is
// exact and is removed by an arithmetic shift (int32 output) or folded into the
// activation scale (floating-point output).  The order in which the codes of a
// 64-wide K step reach the MFMA lanes is a permutation applied identically to
// both operands, which leaves the sum unchanged.
//
// The kernel is bound by vector-ALU issue slots, not by the matrix pipe (one
// 32x32x32 MFMA leaves room for about seven other vector instructions), so the
// expansion is shared by all waves of a workgroup instead of being repeated by
// every wave on its own operands, and the accumulators are never cleared by
// moves: the first MFMA of a tap takes the constant 0 as its addend.
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
    uint32_t pixels;     // rows of the activation matrix (= nb*h*w for a convolution)
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

// 16 packed bytes (32 codes) -> two 16-byte units of int8 (16 * code each)
__device__ __forceinline__ void expand(const v4i &p, v4i &first, v4i &second) {
    const int m = static_cast<int>(0xF0F0F0F0u);
    first = v4i{(p.x << 4) & m, p.x & m, (p.y << 4) & m, p.y & m};
    second = v4i{(p.z << 4) & m, p.z & m, (p.w << 4) & m, p.w & m};
}

// Asynchronous 16-byte global load, written as inline asm so that the waits can be
// placed by hand: requests are issued four K steps ahead and the compiler's own
// wait-count bookkeeping, which is conservative across the loop back-edge, would
// drain them one step after issue.  `base` is wave-uniform, `offset` per lane.
// The result may only be read after wait_vmem<N>() + pin().
__device__ __forceinline__ void load16_async(v4i &dst, const uint8_t *base, uint32_t offset) {
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(dst) : "v"(offset), "s"(base) : "memory");
}

// Waits until at most N of this wave's vector-memory operations are outstanding.
template <int N>
__device__ __forceinline__ void wait_vmem() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

// Ties a register to the point after the preceding hand-placed wait.
__device__ __forceinline__ void pin(v4i &v) { asm volatile("" : "+v"(v)); }

// Bit t set: tap t = (r, s) of a 3x3 / pad 1 window around pixel `pix` lies inside its image.
template <int TAPS>
__device__ __forceinline__ int tap_mask(uint32_t pix, int h, int w) {
    if constexpr (TAPS == 1) {
        return 1;
    } else {
        const uint32_t q = pix / static_cast<uint32_t>(w);
        const int ow = static_cast<int>(pix - q * w);
        const int oh = static_cast<int>(q % static_cast<uint32_t>(h));
        int mask = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int ih = oh + t / 3 - 1, iw = ow + t % 3 - 1;
            mask |= (ih >= 0 && ih < h && iw >= 0 && iw < w) ? (1 << t) : 0;
        }
        return mask;
    }
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
//
// One K step is 64 codes (32 packed bytes per row, two 16-byte pieces).  While
// step s is being multiplied from registers, the MFMA operands of step s+1 are
// read from LDS, the packed pieces of step s+2 (fetched two steps earlier) are
// expanded into a third LDS stage, and the pieces of step s+4 are requested
// from global memory; one barrier per step.  LDS stage layout per operand:
// [unit 0..3][row][16 bytes] with unit = 2 * (k slice) + (lane half).  A thread
// writes units u and u+2 of its row with one instruction each, so the unit
// stride is padded by 64 bytes: two units apart is then half a bank cycle away,
// and both the expanding writes and the operand reads are conflict free.
//
// Rows that do not exist (channels >= n, pixels >= pixels, taps outside the
// image) are loaded from a clamped in-bounds address instead of being zeroed:
// their sums are never stored, and a tap outside the image has scale 0.
template <int TM, int TN, int WAVES_M, int WAVES_N, int TAPS, int OUT, int OCC>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, OCC) void int_gemm_kernel(GemmArgs a) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int NT = 64 * NW;
    constexpr int BCO = 32 * TM * WAVES_M;   // output channels per workgroup
    constexpr int BP = 32 * TN * WAVES_N;    // pixels per workgroup
    constexpr int A_PIECES = 2 * BCO, B_PIECES = 2 * BP;
    constexpr int A_PER_T = (A_PIECES + NT - 1) / NT, B_PER_T = (B_PIECES + NT - 1) / NT;
    static_assert(A_PIECES % 64 == 0 && B_PIECES % 64 == 0, "piece guards must be wave-uniform");
    static_assert(2 * (A_PER_T + B_PER_T) < 64, "vmcnt range");
    constexpr int A_US = BCO * 16 + 64, B_US = BP * 16 + 64;   // unit strides (see below)
    constexpr int A_BYTES = 4 * A_US, STAGE_BYTES = 4 * (A_US + B_US);
    using Out = typename OutT<OUT>::type;

    __shared__ __attribute__((aligned(16))) uint8_t lds[3 * STAGE_BYTES];
    __shared__ float s_sx[TAPS][BP];   // x_scale / 256 of the input pixel under tap t; 0 outside
    __shared__ int s_mask[BP];         // bit t: tap t of this output pixel is inside the image
    __shared__ __attribute__((aligned(16))) float s_sw[BCO];     // w_scale of the tile's channels
    __shared__ __attribute__((aligned(16))) float s_bias[BCO];   // bias (0 if absent)
    constexpr int NL = A_PER_T + B_PER_T;   // loads every thread issues per K step

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
    const int lrow = lane & 31, lhalf = lane >> 5;

    const int tile_co = blockIdx.x % a.n_co_tiles;
    const uint32_t tile_p = blockIdx.x / a.n_co_tiles;
    const int co0 = tile_co * BCO;
    const uint32_t p0 = tile_p * BP;
    const int kbytes = a.k >> 1;      // packed bytes per (row, tap)
    const int kc_steps = a.k >> 6;    // 64-code steps per tap
    const int total_steps = TAPS * kc_steps;

    // ---- this thread's pieces of a K step -----------------------------------------------------
    // Piece = 16 packed bytes of one row: (row, pc) with pc = 0, 1.  Every thread issues the
    // same number of loads per step (the hand-placed wait counts rely on it); with fewer
    // pieces than threads the surplus threads re-load a piece and do not store it.
    uint32_t a_off[A_PER_T];   // byte offset of the piece at flattened step 0
    int a_lds[A_PER_T];
#pragma unroll
    for (int j = 0; j < A_PER_T; ++j) {
        const int piece = (tid + j * NT) % A_PIECES;
        const int row = piece >> 1, pc = piece & 1;
        int co = co0 + (row & ~31) + tile_row_to_channel(row & 31);
        co = co < a.n ? co : a.n - 1;
        a_off[j] = static_cast<uint32_t>(co) * TAPS * kbytes + pc * 16;
        a_lds[j] = (2 * pc) * A_US + row * 16;
    }
    uint32_t b_off[B_PER_T];   // byte offset of the piece at tap "own pixel", k 0
    int b_mask[B_PER_T];       // bit t: tap t of the row's pixel is inside the image
    int b_lds[B_PER_T];
#pragma unroll
    for (int j = 0; j < B_PER_T; ++j) {
        const int piece = (tid + j * NT) % B_PIECES;
        const int row = piece >> 1, pc = piece & 1;
        uint32_t pix = p0 + row;
        pix = pix < a.pixels ? pix : a.pixels - 1;
        b_off[j] = pix * kbytes + pc * 16;
        b_mask[j] = tap_mask<TAPS>(pix, a.h, a.w);
        b_lds[j] = A_BYTES + (2 * pc) * B_US + row * 16;
    }

    v4i ga[2][A_PER_T], gb[2][B_PER_T];   // two register stages of packed pieces
    int ftap = 0, fkc = 0, fstep = 0;     // step being fetched
    // Issues the loads of the next step to fetch (asynchronous; see wait_vmem below).
    auto fetch = [&](v4i(&ra)[A_PER_T], v4i(&rb)[B_PER_T]) {
        if (fstep >= total_steps) return;
        const uint8_t *wbase = a.wq + fstep * 32;      // taps are contiguous in a weight row
        int shift = 0;
        if constexpr (TAPS > 1) shift = ((ftap / 3 - 1) * a.w + (ftap % 3 - 1)) * kbytes;
        const uint8_t *xbase = a.xq + fkc * 32;
#pragma unroll
        for (int j = 0; j < A_PER_T; ++j) load16_async(ra[j], wbase, a_off[j]);
#pragma unroll
        for (int j = 0; j < B_PER_T; ++j)
            load16_async(rb[j], xbase, b_off[j] + (((b_mask[j] >> ftap) & 1) ? shift : 0));
        ++fstep;
        if (++fkc == kc_steps) { fkc = 0; ++ftap; }
    };
    auto expand_to_lds = [&](int stage, v4i(&ra)[A_PER_T], v4i(&rb)[B_PER_T]) {
        uint8_t *base = lds + stage * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < A_PER_T; ++j) {
            pin(ra[j]);
            if ((j + 1) * NT <= A_PIECES || tid + j * NT < A_PIECES) {
                v4i u0, u1;
                expand(ra[j], u0, u1);
                *reinterpret_cast<v4i *>(base + a_lds[j]) = u0;
                *reinterpret_cast<v4i *>(base + a_lds[j] + A_US) = u1;
            }
        }
#pragma unroll
        for (int j = 0; j < B_PER_T; ++j) {
            pin(rb[j]);
            if ((j + 1) * NT <= B_PIECES || tid + j * NT < B_PIECES) {
                v4i u0, u1;
                expand(rb[j], u0, u1);
                *reinterpret_cast<v4i *>(base + b_lds[j]) = u0;
                *reinterpret_cast<v4i *>(base + b_lds[j] + B_US) = u1;
            }
        }
    };

    // ---- prologue, part 1: the first four steps are requested before anything else ---------
    fetch(ga[0], gb[0]);
    fetch(ga[1], gb[1]);

    // ---- per-pixel and per-channel tables (their loads overlap the requests above) ----------
    for (int p = tid; p < BP; p += NT) {
        const uint32_t pix = p0 + p;
        const bool valid = pix < a.pixels;
        const int mask = valid ? tap_mask<TAPS>(pix, a.h, a.w) : 0;
        if constexpr (OUT != kOutI32) {
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                const int delta = TAPS > 1 ? (t / 3 - 1) * a.w + (t % 3 - 1) : 0;
                s_sx[t][p] = ((mask >> t) & 1) ? a.sx[static_cast<int64_t>(pix) + delta] * (1.0f / 256.0f) : 0.f;
            }
        }
        s_mask[p] = mask;
    }
    if constexpr (OUT != kOutI32) {
        const Out *bias = static_cast<const Out *>(a.bias);
        for (int c = tid; c < BCO; c += NT) {
            const int co = co0 + c;
            s_sw[c] = co < a.n ? a.sw[co] : 0.f;
            s_bias[c] = (co < a.n && bias) ? to_float(bias[co]) : 0.f;
        }
    }

    v16i acc[TM][TN];
    float facc[TAPS > 1 ? TM : 1][TAPS > 1 ? TN : 1][16];
    if constexpr (TAPS > 1) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) facc[tm][tn][r] = 0.f;
    }

    const int rd_a = lhalf * A_US + (wave_m * TM * 32 + lrow) * 16;
    const int rd_b = A_BYTES + lhalf * B_US + (wave_n * TN * 32 + lrow) * 16;

    // MFMA operands of one K step: [k slice][tile]
    struct Operands { v4i a[2][TM]; v4i b[2][TN]; };
    auto read_operands = [&](int stage, Operands &o) {
        const uint8_t *sa = lds + stage * STAGE_BYTES + rd_a;
        const uint8_t *sb = lds + stage * STAGE_BYTES + rd_b;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                o.a[ks][tm] = *reinterpret_cast<const v4i *>(sa + tm * 512 + 2 * ks * A_US);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                o.b[ks][tn] = *reinterpret_cast<const v4i *>(sb + tn * 512 + 2 * ks * B_US);
        }
    };

    int tap = 0, kc = 0;   // step being multiplied
    int st_cur = 0;        // LDS stage of the step being multiplied (step % 3)
    // One K step s.  On entry `cur` holds the operands of s, LDS stage (s+1)%3 holds step
    // s+1, and `g` holds the packed pieces of step s+2 (requested two iterations ago; the
    // only requests issued since are the NL of the previous iteration).
    auto iteration = [&](int step, const Operands &cur, Operands &nxt, v4i(&g_a)[A_PER_T],
                         v4i(&g_b)[B_PER_T]) {
        const int st_next = st_cur == 2 ? 0 : st_cur + 1;
        const int st_far = st_next == 2 ? 0 : st_next + 1;
        if (step + 1 < total_steps) read_operands(st_next, nxt);

        if (kc == 0) {
            const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur.a[0][tm], cur.b[0][tn], zero, 0, 0, 0);
        } else {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur.a[0][tm], cur.b[0][tn], acc[tm][tn], 0, 0, 0);
        }
        if (step + 2 < total_steps) {
            if (step + 3 < total_steps) wait_vmem<NL>();   // the previous iteration's requests may stay pending
            else wait_vmem<0>();
            expand_to_lds(st_far, g_a, g_b);
        }
        fetch(g_a, g_b);   // step + 4
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(cur.a[1][tm], cur.b[1][tn], acc[tm][tn], 0, 0, 0);

        if (++kc == kc_steps) {
            kc = 0;
            // ---- end of a tap: fold the integer sums into the result ----------------------
            if constexpr (OUT == kOutI32) {
                int *yi = static_cast<int *>(a.y);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const int prow = (wave_n * TN + tn) * 32 + lrow;
                    const uint32_t pix = p0 + prow;
                    const bool inside = (s_mask[prow] >> tap) & 1;   // also false for pixels >= pixels
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
                        const int cbase = co0 + (wave_m * TM + tm) * 32 + 16 * lhalf;
                        if (pix < a.pixels) {
                            int *dst = yi + (static_cast<int64_t>(pix) * TAPS + tap) * a.n + cbase;
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (cbase + r < a.n) dst[r] = inside ? (acc[tm][tn][r] >> 8) : 0;
                        }
                    }
                }
            } else if constexpr (TAPS > 1) {
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const float s = s_sx[tap][(wave_n * TN + tn) * 32 + lrow];
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            facc[tm][tn][r] += s * static_cast<float>(acc[tm][tn][r]);
                }
            }
            ++tap;
        }
        st_cur = st_next;
        __syncthreads();
    };

    // ---- prologue, part 2: steps 0 and 1 into LDS, steps 2 and 3 requested ----------------------
    wait_vmem<0>();
    expand_to_lds(0, ga[0], gb[0]);
    if (total_steps > 1) expand_to_lds(1, ga[1], gb[1]);
    fetch(ga[0], gb[0]);
    fetch(ga[1], gb[1]);
    __syncthreads();
    Operands op0, op1;
    read_operands(0, op0);
    for (int step = 0; step < total_steps; step += 2) {
        iteration(step, op0, op1, ga[0], gb[0]);
        if (step + 1 < total_steps) iteration(step + 1, op1, op0, ga[1], gb[1]);
    }

    // ---- dequantising epilogue -------------------------------------------------------------
    if constexpr (OUT != kOutI32) {
        Out *y = static_cast<Out *>(a.y);
        const bool vec_ok = (a.n & 15) == 0;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int clocal = (wave_m * TM + tm) * 32 + 16 * lhalf;
            const int cbase = co0 + clocal;
            float swv[16], bv[16];
#pragma unroll
            for (int r = 0; r < 16; r += 4) {
                const float4 s4 = *reinterpret_cast<const float4 *>(&s_sw[clocal + r]);
                const float4 b4 = *reinterpret_cast<const float4 *>(&s_bias[clocal + r]);
                swv[r] = s4.x; swv[r + 1] = s4.y; swv[r + 2] = s4.z; swv[r + 3] = s4.w;
                bv[r] = b4.x; bv[r + 1] = b4.y; bv[r + 2] = b4.z; bv[r + 3] = b4.w;
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int prow = (wave_n * TN + tn) * 32 + lrow;
                const uint32_t pix = p0 + prow;
                if (pix >= a.pixels) continue;
                float out[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float s;
                    if constexpr (TAPS > 1) s = facc[tm][tn][r];
                    else s = s_sx[0][prow] * static_cast<float>(acc[tm][tn][r]);
                    out[r] = s * swv[r] + bv[r];
                }
                Out *dst = y + static_cast<int64_t>(pix) * a.n + cbase;
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

template <int TM, int TN, int WAVES_M, int WAVES_N, int TAPS, int OUT, int OCC>
hq_status launch_tile(GemmArgs a, hipStream_t stream) {
    constexpr int BCO = 32 * TM * WAVES_M, BP = 32 * TN * WAVES_N;
    a.n_co_tiles = (a.n + BCO - 1) / BCO;
    const int64_t p_tiles = (static_cast<int64_t>(a.pixels) + BP - 1) / BP;
    const int64_t grid = p_tiles * a.n_co_tiles;
    if (grid > 0x7fffffffLL) return HQ_ERR_SHAPE;
    hipLaunchKernelGGL((int_gemm_kernel<TM, TN, WAVES_M, WAVES_N, TAPS, OUT, OCC>),
                       dim3(static_cast<unsigned>(grid)), dim3(64 * WAVES_M * WAVES_N), 0, stream, a);
    return hq::launch_status();
}

template <int TAPS, int OUT>
hq_status launch_shape(const GemmArgs &a, hipStream_t stream) {
    return launch_tile<2, 2, 2, 2, TAPS, OUT, 2>(a, stream);
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

// The kernels index pixels with 32 bits and address the packed operands with
// 32-bit byte offsets.
bool fits_32bit(int64_t pixels, int n, int taps, int k) {
    const int64_t lim = 0xFFFFFFFFLL;
    return pixels < 0x7FFFFFFFLL && pixels * (k / 2) <= lim &&
           static_cast<int64_t>(n) * taps * (k / 2) <= lim;
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
    if (!fits_32bit(m, n, 1, k)) return HQ_ERR_UNSUPPORTED;
    GemmArgs a{xq, x_scale, wq, w_scale, bias, y, static_cast<uint32_t>(m), n, k, 1, 1, 0};
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
    if (!fits_32bit(pixels, c_out, r * s, c_in)) return HQ_ERR_UNSUPPORTED;
    GemmArgs a{xq, x_scale, wq, w_scale, bias, y, static_cast<uint32_t>(pixels), c_out, c_in, h, w, 0};
    hipStream_t st_ = static_cast<hipStream_t>(stream);
    return r == 1 ? launch_out<1>(a, y_dtype, st_) : launch_out<9>(a, y_dtype, st_);
}
