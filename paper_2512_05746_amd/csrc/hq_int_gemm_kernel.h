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
// Nibble handling.  Codes stay packed (two per byte) in HBM and in LDS; the copy
// from global memory to LDS is a direct-to-LDS load that touches no register.
// A wave expands the packed operands it has read from LDS in registers: a packed
// dword w becomes the two int8x4 vectors
//     lo = (w << 4) & 0xF0F0F0F0,   hi = w & 0xF0F0F0F0,
// each byte holding 16 * code exactly (two's complement).  Both operands are
// fed that way, so the MFMA accumulates 256 * sum(xq * wq); the factor is exact
// and is removed by an arithmetic shift (int32 output) or folded into the
// activation scale (floating-point output).  The order in which the codes of a
// 64-wide K step reach the MFMA lanes is a permutation applied identically to
// both operands, which leaves the sum unchanged.
//
// Why packed in LDS: measured on MI355X, LDS accepts writes at about 64 bytes per
// clock per CU (reads: about 256), and one 32x32x32 int8 MFMA leaves issue room
// for about seven other vector instructions.  Expanding to int8 before LDS
// doubles the LDS write volume and made that the bound; expanding after the read
// costs three vector instructions per packed dword instead.  The accumulators
// are never cleared by moves: the first MFMA of a tap takes the constant 0 as
// its addend.
#pragma once
#include <hip/hip_fp16.h>

#include "hq_common.h"

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
    uint32_t n_tiles;    // pixel tiles * channel tiles
    uint32_t xcds;       // 1: deal the tiles out per XCD (grid is a multiple of 8); 0: plain grid stride
    uint32_t cus;        // compute units of the device (workgroups b and b + cus tend to share a CU)
    int sx_static;       // sx is ONE scale for the whole activation tensor (a 3x3 convolution then keeps
                         // one integer sum over all taps)
    float out_scale;     // factor applied with w_scale (1, or 2^(-log2(block)/2) for digit-plane weights)
    int bits;            // 4: two codes per byte (3-bit codes included); 8: one int8 code per byte
    // 3x3 convolution with stride 2 (pad 1): `pixels` counts OUTPUT pixels [nb, h_out, w_out], h and w
    // are the INPUT image size, in_pixels = nb * h * w.  stride 0 or 1: same-size output.
    int stride;
    int h_out, w_out;
    uint32_t in_pixels;
};

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kOutF16 = 0, kOutF32 = 1, kOutI32 = 2;
// What a kernel instance computes: a linear layer / 1x1 convolution; a 3x3 convolution whose
// integer sums are kept per tap (every input pixel has its own scale); a 3x3 convolution with
// one integer sum over all taps (one scale for the tensor); a linear layer whose weights are
// three base-16 digit planes [n, 3, k/2] of wider integers (one integer sum per plane, plane p
// weighted by 16^p when the sums are combined in fp32) - three "taps" that all read the same row;
// a 3x3 convolution whose ACTIVATIONS are three such digit planes [3, pixels, k/2] (one scale for
// the tensor): 27 steps, plane-major, one integer sum per plane over its nine taps.
constexpr int kLinear = 0, kConvPerTap = 1, kConvSum = 2, kPlanes = 3, kConvPlanes = 4;
// The same two kinds walking only the two low digit planes (the third is known to be zero when the
// integers it encodes cannot exceed two signed base-16 digits, i.e. 8 x block <= 119).
constexpr int kPlanes2 = 5, kConvPlanes2 = 6;
constexpr bool is_planes(int kind) { return kind == kPlanes || kind == kPlanes2; }
constexpr bool is_conv_planes(int kind) { return kind == kConvPlanes || kind == kConvPlanes2; }

// steps of a tile's tap loop
constexpr int taps_of(int kind) {
    return kind == kLinear ? 1 : kind == kPlanes ? 3 : kind == kPlanes2 ? 2 : kind == kConvPlanes ? 27
           : kind == kConvPlanes2 ? 18 : 9;
}


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

// Waits until at most N of this wave's vector-memory operations are outstanding.
template <int N>
__device__ __forceinline__ void wait_vmem() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

// Waits until at most N of this wave's LDS / scalar-memory operations are outstanding.
template <int N>
__device__ __forceinline__ void wait_lds() {
    static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit counter");
    __builtin_amdgcn_s_waitcnt(0xC07F | (N << 8));
}

// Direct-to-LDS load: lane i's 16 bytes land at lds_wave_base + 16 * i (the LDS base is
// wave-uniform).  Completion is tracked by vmcnt only.
__device__ __forceinline__ void load_to_lds16(const uint8_t *src, uint8_t *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

// LDS reads of the DMA-filled stages are inline asm: the compiler cannot tell which
// stage a direct-to-LDS load targets and would drain every outstanding load (vmcnt(0))
// before each LDS read it knows of, which serialises the pipeline.  The waits these
// reads need (wait_lds) and the register pinning after them are placed by hand.
__device__ __forceinline__ uint32_t lds_address(const void *p) {
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((const __attribute__((address_space(3))) void *)p));
}

template <int OFFSET>
__device__ __forceinline__ void lds_read16(v4i &dst, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFFSET) : "memory");
}

template <int OFFSET>
__device__ __forceinline__ void lds_read_f32(float &dst, uint32_t addr) {
    asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFFSET) : "memory");
}

template <int OFFSET>
__device__ __forceinline__ void lds_write16(uint32_t addr, const v4i &v) {
    asm volatile("ds_write_b128 %0, %1 offset:%2" : : "v"(addr), "v"(v), "n"(OFFSET) : "memory");
}

// fp16 results of a 32-channel x 32-pixel MFMA tile (v: the lane's 16 consecutive channels of pixel
// lane % 32, channel half lane / 32) through a 2 KiB staging area of the wave in LDS, laid out
// [pixel][32 channels]: afterwards lane l holds the 16-byte piece l % 4 of pixels l / 4 (r0) and
// 16 + l / 4 (r1), so that four neighbouring lanes store the 64 contiguous bytes of one pixel
// instead of every lane storing a piece 2 n bytes away from its neighbour's.
__device__ __forceinline__ void transpose_tile_f16(const float (&v)[16], uint32_t staging, int lane, v4i &r0, v4i &r1) {
    uint32_t h[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const __half2 two = __floats2half2_rn(v[2 * i], v[2 * i + 1]);
        h[i] = *reinterpret_cast<const uint32_t *>(&two);
    }
    const v4i w0 = {static_cast<int>(h[0]), static_cast<int>(h[1]), static_cast<int>(h[2]), static_cast<int>(h[3])};
    const v4i w1 = {static_cast<int>(h[4]), static_cast<int>(h[5]), static_cast<int>(h[6]), static_cast<int>(h[7])};
    const uint32_t wr = staging + (lane & 31) * 64 + (lane >> 5) * 32;
    lds_write16<0>(wr, w0);
    lds_write16<16>(wr, w1);
    __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0): the wave's own stores are in LDS
    asm volatile("ds_read_b128 %0, %1" : "=v"(r0) : "v"(staging + lane * 16) : "memory");
    asm volatile("ds_read_b128 %0, %1 offset:1024" : "=v"(r1) : "v"(staging + lane * 16) : "memory");
    __builtin_amdgcn_s_waitcnt(0xC07F);
    asm volatile("" : "+v"(r0), "+v"(r1));
}

// Ties a register to the point after the preceding hand-placed wait.
__device__ __forceinline__ void pin(v4i &v) { asm volatile("" : "+v"(v)); }

// Source of the activation rows of taps that fall outside the image when all taps share one
// integer sum (they must then contribute zeros, not merely be ignored).
__device__ __attribute__((aligned(128))) const uint8_t g_zero_row[128] = {0};

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

// Packed MFMA operands of one 64-code K step, as read from LDS.
template <int TM, int TN>
struct Packed {
    v4i a[TM];
    v4i b[TN];
};

// KOFF: byte offset of the K step inside the chunk row (an immediate of the read)
template <int TM, int TN, int ROWB, int KOFF, int I = 0>
__device__ __forceinline__ void read_packed(Packed<TM, TN> &o, uint32_t addr_a, uint32_t addr_b) {
    if constexpr (I < TM) {
        lds_read16<I * 32 * ROWB + KOFF>(o.a[I], addr_a);
        read_packed<TM, TN, ROWB, KOFF, I + 1>(o, addr_a, addr_b);
    } else if constexpr (I < TM + TN) {
        lds_read16<(I - TM) * 32 * ROWB + KOFF>(o.b[I - TM], addr_b);
        read_packed<TM, TN, ROWB, KOFF, I + 1>(o, addr_a, addr_b);
    }
}

// The K steps of one chunk: the packed operands of step K+1 are requested before the MFMAs of
// step K are issued.  mul(operands, first) multiplies one step; first: the sums start from 0.
template <int K, int KS, int TM, int TN, int ROWB, class Mul>
__device__ __forceinline__ void chunk_steps(Packed<TM, TN> (&op)[2], uint32_t addr_a, uint32_t addr_b,
                                            bool first_of_tap, Mul &mul) {
    if constexpr (K < KS) {
        if constexpr (K + 1 < KS) {
            read_packed<TM, TN, ROWB, (K + 1) * 32>(op[(K + 1) & 1], addr_a, addr_b);
            wait_lds<TM + TN>();   // everything but the reads just issued
        } else {
            wait_lds<0>();
        }
        mul(op[K & 1], K == 0 && first_of_tap);
        chunk_steps<K + 1, KS, TM, TN, ROWB>(op, addr_a, addr_b, first_of_tap, mul);
    }
}

// The TN per-pixel scales of one tap (32 pixels apart in the table), read together.
template <int TN, int I = 0>
__device__ __forceinline__ void read_tap_scales(float (&s)[TN], uint32_t addr) {
    if constexpr (I < TN) {
        lds_read_f32<I * 32 * 4>(s[I], addr);
        read_tap_scales<TN, I + 1>(s, addr);
    } else {
        wait_lds<0>();
#pragma unroll
        for (int i = 0; i < TN; ++i) asm volatile("" : "+v"(s[i]));
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
// The tap loop of a tile has 1 step (linear / 1x1), 9 (3x3, stride 1, pad 1), 3 (weight digit
// planes) or 27 (activation digit planes of a 3x3 convolution); see the kinds above.
//
// Persistent workgroups: the grid is sized to the machine and every workgroup
// walks a contiguous run of tiles (output-channel tiles of one pixel tile are
// adjacent).  With a.xcds set, workgroup b is taken to run on XCD b % 8 (the
// dispatcher deals workgroups round-robin over the eight XCDs) and each XCD
// gets one contiguous eighth of the tiles, so the activation rows a tile shares
// with its neighbours are fetched into one L2 only.  All chunks of all tiles of a
// workgroup form ONE stream through the LDS stages, so the loads of the next
// tile's first chunks are in flight while the current tile is finished and
// written out, and the scale tables of the next tile are built during the
// current one (two table sets).
//
// K is consumed in chunks of KCH 16-byte pieces per row (KCH * 32 codes); NSTAGE
// chunks of both operands live in LDS, filled by direct-to-LDS loads issued
// NSTAGE-1 chunks ahead of the MFMAs; one barrier per chunk.  Inside a wave-wide
// load, KCH consecutive lanes fetch one row's contiguous KCH*16 bytes and
// consecutive lane groups fetch consecutive rows, so a load of activation rows
// reads one contiguous KiB.  The LDS image of a stage is row-major
// [row][KCH*16 bytes]; in rows 8..15 (mod 16) adjacent pieces are swapped, which
// makes the 16-byte operand reads of 16 consecutive rows hit 16 different bank
// groups.  Inside a chunk the packed operands of K step k+1 are read from LDS
// while the MFMAs of step k run.
//
// Addresses.  A load is "uniform base + per-lane 32-bit offset".  The per-lane
// offsets are set once per tile; the position inside the row (chunk) and the
// weight tap move the uniform base only.  For a 3x3 tap the activation offset
// is shifted by a uniform number of pixels and clamped to the last pixel
// (unsigned: a shift below pixel 0 wraps and clamps too), two vector
// instructions per load and tap.  So rows that do not exist (channels >= n,
// pixels >= pixels) and taps outside the image read some other in-bounds row
// instead of zeros: their sums are never stored, and a tap outside the image
// has scale 0 (int32 output: written as 0).  The kinds with one integer sum over several taps
// load such rows from a row of zeros instead.
//
// XB = 8: the operands are int8 codes, one per byte.  The 16 bytes a lane reads are one MFMA
// operand as they are (no expansion, one MFMA per read instead of two), the sums carry no factor
// 256, and a chunk row of KCH * 16 bytes holds KCH * 16 codes.
//
// S2: 3x3 window with stride 2.  Output pixel (image, oh, ow) sits over input pixel (2 oh, 2 ow):
// the activation row of a tile row is that input pixel's (a per-tile table of "centres" beside
// the tap masks), a tap still shifts it by a uniform (dr * w + ds) input pixels, and everything
// on the output side (tiles, scales of the channels, stores) counts output pixels.
template <int TM, int TN, int WAVES_M, int WAVES_N, int KIND, int OUT, int KCH, int NSTAGE, int OCC, int XB = 4,
          bool S2 = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, OCC) void int_gemm_kernel(GemmArgs a) {
    static_assert(XB == 4 || XB == 8, "4-bit codes in pairs or int8 codes");
    static_assert(!S2 || KIND == kConvPerTap || KIND == kConvSum || is_conv_planes(KIND), "stride 2 is a 3x3 window's");
    constexpr int SHIFT = XB == 8 ? 0 : 8;                    // log2 of the factor the integer sums carry
    constexpr float UNIT = XB == 8 ? 1.0f : 1.0f / 256.0f;
    constexpr int TAPS = taps_of(KIND);
    constexpr int WTAPS = is_conv_planes(KIND) ? 9 : (is_planes(KIND) ? 3 : TAPS);   // taps of the weight tensor [n, WTAPS, k/2]
    constexpr bool CONV = KIND == kConvPerTap || KIND == kConvSum || is_conv_planes(KIND);   // taps read shifted pixels
    constexpr bool PER_TAP = KIND == kConvPerTap || is_planes(KIND);  // one integer sum and one scale row per tap
    constexpr bool SUM = KIND == kConvSum;                            // one integer sum over all taps
    constexpr bool ZPAD = KIND == kConvSum || is_conv_planes(KIND);    // taps outside the image load zeros
    constexpr bool FACC = PER_TAP || is_conv_planes(KIND);             // integer sums are folded into fp32 sums
    constexpr int STAPS = PER_TAP ? TAPS : 1;       // rows of the activation-scale table
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int NT = 64 * NW;
    constexpr int BCO = 32 * TM * WAVES_M;   // output channels per workgroup
    constexpr int BP = 32 * TN * WAVES_N;    // pixels per workgroup
    constexpr int ROWB = KCH * 16;           // bytes per row per chunk
    constexpr int KS = KCH / 2;              // 64-code K steps per chunk
    static_assert(KCH % 2 == 0, "a 64-code K step is two pieces");
    static_assert((BCO * KCH) % 64 == 0 && (BP * KCH) % 64 == 0, "whole wave-wide loads only");
    constexpr int A_INSTR = BCO * KCH / 64, B_INSTR = BP * KCH / 64;   // 1 KiB loads per chunk
    // Load i of an operand belongs to wave i % NW: every wave has A_SLOTS slots for weight rows
    // and B_SLOTS for activation rows and skips a slot whose load does not exist (only the last
    // slot of an operand can be missing; the counted waits below take that into account).
    constexpr int A_SLOTS = (A_INSTR + NW - 1) / NW, B_SLOTS = (B_INSTR + NW - 1) / NW;
    constexpr int LPW = A_SLOTS + B_SLOTS;
    static_assert((NSTAGE - 2) * LPW < 64, "vmcnt range");
    static_assert(TM + TN < 16, "lgkmcnt range");
    static_assert(BP <= NT && BCO <= NT, "one table entry per thread");
    constexpr int STAGE_BYTES = (BCO + BP) * ROWB;
    constexpr int SX_PER_T = (STAPS * BP + NT - 1) / NT;   // scale-table entries per thread
    constexpr uint32_t XCDS = 8;
    using Out = typename OutT<OUT>::type;
    using Ops = Packed<TM, TN>;

    // [stage][operand][row][ROWB bytes]
    __shared__ __attribute__((aligned(16))) uint8_t lds[NSTAGE * STAGE_BYTES];
    // two sets of per-tile tables: the set of tile k+1 is built while tile k is multiplied
    __shared__ float s_sx[2][STAPS][BP];   // x_scale / 256 of the input pixel under tap t; 0 outside
    __shared__ int s_mask[2][BP];         // bit t: tap t of this output pixel is inside the image
    __shared__ uint32_t s_center[2][S2 ? BP : 1];   // stride 2: input pixel under the window's centre
    __shared__ __attribute__((aligned(16))) float s_sw[2][BCO];     // w_scale of the tile's channels
    __shared__ __attribute__((aligned(16))) float s_bias[2][BCO];   // bias (0 if absent)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
    const int lrow = lane & 31, lhalf = lane >> 5;

    const int kbytes = XB == 8 ? a.k : a.k >> 1;   // operand bytes per (row, tap)
    const int chunks_per_tap = kbytes / ROWB;    // host guarantees divisibility
    const int total_chunks = TAPS * chunks_per_tap;
    const uint32_t lds_row = lds_address(lds) + lrow * ROWB + (lhalf ^ ((lrow >> 3) & 1)) * 16;
    const uint32_t lds_b = lds_row + (BCO + wave_n * TN * 32) * ROWB;
    const uint32_t lds_sx = lds_address(&s_sx[0][0][0]) + (wave_n * TN * 32 + lrow) * 4;

    // ---- this workgroup's tiles: a contiguous run t_first .. t_first + my_tiles - 1 -------------
    // (consecutive tiles are the channel tiles of one pixel tile, so a run reuses the pixel
    // rows from L2 and mixes full and cut-off channel tiles evenly over the workgroups)
    uint32_t lo = 0, hi = a.n_tiles, j = blockIdx.x, sharers = gridDim.x;
    if (a.xcds) {   // gridDim.x is a multiple of XCDS then
        const uint32_t x = blockIdx.x % XCDS;
        lo = static_cast<uint32_t>(static_cast<uint64_t>(a.n_tiles) * x / XCDS);
        hi = static_cast<uint32_t>(static_cast<uint64_t>(a.n_tiles) * (x + 1) / XCDS);
        j = blockIdx.x / XCDS;
        sharers = gridDim.x / XCDS;
    }
    const uint32_t per = (hi - lo) / sharers, rem = (hi - lo) % sharers;
    const uint32_t t_first = lo + j * per + (j < rem ? j : rem);
    const uint32_t my_tiles = per + (j < rem ? 1 : 0);
    if (my_tiles == 0) return;
    const uint32_t stream_chunks = my_tiles * total_chunks;   // < 2^31, checked on the host
    auto tile_origin = [&](uint32_t k, int &co0, uint32_t &p0) {
        const uint32_t tile = t_first + k;
        co0 = static_cast<int>(tile % a.n_co_tiles) * BCO;
        p0 = (tile / a.n_co_tiles) * BP;
    };

    // ---- per-tile tables ---------------------------------------------------------------------
    auto build_masks = [&](uint32_t k) {   // no memory reads
        int co0; uint32_t p0;
        tile_origin(k, co0, p0);
        if (tid < BP) {
            const uint32_t pix = p0 + tid;
            int mask = 0;
            if constexpr (S2) {
                uint32_t center = 0;
                if (pix < a.pixels) {
                    const uint32_t q = pix / static_cast<uint32_t>(a.w_out);
                    const int ow = static_cast<int>(pix - q * a.w_out);
                    const uint32_t img = q / static_cast<uint32_t>(a.h_out);
                    const int oh = static_cast<int>(q - img * a.h_out);
#pragma unroll
                    for (int t = 0; t < 9; ++t) {
                        const int ih = 2 * oh + t / 3 - 1, iw = 2 * ow + t % 3 - 1;
                        mask |= (ih >= 0 && ih < a.h && iw >= 0 && iw < a.w) ? (1 << t) : 0;
                    }
                    center = (img * a.h + 2 * oh) * a.w + 2 * ow;
                }
                s_center[k & 1][tid] = center;
            } else if (pix < a.pixels) {
                if constexpr (CONV) mask = tap_mask<9>(pix, a.h, a.w);
                else mask = (1 << TAPS) - 1;
            }
            s_mask[k & 1][tid] = mask;
        }
    };
    float t_sx[SX_PER_T], t_sw = 0.f, t_bias = 0.f;
    auto load_scales = [&](uint32_t k) {   // needs the masks of tile k to be visible
        if constexpr (OUT != kOutI32) {
            int co0; uint32_t p0;
            tile_origin(k, co0, p0);
#pragma unroll
            for (int j = 0; j < SX_PER_T; ++j) {
                const int e = tid + j * NT;
                const int t = e / BP, p = e % BP;
                t_sx[j] = 0.f;
                if (e < STAPS * BP) {
                    const int mask = s_mask[k & 1][p];
                    if (PER_TAP ? ((mask >> t) & 1) : (mask != 0)) {
                        const int delta = KIND == kConvPerTap ? (t / 3 - 1) * a.w + (t % 3 - 1) : 0;
                        int64_t at = static_cast<int64_t>(p0 + p);
                        if constexpr (S2) at = s_center[k & 1][p];
                        t_sx[j] = a.sx[a.sx_static ? 0 : at + delta];
                    }
                }
            }
            if (tid < BCO && co0 + tid < a.n) {
                t_sw = a.sw[co0 + tid] * a.out_scale;
                const Out *bias = static_cast<const Out *>(a.bias);
                t_bias = bias ? to_float(bias[co0 + tid]) : 0.f;
            } else {
                t_sw = 0.f;
                t_bias = 0.f;
            }
        }
    };
    auto store_scales = [&](uint32_t k) {
        if constexpr (OUT != kOutI32) {
#pragma unroll
            for (int j = 0; j < SX_PER_T; ++j) {
                const int e = tid + j * NT;
                // the sums carry a factor 256 (both operands are 16 x code); digit plane t weighs 16^t
                const float unit = is_planes(KIND) ? static_cast<float>(1 << (4 * (e / BP))) * UNIT : UNIT;
                if (e < STAPS * BP) (&s_sx[k & 1][0][0])[e] = t_sx[j] * unit;
            }
            if (tid < BCO) {
                s_sw[k & 1][tid] = t_sw;
                s_bias[k & 1][tid] = t_bias;
            }
        }
    };

    // ---- this wave's share of the direct-to-LDS loads -------------------------------------------
    uint32_t ld_a[A_SLOTS];      // weight rows: byte offset of this lane's piece at tap 0, chunk 0
    uint32_t ld_b[B_SLOTS];      // activation rows: the same, at the tile's own pixel
    uint32_t ld_bmax[B_SLOTS];   // ... at the last pixel of the tensor
    uint32_t ld_bcur[B_SLOTS];   // ... at the pixel under the tap being fetched
    int ld_mask[ZPAD ? B_SLOTS : 1];        // zeros outside the image: the row's tap mask ...
    uint32_t ld_zero[ZPAD ? B_SLOTS : 1];   // ... and this lane's piece of the zero row
    uint32_t a_tap_off = 0;      // uniform: tap being fetched * kbytes
    uint32_t fk = 0;             // tile (index in this workgroup's list) being fetched
    int ftap = 0, fch = 0;
    uint32_t fetched = 0;        // chunks of the stream requested so far
    // lane's 16-byte slot in load i of an operand: row of the tile, byte offset inside the chunk row
    auto slot_row = [&](int i) { return (i * 64 + lane) / KCH; };
    auto slot_byte = [&](int i) {
        const int q = i * 64 + lane, row = q / KCH;
        return static_cast<uint32_t>(((q % KCH) ^ ((row >> 3) & 1)) * 16);   // swizzle, see above
    };
#pragma unroll
    for (int j = 0; j < B_SLOTS; ++j)
        ld_bmax[j] = ((S2 ? a.in_pixels : a.pixels) - 1) * kbytes + slot_byte(j * NW + wave);
    auto set_fetch_tap = [&](int step) {
        const int t = step % WTAPS;   // tap of the 3x3 window (digit planes: step = plane * 9 + tap)
        a_tap_off = static_cast<uint32_t>(t) * kbytes;
#pragma unroll
        for (int j = 0; j < B_SLOTS; ++j) {
            if constexpr (CONV) {
                const uint32_t shift = static_cast<uint32_t>(((t / 3 - 1) * a.w + (t % 3 - 1)) * kbytes);
                const uint32_t o = ld_b[j] + shift;
                ld_bcur[j] = o < ld_bmax[j] ? o : ld_bmax[j];
                // (the digit planes are planes of the INPUT tensor)
                if constexpr (is_conv_planes(KIND))
                    ld_bcur[j] += static_cast<uint32_t>(step / 9) * ((S2 ? a.in_pixels : a.pixels) * kbytes);
            } else {
                ld_bcur[j] = ld_b[j];
            }
        }
    };
    auto set_fetch_tile = [&](uint32_t k) {
        int co0; uint32_t p0;
        tile_origin(k, co0, p0);
#pragma unroll
        for (int j = 0; j < A_SLOTS; ++j) {
            const int i = j * NW + wave, row = slot_row(i);
            int co = co0 + (row & ~31) + tile_row_to_channel(row & 31);
            co = co < a.n ? co : a.n - 1;
            ld_a[j] = static_cast<uint32_t>(co) * WTAPS * kbytes + slot_byte(i);
        }
#pragma unroll
        for (int j = 0; j < B_SLOTS; ++j) {
            const int i = j * NW + wave;
            uint32_t pix = p0 + slot_row(i);
            pix = pix < a.pixels ? pix : a.pixels - 1;
            if constexpr (S2) pix = i < B_INSTR ? s_center[k & 1][slot_row(i)] : 0;   // needs the tables of tile k
            ld_b[j] = pix * kbytes + slot_byte(i);
            if constexpr (ZPAD) {   // needs the masks of tile k to be visible
                ld_mask[j] = i < B_INSTR ? s_mask[k & 1][slot_row(i)] : 0;
                ld_zero[j] = slot_byte(i);
            }
        }
        set_fetch_tap(0);
    };
    auto issue_loads = [&](int stage) {
        const uint8_t *base_a = a.wq + (a_tap_off + static_cast<uint32_t>(fch * ROWB));
        const uint8_t *base_b = a.xq + fch * ROWB;
        uint8_t *image = lds + stage * STAGE_BYTES;   // weight rows, then activation rows; 1 KiB per load
#pragma unroll
        for (int j = 0; j < A_SLOTS; ++j) {
            const int i = j * NW + wave;
            if (i < A_INSTR) load_to_lds16(base_a + ld_a[j], image + i * 1024);
        }
#pragma unroll
        for (int j = 0; j < B_SLOTS; ++j) {
            const int i = j * NW + wave;
            if (i < B_INSTR) {
                const uint8_t *src = base_b + ld_bcur[j];
                if constexpr (ZPAD) {
                    if (!((ld_mask[j] >> (ftap % WTAPS)) & 1)) src = g_zero_row + ld_zero[j];
                }
                load_to_lds16(src, image + BCO * ROWB + i * 1024);
            }
        }
        ++fetched;
        if (++fch == chunks_per_tap) {
            fch = 0;
            if (++ftap < TAPS) {
                set_fetch_tap(ftap);
            } else {
                ftap = 0;
                if (++fk < my_tiles) set_fetch_tile(fk);   // the stream runs on into the next tile
            }
        }
    };

    // ---- prologue of the stream ---------------------------------------------------------------
    build_masks(0);
    if (my_tiles > 1) build_masks(1);
    __syncthreads();
    set_fetch_tile(0);
#pragma unroll
    for (int st = 0; st < NSTAGE - 1; ++st)
        if (fetched < stream_chunks) issue_loads(st);
    load_scales(0);
    store_scales(0);
    __syncthreads();   // tables visible to every wave before the first raw barrier below

    int stage = 0;
    uint32_t g = 0;    // position in the chunk stream
    for (uint32_t k = 0; k < my_tiles; ++k) {
        int co0; uint32_t p0;
        tile_origin(k, co0, p0);
        const int tb = k & 1;   // table set of this tile
        // A wave whose channels or pixels all lie outside the tensor skips the arithmetic of the
        // tile (it still loads, waits and meets the barriers).  In a tile that is cut off in the
        // channel direction, every second workgroup (by residency round) rotates which waves own
        // the existing channels, so that the SIMDs a CU's workgroups leave idle differ.
        const int rot = (co0 + BCO > a.n && ((blockIdx.x / a.cus) & 1)) ? 1 : 0;
        const int wm = (wave_m + rot) % WAVES_M;   // channel block of this wave in this tile
        const bool active = co0 + wm * TM * 32 < a.n && p0 + wave_n * TN * 32 < a.pixels;
        const uint32_t lds_a = lds_row + wm * TM * 32 * ROWB;

        v16i acc[TM][TN];
        float facc[FACC ? TM : 1][FACC ? TN : 1][16];
        if constexpr (FACC) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) facc[tm][tn][r] = 0.f;
        }
        // digit planes of the activations, integer output: the exact sum over the planes
        constexpr bool ISUM = is_conv_planes(KIND) && OUT == kOutI32;
        int iacc[ISUM ? TM : 1][ISUM ? TN : 1][16];
        if constexpr (ISUM) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int r = 0; r < 16; ++r) iacc[tm][tn][r] = 0;
        }

        // MFMAs of one K step; first: the sums of a tap start from 0
        auto multiply = [&](Ops &o, bool first) {
            if constexpr (XB == 8) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) pin(o.a[tm]);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) pin(o.b[tn]);
                const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(o.a[tm], o.b[tn], first ? zero : acc[tm][tn], 0, 0, 0);
                return;
            }
            v4i a0[TM], a1[TM], b0[TN], b1[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) { pin(o.a[tm]); expand(o.a[tm], a0[tm], a1[tm]); }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) { pin(o.b[tn]); expand(o.b[tn], b0[tn], b1[tn]); }
            if (first) {
                const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[tm], b0[tn], zero, 0, 0, 0);
            } else {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[tm], b0[tn], acc[tm][tn], 0, 0, 0);
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[tm], b1[tn], acc[tm][tn], 0, 0, 0);
        };

        // this lane's tap masks, taken before chunk 0 lets the masks of tile k+2 into this set
        int my_mask[TN];
        if constexpr (OUT == kOutI32) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) my_mask[tn] = s_mask[tb][(wave_n * TN + tn) * 32 + lrow];
        }

        int tap = 0, ch = 0;
        for (int chunk = 0; chunk < total_chunks; ++chunk, ++g) {
            // this chunk has landed once at most the later (NSTAGE-2) chunks' loads are pending
            if constexpr (NSTAGE == 2) {
                wait_vmem<0>();
            } else if (g + NSTAGE - 2 < stream_chunks) {
                const int missing = ((A_SLOTS - 1) * NW + wave >= A_INSTR) + ((B_SLOTS - 1) * NW + wave >= B_INSTR);
                if (missing == 0) wait_vmem<(NSTAGE - 2) * LPW>();
                else if (missing == 1) wait_vmem<(NSTAGE - 2) * (LPW - 1)>();
                else wait_vmem<(NSTAGE - 2) * (LPW - 2)>();
            } else {
                wait_vmem<0>();
            }
            __builtin_amdgcn_s_barrier();   // every wave's share has landed; the previous stage is free
            if (fetched < stream_chunks) issue_loads(stage == 0 ? NSTAGE - 1 : stage - 1);

            // tables of the next tile, spread over this tile's first chunks: the masks of tile
            // k+1 are already there (built one tile ahead); its scales are loaded in chunk 0
            // and stored at the end of it; the masks of tile k+2 follow.
            const bool tables_now = chunk == 0 && k + 1 < my_tiles;
            if (tables_now) load_scales(k + 1);

            if (active) {
                const uint32_t sa = lds_a + stage * STAGE_BYTES, sb = lds_b + stage * STAGE_BYTES;
                Ops op[2];
                read_packed<TM, TN, ROWB, 0>(op[0], sa, sb);
                const bool sum_starts = SUM ? chunk == 0 : (is_conv_planes(KIND) ? ch == 0 && tap % 9 == 0 : ch == 0);
                chunk_steps<0, KS, TM, TN, ROWB>(op, sa, sb, sum_starts, multiply);
            }

            if (++ch == chunks_per_tap) {
                ch = 0;
                // ---- end of a tap: fold the integer sums into the result (one sum over all taps:
                // nothing to do before the last tap) ---------------------------------------------
                const bool sum_ends = SUM ? tap == TAPS - 1 : (is_conv_planes(KIND) ? tap % 9 == 8 : true);
                if (active && sum_ends) {
                if constexpr (ISUM) {
                    // 256 x the plane's sum, weighted by 16^plane; stored after the last plane
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                            for (int r = 0; r < 16; ++r) iacc[tm][tn][r] += (acc[tm][tn][r] >> SHIFT) * (1 << (4 * (tap / 9)));
                    if (tap == TAPS - 1) {
                        int *yi = static_cast<int *>(a.y);
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn) {
                            const uint32_t pix = p0 + (wave_n * TN + tn) * 32 + lrow;
#pragma unroll
                            for (int tm = 0; tm < TM; ++tm) {
                                const int cbase = co0 + (wm * TM + tm) * 32 + 16 * lhalf;
                                if (pix < a.pixels) {
                                    int *dst = yi + static_cast<int64_t>(pix) * a.n + cbase;
#pragma unroll
                                    for (int r = 0; r < 16; ++r)
                                        if (cbase + r < a.n) dst[r] = iacc[tm][tn][r];
                                }
                            }
                        }
                    }
                } else if constexpr (OUT == kOutI32) {
                    int *yi = static_cast<int *>(a.y);
                    constexpr int OUT_TAPS = SUM ? 1 : TAPS;   // sums stored per output pixel
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const int prow = (wave_n * TN + tn) * 32 + lrow;
                        const uint32_t pix = p0 + prow;
                        // a tap outside the image is written as 0 (also false for pixels >= pixels)
                        const bool inside = SUM || ((my_mask[tn] >> tap) & 1);
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm) {
                            const int cbase = co0 + (wm * TM + tm) * 32 + 16 * lhalf;
                            if (pix < a.pixels) {
                                int *dst = yi + (static_cast<int64_t>(pix) * OUT_TAPS + (SUM ? 0 : tap)) * a.n + cbase;
#pragma unroll
                                for (int r = 0; r < 16; ++r)
                                    if (cbase + r < a.n) dst[r] = inside ? (acc[tm][tn][r] >> SHIFT) : 0;
                            }
                        }
                    }
                } else if constexpr (FACC) {
                    float s[TN];
                    read_tap_scales<TN>(s, lds_sx + (tb * STAPS + (PER_TAP ? tap : 0)) * BP * 4);
                    if constexpr (is_conv_planes(KIND)) {   // the plane's weight 16^plane
                        const float weight = static_cast<float>(1 << (4 * (tap / 9)));
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn) s[tn] *= weight;
                    }
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                facc[tm][tn][r] += s[tn] * static_cast<float>(acc[tm][tn][r]);
                }
                }
                ++tap;
            }
            if (tables_now) {
                store_scales(k + 1);
                if (k + 2 < my_tiles) build_masks(k + 2);   // into this tile's own set: no longer read
            }
            stage = stage + 1 == NSTAGE ? 0 : stage + 1;
        }

        // ---- dequantising epilogue -------------------------------------------------------------
        if constexpr (OUT != kOutI32) {
            if (!active) continue;   // next tile
            Out *y = static_cast<Out *>(a.y);
            const bool vec_ok = (a.n & 15) == 0;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int clocal = (wm * TM + tm) * 32 + 16 * lhalf;
                const int cbase = co0 + clocal;
                float swv[16], bv[16];
#pragma unroll
                for (int r = 0; r < 16; r += 4) {
                    const float4 s4 = *reinterpret_cast<const float4 *>(&s_sw[tb][clocal + r]);
                    const float4 b4 = *reinterpret_cast<const float4 *>(&s_bias[tb][clocal + r]);
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
                        if constexpr (FACC) s = facc[tm][tn][r];
                        else s = s_sx[tb][0][prow] * static_cast<float>(acc[tm][tn][r]);
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
}

template <int TM, int TN, int WAVES_M, int WAVES_N, int KIND, int OUT, int KCH, int NSTAGE, int OCC, int XB = 4,
          bool S2 = false>
hq_status launch_tile(GemmArgs a, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    constexpr int TAPS = taps_of(KIND);
    constexpr int BCO = 32 * TM * WAVES_M, BP = 32 * TN * WAVES_N;
    a.n_co_tiles = (a.n + BCO - 1) / BCO;
    const int64_t p_tiles = (static_cast<int64_t>(a.pixels) + BP - 1) / BP;
    const int64_t tiles = p_tiles * a.n_co_tiles;
    if (tiles * ((a.bits == 8 ? a.k : a.k / 2) / 32) * TAPS > 0x7fffffffLL) return HQ_ERR_SHAPE;   // chunk-stream counters are 32 bit
    a.n_tiles = static_cast<uint32_t>(tiles);
    const int64_t slots = static_cast<int64_t>(hq::compute_units()) * OCC;   // co-resident workgroups
    const unsigned grid = static_cast<unsigned>(tiles < slots ? tiles : slots);
    a.xcds = grid % 8 == 0 ? 1 : 0;
    a.cus = static_cast<uint32_t>(hq::compute_units());
    hipLaunchKernelGGL((int_gemm_kernel<TM, TN, WAVES_M, WAVES_N, KIND, OUT, KCH, NSTAGE, OCC, XB, S2>),
                       dim3(grid), dim3(64 * WAVES_M * WAVES_N), 0, stream, a);
    return check.status();
}

// All instantiations of one tile configuration: the four kernel kinds (taps = 1: linear;
// taps = 9: per-tap sums, or one sum if the activation scale is static; taps = 3: digit planes), the three output
// types, and K chunks of 192 codes (96 contiguous bytes per row) or, if WITH_64 is set, the
// 64-code fallback for channel counts that are not a multiple of 192.
// WITH_S2: this configuration also carries the stride-2 forms of the two 3x3 kinds (4-bit codes).
template <int TM, int TN, int WAVES_M, int WAVES_N, int OCC, bool WITH_64, int NSTAGE_WIDE = 2, bool WITH_S2 = false>
hq_status launch_config(const GemmArgs &a, int taps, hq_dtype y_dtype, hipStream_t stream) {
    const bool wide = (a.bits == 8 ? a.k : a.k / 2) % 96 == 0;   // whole chunks of six 16-byte pieces per row
    if (a.stride == 2) {
        if constexpr (WITH_S2) {
#define HQ_GEMM_CASE_S2(KIND, OUT, XB)                                                                    \
    if (wide) return launch_tile<TM, TN, WAVES_M, WAVES_N, KIND, OUT, 6, NSTAGE_WIDE, OCC, XB, true>(a, stream); \
    return launch_tile<TM, TN, WAVES_M, WAVES_N, KIND, OUT, 2, 4, OCC, XB, true>(a, stream);
            if (a.bits == 8) {   // int8 codes: per-pixel scales only
                if (taps != 9 || a.sx_static) return HQ_ERR_UNSUPPORTED;
                if (y_dtype == HQ_F16) { HQ_GEMM_CASE_S2(kConvPerTap, kOutF16, 8) }
                if (y_dtype == HQ_F32) { HQ_GEMM_CASE_S2(kConvPerTap, kOutF32, 8) }
                if (y_dtype == HQ_I32) { HQ_GEMM_CASE_S2(kConvPerTap, kOutI32, 8) }
                return HQ_ERR_DTYPE;
            }
            if (taps == 27 || taps == 18) {   // digit planes of the activations (width-axis convolution)
                if (taps == 27) {
                    if (y_dtype == HQ_F16) { HQ_GEMM_CASE_S2(kConvPlanes, kOutF16, 4) }
                    if (y_dtype == HQ_F32) { HQ_GEMM_CASE_S2(kConvPlanes, kOutF32, 4) }
                    if (y_dtype == HQ_I32) { HQ_GEMM_CASE_S2(kConvPlanes, kOutI32, 4) }
                } else {
                    if (y_dtype == HQ_F16) { HQ_GEMM_CASE_S2(kConvPlanes2, kOutF16, 4) }
                    if (y_dtype == HQ_F32) { HQ_GEMM_CASE_S2(kConvPlanes2, kOutF32, 4) }
                    if (y_dtype == HQ_I32) { HQ_GEMM_CASE_S2(kConvPlanes2, kOutI32, 4) }
                }
                return HQ_ERR_DTYPE;
            }
            if (taps != 9) return HQ_ERR_UNSUPPORTED;
            if (a.sx_static) {
                if (y_dtype == HQ_F16) { HQ_GEMM_CASE_S2(kConvSum, kOutF16, 4) }
                if (y_dtype == HQ_F32) { HQ_GEMM_CASE_S2(kConvSum, kOutF32, 4) }
                if (y_dtype == HQ_I32) { HQ_GEMM_CASE_S2(kConvSum, kOutI32, 4) }
            } else {
                if (y_dtype == HQ_F16) { HQ_GEMM_CASE_S2(kConvPerTap, kOutF16, 4) }
                if (y_dtype == HQ_F32) { HQ_GEMM_CASE_S2(kConvPerTap, kOutF32, 4) }
                if (y_dtype == HQ_I32) { HQ_GEMM_CASE_S2(kConvPerTap, kOutI32, 4) }
            }
#undef HQ_GEMM_CASE_S2
            return HQ_ERR_DTYPE;
        }
        return HQ_ERR_UNSUPPORTED;
    }
    if (!wide && !WITH_64) return HQ_ERR_UNSUPPORTED;
    if (a.bits == 8) {   // int8 codes: linear layers and 3x3 convolutions with per-pixel scales
#define HQ_GEMM_CASE8(KIND, OUT)                                                                           \
    if (wide) return launch_tile<TM, TN, WAVES_M, WAVES_N, KIND, OUT, 6, NSTAGE_WIDE, OCC, 8>(a, stream);  \
    if constexpr (WITH_64) return launch_tile<TM, TN, WAVES_M, WAVES_N, KIND, OUT, 2, 4, OCC, 8>(a, stream); \
    return HQ_ERR_UNSUPPORTED;
        if (taps == 1) {
            if (y_dtype == HQ_F16) { HQ_GEMM_CASE8(kLinear, kOutF16) }
            if (y_dtype == HQ_F32) { HQ_GEMM_CASE8(kLinear, kOutF32) }
            if (y_dtype == HQ_I32) { HQ_GEMM_CASE8(kLinear, kOutI32) }
        } else if (taps == 9 && !a.sx_static) {
            if (y_dtype == HQ_F16) { HQ_GEMM_CASE8(kConvPerTap, kOutF16) }
            if (y_dtype == HQ_F32) { HQ_GEMM_CASE8(kConvPerTap, kOutF32) }
            if (y_dtype == HQ_I32) { HQ_GEMM_CASE8(kConvPerTap, kOutI32) }
        }
#undef HQ_GEMM_CASE8
        return HQ_ERR_UNSUPPORTED;
    }
#define HQ_GEMM_CASE(KIND, OUT)                                                                        \
    if (wide) return launch_tile<TM, TN, WAVES_M, WAVES_N, KIND, OUT, 6, NSTAGE_WIDE, OCC>(a, stream);           \
    if constexpr (WITH_64) return launch_tile<TM, TN, WAVES_M, WAVES_N, KIND, OUT, 2, 4, OCC>(a, stream); \
    return HQ_ERR_UNSUPPORTED;
    if (taps == 1) {
        if (y_dtype == HQ_F16) { HQ_GEMM_CASE(kLinear, kOutF16) }
        if (y_dtype == HQ_F32) { HQ_GEMM_CASE(kLinear, kOutF32) }
        if (y_dtype == HQ_I32) { HQ_GEMM_CASE(kLinear, kOutI32) }
    } else if (taps == 9 && !a.sx_static) {
        if (y_dtype == HQ_F16) { HQ_GEMM_CASE(kConvPerTap, kOutF16) }
        if (y_dtype == HQ_F32) { HQ_GEMM_CASE(kConvPerTap, kOutF32) }
        if (y_dtype == HQ_I32) { HQ_GEMM_CASE(kConvPerTap, kOutI32) }
    } else if (taps == 9) {
        if (y_dtype == HQ_F16) { HQ_GEMM_CASE(kConvSum, kOutF16) }
        if (y_dtype == HQ_F32) { HQ_GEMM_CASE(kConvSum, kOutF32) }
        if (y_dtype == HQ_I32) { HQ_GEMM_CASE(kConvSum, kOutI32) }
    } else if (taps == 3) {
        if (y_dtype == HQ_F16) { HQ_GEMM_CASE(kPlanes, kOutF16) }
        if (y_dtype == HQ_F32) { HQ_GEMM_CASE(kPlanes, kOutF32) }
        if (y_dtype == HQ_I32) { HQ_GEMM_CASE(kPlanes, kOutI32) }
    } else if (taps == 2) {    // two digit planes of the weights (floating-point output only)
        if (y_dtype == HQ_F16) { HQ_GEMM_CASE(kPlanes2, kOutF16) }
        if (y_dtype == HQ_F32) { HQ_GEMM_CASE(kPlanes2, kOutF32) }
    } else if (taps == 18) {   // two digit planes of the activations
        if (y_dtype == HQ_F16) { HQ_GEMM_CASE(kConvPlanes2, kOutF16) }
        if (y_dtype == HQ_F32) { HQ_GEMM_CASE(kConvPlanes2, kOutF32) }
        if (y_dtype == HQ_I32) { HQ_GEMM_CASE(kConvPlanes2, kOutI32) }
    } else if (taps == 27) {
        if (y_dtype == HQ_F16) { HQ_GEMM_CASE(kConvPlanes, kOutF16) }
        if (y_dtype == HQ_F32) { HQ_GEMM_CASE(kConvPlanes, kOutF32) }
        if (y_dtype == HQ_I32) { HQ_GEMM_CASE(kConvPlanes, kOutI32) }
    }
#undef HQ_GEMM_CASE
    return HQ_ERR_DTYPE;
}

}  // namespace

// One translation unit per tile configuration (they compile in parallel).
hq_status hq_gemm_launch_128x128(const GemmArgs &a, int taps, hq_dtype y_dtype, hipStream_t stream);
hq_status hq_gemm_launch_64x128(const GemmArgs &a, int taps, hq_dtype y_dtype, hipStream_t stream);
hq_status hq_gemm_launch_64x64(const GemmArgs &a, int taps, hq_dtype y_dtype, hipStream_t stream);
// 3x3 convolution, one wave per 64x64 tile and K share (hq_conv3x3_wave.hip)
hq_status hq_conv3x3_wave_launch(const GemmArgs &a, hq_dtype y_dtype, hipStream_t stream);
// linear / 1x1 / 3x3 (stride 1) for channel counts that are a multiple of 8 but not of 64 (hq_int_gemm_anyk.hip)
hq_status hq_gemm_launch_anyk(const GemmArgs &a, int taps, hq_dtype y_dtype, hipStream_t stream);
hq_status hq_fill_zero_launch(void *dst, uint64_t ints, hipStream_t stream);
// 3x3 convolution, per-pixel scales: eight waves per CU, int8 activation tile resident in LDS (hq_conv3x3_res.hip)
bool hq_conv3x3_res_fits(int64_t pixels, int w, int c_in, int c_out);
int hq_conv3x3_res_tile_pixels(int64_t pixels, int w, int c_in, int c_out);
hq_status hq_conv3x3_res_launch(const GemmArgs &a, hq_dtype y_dtype, hipStream_t stream);
// 3x3 convolution with the activation tile resident in LDS (hq_conv3x3_halo.hip)
bool hq_conv3x3_halo_fits(const GemmArgs &a, hq_dtype y_dtype);
hq_status hq_conv3x3_halo_launch(const GemmArgs &a, hq_dtype y_dtype, hipStream_t stream);
