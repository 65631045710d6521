// 3x3 / stride 1 / pad 1 NHWC convolution on int8 MFMA with the activation tile resident in
// LDS (Method, "Convolution").
//
// Why.  Measured on MI355X, direct-to-LDS loads deliver about 21 bytes per clock per CU, and
// one 32x32x32 int8 MFMA per SIMD every 32 clocks needs an operand stream below about 170 bytes
// per MFMA to stay ahead of that.  A tile kernel that re-fetches both operands for every tap
// needs 256..384 bytes per MFMA and is bound by those loads, not by arithmetic.  The nine taps
// of a 3x3 window read the SAME activation rows shifted by -W-1 .. W+1 pixels, so here a
// workgroup loads the rows of its 256 output pixels plus that halo ONCE per 192-channel slice
// and all nine taps read them from LDS at shifted addresses; only the weights (64 channels x
// 96 bytes per tap) stream through a two-stage buffer (deeper prefetch measured no faster).
// That is about 110 bytes per MFMA.
//
// Shape.  Four waves per workgroup, each a 64-channel x 64-pixel register tile (2 x 2 MFMA
// tiles, six vector instructions of nibble expansion per MFMA); workgroup tile 64 channels x
// 256 consecutive pixels (of the flattened [image, row, column] order, so a tile may span
// image rows and images; what lies outside a pixel's own image is masked per pixel and tap).
// Two workgroups per CU (three for the one-sum kind, which keeps no fp32 sums beside the integer
// ones); persistent, contiguous runs of tiles (the channel tiles of one pixel tile are adjacent,
// and a workgroup keeps the activation slice when only the channel tile changes).
//
// Loop order.  For each 192-channel slice of the input channels: load the activation slice,
// then for each of the nine taps: three K steps of 64 codes against that tap's weight rows.
// KIND = kConvPerTap (every input pixel has its own scale): the integer sums of one (slice,
// tap) are folded into the fp32 result with the scale of the input pixel under the tap right
// away (a partial sum scales linearly, so per-tap sums need not be complete).  KIND = kConvSum
// (one scale for the tensor): one integer sum over everything; a tap outside the image reads
// a row of zeros instead of the activation row.
//
// Folding a (slice, tap) sum into the fp32 result costs one instruction per element, not two:
// the integer accumulators start from the bit pattern of the float 1.5 * 2^23, so after the
// MFMAs their bits, read as a float, are exactly 1.5 * 2^23 + S (|S| = 256 |sum| <= 256 * 192 * 64
// < 2^22), and facc = fma(scale, that, facc) needs no int-to-float conversion.  The surplus
// 1.5 * 2^23 * (sum of the scales used) is known per pixel beforehand and is what facc starts from,
// negated.  The fp32 roundings this adds stay below 0.1 of one code product per output.
//
// Latency.  The loads of a tile's first slice and first weights are issued before the tile's
// tables are built, and those of the next tile before the current tile's results are scaled
// and stored, so neither waits for the other.
#include <type_traits>

#include "hq_int_gemm_kernel.h"

namespace {

constexpr int kHaloRows = 400;   // activation rows a tile can hold: 256 + 2 (W + 1) for W <= 71

struct HaloArgs {
    const uint8_t *xq;   // [pixels, k/2]
    const float *sx;     // [pixels], or one value (sx_static)
    const uint8_t *wq;   // [n, 9, k/2]
    const float *sw;     // [n]
    const void *bias;    // [n] of the output dtype, or null
    void *y;             // [pixels, n]
    uint32_t pixels;
    int n, k, h, w;
    uint32_t w_magic, w_shift, h_magic, h_shift;   // exact division of a pixel index by w and by h
    uint32_t n_co_tiles, n_tiles, xcds;
    int sx_static;
};

template <int KIND, int OUT>
__global__ __launch_bounds__(256, KIND == kConvSum ? 3 : 2) void conv3x3_halo_kernel(HaloArgs a) {
    constexpr bool PER_TAP = KIND == kConvPerTap;
    constexpr bool SUM = KIND == kConvSum;
    constexpr int TM = 2, TN = 2, NW = 4, KCH = 6, ROWB = KCH * 16, TAPS = 9;
    constexpr int BCO = 64, BP = 256;
    constexpr int A_BYTES = BCO * ROWB;               // weight rows of one tap and slice: six 1 KiB loads
    constexpr int NA = 2;                             // stages of the weight stream
    constexpr uint32_t XCDS = 8;
    using Out = typename OutT<OUT>::type;
    using Ops = Packed<TM, TN>;

    // row 0: zeros (source of taps outside the image when all taps share one sum); rows 1..: the slice
    __shared__ __attribute__((aligned(16))) uint8_t s_halo[(kHaloRows + 1) * ROWB];
    __shared__ __attribute__((aligned(16))) uint8_t s_a[NA][A_BYTES];
    __shared__ float s_sx[PER_TAP ? TAPS : 1][BP];    // x_scale / 256 under tap t, 0 outside the image
    __shared__ int s_mask[BP];                        // bit t: tap t of this output pixel is inside its image
    __shared__ __attribute__((aligned(16))) float s_sw[BCO];
    __shared__ __attribute__((aligned(16))) float s_bias[BCO];
    __shared__ float s_start[PER_TAP ? BP : 1];       // what a pixel's fp32 sums start from (see above)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // = pixel block of this wave (1 x 4 layout)
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int kbytes = a.k >> 1;
    const int slices = kbytes / ROWB;                 // host guarantees divisibility
    const int halo = a.w + 1;                         // pixels a tap can reach to either side
    const int rows_needed = BP + 2 * halo;            // <= kHaloRows, checked on the host
    const uint32_t last = a.pixels - 1;

    if (tid < ROWB / 4) reinterpret_cast<uint32_t *>(s_halo)[tid] = 0u;

    // ---- this workgroup's tiles: a contiguous run (as in the tile kernel) ----------------------
    uint32_t lo = 0, hi = a.n_tiles, j = blockIdx.x, sharers = gridDim.x;
    if (a.xcds) {
        const uint32_t x = blockIdx.x % XCDS;
        lo = static_cast<uint32_t>(static_cast<uint64_t>(a.n_tiles) * x / XCDS);
        hi = static_cast<uint32_t>(static_cast<uint64_t>(a.n_tiles) * (x + 1) / XCDS);
        j = blockIdx.x / XCDS;
        sharers = gridDim.x / XCDS;
    }
    const uint32_t per = (hi - lo) / sharers, rem = (hi - lo) % sharers;
    const uint32_t t_first = lo + j * per + (j < rem ? j : rem);
    const uint32_t my_tiles = per + (j < rem ? 1 : 0);

    // ---- per-lane pieces of the loads -----------------------------------------------------------
    // A wave-wide load covers 64 consecutive 16-byte slots q of a row-major [row][6 pieces] image:
    // row q / 6, piece q % 6, with adjacent pieces swapped in rows 8..15 (mod 16) against LDS bank
    // conflicts.  64 * 3 = 32 * 6: loads i and i + 3 repeat the per-lane pattern 32 rows further.
    int pat_row[3];
    uint32_t pat_byte[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int q = 64 * r + lane;
        pat_row[r] = q / KCH;
        pat_byte[r] = static_cast<uint32_t>(((q % KCH) ^ ((pat_row[r] >> 3) & 1)) * 16);
    }

    // weight rows of a tile: this wave's loads i = wave, wave + 4 (< 6) of every (tap, slice)
    uint32_t ld_a[2];
    auto set_weight_rows = [&](int co0) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int i = s * NW + wave, r = i % 3;
            const int row = pat_row[r] + 32 * (i / 3);
            int co = co0 + (row & ~31) + tile_row_to_channel(row & 31);
            co = co < a.n ? co : a.n - 1;
            ld_a[s] = static_cast<uint32_t>(co) * TAPS * kbytes + pat_byte[r];
        }
    };
    auto issue_weights = [&](int tap, int slice, int stage) {
        const uint8_t *base = a.wq + (static_cast<uint32_t>(tap) * kbytes + slice * ROWB);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const int i = s * NW + wave;
            if (i < 6) load_to_lds16(base + ld_a[s], s_a[stage] + i * 1024);
        }
    };
    // activation rows p0 - halo .. of one slice into LDS rows 1..; load i covers rows 32 (i/3) + ...
    auto issue_halo = [&](uint32_t p0, int slice) {
        const int64_t first = static_cast<int64_t>(p0) - halo;
        const bool inside = first >= 0 && first + kHaloRows - 1 <= static_cast<int64_t>(last);
        const int loads = 3 * ((rows_needed + 31) / 32);
        for (int i = wave; i < loads; i += NW) {
            const int r = i % 3, g = i / 3;
            uint8_t *dst = s_halo + ROWB + i * 1024;
            if (32 * g + pat_row[r] >= rows_needed) continue;   // lanes past the last row needed load nothing
            if (inside) {
                const uint8_t *base = a.xq + (static_cast<uint64_t>(first) + 32 * g) * kbytes + slice * ROWB;
                load_to_lds16(base + (static_cast<uint32_t>(pat_row[r]) * kbytes + pat_byte[r]), dst);
            } else {
                int64_t pix = first + 32 * g + pat_row[r];
                pix = pix < 0 ? 0 : (pix > static_cast<int64_t>(last) ? last : pix);
                load_to_lds16(a.xq + (static_cast<uint64_t>(pix) * kbytes + slice * ROWB + pat_byte[r]), dst);
            }
        }
    };

    const uint32_t lds_halo = lds_address(s_halo);
    const uint32_t lds_a0 = lds_address(s_a) + lrow * ROWB + (lhalf ^ ((lrow >> 3) & 1)) * 16;
    const uint32_t lds_sx = lds_address(&s_sx[0][0]) + (wave * 64 + lrow) * 4;
    const uint32_t lds_sw = lds_address(s_sw) + lhalf * 64;
    const uint32_t lds_bias = lds_address(s_bias) + lhalf * 64;

    // integer accumulators start from the bits of 1.5 * 2^23 when their sums are folded per tap
    // (integer output: from 0, the sums themselves are stored)
    constexpr bool INT_OUT = OUT == kOutI32;
    constexpr bool FOLD = PER_TAP && !INT_OUT;
    constexpr int kBiasBits = 0x4B400000;
    constexpr float kBias = 12582912.0f;
    v16i acc_start;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_start[r] = FOLD ? kBiasBits : 0;
    if constexpr (PER_TAP) asm volatile("" : "+v"(acc_start));   // kept in registers, not rebuilt per tap

    if (my_tiles > 0) {   // loads of the first tile (the zero row above is not touched by them)
        set_weight_rows(static_cast<int>(t_first % a.n_co_tiles) * BCO);
        issue_halo((t_first / a.n_co_tiles) * BP, 0);
        issue_weights(0, 0, 0);
    }

    for (uint32_t kt = 0; kt < my_tiles; ++kt) {
        const uint32_t tile = t_first + kt;
        const int co0 = static_cast<int>(tile % a.n_co_tiles) * BCO;
        const uint32_t p0 = (tile / a.n_co_tiles) * BP;

        // ---- tables of the tile (its first loads are in flight) ---------------------------------
        int my_mask;
        {
            const uint32_t pix = p0 + tid;
            const uint32_t q = hq::div_magic31(pix, a.w, a.w_magic, a.w_shift);
            const int ow = static_cast<int>(pix - q * a.w);
            const int oh = static_cast<int>(q - hq::div_magic31(q, a.h, a.h_magic, a.h_shift) * a.h);
            const int cm = (ow > 0 ? 1 : 0) | 2 | (ow + 1 < a.w ? 4 : 0);
            my_mask = (oh > 0 ? cm : 0) | (cm << 3) | (oh + 1 < a.h ? cm << 6 : 0);
            if (pix >= a.pixels) my_mask = 0;
            s_mask[tid] = my_mask;
            if constexpr (INT_OUT) {
                // no scales are read (the pointers may be null)
            } else if constexpr (PER_TAP) {
                float v[TAPS];
#pragma unroll
                for (int t = 0; t < TAPS; ++t) {
                    uint32_t ip = pix + static_cast<uint32_t>((t / 3 - 1) * a.w + (t % 3 - 1));   // wraps below 0
                    ip = ip < last ? ip : last;
                    v[t] = a.sx[ip];
                }
                float total = 0.f;
#pragma unroll
                for (int t = 0; t < TAPS; ++t) {
                    v[t] = ((my_mask >> t) & 1) ? v[t] * (1.0f / 256.0f) : 0.f;
                    s_sx[t][tid] = v[t];
                    total += v[t];
                }
                s_start[tid] = -kBias * static_cast<float>(slices) * total;
            } else {
                s_sx[0][tid] = my_mask ? a.sx[0] * (1.0f / 256.0f) : 0.f;
            }
            if constexpr (!INT_OUT) {
                if (tid < BCO) {
                    const bool ok = co0 + tid < a.n;
                    const Out *bias = static_cast<const Out *>(a.bias);
                    s_sw[tid] = ok ? a.sw[co0 + tid] : 0.f;
                    s_bias[tid] = ok && bias ? to_float(bias[co0 + tid]) : 0.f;
                }
            }
        }

        v16i acc[TM][TN];
        float facc[FOLD ? TM : 1][FOLD ? TN : 1][16];
        auto multiply = [&](Ops &o, bool first) {
            v4i a0[TM], a1[TM], b0[TN], b1[TN];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) { pin(o.a[tm]); expand(o.a[tm], a0[tm], a1[tm]); }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) { pin(o.b[tn]); expand(o.b[tn], b0[tn], b1[tn]); }
            if (first) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[tm], b0[tn], acc_start, 0, 0, 0);
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

        int pix_mask[TN];   // masks of this lane's pixels, local index wave * 64 + tn * 32 + lrow (one sum, integer output)

        for (int slice = 0; slice < slices; ++slice) {
            if (slice > 0) {
                __syncthreads();   // the previous slice is no longer read
                issue_halo(p0, slice);
                issue_weights(0, slice, 0);
            }
            wait_vmem<0>();
            __syncthreads();   // slice, first weights and tables visible
            if (slice == 0) {
                if constexpr (SUM || INT_OUT) {
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) pix_mask[tn] = s_mask[wave * 64 + tn * 32 + lrow];
                }
                if constexpr (FOLD) {
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const float f0 = s_start[wave * 64 + tn * 32 + lrow];
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int r = 0; r < 16; ++r) facc[tm][tn][r] = f0;
                    }
                }
            }

            int stage = 0;
#pragma unroll 1
            for (int tap = 0; tap < TAPS; ++tap) {
                // the stage of the previous tap is free (barrier below): refill it NA - 1 taps ahead
                if (tap + NA - 1 < TAPS) issue_weights(tap + NA - 1, slice, stage == 0 ? NA - 1 : stage - 1);

                // B operand: halo row of this lane's pixel under the tap (LDS row 1 + that)
                const int dpix = (tap / 3 - 1) * a.w + (tap % 3 - 1);
                const int row0 = halo + wave * 64 + lrow + dpix;   // row of the slice image, >= 0
                uint32_t addr_b[TN];
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const int row = row0 + 32 * tn;
                    addr_b[tn] = lds_halo + (1 + row) * ROWB + (lhalf ^ ((row >> 3) & 1)) * 16;
                    if constexpr (SUM) {
                        if (!((pix_mask[tn] >> tap) & 1)) addr_b[tn] = lds_halo + lhalf * 16;   // zeros
                    }
                }
                const uint32_t addr_a = lds_a0 + stage * A_BYTES;
                auto read_step = [&](Ops &o, auto KOFF) {
                    lds_read16<decltype(KOFF)::value>(o.a[0], addr_a);
                    lds_read16<32 * ROWB + decltype(KOFF)::value>(o.a[1], addr_a);
                    lds_read16<decltype(KOFF)::value>(o.b[0], addr_b[0]);
                    lds_read16<decltype(KOFF)::value>(o.b[1], addr_b[1]);
                };
                Ops op[2];
                read_step(op[0], std::integral_constant<int, 0>{});
                read_step(op[1], std::integral_constant<int, 32>{});
                wait_lds<4>();
                multiply(op[0], PER_TAP || (tap == 0 && slice == 0));
                read_step(op[0], std::integral_constant<int, 64>{});
                wait_lds<4>();
                multiply(op[1], false);
                wait_lds<0>();
                multiply(op[0], false);

                if constexpr (PER_TAP && INT_OUT) {
                    // the sums of this (slice, tap), exactly: stored by the first slice, added by the others
                    // (the same lane owns an element in every slice); a tap outside the image is written as 0
                    int *yi = static_cast<int *>(a.y);
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const uint32_t pix = p0 + wave * 64 + tn * 32 + lrow;
                        if (pix >= a.pixels) continue;
                        const bool inside = (pix_mask[tn] >> tap) & 1;
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm) {
                            const int cbase = co0 + tm * 32 + 16 * lhalf;
                            int *dst = yi + (static_cast<int64_t>(pix) * TAPS + tap) * a.n + cbase;
#pragma unroll
                            for (int r = 0; r < 16; ++r) {
                                if (cbase + r >= a.n) continue;
                                const int v = inside ? (acc[tm][tn][r] >> 8) : 0;
                                dst[r] = slice == 0 ? v : dst[r] + v;
                            }
                        }
                    }
                } else if constexpr (PER_TAP) {
                    float s[TN];
                    read_tap_scales<TN>(s, lds_sx + tap * (BP * 4));
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                facc[tm][tn][r] = __builtin_fmaf(s[tn], __int_as_float(acc[tm][tn][r]), facc[tm][tn][r]);
                }
                // this wave's share of the next tap's weights has landed once only the loads of the
                // taps after it are pending (waves 0 and 1 issue two loads per tap, 2 and 3 one)
                {
                    const int ahead = (tap + NA - 1 < TAPS ? tap + NA - 1 : TAPS - 1) - (tap + 1);
                    const int pending = ahead > 0 ? ahead * (wave < 2 ? 2 : 1) : 0;
                    if (pending >= 4) wait_vmem<4>();
                    else if (pending >= 2) wait_vmem<2>();
                    else if (pending == 1) wait_vmem<1>();
                    else wait_vmem<0>();
                }
                __builtin_amdgcn_s_barrier();     // everyone's has landed; this tap's stage is free
                stage = stage + 1 == NA ? 0 : stage + 1;
            }
        }

        // ---- loads of the next tile: the activation slice and the weight stages are free ---------
        if (kt + 1 < my_tiles) {
            const uint32_t next = tile + 1;
            const uint32_t next_p0 = (next / a.n_co_tiles) * BP;
            set_weight_rows(static_cast<int>(next % a.n_co_tiles) * BCO);
            if (!(slices == 1 && next_p0 == p0)) issue_halo(next_p0, 0);
            issue_weights(0, 0, 0);
        }

        // ---- dequantising epilogue (LDS reads by hand: loads of the next tile are in flight) ------
        if constexpr (INT_OUT) {
            if constexpr (SUM) {   // the one sum over all taps and slices
                int *yi = static_cast<int *>(a.y);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const uint32_t pix = p0 + wave * 64 + tn * 32 + lrow;
                    if (pix >= a.pixels) continue;
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
                        const int cbase = co0 + tm * 32 + 16 * lhalf;
                        int *dst = yi + static_cast<int64_t>(pix) * a.n + cbase;
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (cbase + r < a.n) dst[r] = acc[tm][tn][r] >> 8;
                    }
                }
            }
        } else {
        Out *y = static_cast<Out *>(a.y);
        const bool vec_ok = (a.n & 15) == 0;
        float sxv[TN];
        if constexpr (SUM) read_tap_scales<TN>(sxv, lds_sx);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int cbase = co0 + tm * 32 + 16 * lhalf;
            v4i swq[4], bq[4];
            lds_read16<0>(swq[0], lds_sw + tm * 128);
            lds_read16<16>(swq[1], lds_sw + tm * 128);
            lds_read16<32>(swq[2], lds_sw + tm * 128);
            lds_read16<48>(swq[3], lds_sw + tm * 128);
            lds_read16<0>(bq[0], lds_bias + tm * 128);
            lds_read16<16>(bq[1], lds_bias + tm * 128);
            lds_read16<32>(bq[2], lds_bias + tm * 128);
            lds_read16<48>(bq[3], lds_bias + tm * 128);
            wait_lds<0>();
#pragma unroll
            for (int i = 0; i < 4; ++i) { pin(swq[i]); pin(bq[i]); }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const uint32_t pix = p0 + wave * 64 + tn * 32 + lrow;
                if (pix >= a.pixels) continue;
                float out[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v;
                    if constexpr (FOLD) v = facc[tm][tn][r];
                    else v = sxv[tn] * static_cast<float>(acc[tm][tn][r]);
                    out[r] = __builtin_fmaf(v, __int_as_float(swq[r >> 2][r & 3]), __int_as_float(bq[r >> 2][r & 3]));
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
        __syncthreads();   // the tables are free for the next tile
    }
}

}  // namespace

// True if the layer fits this kernel: channel slices of 192, image rows short enough for 256
// pixels plus the halo to fit the LDS buffer.
bool hq_conv3x3_halo_fits(const GemmArgs &g, hq_dtype y_dtype) {
    return g.k % 192 == 0 && (y_dtype == HQ_F16 || y_dtype == HQ_F32 || y_dtype == HQ_I32) &&
           256 + 2 * (g.w + 1) <= kHaloRows && g.pixels >= static_cast<uint32_t>(kHaloRows);
}

hq_status hq_conv3x3_halo_launch(const GemmArgs &g, hq_dtype y_dtype, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    if (!hq_conv3x3_halo_fits(g, y_dtype)) return HQ_ERR_UNSUPPORTED;
    HaloArgs a{};
    a.xq = g.xq; a.sx = g.sx; a.wq = g.wq; a.sw = g.sw; a.bias = g.bias; a.y = g.y;
    a.pixels = g.pixels; a.n = g.n; a.k = g.k; a.h = g.h; a.w = g.w; a.sx_static = g.sx_static;
    const hq::Magic31 mw = hq::magic31(static_cast<uint32_t>(g.w)), mh = hq::magic31(static_cast<uint32_t>(g.h));
    a.w_magic = mw.m; a.w_shift = mw.s; a.h_magic = mh.m; a.h_shift = mh.s;
    a.n_co_tiles = static_cast<uint32_t>((g.n + 63) / 64);
    const int64_t tiles = ((static_cast<int64_t>(g.pixels) + 255) / 256) * a.n_co_tiles;
    if (tiles > 0x7fffffffLL) return HQ_ERR_SHAPE;
    a.n_tiles = static_cast<uint32_t>(tiles);
    // workgroups per CU: the one-sum kernel needs no fp32 sums beside the integer ones and fits three
    const int64_t slots = (g.sx_static ? 3 : 2) * static_cast<int64_t>(hq::compute_units());
    const unsigned grid = static_cast<unsigned>(tiles < slots ? tiles : slots);
    a.xcds = grid % 8 == 0 ? 1 : 0;
    const dim3 block(256);
    if (g.sx_static) {
        if (y_dtype == HQ_F16)
            hipLaunchKernelGGL((conv3x3_halo_kernel<kConvSum, kOutF16>), dim3(grid), block, 0, stream, a);
        else if (y_dtype == HQ_F32)
            hipLaunchKernelGGL((conv3x3_halo_kernel<kConvSum, kOutF32>), dim3(grid), block, 0, stream, a);
        else
            hipLaunchKernelGGL((conv3x3_halo_kernel<kConvSum, kOutI32>), dim3(grid), block, 0, stream, a);
    } else {
        if (y_dtype == HQ_F16)
            hipLaunchKernelGGL((conv3x3_halo_kernel<kConvPerTap, kOutF16>), dim3(grid), block, 0, stream, a);
        else if (y_dtype == HQ_F32)
            hipLaunchKernelGGL((conv3x3_halo_kernel<kConvPerTap, kOutF32>), dim3(grid), block, 0, stream, a);
        else
            hipLaunchKernelGGL((conv3x3_halo_kernel<kConvPerTap, kOutI32>), dim3(grid), block, 0, stream, a);
    }
    return check.status();
}
