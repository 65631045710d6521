// 3x3 / stride 1 / pad 1 NHWC convolution with per-pixel activation scales on int8 MFMA, one
// workgroup of eight waves per CU (or two of four waves), the activation tile expanded to int8
// ONCE and resident in LDS (Method, "Convolution": one integer sum per tap, taps combined in fp32
// with the scale of the input pixel under the tap).
//
// Why.  Three things hold the other 3x3 kernels below a third of the int8 rate on the UNet's
// layers: (1) tile counts that do not divide the machine (768 tiles for 512 resident
// workgroups, 576 for 256 CUs), (2) every wave expanding the packed nibbles of BOTH operands for
// every use, nine times for an activation row, and (3) operand streams of 250..500 bytes per MFMA
// through a copy path that delivers about 170.  Here
//   - a workgroup owns 192 output channels x PX pixels (PX = 256, 128 or 64, chosen on the host so
//     that the layer has about one tile per CU), i.e. 12, 6 or 3 wave tiles of 64 x 64 for eight
//     waves: the work is dealt out in two PHASES, and where a phase has fewer wave tiles than
//     waves a tile's K range (its 9 x C_in/192 "units" of one tap and one 192-channel slice) is
//     split over 2, 4 or 8 waves, whose partial fp32 sums meet in LDS in a fixed order:
//         phase A: channels 0..127   as 2 x PX/64 wave tiles, each split 4 / (PX/64) ways in K,
//         phase B: channels 128..191 as 1 x PX/64 wave tiles, each split 8 / (PX/64) ways in K,
//     so every wave multiplies 1.5 / 0.75 / 0.375 tiles' worth of units, all waves the same amount
//     (four waves: 192 channels x 128 pixels, no split in phase A, two ways in phase B);
//   - the activation rows of the tile's pixels plus W + 1 pixels either side are fetched once (all
//     input channels), expanded to int8 (16 x code) on the way into LDS, and all nine taps of all
//     phases read them at shifted addresses: an activation operand is an LDS read, nothing else;
//   - only the weights stream (direct-to-LDS loads, packed, two or three stages of one unit per K
//     group), 64..128 bytes per MFMA; a wave expands the weight nibbles it reads (three vector
//     instructions per MFMA in the 2 x 2 register tile).
// The sums of one unit are folded into the fp32 result with one fma per element: the integer
// accumulators start from the bit pattern of 1.5 * 2^23, so their bits read as a float are
// 1.5 * 2^23 + S exactly (S = 256 * sum, |S| < 2^22 for 192 codes), and the fp32 sums start from
// minus the known surplus.  A wave requests the activation operands of a unit one step ahead (they
// do not depend on the weight stream), its weight operands after the step's barrier, and refills
// the freed weight stage while those are on their way.  fp16 results are transposed through a
// per-wave LDS staging area so that neighbouring lanes store contiguous bytes.
//
// Integer output (HQ_I32): the same loads, stages, phases and MFMAs; instead of the fold every
// wave adds the exact sums of its units to the zero-filled [pixel, tap, n] output with integer
// atomics (integer addition is exact in any order).
#pragma once
#include "hq_hadamard_mfma.h"
#include "hq_int_gemm_kernel.h"

namespace {

// LDS of a workgroup: all of a CU's 160 KiB for eight waves (one workgroup per CU), half of it for
// four waves (two workgroups per CU, each with its own barrier, so that one multiplies while the
// other folds, waits or synchronises)
constexpr int res_lds(int nwl) { return nwl == 3 ? 163840 : 81920; }
constexpr int kResBlock = 64 * 96;   // weight rows of one 64-channel block of one unit (packed)
constexpr int kRes4WaveCost = 85;    // percent: time of the four-wave form relative to the eight-wave form

struct ResArgs {
    const uint8_t *xq;   // [pixels, k/2]
    const float *sx;     // [pixels]
    const uint8_t *wq;   // [n, 9, k/2]
    const float *sw;     // [n]
    const void *bias;    // [n] of the output dtype, or null
    void *y;             // [pixels, n]; integer output: [pixels, 9, n], zero-filled before the launch
    uint32_t pixels;
    int n, k, h, w;
    uint32_t w_magic, w_shift, h_magic, h_shift;   // exact division of a pixel index by w and by h
    uint32_t s_magic, s_shift;                     // ... of a unit index by the number of slices
    uint32_t p_magic, p_shift;                     // ... of a piece index by the 16-byte pieces per activation row
    int pg_log2;         // PX = 64 << pg_log2
    int slices;          // k / 192
    uint32_t n_co_tiles, n_tiles;
    uint32_t stage_base, stage_bytes, tab_base;    // LDS layout: activations at 0, then stages, then tables
    // transform and quantisation done here (FUSED): the fp16 activations [pixels, k], qmax of the codes, and
    // optional outputs of the codes [pixels, k/2] and scales [pixels] the kernel used (null: not written)
    const __half *x;
    float qmax;
    uint8_t *xq_out;
    float *sx_out;
};

// chunk c (0..15) of a wave's 64 x 64 partial result = sub-tile c / 4 (tm * 2 + tn), registers 4 (c % 4) .. + 3;
// among the KG waves that share a tile, wave c / (16 / KG) finishes chunk c (whole 32 x 32 sub-tiles
// for KG <= 4).  A wave stores the chunks it does not finish compactly: chunk c of wave kg sits at
// position c, or c - 16 / KG if it lies after the chunks kg finishes itself.
__device__ __forceinline__ int exchange_owner(int c, int kgn_log2) { return c >> (4 - kgn_log2); }
__device__ __forceinline__ int exchange_pos(int c, int kg, int kgn_log2) {
    const int g = 16 >> kgn_log2;
    return c < kg * g ? c : c - g;
}

// PGL: log2 of the pixel blocks of 64 per tile (the tile has 64 << PGL pixels)
// weight stages of a tile of 64 << pgl pixels of a workgroup of 1 << nwl waves (a stage is
// (1 << nwl) >> pgl blocks of 6 KiB)
constexpr int res_stages(int pgl, int nwl) { return nwl == 3 ? (pgl == 0 ? 2 : 3) : 2; }

// NWL: log2 of the waves per workgroup (3 or 2).  The K ranges are split (waves / 2) / pgn ways in
// phase A and waves / pgn ways in phase B.
// FUSED: the activations arrive as fp16 and the kernel itself applies the block-64 Hadamard
// transform (on the matrix cores, as the stand-alone transform-quantise kernel does, with the same
// arithmetic and so the same codes) and the per-pixel quantisation to the rows of its tile and
// halo: the codes go straight into the LDS image as int8 and never reach memory, the scales into
// a table (Method, "Matrix Multiplication": X H is only ever consumed by the integer product).
template <int OUT, int PGL, int NWL, bool FUSED>
__global__ __launch_bounds__(64 << NWL, NWL == 3 ? 1 : 2) void conv3x3_res_kernel(ResArgs a) {
    constexpr int NT = 64 << NWL;
    constexpr int kResLds = res_lds(NWL);
    static_assert(NWL - 1 - PGL >= 0, "at least one wave per tile in phase A");
    constexpr bool INT_OUT = OUT == kOutI32;
    constexpr int TM = 2, TN = 2, TAPS = 9, MAXL = (6 + (1 << PGL) - 1) >> PGL;
    constexpr int NSTAGE = res_stages(PGL, NWL);
    constexpr int kBiasBits = 0x4B400000;
    constexpr float kBias = 12582912.0f;
    using Out = typename OutT<OUT>::type;
    using Ops = Packed<TM, 2 * TN>;   // b[2 * tn + m]: int8 operand of pixel block tn, MFMA m of the step

    __shared__ __attribute__((aligned(16))) uint8_t lds[kResLds];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int kbytes = a.k >> 1;
    const int S = a.slices;
    const int NU = TAPS * S;
    constexpr int pgn_log2 = PGL, pgn = 1 << pgn_log2, PX = 64 << pgn_log2;
    const int halo = a.w + 1;
    const int rows = PX + 2 * halo;
    const uint32_t last = a.pixels - 1;

    // tables (at the top of the LDS): scale of the input pixel under tap t for every pixel of the tile,
    // tap masks, scales and bias of the tile's 192 channels
    float *s_sx = reinterpret_cast<float *>(lds + a.tab_base);            // [9][PX], x_scale / 256, 0 outside
    int *s_mask = reinterpret_cast<int *>(s_sx + TAPS * PX);              // [PX]
    float *s_sw = reinterpret_cast<float *>(s_mask + PX);                 // [192]
    float *s_bias = s_sw + 192;                                           // [192]
    float *s_rowscale = s_bias + 192;                                     // [rows] (FUSED): scale of every row of the image

    // ---- tile of this workgroup (XCD-contiguous: workgroup b runs on XCD b % 8) ------------------
    uint32_t tile = blockIdx.x;
    if (gridDim.x % 8 == 0) tile = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
    const int co0 = static_cast<int>(tile % a.n_co_tiles) * 192;
    const uint32_t p0 = (tile / a.n_co_tiles) * PX;

    // ---- phases ------------------------------------------------------------------------------------
    // phase 0: channel blocks 0, 1; K groups 4 / pgn.  phase 1: channel block 2; K groups 8 / pgn.
    // In both phases wave wv works on block wv / pgn of a stage (K group major, then channel block) and
    // the pgn waves of a block (its pixel blocks) fetch that block's weight rows together.
    const int blk = wv >> pgn_log2;           // this wave's block of a stage
    const int ws = wv & (pgn - 1);            // its pixel block = its index among the waves of the block
    auto unit_first = [&](int kg, int kgn_log2) { return (kg * NU) >> kgn_log2; };

    // ---- weight stream -------------------------------------------------------------------------------
    // A block of a stage is the row-major [64 rows][6 pieces of 16 bytes] image of 64 weight rows of one
    // unit: six wave-wide loads of 1 KiB (load r covers slots q = 64 r + lane: row q / 6, piece q % 6),
    // adjacent pieces swapped in rows 8..15 (mod 16) against bank conflicts of the operand reads.  Wave
    // ws of the block issues loads r = ws, ws + pgn, ... < 6.
    uint32_t ld_off[MAXL];     // per lane: byte offset of the piece inside the weight tensor at tap 0, slice 0
    int f_unit = 0, f_slice = 0, f_stage = 0, f_issued = 0;
    uint32_t f_off = 0;        // uniform: tap * kbytes + slice * 96 of the unit fetched next
    auto begin_fetch = [&](int phase, bool continuing) {
        const int kl = phase == 0 ? NWL - 1 - pgn_log2 : NWL - pgn_log2;
        const int cblock = phase == 0 ? (blk & 1) : 2;
        const int kg = phase == 0 ? blk >> 1 : blk;
#pragma unroll
        for (int j = 0; j < MAXL; ++j) {
            const int r = ws + (j << pgn_log2);
            const int q = 64 * r + lane, row = q / 6, piece = (q - 6 * row) ^ ((row >> 3) & 1);
            int co = co0 + 64 * cblock + (row & ~31) + tile_row_to_channel(row & 31);
            co = co < a.n ? co : a.n - 1;
            ld_off[j] = static_cast<uint32_t>(co) * TAPS * kbytes + piece * 16;
        }
        f_unit = unit_first(kg, kl);
        const int tap = static_cast<int>(hq::div_magic31(static_cast<uint32_t>(f_unit), S, a.s_magic, a.s_shift));
        f_slice = f_unit - tap * S;
        f_off = static_cast<uint32_t>(tap) * kbytes + f_slice * 96;
        if (!continuing) f_stage = 0;   // a stream that runs on keeps rotating through the stages
        f_issued = 0;
    };
    // requests the next unit of this wave's block (a K group that has run out of its own units goes on
    // into the following ones, which are not used; the last unit of the tensor is repeated)
    auto issue_step = [&]() {
        uint8_t *image = lds + a.stage_base + f_stage * a.stage_bytes + blk * kResBlock;
        const uint8_t *src = a.wq + f_off;
#pragma unroll
        for (int j = 0; j < MAXL; ++j) {
            const int r = ws + (j << pgn_log2);
            if (r < 6) load_to_lds16(src + ld_off[j], image + r * 1024);
        }
        if (f_unit + 1 < NU) {
            ++f_unit;
            f_off += 96;
            if (++f_slice == S) { f_slice = 0; f_off += kbytes - 96 * S; }
        }
        f_stage = f_stage + 1 == NSTAGE ? 0 : f_stage + 1;
        ++f_issued;
    };
    // waits until this wave's loads of all steps but the youngest have landed
    auto wait_all_but_one_step = [&]() {
        if constexpr (INT_OUT || NSTAGE == 2) wait_vmem<0>();   // (integer output: other memory operations in between)
        else if constexpr (PGL == 0) wait_vmem<6>();
        else if constexpr (PGL == 1) wait_vmem<3>();
        else if (ws < 2) wait_vmem<2>();
        else wait_vmem<1>();
    };
    constexpr int kla = NWL - 1 - pgn_log2, klb = NWL - pgn_log2;   // log2 of the K groups of the two phases
    const int ulen_of[2] = {(NU + (1 << kla) - 1) >> kla, (NU + (1 << klb) - 1) >> klb};
    begin_fetch(0, false);
    for (int st = 0; st < NSTAGE - 1 && st < ulen_of[0]; ++st) issue_step();

    // ---- table entries are requested first, so that their latency and that of the activation rows
    //      below pass together -------------------------------------------------------------------------------
    int t_mask = 0;
    float t_sx[TAPS];
    float t_sw = 0.f, t_bias = 0.f;
    const int t_chan = NT - 1 - tid;   // (the last threads first: they have no pixel to look up)
    if (tid < PX) {
        const uint32_t pix = p0 + tid;
        const uint32_t q = hq::div_magic31(pix, a.w, a.w_magic, a.w_shift);
        const int ow = static_cast<int>(pix - q * a.w);
        const int oh = static_cast<int>(q - hq::div_magic31(q, a.h, a.h_magic, a.h_shift) * a.h);
        const int cm = (ow > 0 ? 1 : 0) | 2 | (ow + 1 < a.w ? 4 : 0);
        t_mask = (oh > 0 ? cm : 0) | (cm << 3) | (oh + 1 < a.h ? cm << 6 : 0);
        if (pix >= a.pixels) t_mask = 0;
        if constexpr (!INT_OUT && !FUSED) {
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                uint32_t ip = pix + static_cast<uint32_t>((t / 3 - 1) * a.w + (t % 3 - 1));   // wraps below 0
                ip = ip < last ? ip : last;
                t_sx[t] = a.sx[ip];
            }
        }
    }
    if constexpr (!INT_OUT) {
        if (t_chan < 192 && co0 + t_chan < a.n) {
            const Out *bias = static_cast<const Out *>(a.bias);
            t_sw = a.sw[co0 + t_chan];
            t_bias = bias ? to_float(bias[co0 + t_chan]) : 0.f;
        }
    }

    // ---- activation tile: packed rows -> int8 (16 x code) in LDS -------------------------------------
    // Row r of the image is pixel p0 - halo + r (clamped into the tensor; rows outside the image are
    // only ever read under taps whose scale is 0).  Plane s (192-channel slice) at s * rows * 192; a row
    // is three 64-byte K steps of four 16-byte pieces [MFMA 0 / lane half 0, 0 / 1, 1 / 0, 1 / 1], the
    // piece index xor-ed with (row / 4) % 4 so that the operand reads of 16 consecutive rows hit 16
    // different bank groups (row stride 192 bytes = 12 groups).
    if constexpr (FUSED) {
        // One wave transforms and quantises 16 rows at a time: lane l owns row l % 16 of the group and
        // K slice q = l / 16; its operands of 64-channel block b are the two 16-byte pieces at channels
        // 64 b + 32 h + 8 q, its 16 results are channels 64 b + 16 q .. + 15.  First pass: the row's
        // abs-max over all blocks; second pass: the transform again (the fp16 pieces are still in
        // registers), eight values to a packed dword exactly as the stand-alone kernel packs them, two dwords
        // expanded to the lane's 16 int8 operand bytes: piece (MFMA q % 2, lane half q / 2) of K step
        // b % 3 of slice b / 3.
        v8h hmat[4][2];
        hadamard64_operands(lane, hmat);
        const int tok = lane & 15, q = lane >> 4;
        const int64_t first = static_cast<int64_t>(p0) - halo;
        const bool writes_debug = a.xq_out != nullptr && co0 == 0;
        // the fp16 pieces of a row: all requested before any is used, and those of the wave's next group
        // of rows before the current group is worked on (up to three slices of three blocks each)
        auto row_source = [&](int g16) {
            const int row = g16 + tok;
            int64_t pix = first + (row < rows ? row : rows - 1);
            pix = pix < 0 ? 0 : (pix > static_cast<int64_t>(last) ? last : pix);
            return pix;
        };
        auto request = [&](v8h (&b)[3][3][2], int64_t pix) {
            const __half *src = a.x + static_cast<uint64_t>(pix) * a.k + 8 * q;
#pragma unroll
            for (int sl = 0; sl < 3; ++sl) {
                if (sl < S) {
#pragma unroll
                    for (int bk = 0; bk < 3; ++bk) {
                        b[sl][bk][0] = *reinterpret_cast<const v8h *>(src + 64 * (3 * sl + bk));
                        b[sl][bk][1] = *reinterpret_cast<const v8h *>(src + 64 * (3 * sl + bk) + 32);
                    }
                }
            }
        };
        v8h b[3][3][2], b_next[3][3][2];
        if (wv * 16 < rows) request(b_next, row_source(wv * 16));
        for (int g16 = wv * 16; g16 < rows; g16 += 16 << NWL) {
            const int row = g16 + tok;
            const int lrow_c = row < rows ? row : rows - 1;
            const int64_t pix = row_source(g16);
#pragma unroll
            for (int sl = 0; sl < 3; ++sl)
#pragma unroll
                for (int bk = 0; bk < 3; ++bk) { b[sl][bk][0] = b_next[sl][bk][0]; b[sl][bk][1] = b_next[sl][bk][1]; }
            if (g16 + (16 << NWL) < rows) request(b_next, row_source(g16 + (16 << NWL)));
            float amax = 0.f;
#pragma unroll
            for (int sl = 0; sl < 3; ++sl) {
                if (sl < S) {
#pragma unroll
                    for (int bk = 0; bk < 3; ++bk) {
                        float v[16];
                        hadamard64_transform(hmat, b[sl][bk], v);
#pragma unroll
                        for (int r = 0; r < 16; ++r) amax = fmaxf(amax, fabsf(v[r]));
                    }
                }
            }
            amax = fmaxf(amax, __shfl_xor(amax, 16));   // the row's other three K slices
            amax = fmaxf(amax, __shfl_xor(amax, 32));
            const float inv = amax > 0.f ? a.qmax / amax : 0.f;
            const float scale = amax > 0.f ? (amax * 0.125f) / a.qmax : 1.0f;
            // rows of this tile's own pixels (not of the halo) that exist: theirs are the codes and scales to report
            const bool own = row >= halo && row < halo + PX && first + row <= static_cast<int64_t>(last);
            if (row < rows && q == 0) {
                s_rowscale[row] = scale;
                if (own && co0 == 0 && a.sx_out) a.sx_out[pix] = scale;
            }
            const uint32_t sw4 = (static_cast<uint32_t>(lrow_c) >> 2) & 3;
            const uint32_t piece = ((((q & 1) << 1) | (q >> 1)) ^ sw4) * 16;
#pragma unroll
            for (int sl = 0; sl < 3; ++sl) {
                if (sl < S) {
#pragma unroll
                    for (int bk = 0; bk < 3; ++bk) {
                        float v[16];
                        hadamard64_transform(hmat, b[sl][bk], v);   // (cheaper than keeping 144 values)
                        v4i p = {0, 0, 0, 0};
                        p.x = static_cast<int>(pack8_magic(v, inv));
                        p.y = static_cast<int>(pack8_magic(v + 8, inv));
                        v4i first_half, second_half;
                        expand(p, first_half, second_half);
                        if (row < rows) {
                            *reinterpret_cast<v4i *>(lds + (sl * rows + row) * 192 + bk * 64 + piece) = first_half;
                            if (writes_debug && own)
                                *reinterpret_cast<uint2 *>(a.xq_out + static_cast<uint64_t>(pix) * kbytes +
                                                           (3 * sl + bk) * 32 + q * 8) =
                                    uint2{static_cast<uint32_t>(p.x), static_cast<uint32_t>(p.y)};
                        }
                    }
                }
            }
        }
    } else
    {
        const uint32_t pieces_per_row = 6u * S;
        const uint32_t total = static_cast<uint32_t>(rows) * pieces_per_row;
        const int64_t first = static_cast<int64_t>(p0) - halo;
        constexpr int BATCH = NWL == 3 ? 5 : 7;   // pieces per thread in flight: one batch covers a tile
        for (uint32_t base = tid; base < total; base += NT * BATCH) {
            v4i p[BATCH];
            uint32_t dst[BATCH];
#pragma unroll
            for (int e = 0; e < BATCH; ++e) {
                const uint32_t q = base + NT * e;
                if (q < total) {
                    const uint32_t row = hq::div_magic31(q, pieces_per_row, a.p_magic, a.p_shift);
                    const uint32_t rem = q - row * pieces_per_row;
                    int64_t pix = first + row;
                    pix = pix < 0 ? 0 : (pix > static_cast<int64_t>(last) ? last : pix);
                    p[e] = *reinterpret_cast<const v4i *>(a.xq + static_cast<uint64_t>(pix) * kbytes + rem * 16);
                    const uint32_t slice = rem / 6, pc = rem - slice * 6;
                    const uint32_t sw = (row >> 2) & 3;
                    // piece index of (MFMA 0, lane half pc & 1); MFMA 1 is that index xor 2
                    dst[e] = (slice * rows + row) * 192 + (pc >> 1) * 64 + (((pc & 1) ^ sw) * 16);
                }
            }
#pragma unroll
            for (int e = 0; e < BATCH; ++e) {
                const uint32_t q = base + NT * e;
                if (q < total) {
                    v4i first_half, second_half;
                    expand(p[e], first_half, second_half);
                    *reinterpret_cast<v4i *>(lds + dst[e]) = first_half;
                    *reinterpret_cast<v4i *>(lds + (dst[e] ^ 32)) = second_half;
                }
            }
        }
    }

    // ---- tables ------------------------------------------------------------------------------------------
    if (tid < PX) {
        s_mask[tid] = t_mask;
        if constexpr (!INT_OUT && !FUSED) {
#pragma unroll
            for (int t = 0; t < TAPS; ++t) s_sx[t * PX + tid] = ((t_mask >> t) & 1) ? t_sx[t] * (1.0f / 256.0f) : 0.f;
        }
    }
    if constexpr (!INT_OUT && FUSED) {
        __syncthreads();   // the scales of all rows are in the table
        if (tid < PX) {
            const int mask = s_mask[tid];
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                const int row = halo + tid + (t / 3 - 1) * a.w + (t % 3 - 1);   // in [0, rows)
                s_sx[t * PX + tid] = ((mask >> t) & 1) ? s_rowscale[row] * (1.0f / 256.0f) : 0.f;
            }
        }
    }
    if constexpr (!INT_OUT) {
        if (t_chan < 192) {
            s_sw[t_chan] = t_sw;
            s_bias[t_chan] = t_bias;
        }
    }
    __syncthreads();   // activations and tables visible (also waits for this wave's first weight loads)

    const uint32_t lds_base = lds_address(lds);
    const uint32_t lds_tab = lds_base + a.tab_base;
    const uint32_t a_lane = lrow * 96 + (lhalf ^ ((lrow >> 3) & 1)) * 16;

    v16i acc_start;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_start[r] = INT_OUT ? 0 : kBiasBits;
    asm volatile("" : "+v"(acc_start));   // kept in registers, not rebuilt per unit

    // Steps of the phase about to start whose stages have landed and are visible to every wave (the
    // phase's first loads are always waited for, and a barrier passed, before the phase starts).
    int pre_landed = f_issued;
    int r_stage = 0;           // stage of the unit multiplied next
    auto run_phase = [&](auto PHASE) {
        constexpr int phase = decltype(PHASE)::value;
        constexpr int kl = phase == 0 ? kla : klb, kgn = 1 << kl;
        constexpr bool whole = kgn == 1;   // one wave per tile: no exchange
        const int ulen = ulen_of[phase];
        // this wave in this phase: pixel block ws, channel block cblock, K group kg
        const int cblock = phase == 0 ? (blk & 1) : 2;
        const int kg = phase == 0 ? blk >> 1 : blk;
        const int u0 = unit_first(kg, kl), u1 = unit_first(kg + 1, kl);
        const int cb = co0 + 64 * cblock;                            // first channel of this wave's tile
        const int px = ws * 64;                                      // first pixel (local) of this wave's tile
        const bool exists = cb < a.n && p0 + px < a.pixels;          // else: nothing to multiply or store

        v16i acc[TM][TN];
        float facc[INT_OUT ? 1 : TM][INT_OUT ? 1 : TN][16];
        int my_mask[TN];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) my_mask[tn] = s_mask[px + tn * 32 + lrow];
        if constexpr (!INT_OUT) {
            // fp32 sums start from minus the surplus of the units this wave folds: tap t counts
            // |[u0, u1) intersected with [t S, (t + 1) S)| times
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                float total = 0.f;
#pragma unroll
                for (int t = 0; t < TAPS; ++t) {
                    const int lo = u0 > t * S ? u0 : t * S, hi = u1 < (t + 1) * S ? u1 : (t + 1) * S;
                    const float cnt = hi > lo ? static_cast<float>(hi - lo) : 0.f;
                    total = __builtin_fmaf(cnt, s_sx[t * PX + px + tn * 32 + lrow], total);
                }
                const float f0 = -kBias * total;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int r = 0; r < 16; ++r) facc[tm][tn][r] = f0;
            }
        }

        auto multiply = [&](Ops &o, bool first) {
            v4i a0[TM], a1[TM];
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) { pin(o.a[tm]); expand(o.a[tm], a0[tm], a1[tm]); }
#pragma unroll
            for (int i = 0; i < 2 * TN; ++i) pin(o.b[i]);
            if (first) {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[tm], o.b[2 * tn], acc_start, 0, 0, 0);
            } else {
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
                        acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[tm], o.b[2 * tn], acc[tm][tn], 0, 0, 0);
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[tm], o.b[2 * tn + 1], acc[tm][tn], 0, 0, 0);
        };

        // operand addresses of a unit: weights in the stage, int8 rows of this lane's pixels under the
        // unit's tap in the unit's slice plane
        uint32_t addr_a = 0, addr_b0[TN] = {0, 0}, addr_b1[TN] = {0, 0};
        int r_tap = static_cast<int>(hq::div_magic31(static_cast<uint32_t>(u0), S, a.s_magic, a.s_shift));
        int r_slice = u0 - r_tap * S;
        int r_dpix = (r_tap / 3 - 1) * a.w + (r_tap % 3 - 1);   // pixels from an output pixel to the one under the tap
        auto set_addresses_b = [&]() {
            const int dpix = r_dpix;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                const int row = halo + px + tn * 32 + lrow + dpix;     // in [0, rows)
                const uint32_t rowaddr = lds_base + (r_slice * rows + row) * 192;
                const uint32_t o0 = (lhalf ^ ((row >> 2) & 3)) * 16;
                addr_b0[tn] = rowaddr + o0;
                addr_b1[tn] = rowaddr + (o0 ^ 32);
            }
        };
        auto set_address_a = [&]() {
            addr_a = lds_base + a.stage_base + r_stage * a.stage_bytes + blk * kResBlock + a_lane;
        };
        auto read_a = [&](Ops &o, auto KS) {
            constexpr int ks = decltype(KS)::value;     // K step of 64 codes
            lds_read16<ks * 32>(o.a[0], addr_a);
            lds_read16<32 * 96 + ks * 32>(o.a[1], addr_a);
        };
        auto read_b = [&](Ops &o, auto KS) {
            constexpr int ks = decltype(KS)::value;
            lds_read16<ks * 64>(o.b[0], addr_b0[0]);
            lds_read16<ks * 64>(o.b[2], addr_b0[1]);
            lds_read16<ks * 64>(o.b[1], addr_b1[0]);
            lds_read16<ks * 64>(o.b[3], addr_b1[1]);
        };

        auto fold = [&](int tap, const float (&s)[TN]) {
            if constexpr (INT_OUT) {
                // the exact sums of the unit, added to the zero-filled output
                int *yi = static_cast<int *>(a.y);
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const uint32_t pix = p0 + px + tn * 32 + lrow;
                    if (pix >= a.pixels || !((my_mask[tn] >> tap) & 1)) continue;
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
                        const int cbase = cb + tm * 32 + 16 * lhalf;
                        int *dst = yi + (static_cast<int64_t>(pix) * TAPS + tap) * a.n + cbase;
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (cbase + r < a.n) atomicAdd(dst + r, acc[tm][tn][r] >> 8);
                    }
                }
            } else {
                // in the order in which the tiles' last MFMAs were issued: the first sums are folded while the
                // last MFMAs still execute
#pragma unroll
                for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            facc[tm][tn][r] = __builtin_fmaf(s[tn], __int_as_float(acc[tm][tn][r]), facc[tm][tn][r]);
            }
        };
        auto read_scales = [&](float (&s)[TN], int tap) {
            if constexpr (!INT_OUT) {
                lds_read_f32<0>(s[0], lds_tab + (tap * PX + px + lrow) * 4);
                lds_read_f32<128>(s[1], lds_tab + (tap * PX + px + lrow) * 4);
            }
        };

        // Stores the 32 x 32 sub-tile (tm, tn) of this wave, v = the lane's 16 finished values (channels
        // cb + tm * 32 + 16 * lhalf + r of pixel tn * 32 + lrow).  fp16 results pass through a 2 KiB staging
        // area of the wave in LDS as [pixel][32 channels], so that four neighbouring lanes store the 64
        // contiguous bytes of one pixel (16 requests per store instead of 64 pieces 2 n bytes apart).
        auto store_subtile = [&](int tm, int tn, const float (&v)[16], uint32_t staging) {
          if constexpr (!INT_OUT) {
            Out *y = static_cast<Out *>(a.y);
            const int csub = cb + tm * 32;
            if constexpr (OUT == kOutF16) {
                if ((a.n & 7) == 0 && csub + 32 <= a.n) {
                    v4i r0, r1;
                    transpose_tile_f16(v, staging, lane, r0, r1);
                    const uint32_t pix0 = p0 + px + tn * 32 + (lane >> 2), pix1 = pix0 + 16;
                    __half *dst = reinterpret_cast<__half *>(y) + csub + (lane & 3) * 8;
                    if (pix0 < a.pixels) *reinterpret_cast<v4i *>(dst + static_cast<int64_t>(pix0) * a.n) = r0;
                    if (pix1 < a.pixels) *reinterpret_cast<v4i *>(dst + static_cast<int64_t>(pix1) * a.n) = r1;
                    return;
                }
            }
            const uint32_t pix = p0 + px + tn * 32 + lrow;
            if (pix >= a.pixels) return;
            const int cbase = csub + 16 * lhalf;
            Out *dst = y + static_cast<int64_t>(pix) * a.n + cbase;
            if ((a.n & 15) == 0 && cbase + 16 <= a.n) {
                store16(dst, v);
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (cbase + r < a.n) dst[r] = static_cast<Out>(v[r]);
            }
          }
        };

        // Step i.  The activation operands of a unit's first two K steps do not depend on the weight
        // stream and are requested one step ahead, before the previous unit's sums are folded.  Once the
        // unit's stage has landed everywhere (barrier) its weight operands are requested, a free stage is
        // refilled while they are on their way, the unit is multiplied, the next unit's activation
        // operands are requested and the sums are folded.
        Ops op[2];
        bool next_begun = false;   // whole tiles: the stream has gone on to the second phase's weights
        if (exists && u0 < u1) {
            set_addresses_b();
            read_b(op[0], std::integral_constant<int, 0>{});
            read_b(op[1], std::integral_constant<int, 1>{});
        }
        for (int i = 0; i < ulen; ++i) {
            if (i >= pre_landed) {
                // unit i's loads have landed once at most one younger step's are pending
                if (!next_begun && f_issued - (i + 1) == 1) wait_all_but_one_step();
                else wait_vmem<0>();
            }
            __builtin_amdgcn_s_barrier();   // every wave's share has landed; the stage of unit i - 1 is no longer read
            const bool active = exists && u0 + i < u1;
            const int tap = r_tap;
            float s[TN] = {0.f, 0.f};
            if (active) {
                read_scales(s, tap);
                set_address_a();
                read_a(op[0], std::integral_constant<int, 0>{});
                read_a(op[1], std::integral_constant<int, 1>{});
            }
            // units 0 .. i - 1 are done with their stages: units up to i + NSTAGE - 1 may be on their way
            // (more than one request only right after a phase that began with a single prefetched stage)
            while (f_issued < ulen && f_issued < i + NSTAGE && !next_begun) issue_step();
            if (whole && i + NSTAGE - 1 == ulen) {
                // the stream goes on to the second phase's first unit (one stage only: the others serve as
                // staging for the stores of this phase's results)
                begin_fetch(1, true);
                next_begun = true;
                issue_step();
            }
            const bool next_active = exists && i + 1 < ulen && u0 + i + 1 < u1;
            if (active) {
                wait_lds<2>();   // LDS operations return in order: all but the weights of the second K step are there
                if constexpr (!INT_OUT) asm volatile("" : "+v"(s[0]), "+v"(s[1]));
                multiply(op[0], true);
                read_a(op[0], std::integral_constant<int, 2>{});
                read_b(op[0], std::integral_constant<int, 2>{});
                wait_lds<6>();
                multiply(op[1], false);
                wait_lds<0>();
                multiply(op[0], false);
            }
            if (++r_slice == S) {
                r_slice = 0;
                ++r_tap;
                r_dpix = (r_tap / 3 - 1) * a.w + (r_tap % 3 - 1);
            }
            r_stage = r_stage + 1 == NSTAGE ? 0 : r_stage + 1;
            if (next_active) {
                set_addresses_b();
                read_b(op[0], std::integral_constant<int, 0>{});
                read_b(op[1], std::integral_constant<int, 1>{});
            }
            if (active) fold(tap, s);
        }
        // whole tiles: the second phase's first stages were requested during the last steps; they must have
        // landed before the results are stored (stores would sit between them and a later counted wait)
        if (whole) wait_vmem<0>();
        __builtin_amdgcn_s_barrier();   // every wave has finished reading the last stage (and its loads have landed)
        if (whole) pre_landed = next_begun ? f_issued : 0;

        if constexpr (INT_OUT) {
            if (phase == 0 && !whole) {   // the stream starts again
                begin_fetch(1, false);
                r_stage = 0;
                for (int st = 0; st < NSTAGE - 1 && st < ulen_of[1]; ++st) issue_step();
                wait_vmem<0>();
                __builtin_amdgcn_s_barrier();
                pre_landed = f_issued;
            }
        } else {
            Out *y = static_cast<Out *>(a.y);
            if (whole) {
                // ---- whole tiles: scale and store -----------------------------------------------------
                // (staging: a weight stage that does not hold the second phase's first unit)
                const int free_stage = (r_stage + 1 + (NSTAGE == 3 && wv >= 4 ? 1 : 0)) % NSTAGE;
                const uint32_t staging = lds_base + a.stage_base + free_stage * a.stage_bytes + (wv & 3) * 2048;
                if (exists) {
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
                        const int clocal = 64 * cblock + tm * 32 + 16 * lhalf;
                        float swv[16], bv[16];
#pragma unroll
                        for (int r = 0; r < 16; r += 4) {
                            const float4 s4 = *reinterpret_cast<const float4 *>(s_sw + clocal + r);
                            const float4 b4 = *reinterpret_cast<const float4 *>(s_bias + clocal + r);
                            swv[r] = s4.x; swv[r + 1] = s4.y; swv[r + 2] = s4.z; swv[r + 3] = s4.w;
                            bv[r] = b4.x; bv[r + 1] = b4.y; bv[r + 2] = b4.z; bv[r + 3] = b4.w;
                        }
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn) {
                            float out[16];
#pragma unroll
                            for (int r = 0; r < 16; ++r) out[r] = __builtin_fmaf(facc[tm][tn][r], swv[r], bv[r]);
                            store_subtile(tm, tn, out, staging);
                        }
                    }
                }
            } else {
                // ---- the K groups of a tile exchange their partial sums through LDS ---------------------
                // Chunk c of a wave's 64 x 64 partial result (sub-tile c / 4, registers 4 (c % 4) .. + 3) is
                // finished by the wave of K group c / (16 / kgn).  The first phase uses the (idle) weight stages and
                // what lies between them and the tables, the second phase everything below the tables.
                const uint32_t xbase = phase == 0 ? a.stage_base : 0;
                const uint32_t per_wave = (16 - (16 >> kl)) * 1024;
                const int wstride = phase == 0 ? 2 * pgn : pgn;          // waves of consecutive K groups of a tile
                const int wave0 = wv - kg * wstride;                     // the tile's wave of K group 0
                // (written with hand-placed LDS stores: stores the compiler knows of would first wait for every
                // outstanding memory operation, i.e. for the first phase's results to reach memory)
                const uint32_t mine = lds_base + xbase + wv * per_wave + lane * 16;
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    if (exchange_owner(c, kl) == kg) continue;   // finished here
                    const int tm = c >> 3, tn = (c >> 2) & 1, q4 = c & 3;
                    const v4i bits = {__float_as_int(facc[tm][tn][4 * q4]), __float_as_int(facc[tm][tn][4 * q4 + 1]),
                                      __float_as_int(facc[tm][tn][4 * q4 + 2]), __float_as_int(facc[tm][tn][4 * q4 + 3])};
                    asm volatile("ds_write_b128 %0, %1" : : "v"(mine + exchange_pos(c, kg, kl) * 1024), "v"(bits) : "memory");
                }
                wait_lds<0>();
                __builtin_amdgcn_s_barrier();
                // the chunks this wave finishes: their totals replace its own shares in the registers
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    if (exchange_owner(c, kl) != kg) continue;   // uniform
                    const int tm = c >> 3, tn = (c >> 2) & 1, q4 = c & 3;
                    float4 total = float4{0.f, 0.f, 0.f, 0.f};
                    for (int j = 0; j < kgn; ++j) {   // fixed order: the result does not depend on timing
                        float4 t;
                        if (j == kg) {
                            t = float4{facc[tm][tn][4 * q4], facc[tm][tn][4 * q4 + 1], facc[tm][tn][4 * q4 + 2],
                                       facc[tm][tn][4 * q4 + 3]};
                        } else {
                            const float4 *theirs =
                                reinterpret_cast<const float4 *>(lds + xbase + (wave0 + j * wstride) * per_wave);
                            t = theirs[exchange_pos(c, j, kl) * 64 + lane];
                        }
                        total.x += t.x; total.y += t.y; total.z += t.z; total.w += t.w;
                    }
                    const int clocal = 64 * cblock + tm * 32 + 16 * lhalf + 4 * q4;
                    const float4 s4 = *reinterpret_cast<const float4 *>(s_sw + clocal);
                    const float4 b4 = *reinterpret_cast<const float4 *>(s_bias + clocal);
                    facc[tm][tn][4 * q4] = __builtin_fmaf(total.x, s4.x, b4.x);
                    facc[tm][tn][4 * q4 + 1] = __builtin_fmaf(total.y, s4.y, b4.y);
                    facc[tm][tn][4 * q4 + 2] = __builtin_fmaf(total.z, s4.z, b4.z);
                    facc[tm][tn][4 * q4 + 3] = __builtin_fmaf(total.w, s4.w, b4.w);
                }
                if (phase == 0) {
                    // the stages are free again: the second phase's weights are requested and waited for
                    // before the results are stored
                    __syncthreads();
                    begin_fetch(1, false);
                    r_stage = 0;
                    for (int st = 0; st < NSTAGE - 1 && st < ulen_of[1]; ++st) issue_step();
                }
                if (phase == 0) {
                    wait_vmem<0>();
                    __builtin_amdgcn_s_barrier();
                    pre_landed = f_issued;
                }
                // staging for the stores: phase A - the last weight stage (the second phase's first units sit
                // in the stages before it); phase B - just below the tables, above the exchanged sums
                const uint32_t staging = lds_base + (phase == 0 ? a.stage_base + (NSTAGE - 1) * a.stage_bytes
                                                                : a.tab_base - (2048u << NWL)) + wv * 2048;
                if constexpr (kgn <= 4) {
#pragma unroll
                    for (int sub = 0; sub < 4; ++sub) {
                        if (exchange_owner(4 * sub, kl) != kg) continue;   // uniform
                        if (exists) store_subtile(sub >> 1, sub & 1, facc[sub >> 1][sub & 1], staging);
                    }
                } else {
                    // eight K groups: this wave finishes half a sub-tile, 8 channels of every pixel
#pragma unroll
                    for (int c = 0; c < 16; ++c) {
                        if (exchange_owner(c, kl) != kg) continue;   // uniform
                        const int tm = c >> 3, tn = (c >> 2) & 1, q4 = c & 3;
                        const int cbase = cb + tm * 32 + 16 * lhalf + 4 * q4;
                        const uint32_t pix = p0 + px + tn * 32 + lrow;
                        if (!exists || pix >= a.pixels) continue;
                        const float out[4] = {facc[tm][tn][4 * q4], facc[tm][tn][4 * q4 + 1], facc[tm][tn][4 * q4 + 2],
                                              facc[tm][tn][4 * q4 + 3]};
                        Out *dst = y + static_cast<int64_t>(pix) * a.n + cbase;
                        if ((a.n & 3) == 0 && cbase + 4 <= a.n) {
                            if constexpr (OUT == kOutF16) {
                                __half2 h01 = __floats2half2_rn(out[0], out[1]), h23 = __floats2half2_rn(out[2], out[3]);
                                uint2 w2;
                                w2.x = *reinterpret_cast<uint32_t *>(&h01);
                                w2.y = *reinterpret_cast<uint32_t *>(&h23);
                                *reinterpret_cast<uint2 *>(dst) = w2;
                            } else {
                                *reinterpret_cast<float4 *>(dst) = float4{out[0], out[1], out[2], out[3]};
                            }
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                if (cbase + r < a.n) dst[r] = static_cast<Out>(out[r]);
                        }
                    }
                }
            }
        }
    };
    run_phase(std::integral_constant<int, 0>{});
    run_phase(std::integral_constant<int, 1>{});
}

struct ResPlan {
    int pg_log2, nw_log2;
    uint32_t stage_base, stage_bytes, tab_base;
    int64_t tiles;
};

// LDS layout of a tile of 64 << pg_log2 pixels for a workgroup of 1 << nw_log2 waves, or false if it
// does not fit.
bool res_plan(int64_t pixels, int w, int c_in, int c_out, int pg_log2, int nw_log2, bool fused, ResPlan &p) {
    if (nw_log2 - 1 - pg_log2 < 0) return false;
    const int px = 64 << pg_log2, nw = 1 << nw_log2;
    const int lds = res_lds(nw_log2);
    const int slices = c_in / 192;
    const int64_t rows = px + 2 * (static_cast<int64_t>(w) + 1);
    const int64_t act = rows * slices * 192;
    const int64_t tab = ((9 * px + px + 2 * 192 + (fused ? rows : 0)) * 4 + 15) & ~static_cast<int64_t>(15);
    const int64_t stage = static_cast<int64_t>(nw >> pg_log2) * kResBlock;
    const int64_t nstage = res_stages(pg_log2, nw_log2);
    if (act + nstage * stage + tab > lds) return false;
    // the exchange of phase A (K groups (waves / 2) / pgn > 1) happens between the activations and the tables
    const int kgn_a = (nw / 2) >> pg_log2;
    if (kgn_a > 1 && lds - tab - act < nw * (16 - 16 / kgn_a) * 1024) return false;
    // ... and that of phase B below the tables
    const int kgn_b = nw >> pg_log2;
    if (lds - tab < nw * (16 - 16 / kgn_b) * 1024 + nw * 2048) return false;   // (+ staging of the stores)
    if (stage < 4 * 2048) return false;
    p.pg_log2 = pg_log2;
    p.nw_log2 = nw_log2;
    p.stage_base = static_cast<uint32_t>(act);
    p.stage_bytes = static_cast<uint32_t>(stage);
    p.tab_base = static_cast<uint32_t>(lds - tab);
    p.tiles = ((pixels + px - 1) / px) * ((c_out + 191) / 192);
    return true;
}

// The configuration that minimises rounds x (time of a tile + fixed cost) on `cus` CUs.  Eight waves:
// one tile per CU at a time.  Four waves and 128 pixels: two tiles per CU at a time, each at half
// the rate, but the two workgroups of a CU are not in step with each other (measured faster
// wherever the layer fills the CUs twice over).
bool res_choose(int64_t pixels, int w, int c_in, int c_out, int cus, bool fused, ResPlan &best) {
    if (c_in % 192 != 0 || c_in <= 0 || c_in > 192 * 16) return false;
    bool found = false;
    int64_t best_cost = 0;
    for (int l = 2; l >= 0; --l) {
        ResPlan p;
        if (!res_plan(pixels, w, c_in, c_out, l, 3, fused, p)) continue;
        const int64_t rounds = (p.tiles + cus - 1) / cus;
        const int64_t cost = rounds * ((64 << l) + 48);
        if (!found || cost < best_cost) { best = p; best_cost = cost; found = true; }
    }
    ResPlan p4;
    if (res_plan(pixels, w, c_in, c_out, 1, 2, fused, p4)) {
        const int64_t rounds = (p4.tiles + 2 * cus - 1) / (2 * cus);
        const int64_t cost = rounds * (2 * 128 + 48) * kRes4WaveCost / 100;
        if (!found || cost < best_cost) { best = p4; best_cost = cost; found = true; }
    }
    return found;
}


// Fills the geometry, divisions and LDS layout of a launch.
inline void res_fill_args(ResArgs &a, const GemmArgs &g, const ResPlan &p) {
    a.xq = g.xq; a.sx = g.sx; a.wq = g.wq; a.sw = g.sw; a.bias = g.bias; a.y = g.y;
    a.pixels = g.pixels; a.n = g.n; a.k = g.k; a.h = g.h; a.w = g.w;
    const hq::Magic31 mw = hq::magic31(static_cast<uint32_t>(g.w)), mh = hq::magic31(static_cast<uint32_t>(g.h));
    a.w_magic = mw.m; a.w_shift = mw.s; a.h_magic = mh.m; a.h_shift = mh.s;
    a.slices = g.k / 192;
    const hq::Magic31 ms = hq::magic31(static_cast<uint32_t>(a.slices));
    a.s_magic = ms.m; a.s_shift = ms.s;
    const hq::Magic31 mp = hq::magic31(static_cast<uint32_t>(6 * a.slices));
    a.p_magic = mp.m; a.p_shift = mp.s;
    a.pg_log2 = p.pg_log2;
    a.n_co_tiles = static_cast<uint32_t>((g.n + 191) / 192);
    a.n_tiles = static_cast<uint32_t>(p.tiles);
    a.stage_base = p.stage_base; a.stage_bytes = p.stage_bytes; a.tab_base = p.tab_base;
}

// Launches the configuration of the plan (integer output: the caller has zero-filled it).
template <bool FUSED>
void res_launch_plan(const ResArgs &a, const ResPlan &p, hq_dtype y_dtype, hipStream_t stream) {
    const dim3 grid(a.n_tiles), block(64 << p.nw_log2);
#define HQ_RES_CASE(PGL, NWL)                                                                                      \
    if (y_dtype == HQ_I32) hipLaunchKernelGGL((conv3x3_res_kernel<kOutI32, PGL, NWL, FUSED>), grid, block, 0, stream, a);      \
    else if (y_dtype == HQ_F16) hipLaunchKernelGGL((conv3x3_res_kernel<kOutF16, PGL, NWL, FUSED>), grid, block, 0, stream, a); \
    else hipLaunchKernelGGL((conv3x3_res_kernel<kOutF32, PGL, NWL, FUSED>), grid, block, 0, stream, a);
    if (p.nw_log2 == 2) { HQ_RES_CASE(1, 2) }
    else if (p.pg_log2 == 2) { HQ_RES_CASE(2, 3) }
    else if (p.pg_log2 == 1) { HQ_RES_CASE(1, 3) }
    else { HQ_RES_CASE(0, 3) }
#undef HQ_RES_CASE
}

}  // namespace
