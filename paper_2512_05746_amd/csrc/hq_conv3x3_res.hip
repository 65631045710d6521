// 3x3 / stride 1 / pad 1 NHWC convolution with per-pixel activation scales on int8 MFMA, one
// workgroup of eight waves per CU, the activation tile expanded to int8 ONCE and resident in LDS
// (Method, "Convolution": one integer sum per tap, taps combined in fp32 with the scale of the
// input pixel under the tap).
//
// Why another kernel.  Three things held the other 3x3 kernels below a third of the int8 rate on
// the UNet's layers: (1) tile counts that do not divide the machine (768 tiles for 512 resident
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
//     so every wave multiplies 1.5 / 0.75 / 0.375 tiles' worth of units, all waves the same amount;
//   - the activation rows of the tile's pixels plus W + 1 pixels either side are fetched once (all
//     input channels), expanded to int8 (16 x code) on the way into LDS, and all nine taps of all
//     phases read them at shifted addresses: an activation operand is an LDS read, nothing else;
//   - only the weights stream (direct-to-LDS loads, packed, two or three stages of one unit per K
//     group), 64..128 bytes per MFMA; a wave expands the weight nibbles it reads (three vector
//     instructions per MFMA in the 2 x 2 register tile).
// The sums of one unit are folded into the fp32 result with one fma per element: the integer
// accumulators start from the bit pattern of 1.5 * 2^23, so their bits read as a float are
// 1.5 * 2^23 + S exactly (S = 256 * sum, |S| < 2^22 for 192 codes), and the fp32 sums start from
// minus the known surplus.
//
// Integer output (HQ_I32): the same loads, stages, phases and MFMAs; instead of the fold every
// wave adds the exact sums of its units to the zero-filled [pixel, tap, n] output with integer
// atomics (integer addition is exact in any order).
#include "hq_int_gemm_kernel.h"

namespace {

constexpr int kResLds = 163840;      // all of a CU's LDS: one workgroup per CU
constexpr int kResBlock = 64 * 96;   // weight rows of one 64-channel block of one unit (packed)

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
    int nstage;          // weight stages (2 or 3)
    uint32_t stage_base, stage_bytes, tab_base;    // LDS layout: activations at 0, then stages, then tables
    int continuous;      // the weight stream runs on from phase A into phase B (phase A needs no exchange)
};

// chunk c (0..15) of a wave's 64 x 64 partial result = sub-tile c / 4 (tm * 2 + tn), registers 4 (c % 4) .. + 3;
// among the KG waves that share a tile, wave c % KG finishes chunk c.  A wave stores the chunks it
// does not finish compactly: chunk c of wave kg sits at position c - (chunks below c that kg finishes).
__device__ __forceinline__ int exchange_pos(int c, int kg, int kgn_log2) {
    return c - ((c + (1 << kgn_log2) - 1 - kg) >> kgn_log2);
}

template <int OUT>
__global__ __launch_bounds__(512) void conv3x3_res_kernel(ResArgs a) {
    constexpr bool INT_OUT = OUT == kOutI32;
    constexpr int TM = 2, TN = 2, TAPS = 9, NWAVE = 8, MAXL = 6;
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
    const int pgn_log2 = a.pg_log2, pgn = 1 << pgn_log2, PX = 64 << pgn_log2;
    const int halo = a.w + 1;
    const int rows = PX + 2 * halo;
    const uint32_t last = a.pixels - 1;
    const int nb_log2 = 3 - pgn_log2;                   // blocks of 64 weight rows per stage: 8 / pgn
    const int nloads = 6 << nb_log2;                    // 1 KiB loads per stage

    // tables (at the top of the LDS): scale of the input pixel under tap t for every pixel of the tile,
    // tap masks, scales and bias of the tile's 192 channels
    float *s_sx = reinterpret_cast<float *>(lds + a.tab_base);            // [9][PX], x_scale / 256, 0 outside
    int *s_mask = reinterpret_cast<int *>(s_sx + TAPS * PX);              // [PX]
    float *s_sw = reinterpret_cast<float *>(s_mask + PX);                 // [192]
    float *s_bias = s_sw + 192;                                           // [192]

    // ---- tile of this workgroup (XCD-contiguous: workgroup b runs on XCD b % 8) ------------------
    uint32_t tile = blockIdx.x;
    if (gridDim.x % 8 == 0) tile = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
    const int co0 = static_cast<int>(tile % a.n_co_tiles) * 192;
    const uint32_t p0 = (tile / a.n_co_tiles) * PX;

    // ---- phases ------------------------------------------------------------------------------------
    // phase 0: channel blocks 0, 1; K groups 4 / pgn.  phase 1: channel block 2; K groups 8 / pgn.
    const int kgn_log2_of[2] = {2 - pgn_log2, 3 - pgn_log2};
    const int ulen_of[2] = {(NU + (1 << kgn_log2_of[0]) - 1) >> kgn_log2_of[0],
                            (NU + (1 << kgn_log2_of[1]) - 1) >> kgn_log2_of[1]};
    const int total_steps = ulen_of[0] + ulen_of[1];
    auto unit_first = [&](int kg, int kgn_log2) { return (kg * NU) >> kgn_log2; };

    // ---- weight stream: this wave's loads L = wv + 8 j < nloads of every stage ----------------------
    // load L fills LDS bytes [L * 1024, + 1024) of the stage: block L / 6 (K group major, then channel
    // block), 16-byte slots q = 64 (L % 6) + lane of the block's row-major [64 rows][6 pieces] image,
    // adjacent pieces swapped in rows 8..15 (mod 16) against bank conflicts of the operand reads.
    uint32_t ld_off[MAXL];     // per lane: byte offset of the piece inside the weight tensor at tap 0, slice 0
    int fetch_phase = -1;
    auto setup_fetch = [&](int phase) {
        fetch_phase = phase;
#pragma unroll
        for (int j = 0; j < MAXL; ++j) {
            const int L = wv + NWAVE * j;
            const int b = L / 6, r = L - 6 * b;
            const int q = 64 * r + lane, row = q / 6, piece = (q - 6 * row) ^ ((row >> 3) & 1);
            const int cblock = phase == 0 ? (b & 1) : 2;
            int co = co0 + 64 * cblock + (row & ~31) + tile_row_to_channel(row & 31);
            co = co < a.n ? co : a.n - 1;
            ld_off[j] = static_cast<uint32_t>(co) * TAPS * kbytes + piece * 16;
        }
    };
    int issued = 0;            // steps of the stream requested so far
    int issue_stage = 0;
    auto issue_step = [&]() {
        const int phase = issued >= ulen_of[0] ? 1 : 0;
        const int i = issued - (phase ? ulen_of[0] : 0);
        if (fetch_phase != phase) setup_fetch(phase);
        const int kl = kgn_log2_of[phase];
        uint8_t *image = lds + a.stage_base + issue_stage * a.stage_bytes;
#pragma unroll
        for (int j = 0; j < MAXL; ++j) {
            const int L = wv + NWAVE * j;
            if (L < nloads) {
                const int b = L / 6;
                const int kg = phase == 0 ? b >> 1 : b;
                int u = unit_first(kg, kl) + i;
                const int u_end = unit_first(kg + 1, kl);
                u = u < u_end ? u : u_end - 1;     // a K group that has run out repeats its last unit (not used)
                u = u < 0 ? 0 : u;
                const uint32_t tap = hq::div_magic31(static_cast<uint32_t>(u), S, a.s_magic, a.s_shift);
                const uint32_t slice = u - tap * S;
                load_to_lds16(a.wq + (tap * kbytes + slice * 96) + ld_off[j], image + L * 1024);
            }
        }
        ++issued;
        issue_stage = issue_stage + 1 == a.nstage ? 0 : issue_stage + 1;
    };
    const int my_loads = (nloads - wv + NWAVE - 1) / NWAVE;   // loads per step of this wave
    // waits until this wave's loads of the step being consumed have landed: at most `later` younger
    // steps' loads may still be pending
    auto wait_step = [&](int later) {
        const int pending = later * my_loads;
        if (pending >= 12) wait_vmem<12>();
        else if (pending >= 6) wait_vmem<6>();
        else if (pending >= 4) wait_vmem<4>();
        else if (pending >= 3) wait_vmem<3>();
        else if (pending >= 2) wait_vmem<2>();
        else if (pending >= 1) wait_vmem<1>();
        else wait_vmem<0>();
    };
    const int stream_end = a.continuous ? total_steps : ulen_of[0];
    for (int st = 0; st < a.nstage - 1 && issued < stream_end; ++st) issue_step();

    // ---- activation tile: packed rows -> int8 (16 x code) in LDS -------------------------------------
    // Row r of the image is pixel p0 - halo + r (clamped into the tensor; rows outside the image are
    // only ever read under taps whose scale is 0).  Plane s (192-channel slice) at s * rows * 192; a row
    // is three 64-byte K steps of four 16-byte pieces [MFMA 0 / lane half 0, 0 / 1, 1 / 0, 1 / 1], the
    // piece index xor-ed with (row / 4) % 4 so that the operand reads of 16 consecutive rows hit 16
    // different bank groups (row stride 192 bytes = 12 groups).
    {
        const uint32_t pieces_per_row = 6u * S;
        const uint32_t total = static_cast<uint32_t>(rows) * pieces_per_row;
        const int64_t first = static_cast<int64_t>(p0) - halo;
        for (uint32_t base = tid; base < total; base += 512 * 4) {
            v4i p[4];
            uint32_t dst[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t q = base + 512 * e;
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
            for (int e = 0; e < 4; ++e) {
                const uint32_t q = base + 512 * e;
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
        const uint32_t pix = p0 + tid;
        const uint32_t q = hq::div_magic31(pix, a.w, a.w_magic, a.w_shift);
        const int ow = static_cast<int>(pix - q * a.w);
        const int oh = static_cast<int>(q - hq::div_magic31(q, a.h, a.h_magic, a.h_shift) * a.h);
        const int cm = (ow > 0 ? 1 : 0) | 2 | (ow + 1 < a.w ? 4 : 0);
        int mask = (oh > 0 ? cm : 0) | (cm << 3) | (oh + 1 < a.h ? cm << 6 : 0);
        if (pix >= a.pixels) mask = 0;
        s_mask[tid] = mask;
        if constexpr (!INT_OUT) {
            float v[TAPS];
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                uint32_t ip = pix + static_cast<uint32_t>((t / 3 - 1) * a.w + (t % 3 - 1));   // wraps below 0
                ip = ip < last ? ip : last;
                v[t] = a.sx[ip];
            }
#pragma unroll
            for (int t = 0; t < TAPS; ++t) s_sx[t * PX + tid] = ((mask >> t) & 1) ? v[t] * (1.0f / 256.0f) : 0.f;
        }
    }
    if constexpr (!INT_OUT) {
        if (tid >= 256 && tid < 256 + 192) {
            const int c = tid - 256;
            const bool ok = co0 + c < a.n;
            const Out *bias = static_cast<const Out *>(a.bias);
            s_sw[c] = ok ? a.sw[co0 + c] : 0.f;
            s_bias[c] = ok && bias ? to_float(bias[co0 + c]) : 0.f;
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

    int g = 0;           // step of the stream being consumed
    int stage = 0;
    for (int phase = 0; phase < 2; ++phase) {
        const int kl = kgn_log2_of[phase], kgn = 1 << kl, ulen = ulen_of[phase];
        // this wave in this phase: pixel block pg, channel block cg (of the phase), K group kg
        const int pg = wv & (pgn - 1);
        const int cg = phase == 0 ? (wv >> pgn_log2) & 1 : 0;
        const int kg = phase == 0 ? wv >> (pgn_log2 + 1) : wv >> pgn_log2;
        const int cblock = phase == 0 ? cg : 2;
        const int u0 = unit_first(kg, kl), u1 = unit_first(kg + 1, kl);
        const int block = phase == 0 ? 2 * kg + cg : kg;             // of the stage
        const int cb = co0 + 64 * cblock;                            // first channel of this wave's tile
        const int px = pg * 64;                                      // first pixel (local) of this wave's tile
        const bool exists = cb < a.n && p0 + px < a.pixels;          // else: nothing to multiply or store

        if (phase == 1 && !a.continuous) {   // the stream was drained for the exchange: start it again
            for (int st = 0; st < a.nstage - 1 && issued < total_steps; ++st) issue_step();
        }

        v16i acc[TM][TN];
        float facc[INT_OUT ? 1 : TM][INT_OUT ? 1 : TN][16];
        int my_mask[TN];
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) my_mask[tn] = s_mask[px + tn * 32 + lrow];
        if constexpr (!INT_OUT) {
            // fp32 sums start from minus the surplus of the units this wave folds
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                float total = 0.f;
                for (int u = u0; u < u1; ++u) {
                    const uint32_t tap = hq::div_magic31(static_cast<uint32_t>(u), S, a.s_magic, a.s_shift);
                    total += s_sx[tap * PX + px + tn * 32 + lrow];
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

        for (int i = 0; i < ulen; ++i, ++g) {
            // the stage of this step has landed once only younger steps' loads are pending
            if (i == 0) {
                wait_vmem<0>();     // also the stores and table loads issued before the phase
            } else {
                const int younger = issued - g - 1;
                wait_step(younger < a.nstage - 2 ? younger : a.nstage - 2);
            }
            __builtin_amdgcn_s_barrier();   // every wave's share has landed; the previous stage is free
            {
                const int limit = (phase == 0 && !a.continuous) ? ulen_of[0] : total_steps;
                if (issued < limit) issue_step();
            }

            const int u = u0 + i;
            if (exists && u < u1) {
                const uint32_t tap = hq::div_magic31(static_cast<uint32_t>(u), S, a.s_magic, a.s_shift);
                const int slice = u - static_cast<int>(tap) * S;
                const int dpix = (static_cast<int>(tap) / 3 - 1) * a.w + (static_cast<int>(tap) % 3 - 1);
                // B: int8 rows of this lane's pixels under the tap
                uint32_t addr_b0[TN], addr_b1[TN];
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const int row = halo + px + tn * 32 + lrow + dpix;     // in [0, rows)
                    const uint32_t rowaddr = lds_base + (slice * rows + row) * 192;
                    const uint32_t o0 = (lhalf ^ ((row >> 2) & 3)) * 16;
                    addr_b0[tn] = rowaddr + o0;
                    addr_b1[tn] = rowaddr + (o0 ^ 32);
                }
                const uint32_t addr_a = lds_base + a.stage_base + stage * a.stage_bytes + block * kResBlock + a_lane;
                auto read_step = [&](Ops &o, auto KS) {
                    constexpr int ks = decltype(KS)::value;     // K step of 64 codes
                    lds_read16<ks * 32>(o.a[0], addr_a);
                    lds_read16<32 * 96 + ks * 32>(o.a[1], addr_a);
                    lds_read16<ks * 64>(o.b[0], addr_b0[0]);
                    lds_read16<ks * 64>(o.b[2], addr_b0[1]);
                    lds_read16<ks * 64>(o.b[1], addr_b1[0]);
                    lds_read16<ks * 64>(o.b[3], addr_b1[1]);
                };
                Ops op[2];
                read_step(op[0], std::integral_constant<int, 0>{});
                read_step(op[1], std::integral_constant<int, 1>{});
                wait_lds<6>();
                multiply(op[0], true);
                read_step(op[0], std::integral_constant<int, 2>{});
                wait_lds<6>();
                multiply(op[1], false);
                wait_lds<0>();
                multiply(op[0], false);

                if constexpr (INT_OUT) {
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
                    float s[TN];
                    read_tap_scales<TN>(s, lds_tab + (tap * PX + px + lrow) * 4);
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                facc[tm][tn][r] = __builtin_fmaf(s[tn], __int_as_float(acc[tm][tn][r]), facc[tm][tn][r]);
                }
            }
            stage = stage + 1 == a.nstage ? 0 : stage + 1;
        }

        if constexpr (!INT_OUT) {
            Out *y = static_cast<Out *>(a.y);
            const bool vec_ok = (a.n & 15) == 0;
            if (kgn == 1) {
                // ---- whole tiles: scale and store -----------------------------------------------------
                if (exists) {
#pragma unroll
                    for (int tm = 0; tm < TM; ++tm) {
                        const int clocal = 64 * cblock + tm * 32 + 16 * lhalf;
                        const int cbase = co0 + clocal;
                        float swv[16], bv[16];
#pragma unroll
                        for (int r = 0; r < 16; ++r) { swv[r] = s_sw[clocal + r]; bv[r] = s_bias[clocal + r]; }
#pragma unroll
                        for (int tn = 0; tn < TN; ++tn) {
                            const uint32_t pix = p0 + px + tn * 32 + lrow;
                            if (pix >= a.pixels) continue;
                            float out[16];
#pragma unroll
                            for (int r = 0; r < 16; ++r) out[r] = __builtin_fmaf(facc[tm][tn][r], swv[r], bv[r]);
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
            } else {
                // ---- the K groups of a tile exchange their partial sums through LDS ---------------------
                // Phase A uses the (drained) weight stages, phase B everything below the tables.
                __syncthreads();   // every wave is done with the stages (and, in phase B, the activations)
                const uint32_t xbase = phase == 0 ? a.stage_base : 0;
                const uint32_t per_wave = (16 - (16 >> kl)) * 1024;
                float4 *mine = reinterpret_cast<float4 *>(lds + xbase + wv * per_wave);
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    if ((c & (kgn - 1)) == kg) continue;   // finished here
                    const int tm = c >> 3, tn = (c >> 2) & 1, q4 = c & 3;
                    mine[exchange_pos(c, kg, kl) * 64 + lane] =
                        float4{facc[tm][tn][4 * q4], facc[tm][tn][4 * q4 + 1], facc[tm][tn][4 * q4 + 2],
                               facc[tm][tn][4 * q4 + 3]};
                }
                __syncthreads();
                const int wave0 = wv - kg * (phase == 0 ? 2 * pgn : pgn);   // the tile's wave of K group 0
                const int wstride = phase == 0 ? 2 * pgn : pgn;
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    if ((c & (kgn - 1)) != kg) continue;
                    const int tm = c >> 3, tn = (c >> 2) & 1, q4 = c & 3;
                    float v[4] = {0.f, 0.f, 0.f, 0.f};
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
                        v[0] += t.x; v[1] += t.y; v[2] += t.z; v[3] += t.w;
                    }
                    const int clocal = 64 * cblock + tm * 32 + 16 * lhalf + 4 * q4;
                    const int cbase = co0 + clocal;
                    const uint32_t pix = p0 + px + tn * 32 + lrow;
                    if (!exists || pix >= a.pixels) continue;
                    float out[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) out[r] = __builtin_fmaf(v[r], s_sw[clocal + r], s_bias[clocal + r]);
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
                if (phase == 0) __syncthreads();   // the stages are free for phase B's weights
            }
        }
    }
}

struct ResPlan {
    int pg_log2, nstage;
    uint32_t stage_base, stage_bytes, tab_base;
    int64_t tiles;
};

// LDS layout of pixel-tile size 64 << pg_log2, or false if it does not fit.
bool res_plan(int64_t pixels, int w, int c_in, int c_out, int pg_log2, ResPlan &p) {
    const int px = 64 << pg_log2;
    const int slices = c_in / 192;
    const int64_t rows = px + 2 * (static_cast<int64_t>(w) + 1);
    const int64_t act = rows * slices * 192;
    const int64_t tab = (9 * px + px + 2 * 192) * 4;
    const int64_t stage = static_cast<int64_t>(8 >> pg_log2) * kResBlock;
    int64_t nstage = (kResLds - tab - act) / stage;
    if (nstage < 2) return false;
    if (nstage > 3) nstage = 3;
    // the exchange of phase A (K groups 4 / pgn > 1) happens inside the stages
    const int kgn_a = 4 >> pg_log2;
    if (kgn_a > 1 && nstage * stage < 8 * (16 - 16 / kgn_a) * 1024) return false;
    // ... and that of phase B below the tables
    const int kgn_b = 8 >> pg_log2;
    if (act + nstage * stage < 8 * (16 - 16 / kgn_b) * 1024) return false;
    p.pg_log2 = pg_log2;
    p.nstage = static_cast<int>(nstage);
    p.stage_base = static_cast<uint32_t>(act);
    p.stage_bytes = static_cast<uint32_t>(stage);
    p.tab_base = static_cast<uint32_t>(act + nstage * stage);
    p.tiles = ((pixels + px - 1) / px) * ((c_out + 191) / 192);
    return true;
}

// The pixel-tile size that minimises rounds x (tile size + fixed cost) on `cus` CUs.
bool res_choose(int64_t pixels, int w, int c_in, int c_out, int cus, ResPlan &best) {
    if (c_in % 192 != 0 || c_in <= 0 || c_in > 192 * 16) return false;
    bool found = false;
    int64_t best_cost = 0;
    for (int l = 2; l >= 0; --l) {
        ResPlan p;
        if (!res_plan(pixels, w, c_in, c_out, l, p)) continue;
        const int64_t rounds = (p.tiles + cus - 1) / cus;
        const int64_t cost = rounds * ((64 << l) + 48);
        if (!found || cost < best_cost) { best = p; best_cost = cost; found = true; }
    }
    return found;
}

}  // namespace

// True if the layer is one for this kernel: per-pixel scales, channel slices of 192, a pixel tile
// whose activations fit the LDS, and enough tiles to occupy at least half of the CUs.
bool hq_conv3x3_res_fits(int64_t pixels, int w, int c_in, int c_out) {
    ResPlan p;
    const int cus = hq::compute_units();
    return res_choose(pixels, w, c_in, c_out, cus, p) && 2 * p.tiles >= cus;
}

// Pixels per workgroup tile (256, 128 or 64) the kernel takes for this layer; 0 if it does not serve it.
int hq_conv3x3_res_tile_pixels(int64_t pixels, int w, int c_in, int c_out) {
    ResPlan p;
    const int cus = hq::compute_units();
    if (!res_choose(pixels, w, c_in, c_out, cus, p) || 2 * p.tiles < cus) return 0;
    return 64 << p.pg_log2;
}

hq_status hq_conv3x3_res_launch(const GemmArgs &g, hq_dtype y_dtype, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    ResPlan p;
    if (g.sx_static || !res_choose(g.pixels, g.w, g.k, g.n, hq::compute_units(), p)) return HQ_ERR_UNSUPPORTED;
    if (p.tiles > 0x7fffffffLL) return HQ_ERR_SHAPE;
    ResArgs a{};
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
    a.nstage = p.nstage;
    a.stage_base = p.stage_base; a.stage_bytes = p.stage_bytes; a.tab_base = p.tab_base;
    a.continuous = (4 >> p.pg_log2) == 1 ? 1 : 0;
    const dim3 grid(a.n_tiles), block(512);
    if (y_dtype == HQ_I32) {
        const hq_status st = hq_fill_zero_launch(g.y, static_cast<uint64_t>(g.pixels) * 9 * g.n, stream);
        if (st != HQ_OK) return st;
        hipLaunchKernelGGL((conv3x3_res_kernel<kOutI32>), grid, block, 0, stream, a);
    } else if (y_dtype == HQ_F16) {
        hipLaunchKernelGGL((conv3x3_res_kernel<kOutF16>), grid, block, 0, stream, a);
    } else if (y_dtype == HQ_F32) {
        hipLaunchKernelGGL((conv3x3_res_kernel<kOutF32>), grid, block, 0, stream, a);
    } else {
        return HQ_ERR_DTYPE;
    }
    return check.status();
}
