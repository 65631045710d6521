// 3x3 / stride 1 / pad 1 NHWC convolution for layers with few pixels and many channels, with the K
// range of an output tile split ACROSS workgroups (Method, "Convolution": one integer sum per tap,
// taps combined in fp32 with the scale of the input pixel under the tap).
//
// Why.  A 16 x 16 or 8 x 8 feature map at batch 16 has 4096 or 1024 pixels: tiles small enough to
// occupy 256 CUs (64 x 64) need 512 operand bytes per MFMA, three times what the direct-to-LDS path
// delivers, and a K range split over the waves of ONE workgroup shares no operands.  Here a
// workgroup of four waves owns a 128-channel x 128-pixel tile (four 64 x 64 wave tiles that share
// both operands: 256 bytes per MFMA) and ONE contiguous share of the tile's 9 x C_in/192 chunks; the
// shares of a tile run on different CUs.  Every workgroup writes its partial fp32 sums (per-tap
// integer sums already folded with the scales of the input pixels, so they simply add) to its plane
// of a caller-supplied workspace [splits][pixels][n]; a second launch adds the planes in a fixed
// order, applies the channel scale and the bias and writes the result.  No atomics, no
// allocation: the workspace is the caller's.
//
// Chunks stream through three LDS stages (24 KiB each: 128 weight rows and 128 activation rows of
// 96 packed bytes) filled by direct-to-LDS loads, one barrier per chunk; rows that do not exist
// (channels >= n, pixels outside the tensor) are clamped to an in-bounds row, never stored, and
// taps outside the image carry scale 0.
//
// Integer output (HQ_I32): the same tiles, shares and loop; every workgroup adds the exact sums of
// its share of a tap to the zero-filled output with integer atomics (exact in any order).
#include "hq_int_gemm_kernel.h"

namespace {

struct SplitArgs {
    const uint8_t *xq;   // [pixels, k/2]
    const float *sx;     // [pixels], or one value for the whole tensor (sx_static)
    const uint8_t *wq;   // [n, 9, k/2]
    float *partial;      // workspace [splits, pixels, n] fp32 (floating-point outputs)
    int *yi;             // integer output [pixels, 9, n] or [pixels, n] (one scale), zero-filled
    uint32_t pixels;
    int n, k, h, w;
    uint32_t w_magic, w_shift, h_magic, h_shift;   // exact division of a pixel index by w and by h
    uint32_t n_px_tiles, n_tiles;
    int splits;
    int sx_static;
};

template <bool INT_OUT>
__global__ __launch_bounds__(256, 2) void conv3x3_split_kernel(SplitArgs a) {
    constexpr int TM = 2, TN = 2, KCH = 6, ROWB = KCH * 16, KS = KCH / 2, TAPS = 9, NSTAGE = 3;
    constexpr int BCO = 128, BP = 128;
    constexpr int STAGE_BYTES = (BCO + BP) * ROWB;   // 24 KiB: twelve 1 KiB loads per operand
    constexpr int LPW = 6;                            // loads per chunk of one wave (three per operand)
    using Ops = Packed<TM, TN>;

    __shared__ __attribute__((aligned(16))) uint8_t lds[NSTAGE * STAGE_BYTES];
    __shared__ float s_sx[TAPS][BP];   // x_scale / 256 of the input pixel under tap t, 0 outside the image
    __shared__ int s_mask[BP];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;     // channel half, pixel half of the tile
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int kbytes = a.k >> 1;
    const int cpt = kbytes / ROWB;               // chunks per tap (host guarantees divisibility)
    const int chunks = TAPS * cpt;
    const uint32_t last = a.pixels - 1;

    // ---- this workgroup's unit: tile and share of its chunks (XCD-contiguous, channel-tile major) ---
    uint32_t unit = blockIdx.x;
    if (gridDim.x % 8 == 0) unit = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
    const uint32_t tile = unit / a.splits;
    const int sp = static_cast<int>(unit - tile * a.splits);
    const int c0 = (sp * chunks) / a.splits, c1 = ((sp + 1) * chunks) / a.splits;
    const int co0 = static_cast<int>(tile / a.n_px_tiles) * BCO;
    const uint32_t p0 = (tile % a.n_px_tiles) * BP;

    // ---- tables: tap masks and scales of the tile's pixels -----------------------------------------
    if (tid < BP) {
        const uint32_t pix = p0 + tid;
        const uint32_t q = hq::div_magic31(pix, a.w, a.w_magic, a.w_shift);
        const int ow = static_cast<int>(pix - q * a.w);
        const int oh = static_cast<int>(q - hq::div_magic31(q, a.h, a.h_magic, a.h_shift) * a.h);
        const int cm = (ow > 0 ? 1 : 0) | 2 | (ow + 1 < a.w ? 4 : 0);
        int mask = (oh > 0 ? cm : 0) | (cm << 3) | (oh + 1 < a.h ? cm << 6 : 0);
        if (pix >= a.pixels) mask = 0;
        s_mask[tid] = mask;
        if constexpr (!INT_OUT) {
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                uint32_t ip = pix + static_cast<uint32_t>((t / 3 - 1) * a.w + (t % 3 - 1));   // wraps below 0
                ip = ip < last ? ip : last;
                const float v = a.sx[a.sx_static ? 0 : ip];
                s_sx[t][tid] = ((mask >> t) & 1) ? v * (1.0f / 256.0f) : 0.f;
            }
        }
    }

    // ---- this wave's loads: i = wave, wave + 4, wave + 8 of the twelve of each operand ------------------
    // load i covers the 16-byte slots q = 64 i + lane of a row-major [128 rows][6 pieces] image
    // (row q / 6, piece q % 6, adjacent pieces swapped in rows 8..15 mod 16 against bank conflicts)
    uint32_t off_a[3];       // weight rows: byte offset at tap 0, chunk 0
    uint32_t row_b[3], piece_b[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        const int q = 64 * (wave + 4 * j) + lane, row = q / KCH, piece = (q - KCH * row) ^ ((row >> 3) & 1);
        int co = co0 + (row & ~31) + tile_row_to_channel(row & 31);
        co = co < a.n ? co : a.n - 1;
        off_a[j] = static_cast<uint32_t>(co) * TAPS * kbytes + piece * 16;
        row_b[j] = p0 + row;
        piece_b[j] = piece * 16;
    }
    int ftap = c0 / cpt, fch = c0 - ftap * cpt;   // chunk being fetched
    auto issue_loads = [&](int stage) {
        const uint32_t dpix = static_cast<uint32_t>((ftap / 3 - 1) * a.w + (ftap % 3 - 1));
        uint8_t *image = lds + stage * STAGE_BYTES;
        const uint8_t *base_a = a.wq + (static_cast<uint32_t>(ftap) * kbytes + fch * ROWB);
        const uint8_t *base_b = a.xq + fch * ROWB;
#pragma unroll
        for (int j = 0; j < 3; ++j) load_to_lds16(base_a + off_a[j], image + (wave + 4 * j) * 1024);
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            uint32_t pix = row_b[j] + dpix;   // wraps below pixel 0
            pix = pix < last ? pix : last;
            load_to_lds16(base_b + (pix * kbytes + piece_b[j]), image + BCO * ROWB + (wave + 4 * j) * 1024);
        }
        if (++fch == cpt) { fch = 0; ++ftap; }
    };
#pragma unroll
    for (int st = 0; st < NSTAGE - 1; ++st)
        if (c0 + st < c1) issue_loads(st);
    __syncthreads();   // tables visible (the compiler also waits for the first loads here)

    const uint32_t lds_row = lds_address(lds) + lrow * ROWB + (lhalf ^ ((lrow >> 3) & 1)) * 16;
    const uint32_t lds_a = lds_row + wm * 64 * ROWB;
    const uint32_t lds_b = lds_row + (BCO + wn * 64) * ROWB;
    const uint32_t lds_sx = lds_address(&s_sx[0][0]) + (wn * 64 + lrow) * 4;
    const bool exists = co0 + wm * 64 < a.n && p0 + wn * 64 < a.pixels;

    float facc[INT_OUT ? 1 : TM][INT_OUT ? 1 : TN][16];
    if constexpr (!INT_OUT) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) facc[tm][tn][r] = 0.f;
    }
    int my_mask[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) my_mask[tn] = s_mask[wn * 64 + tn * 32 + lrow];

    v16i acc[TM][TN];
    auto multiply = [&](Ops &o, bool first) {
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

    int tap = c0 / cpt, ch = c0 - tap * cpt;
    int stage = 0;
    for (int c = c0; c < c1; ++c) {
        // chunk c has landed once only the loads of the chunk after it are pending
        if (c + 1 < c1) wait_vmem<LPW>();
        else wait_vmem<0>();
        __builtin_amdgcn_s_barrier();   // every wave's share has landed; the stage of chunk c - 1 is free
        if (c + NSTAGE - 1 < c1) issue_loads(stage == 0 ? NSTAGE - 1 : stage - 1);

        if (exists) {
            const uint32_t sa = lds_a + stage * STAGE_BYTES, sb = lds_b + stage * STAGE_BYTES;
            Ops op[2];
            read_packed<TM, TN, ROWB, 0>(op[0], sa, sb);
            chunk_steps<0, KS, TM, TN, ROWB>(op, sa, sb, ch == 0 || c == c0, multiply);

            const bool tap_ends = ch + 1 == cpt;
            if (tap_ends || c + 1 == c1) {
                if constexpr (INT_OUT) {
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const uint32_t pix = p0 + wn * 64 + tn * 32 + lrow;
                        if (pix >= a.pixels || !((my_mask[tn] >> tap) & 1)) continue;
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm) {
                            const int cbase = co0 + wm * 64 + tm * 32 + 16 * lhalf;
                            int *dst = a.yi + (a.sx_static ? static_cast<int64_t>(pix)
                                                           : static_cast<int64_t>(pix) * TAPS + tap) * a.n + cbase;
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (cbase + r < a.n) atomicAdd(dst + r, acc[tm][tn][r] >> 8);
                        }
                    }
                } else {
                    float s[TN];
                    read_tap_scales<TN>(s, lds_sx + tap * (BP * 4));
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                facc[tm][tn][r] += s[tn] * static_cast<float>(acc[tm][tn][r]);
                }
            }
        }
        if (ch + 1 == cpt) { ch = 0; ++tap; } else { ++ch; }
        stage = stage + 1 == NSTAGE ? 0 : stage + 1;
    }

    // ---- this share's partial sums to its plane of the workspace ---------------------------------------
    if constexpr (!INT_OUT) {
        if (!exists) return;
        float *plane = a.partial + static_cast<uint64_t>(sp) * a.pixels * a.n;
        const bool vec_ok = (a.n & 3) == 0;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const uint32_t pix = p0 + wn * 64 + tn * 32 + lrow;
            if (pix >= a.pixels) continue;
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int cbase = co0 + wm * 64 + tm * 32 + 16 * lhalf;
                float *dst = plane + static_cast<uint64_t>(pix) * a.n + cbase;
                if (vec_ok && cbase + 16 <= a.n) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        reinterpret_cast<float4 *>(dst)[i] = float4{facc[tm][tn][4 * i], facc[tm][tn][4 * i + 1],
                                                                    facc[tm][tn][4 * i + 2], facc[tm][tn][4 * i + 3]};
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (cbase + r < a.n) dst[r] = facc[tm][tn][r];
                }
            }
        }
    }
}

// y[p, c] = (sum over the planes, in order, of partial[s][p][c]) * w_scale[c] + bias[c]; four channels per thread
template <int OUT>
__global__ __launch_bounds__(256) void split_reduce_kernel(const float *__restrict__ partial, int splits, uint64_t plane,
                                                           const float *__restrict__ sw, const void *__restrict__ bias_,
                                                           void *__restrict__ y_, uint64_t quads, int n) {
    using Out = typename OutT<OUT>::type;
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * 256 + threadIdx.x;
    if (i >= quads) return;
    const uint64_t e = i * 4;                  // n is a multiple of 4: a quad never straddles rows
    const int c = static_cast<int>(e % static_cast<uint64_t>(n));
    float4 t = *reinterpret_cast<const float4 *>(partial + e);
    for (int s = 1; s < splits; ++s) {
        const float4 u = *reinterpret_cast<const float4 *>(partial + s * plane + e);
        t.x += u.x; t.y += u.y; t.z += u.z; t.w += u.w;
    }
    const float4 w4 = *reinterpret_cast<const float4 *>(sw + c);
    const Out *bias = static_cast<const Out *>(bias_);
    float b[4] = {0.f, 0.f, 0.f, 0.f};
    if (bias) {
#pragma unroll
        for (int r = 0; r < 4; ++r) b[r] = to_float(bias[c + r]);
    }
    const float o[4] = {t.x * w4.x + b[0], t.y * w4.y + b[1], t.z * w4.z + b[2], t.w * w4.w + b[3]};
    Out *y = static_cast<Out *>(y_) + e;
    if constexpr (OUT == kOutF16) {
        const __half2 h01 = __floats2half2_rn(o[0], o[1]), h23 = __floats2half2_rn(o[2], o[3]);
        uint2 w2;
        w2.x = *reinterpret_cast<const uint32_t *>(&h01);
        w2.y = *reinterpret_cast<const uint32_t *>(&h23);
        *reinterpret_cast<uint2 *>(y) = w2;
    } else {
        *reinterpret_cast<float4 *>(y) = float4{o[0], o[1], o[2], o[3]};
    }
}

}  // namespace

// Shares per tile with which this kernel serves the layer, or 0 if it does not: channel slices of
// 192, a channel count that is a multiple of 4, fewer than two 128 x 128 tiles per CU (layers with
// more do not need the split), and at least three chunks per share.
int hq_conv3x3_split_shares(int64_t pixels, int c_in, int c_out) {
    if (c_in % 192 != 0 || (c_out & 3) != 0 || pixels <= 0) return 0;
    const int64_t cus = hq::compute_units();
    const int64_t tiles = ((pixels + 127) / 128) * ((c_out + 127) / 128);
    if (tiles >= 2 * cus) return 0;
    const int chunks = 9 * (c_in / 192);
    int64_t shares = (2 * cus + tiles - 1) / tiles;
    if (shares > chunks / 3) shares = chunks / 3;
    if (shares > 16) shares = 16;
    return shares >= 2 ? static_cast<int>(shares) : 0;
}

hq_status hq_conv3x3_split_launch(const GemmArgs &g, hq_dtype y_dtype, void *workspace, size_t workspace_bytes,
                                  hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    const int shares = hq_conv3x3_split_shares(g.pixels, g.k, g.n);
    if (shares == 0) return HQ_ERR_UNSUPPORTED;
    const uint64_t plane = static_cast<uint64_t>(g.pixels) * g.n;
    if (y_dtype != HQ_I32) {
        if (!workspace || workspace_bytes < plane * shares * sizeof(float)) return HQ_ERR_SHAPE;
        if (reinterpret_cast<uintptr_t>(workspace) & 15u) return HQ_ERR_ALIGN;
    }
    SplitArgs a{};
    a.xq = g.xq; a.sx = g.sx; a.wq = g.wq; a.partial = static_cast<float *>(workspace); a.yi = static_cast<int *>(g.y);
    a.pixels = g.pixels; a.n = g.n; a.k = g.k; a.h = g.h; a.w = g.w; a.sx_static = g.sx_static;
    const hq::Magic31 mw = hq::magic31(static_cast<uint32_t>(g.w)), mh = hq::magic31(static_cast<uint32_t>(g.h));
    a.w_magic = mw.m; a.w_shift = mw.s; a.h_magic = mh.m; a.h_shift = mh.s;
    a.n_px_tiles = static_cast<uint32_t>((static_cast<int64_t>(g.pixels) + 127) / 128);
    const int64_t tiles = static_cast<int64_t>(a.n_px_tiles) * ((g.n + 127) / 128);
    a.n_tiles = static_cast<uint32_t>(tiles);
    a.splits = shares;
    const unsigned grid = static_cast<unsigned>(tiles * shares);
    if (y_dtype == HQ_I32) {
        const hq_status st = hq_fill_zero_launch(g.y, plane * (g.sx_static ? 1 : 9), stream);
        if (st != HQ_OK) return st;
        hipLaunchKernelGGL((conv3x3_split_kernel<true>), dim3(grid), dim3(256), 0, stream, a);
        return check.status();
    }
    hipLaunchKernelGGL((conv3x3_split_kernel<false>), dim3(grid), dim3(256), 0, stream, a);
    const uint64_t quads = plane / 4;
    const unsigned rgrid = static_cast<unsigned>((quads + 255) / 256);
    if (y_dtype == HQ_F16)
        hipLaunchKernelGGL((split_reduce_kernel<kOutF16>), dim3(rgrid), dim3(256), 0, stream, a.partial, shares, plane,
                           g.sw, g.bias, g.y, quads, g.n);
    else
        hipLaunchKernelGGL((split_reduce_kernel<kOutF32>), dim3(rgrid), dim3(256), 0, stream, a.partial, shares, plane,
                           g.sw, g.bias, g.y, quads, g.n);
    return check.status();
}
