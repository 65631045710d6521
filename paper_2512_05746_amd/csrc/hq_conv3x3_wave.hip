// 3x3 / stride 1 / pad 1 NHWC convolution on int8 MFMA for layers with few output tiles:
// every WAVE works alone on one 64-channel x 64-pixel output tile (2 x 2 MFMA tiles of
// 32x32) and on one contiguous share of that tile's K range (Method, "Convolution":
// one integer sum per tap, taps combined in fp32 with the scale of the input pixel
// under the tap).
//
// Why.  With 64x64 output tiles a layer of 1024 pixels x 960 channels has 240 tiles for
// 1024 SIMDs.  Splitting every tile's 9 * C_in / 192 chunks over KG = 1, 2 or 4 waves of
// one workgroup fills the machine, keeps the efficient 2 x 2 register tile (six vector
// instructions of nibble expansion per MFMA instead of twelve for a 32x32 wave tile) and
// needs no exchange through global memory: the KG partial fp32 results of a tile meet in
// LDS and each of the KG waves finishes a quarter (or half) of the tile.
//
// A wave owns its LDS stages, issues its own direct-to-LDS loads (12 KiB per chunk: 64
// weight rows and 64 activation rows of 96 packed bytes) and waits only for its own loads:
// there is no barrier in the K loop.  One workgroup of four waves (one per SIMD) per CU.
//
// Addresses.  Lane l of load i fetches 16-byte slot q = 64 i + l of the operand image
// (row q / 6, piece q % 6).  64 * 3 = 32 * 6, so loads i and i + 3 have the same per-lane
// pattern 32 rows apart: three per-lane offsets per operand, computed once, serve the whole
// kernel, and tile, tap, chunk and row half move a uniform base only.  A tile or tap that
// touches the end of a tensor (channels >= n, pixels >= pixels, a shifted row before pixel
// 0 or after the last pixel) takes a per-lane path that clamps every row to an in-bounds
// one instead; such rows are never stored and taps outside the image have scale 0.
#include "hq_int_gemm_kernel.h"

namespace {

struct WaveConvArgs {
    const uint8_t *xq;   // [pixels, k/2]
    const float *sx;     // [pixels], or one value for the whole tensor (sx_static)
    const uint8_t *wq;   // [n, 9, k/2]
    const float *sw;     // [n]
    const void *bias;    // [n] of the output dtype, or null
    void *y;             // [pixels, n]
    uint32_t pixels;
    int n, k, h, w;
    uint32_t w_magic, w_shift, h_magic, h_shift;   // exact division of a pixel index by w and by h
    uint32_t n_px_tiles, n_tiles;
    int kg_log2;         // waves per tile: 1 << kg_log2 (1, 2 or 4)
    int sx_static;       // one activation scale for the tensor: the per-tap sums are then combined with
                         // that one scale, which equals one integer sum times one product of scales
};

template <int OUT, int NSTAGE>
__global__ __launch_bounds__(256, 1) void conv3x3_wave_kernel(WaveConvArgs a) {
    constexpr int TM = 2, TN = 2, KCH = 6, ROWB = KCH * 16, KS = KCH / 2, TAPS = 9;
    constexpr int OP_BYTES = 64 * ROWB;             // one operand of one chunk: six 1 KiB loads
    constexpr int STAGE_BYTES = 2 * OP_BYTES;       // weight rows, then activation rows
    constexpr int WAVE_BYTES = NSTAGE * STAGE_BYTES;
    constexpr int LOADS = 12;                       // per chunk
    static_assert(WAVE_BYTES >= 64 * 64 * 4, "a wave's stages later hold its 64x64 fp32 partial result");
    static_assert(NSTAGE >= 2 && (NSTAGE - 2) * LOADS < 64, "vmcnt range");
    using Out = typename OutT<OUT>::type;
    using Ops = Packed<TM, TN>;

    __shared__ __attribute__((aligned(16))) uint8_t lds[4 * WAVE_BYTES];
    __shared__ float s_sx[4][TAPS][TN][32];   // per wave: x_scale / 256 under tap t, 0 outside the image

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int kbytes = a.k >> 1;
    const int cpt = kbytes / ROWB;               // chunks per tap (host guarantees divisibility)
    const int chunks = TAPS * cpt;
    const uint32_t last = a.pixels - 1;

    // ---- this wave's unit: tile and chunk range ---------------------------------------------
    // Workgroup b runs on XCD b % 8 (round-robin dispatch): give every XCD a contiguous range of
    // units, and order the tiles channel-tile major, so that an XCD's L2 fetches only the weight
    // rows of a few channel tiles (the weights are the large operand of the layers this kernel serves).
    uint32_t wg = blockIdx.x;
    if (gridDim.x % 8 == 0) wg = (blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
    const uint32_t unit = wg * 4 + wave;
    const int kg = 1 << a.kg_log2;
    const int g = static_cast<int>(unit & (kg - 1));
    uint32_t tile = unit >> a.kg_log2;
    const bool active = tile < a.n_tiles;        // the same for all waves of a tile
    if (!active) tile = a.n_tiles - 1;
    const int c0 = active ? (g * chunks) >> a.kg_log2 : 0;
    const int c1 = active ? ((g + 1) * chunks) >> a.kg_log2 : 0;
    const int co0 = static_cast<int>(tile / a.n_px_tiles) * 64;
    const uint32_t p0 = (tile % a.n_px_tiles) * 64;

    const uint32_t wave_base = lds_address(lds) + wave * WAVE_BYTES;
    const uint32_t lds_a = wave_base + lrow * ROWB + (lhalf ^ ((lrow >> 3) & 1)) * 16;
    const uint32_t lds_b = lds_a + OP_BYTES;
    const uint32_t lds_sx = lds_address(&s_sx[wave][0][0][0]) + lrow * 4;

    // ---- per-lane load patterns (see above) ---------------------------------------------------
    uint32_t pat_a[3], pat_b[3];
#pragma unroll
    for (int r = 0; r < 3; ++r) {
        const int q = 64 * r + lane, row = q / KCH, piece = (q % KCH) ^ ((row >> 3) & 1);
        pat_a[r] = static_cast<uint32_t>(tile_row_to_channel(row)) * TAPS * kbytes + piece * 16;
        pat_b[r] = static_cast<uint32_t>(row) * kbytes + piece * 16;
    }
    const bool rows_inside = co0 + 64 <= a.n && p0 + 64 <= a.pixels;
    int ftap = c0 / cpt, fch = c0 - ftap * cpt;   // chunk being fetched
    auto issue_loads = [&](int stage) {
        const int dpix = (ftap / 3 - 1) * a.w + (ftap % 3 - 1);
        uint8_t *image = lds + wave * WAVE_BYTES + stage * STAGE_BYTES;
        const int64_t first = static_cast<int64_t>(p0) + dpix;
        if (rows_inside && first >= 0 && first + 63 <= static_cast<int64_t>(last)) {
            const uint8_t *base_a = a.wq + (static_cast<uint64_t>(co0) * TAPS + ftap) * kbytes + fch * ROWB;
            const uint8_t *base_b = a.xq + static_cast<uint64_t>(first) * kbytes + fch * ROWB;
#pragma unroll
            for (int i = 0; i < 6; ++i)
                load_to_lds16(base_a + (i >= 3 ? static_cast<uint64_t>(32) * TAPS * kbytes : 0) + pat_a[i % 3],
                              image + i * 1024);
#pragma unroll
            for (int i = 0; i < 6; ++i)
                load_to_lds16(base_b + (i >= 3 ? static_cast<uint64_t>(32) * kbytes : 0) + pat_b[i % 3],
                              image + OP_BYTES + i * 1024);
        } else {
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                const int q = 64 * i + lane, row = q / KCH, piece = (q % KCH) ^ ((row >> 3) & 1);
                int co = co0 + (row & ~31) + tile_row_to_channel(row & 31);
                co = co < a.n ? co : a.n - 1;
                const uint32_t off = (static_cast<uint32_t>(co) * TAPS + ftap) * kbytes + fch * ROWB + piece * 16;
                load_to_lds16(a.wq + off, image + i * 1024);
            }
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                const int q = 64 * i + lane, row = q / KCH, piece = (q % KCH) ^ ((row >> 3) & 1);
                uint32_t pix = p0 + row + static_cast<uint32_t>(dpix);   // wraps below pixel 0
                pix = pix < last ? pix : last;
                const uint32_t off = pix * kbytes + fch * ROWB + piece * 16;
                load_to_lds16(a.xq + off, image + OP_BYTES + i * 1024);
            }
        }
        if (++fch == cpt) { fch = 0; ++ftap; }
    };

    constexpr bool INT_OUT = OUT == kOutI32;
    float facc[INT_OUT ? 1 : TM][INT_OUT ? 1 : TN][16];
    if constexpr (!INT_OUT) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int r = 0; r < 16; ++r) facc[tm][tn][r] = 0.f;
    }
    int my_mask[TN];   // integer output: tap masks of this lane's two pixels (pixel tn * 32 + lrow)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) my_mask[tn] = 0;

    if (c0 < c1) {
        // ---- scales of the nine input pixels of this lane's output pixel (pixel lhalf*32 + lrow)
        {
            const uint32_t pix = p0 + lhalf * 32 + lrow;
            const uint32_t q = hq::div_magic31(pix, a.w, a.w_magic, a.w_shift);
            const int ow = static_cast<int>(pix - q * a.w);
            const int oh = static_cast<int>(q - hq::div_magic31(q, a.h, a.h_magic, a.h_shift) * a.h);
            const int cm = (ow > 0 ? 1 : 0) | 2 | (ow + 1 < a.w ? 4 : 0);
            int mask = (oh > 0 ? cm : 0) | (cm << 3) | (oh + 1 < a.h ? cm << 6 : 0);
            if (pix >= a.pixels) mask = 0;
            float v[TAPS];
#pragma unroll
            for (int t = 0; t < TAPS; ++t) {
                uint32_t ip = pix + static_cast<uint32_t>((t / 3 - 1) * a.w + (t % 3 - 1));
                ip = ip < last ? ip : last;
                v[t] = INT_OUT ? 0.f : a.sx[a.sx_static ? 0 : ip];   // integer output: no scales (null allowed)
            }
            if constexpr (INT_OUT) {   // lane (lhalf, lrow) computed the mask of pixel lhalf * 32 + lrow
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) my_mask[tn] = __shfl(mask, tn * 32 + lrow, 64);
            }
            // the chunks in flight first, then the table: the table's loads are older than the
            // chunk loads, so waiting for them leaves the chunk loads in flight
#pragma unroll
            for (int st = 0; st < NSTAGE - 1; ++st)
                if (c0 + st < c1) issue_loads(st);
#pragma unroll
            for (int t = 0; t < TAPS; ++t)
                s_sx[wave][t][lhalf][lrow] = ((mask >> t) & 1) ? v[t] * (1.0f / 256.0f) : 0.f;
        }

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
            // chunk c has landed once only the loads of the later chunks in flight are pending
            if (c + NSTAGE - 2 < c1) wait_vmem<(NSTAGE - 2) * LOADS>();
            else wait_vmem<0>();
            if (c + NSTAGE - 1 < c1) issue_loads(stage == 0 ? NSTAGE - 1 : stage - 1);

            const uint32_t sa = lds_a + stage * STAGE_BYTES, sb = lds_b + stage * STAGE_BYTES;
            Ops op[2];
            read_packed<TM, TN, ROWB, 0>(op[0], sa, sb);
            chunk_steps<0, KS, TM, TN, ROWB>(op, sa, sb, ch == 0 || c == c0, multiply);

            const bool tap_ends = ch + 1 == cpt;
            if (tap_ends || c + 1 == c1) {
                if constexpr (INT_OUT) {
                    // This wave's share of the tap's sum, added to the zero-filled output: integer
                    // additions are exact, so the order in which the waves of a tile arrive does not
                    // matter.  Per-tap sums [pixel, tap, n]; one sum over all taps [pixel, n] when the
                    // tensor has one scale (then taps outside the image must not count either).
                    int *yi = static_cast<int *>(a.y);
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        const uint32_t pix = p0 + tn * 32 + lrow;
                        if (pix >= a.pixels || !((my_mask[tn] >> tap) & 1)) continue;
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm) {
                            const int cbase = co0 + tm * 32 + 16 * lhalf;
                            int *dst = yi + (a.sx_static ? static_cast<int64_t>(pix)
                                                         : static_cast<int64_t>(pix) * TAPS + tap) * a.n + cbase;
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (cbase + r < a.n) atomicAdd(dst + r, acc[tm][tn][r] >> 8);
                        }
                    }
                } else {
                    float s[TN];
                    read_tap_scales<TN>(s, lds_sx + tap * (TN * 32 * 4));
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                facc[tm][tn][r] += s[tn] * static_cast<float>(acc[tm][tn][r]);
                }
            }
            if (tap_ends) { ch = 0; ++tap; } else { ++ch; }
            stage = stage + 1 == NSTAGE ? 0 : stage + 1;
        }
    }

    if constexpr (INT_OUT) {
        return;   // everything was added to the output above
    } else {
    // ---- the KG partial results of a tile meet in LDS; each wave finishes its share -----------
    // partial of a wave: [sub-tile tm*2+tn][r/4][lane] float4 in its own (now idle) stages
    Out *y = static_cast<Out *>(a.y);
    const Out *bias = static_cast<const Out *>(a.bias);
    auto finish = [&](int tm, int tn, const float (&v)[16]) {
        const int cbase = co0 + tm * 32 + 16 * lhalf;
        const uint32_t pix = p0 + tn * 32 + lrow;
        float swv[16], bv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const bool ok = cbase + r < a.n;
            swv[r] = ok ? a.sw[cbase + r] : 0.f;
            bv[r] = ok && bias ? to_float(bias[cbase + r]) : 0.f;
        }
        if (pix >= a.pixels) return;
        float out[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) out[r] = v[r] * swv[r] + bv[r];
        Out *dst = y + static_cast<int64_t>(pix) * a.n + cbase;
        if ((a.n & 15) == 0 && cbase + 16 <= a.n) {
            store16(dst, out);
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (cbase + r < a.n) dst[r] = static_cast<Out>(out[r]);
        }
    };

    if (kg == 1) {
        if (!active) return;
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) finish(tm, tn, facc[tm][tn]);
        return;
    }

    float4 *mine = reinterpret_cast<float4 *>(lds + wave * WAVE_BYTES);
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                mine[((tm * 2 + tn) * 4 + q) * 64 + lane] =
                    float4{facc[tm][tn][4 * q], facc[tm][tn][4 * q + 1], facc[tm][tn][4 * q + 2], facc[tm][tn][4 * q + 3]};
    __syncthreads();
    if (!active) return;
    const int first_wave = wave & ~(kg - 1);     // the waves first_wave .. first_wave + kg - 1 share the tile
    const int subs = 4 >> a.kg_log2;             // sub-tiles this wave finishes: g*subs .. g*subs + subs - 1
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
        if (sub / subs != g) continue;           // uniform
        float v[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) v[r] = 0.f;
        for (int j = 0; j < kg; ++j) {           // fixed order: results do not depend on timing
            const float4 *part = reinterpret_cast<const float4 *>(lds + (first_wave + j) * WAVE_BYTES);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 t = part[(sub * 4 + q) * 64 + lane];
                v[4 * q] += t.x; v[4 * q + 1] += t.y; v[4 * q + 2] += t.z; v[4 * q + 3] += t.w;
            }
        }
        finish(sub >> 1, sub & 1, v);
    }
    }
}

// Zero fill of the integer output (its sums are accumulated with integer atomics).
__global__ void fill_zero_kernel(int4 *dst, uint64_t n16, int *tail, int n_tail) {
    const uint64_t i = static_cast<uint64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n16) dst[i] = int4{0, 0, 0, 0};
    if (i < static_cast<uint64_t>(n_tail)) tail[i] = 0;
}

}  // namespace

// Waves per tile that minimise rounds * (chunks per wave + fixed cost) on `cus` CUs of four SIMDs.
int hq_conv3x3_wave_split(int64_t tiles, int chunks, int cus) {
    int best = 0;
    int64_t best_cost = -1;
    for (int l = 0; l <= 2; ++l) {
        const int64_t waves = tiles << l;
        const int64_t rounds = (waves + 4 * cus - 1) / (4 * cus);
        const int64_t cost = rounds * ((chunks + (1 << l) - 1) / (1 << l) + 3);
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = l; }
    }
    return best;
}

// Zero fill of `ints` int32 values at a 16-byte aligned address (a kernel, so that it can be captured).
hq_status hq_fill_zero_launch(void *dst, uint64_t ints, hipStream_t stream) {
    const uint64_t n16 = ints / 4;
    const int n_tail = static_cast<int>(ints % 4);
    const uint64_t blocks = (n16 + 255) / 256;
    if (blocks > 0x7fffffffULL) return HQ_ERR_SHAPE;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(static_cast<unsigned>(blocks ? blocks : 1)), dim3(256), 0, stream,
                       static_cast<int4 *>(dst), n16, static_cast<int *>(dst) + n16 * 4, n_tail);
    return HQ_OK;
}

hq_status hq_conv3x3_wave_launch(const GemmArgs &g, hq_dtype y_dtype, hipStream_t stream) {
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    if (g.k % 192 != 0 || (y_dtype != HQ_F16 && y_dtype != HQ_F32 && y_dtype != HQ_I32)) return HQ_ERR_UNSUPPORTED;
    WaveConvArgs a{};
    a.xq = g.xq; a.sx = g.sx; a.wq = g.wq; a.sw = g.sw; a.bias = g.bias; a.y = g.y;
    a.pixels = g.pixels; a.n = g.n; a.k = g.k; a.h = g.h; a.w = g.w; a.sx_static = g.sx_static;
    const hq::Magic31 mw = hq::magic31(static_cast<uint32_t>(g.w)), mh = hq::magic31(static_cast<uint32_t>(g.h));
    a.w_magic = mw.m; a.w_shift = mw.s; a.h_magic = mh.m; a.h_shift = mh.s;
    a.n_px_tiles = static_cast<uint32_t>((static_cast<int64_t>(g.pixels) + 63) / 64);
    const int64_t tiles = static_cast<int64_t>(a.n_px_tiles) * ((g.n + 63) / 64);
    if (tiles > 0x1fffffff) return HQ_ERR_SHAPE;
    a.n_tiles = static_cast<uint32_t>(tiles);
    a.kg_log2 = hq_conv3x3_wave_split(tiles, 9 * (g.k / 192), hq::compute_units());
    const unsigned grid = static_cast<unsigned>(((tiles << a.kg_log2) + 3) / 4);
    if (y_dtype == HQ_I32) {
        // integer output [pixels, 9, n] (per-tap sums) or [pixels, n] (one scale: one sum): zero it, then
        // every wave adds its share of a tap's sum
        const hq_status st = hq_fill_zero_launch(g.y, static_cast<uint64_t>(g.pixels) * (g.sx_static ? 1 : 9) * g.n,
                                                 stream);
        if (st != HQ_OK) return st;
        hipLaunchKernelGGL((conv3x3_wave_kernel<kOutI32, 3>), dim3(grid), dim3(256), 0, stream, a);
    } else if (y_dtype == HQ_F16)
        hipLaunchKernelGGL((conv3x3_wave_kernel<kOutF16, 3>), dim3(grid), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((conv3x3_wave_kernel<kOutF32, 3>), dim3(grid), dim3(256), 0, stream, a);
    return check.status();
}
