// hq_act_quant_int_linear: a linear layer / 1x1 convolution in one launch.  (Method, "Matrix
// Multiplication": the transformed activations X H are only ever an operand of the integer
// product, so they need not exist outside the kernel that multiplies them.)
//
// Linear and 1x1 layers of a UNet are bound by reading their fp16 input and writing their fp16
// output (arithmetic intensity below the machine balance); through two calls they also write and
// re-read the codes and pay a second launch.  Here a workgroup of four waves owns 64 rows (tokens)
// and a range of output columns:
//   1. every wave transforms and quantises 16 of the rows exactly as the stand-alone kernel does
//      (v_mfma_f32_16x16x32_f16 against the +-1 matrix, abs-max over the row, eight values to a
//      packed dword: the same arithmetic, hence the same codes and scales), expands the packed
//      dwords to int8 (16 x code) and stores them to LDS as the "B" operand image [row][K] (rows
//      padded by 16 bytes so that the operand reads of 16 consecutive rows hit 16 bank groups);
//   2. every wave then walks its 32-column blocks: per 64-code K step its lanes fetch their packed
//      weight pieces straight from memory (the weights of such layers are small and stay in L2; four
//      steps ahead of the MFMAs), expand them and multiply a 32 x 64 register tile against the
//      resident int8 rows; the sums carry 256 and are scaled by x_scale[row] w_scale[col] / 256;
//   3. fp16 results pass through a per-wave LDS staging area so that neighbouring lanes store
//      contiguous bytes.
#include "hq_hadamard_mfma.h"
#include "hq_int_gemm_kernel.h"

namespace {

constexpr int kLinRows = 64;          // rows of a workgroup
constexpr int kLinMaxK = 1024;

struct LinFusedArgs {
    const __half *x;     // [m, k]
    const uint8_t *wq;   // [n, k/2]
    const float *sw;     // [n]
    const void *bias;    // [n] of the output dtype, or null
    void *y;             // [m, n]
    uint8_t *xq_out;     // null, or [m, k/2]
    float *sx_out;       // null, or [m]
    int64_t m;
    int n, k;
    float qmax;
    int col_splits;      // workgroups per row tile; each takes every col_splits-th group of 128 columns
};

template <int OUT>
__global__ __launch_bounds__(256, 4) void linear_fused_kernel(LinFusedArgs a) {
    constexpr bool INT_OUT = OUT == kOutI32;
    using Out = typename OutT<OUT>::type;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];   // [64 rows][k + 16] int8, then scales, then staging

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int K = a.k, kbytes = K >> 1, nblk = K >> 6;
    const int stride = K + 16;
    float *s_sx = reinterpret_cast<float *>(lds + kLinRows * stride);          // [64]
    const uint32_t lds_base = lds_address(lds);
    const uint32_t staging = lds_base + kLinRows * stride + kLinRows * 4 + wave * 2048;

    const int64_t row_tile = blockIdx.x / a.col_splits;
    const int split = static_cast<int>(blockIdx.x - row_tile * a.col_splits);
    const int64_t r0 = row_tile * kLinRows;

    // ---- 1. transform + quantise 16 rows per wave into the int8 image ---------------------------------
    {
        v8h hmat[4][2];
        hadamard64_operands(lane, hmat);
        const int tok = lane & 15, q = lane >> 4;
        const int row = wave * 16 + tok;
        int64_t token = r0 + row;
        const bool live = token < a.m;
        token = live ? token : a.m - 1;
        const __half *src = a.x + token * K + 8 * q;
        // the fp16 pieces are requested four blocks at a time (eight 16-byte loads in flight per lane);
        // rows of up to four blocks keep them in registers for the second pass
        v8h bb[4][2];
        auto request = [&](int b0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (b0 + j < nblk) {
                    bb[j][0] = *reinterpret_cast<const v8h *>(src + 64 * (b0 + j));
                    bb[j][1] = *reinterpret_cast<const v8h *>(src + 64 * (b0 + j) + 32);
                }
            }
        };
        float amax = 0.f;
        for (int b0 = 0; b0 < nblk; b0 += 4) {
            request(b0);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (b0 + j < nblk) {
                    float v[16];
                    hadamard64_transform(hmat, bb[j], v);
#pragma unroll
                    for (int r = 0; r < 16; ++r) amax = fmaxf(amax, fabsf(v[r]));
                }
            }
        }
        amax = fmaxf(amax, __shfl_xor(amax, 16));   // the row's other three K slices
        amax = fmaxf(amax, __shfl_xor(amax, 32));
        const float inv = amax > 0.f ? a.qmax / amax : 0.f;
        const float scale = amax > 0.f ? (amax * 0.125f) / a.qmax : 1.0f;
        if (q == 0) {
            s_sx[row] = live ? scale * (1.0f / 256.0f) : 0.f;
            if (live && split == 0 && a.sx_out) a.sx_out[token] = scale;
        }
        // piece (MFMA q % 2, lane half q / 2) of the block's 64 bytes
        const uint32_t piece = (((q & 1) << 1) | (q >> 1)) * 16;
        for (int b0 = 0; b0 < nblk; b0 += 4) {
            if (nblk > 4) request(b0);   // (from cache)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (b0 + j < nblk) {
                    const int blk = b0 + j;
                    float v[16];
                    hadamard64_transform(hmat, bb[j], v);
                    v4i p = {0, 0, 0, 0};
                    p.x = static_cast<int>(pack8_magic(v, inv));
                    p.y = static_cast<int>(pack8_magic(v + 8, inv));
                    v4i first_half, second_half;
                    expand(p, first_half, second_half);
                    *reinterpret_cast<v4i *>(lds + row * stride + blk * 64 + piece) = first_half;
                    if (live && split == 0 && a.xq_out)
                        *reinterpret_cast<uint2 *>(a.xq_out + token * kbytes + blk * 32 + q * 8) =
                            uint2{static_cast<uint32_t>(p.x), static_cast<uint32_t>(p.y)};
                }
            }
        }
    }
    __syncthreads();

    // ---- 2. 32-column blocks of this wave (a 32 x 64 register tile: two MFMA tiles, which leaves
    //         registers for four workgroups per CU - these layers need the occupancy, not the reuse) ------
    const int n_cb = (a.n + 31) / 32;
    // B operand addresses: rows tn * 32 + lrow, pieces (m * 2 + lhalf) of a K step
    uint32_t off_b[2];
#pragma unroll
    for (int tn = 0; tn < 2; ++tn) off_b[tn] = (tn * 32 + lrow) * stride + lhalf * 16;

    for (int cb = split * 4 + wave; cb < n_cb; cb += 4 * a.col_splits) {
        const int c0 = cb * 32;
        // this lane's weight row: column c0 + (row of the MFMA tile -> channel), clamped
        int c = c0 + tile_row_to_channel(lrow);
        c = c < a.n ? c : a.n - 1;
        const uint8_t *wrow = a.wq + static_cast<int64_t>(c) * kbytes + lhalf * 16;
        v16i acc[2];
#pragma unroll
        for (int tn = 0; tn < 2; ++tn)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[tn][r] = 0;
        // the lane's packed weight pieces are requested four K steps ahead of their use
        v4i wr[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (j < nblk) wr[j] = *reinterpret_cast<const v4i *>(wrow + j * 32);
        for (int k4 = 0; k4 < nblk; k4 += 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int ks = k4 + j;
                if (ks < nblk) {
                    v4i a0, a1;
                    expand(wr[j], a0, a1);
                    if (ks + 4 < nblk) wr[j] = *reinterpret_cast<const v4i *>(wrow + (ks + 4) * 32);
#pragma unroll
                    for (int tn = 0; tn < 2; ++tn) {
                        const v4i b0v = *reinterpret_cast<const v4i *>(lds + off_b[tn] + ks * 64);
                        const v4i b1v = *reinterpret_cast<const v4i *>(lds + off_b[tn] + ks * 64 + 32);
                        acc[tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b0v, acc[tn], 0, 0, 0);
                        acc[tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b1v, acc[tn], 0, 0, 0);
                    }
                }
            }
        }
        // ---- 3. scale and store ------------------------------------------------------------------------------
        const int cbase = c0 + 16 * lhalf;
        if constexpr (INT_OUT) {
            int *yi = static_cast<int *>(a.y);
#pragma unroll
            for (int tn = 0; tn < 2; ++tn) {
                const int64_t row = r0 + tn * 32 + lrow;
                if (row >= a.m) continue;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (cbase + r < a.n) yi[row * a.n + cbase + r] = acc[tn][r] >> 8;
            }
        } else {
            Out *y = static_cast<Out *>(a.y);
            const Out *bias = static_cast<const Out *>(a.bias);
            float swv[16], bv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const bool ok = cbase + r < a.n;
                swv[r] = ok ? a.sw[cbase + r] : 0.f;
                bv[r] = ok && bias ? to_float(bias[cbase + r]) : 0.f;
            }
#pragma unroll
            for (int tn = 0; tn < 2; ++tn) {
                const float sx = s_sx[tn * 32 + lrow];
                float out[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) out[r] = __builtin_fmaf(sx * static_cast<float>(acc[tn][r]), swv[r], bv[r]);
                if constexpr (OUT == kOutF16) {
                    if ((a.n & 7) == 0 && c0 + 32 <= a.n) {   // uniform
                        v4i q0, q1;
                        transpose_tile_f16(out, staging, lane, q0, q1);
                        const int64_t row0 = r0 + tn * 32 + (lane >> 2), row1 = row0 + 16;
                        __half *dst = reinterpret_cast<__half *>(y) + c0 + (lane & 3) * 8;
                        if (row0 < a.m) *reinterpret_cast<v4i *>(dst + row0 * a.n) = q0;
                        if (row1 < a.m) *reinterpret_cast<v4i *>(dst + row1 * a.n) = q1;
                        continue;
                    }
                }
                const int64_t row = r0 + tn * 32 + lrow;
                if (row >= a.m) continue;
                Out *dst = y + row * a.n + cbase;
                if ((a.n & 15) == 0 && cbase + 16 <= a.n) {
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

// The kernel's LDS is sized per launch (64 rows of K + 16 bytes); above the default limit of dynamic
// LDS the limit is raised once per device and output type (a property of the kernel, not state of a call).
template <int OUT>
hq_status launch_linear_fused(const LinFusedArgs &a, unsigned grid, size_t lds_bytes, hipStream_t stream) {
    static std::atomic<int> raised[64];
    int dev = 0;
    if (lds_bytes > 48 * 1024 && hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64 &&
        raised[dev].load(std::memory_order_relaxed) == 0) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&linear_fused_kernel<OUT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                kLinRows * (kLinMaxK + 16) + kLinRows * 4 + 4 * 2048) != hipSuccess)
            return HQ_ERR_LAUNCH;
        raised[dev].store(1, std::memory_order_relaxed);
    }
    hipLaunchKernelGGL((linear_fused_kernel<OUT>), dim3(grid), dim3(256), lds_bytes, stream, a);
    return HQ_OK;
}

}  // namespace

extern "C" hq_status hq_act_quant_int_linear(const void *x, hq_dtype x_dtype, const uint8_t *wq, const float *w_scale,
                                             const void *bias, int64_t m, int n, int k, int had_block, int a_bits,
                                             void *y, hq_dtype y_dtype, uint8_t *xq_out, float *x_scale_out,
                                             void *stream) {
    if (!x || !wq || !y) return HQ_ERR_NULL;
    if (y_dtype != HQ_F16 && y_dtype != HQ_F32 && y_dtype != HQ_I32) return HQ_ERR_DTYPE;
    if (y_dtype != HQ_I32 && !w_scale) return HQ_ERR_NULL;
    if (x_dtype != HQ_F16 && x_dtype != HQ_F32) return HQ_ERR_DTYPE;
    if (m <= 0 || n <= 0 || k <= 0) return HQ_ERR_SHAPE;
    if (a_bits < 2 || a_bits > 4) return HQ_ERR_BITS;
    if (!hq::pow2_upto_128(had_block) || k % had_block != 0 || (k & 7) != 0 || k >= 131072) return HQ_ERR_SHAPE;
    if (!hq::aligned16(x) || !hq::aligned16(wq) || !hq::aligned16(y) || (xq_out && !hq::aligned16(xq_out)))
        return HQ_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(w_scale) & 3u) || (reinterpret_cast<uintptr_t>(x_scale_out) & 3u) ||
        (reinterpret_cast<uintptr_t>(bias) & 1u))
        return HQ_ERR_ALIGN;
    // built: fp16 activations, block 64, rows of at most 1024 channels
    if (x_dtype != HQ_F16 || had_block != 64 || k % 64 != 0 || k > kLinMaxK) return HQ_ERR_UNSUPPORTED;
    const int64_t row_tiles = (m + kLinRows - 1) / kLinRows;
    // enough workgroups for four per CU, but never fewer than one group of four 32-column blocks each
    const int col_groups = (n + 127) / 128;
    int64_t splits = (4 * static_cast<int64_t>(hq::compute_units()) + row_tiles - 1) / row_tiles;
    splits = splits < 1 ? 1 : (splits > col_groups ? col_groups : splits);
    if (row_tiles * splits > 0x7fffffffLL) return HQ_ERR_SHAPE;
    const hq::LaunchCheck check;   // samples the thread's error state before anything is launched
    LinFusedArgs a{};
    a.x = static_cast<const __half *>(x); a.wq = wq; a.sw = w_scale; a.bias = bias; a.y = y;
    a.xq_out = xq_out; a.sx_out = x_scale_out; a.m = m; a.n = n; a.k = k;
    a.qmax = static_cast<float>((1 << (a_bits - 1)) - 1);
    a.col_splits = static_cast<int>(splits);
    const size_t lds_bytes = static_cast<size_t>(kLinRows) * (k + 16) + kLinRows * 4 + 4 * 2048;
    const unsigned grid = static_cast<unsigned>(row_tiles * splits);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hq_status rc;
    if (y_dtype == HQ_I32) rc = launch_linear_fused<kOutI32>(a, grid, lds_bytes, st);
    else if (y_dtype == HQ_F16) rc = launch_linear_fused<kOutF16>(a, grid, lds_bytes, st);
    else rc = launch_linear_fused<kOutF32>(a, grid, lds_bytes, st);
    if (rc != HQ_OK) return rc;
    return check.status();
}
