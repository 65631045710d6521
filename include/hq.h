/*
 * hq.h - C ABI of the Hadamard-quantised layer of HQ-DM (arxiv 2512.05746) for
 * AMD MI355X (gfx950).
 *
 * The layer replaces every linear / convolution of a diffusion UNet by
 *   1. a block-diagonal Hadamard transform over the input-channel axis
 *      (Method, "Matrix Multiplication": H = BlockDiag(H_k, ..., H_k)),
 *   2. symmetric low-bit quantisation (Background, "Model Quantization":
 *      X_int = clamp(round(X / S), min, max)),
 *   3. an integer product with int32 accumulation, and
 *   4. dequantisation by the product of scales (Method: Y ~ S_XH S_W (...)).
 *
 * Conventions shared by every call
 *   - Every pointer is a DEVICE pointer owned by the caller (the library never
 *     allocates, frees or keeps one), 16-byte aligned unless stated otherwise.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it; they never synchronise.
 *   - All arguments are validated on the host before anything is launched; a
 *     bad argument returns the matching HQ_ERR_* and launches nothing.
 *   - Tensors are row-major and dense (no strides).
 *   - Packed codes: two 4-bit two's-complement codes per byte; element 2j of a
 *     row sits in bits 0..3 of byte j and element 2j+1 in bits 4..7.  3-bit
 *     codes are stored sign-extended in the same 4-bit container.
 *   - Scales use the orthonormal convention H_k = 2^{-k/2} H_k^raw, so that
 *     acc * x_scale * w_scale needs no further factor (the paper absorbs
 *     2^{-k/2} into the scales in the same way).
 *   - Rounding is round-half-to-even.  Non-finite inputs are undefined.
 *   - The library is stateless and may be called from several host threads.
 *   - HQ_ERR_LAUNCH reports a launch the HIP runtime refused.  The runtime's per-thread
 *     "last error" is sampled before a call launches anything: an error that the caller's own
 *     earlier HIP calls left pending there is neither reported as the library's nor cleared.
 *   - Size limit of the integer stage: the packed operands are addressed with
 *     32-bit byte offsets.  (rows + image width + 2) * bytes per activation row
 *     and n * taps * bytes per weight row must stay below 2^32 (4 GiB of codes
 *     per operand); a larger call returns HQ_ERR_UNSUPPORTED and launches nothing.
 */
#ifndef HQ_H
#define HQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    HQ_OK = 0,
    HQ_ERR_NULL = 1,        /* a required pointer is NULL */
    HQ_ERR_SHAPE = 2,       /* a size is non-positive, odd where even is needed, or k % had_block != 0 */
    HQ_ERR_DTYPE = 3,       /* dtype enum not valid for this argument */
    HQ_ERR_BITS = 4,        /* unsupported bit width */
    HQ_ERR_ALIGN = 5,       /* pointer not 16-byte aligned */
    HQ_ERR_UNSUPPORTED = 6, /* valid in principle, not built (e.g. stride 3, a 5x5 window) or beyond the size limit below */
    HQ_ERR_LAUNCH = 7       /* the HIP runtime refused the launch */
} hq_status;

typedef enum {
    HQ_F16 = 0, /* IEEE half */
    HQ_F32 = 1, /* IEEE single */
    HQ_I32 = 2  /* raw int32 accumulators: outputs of the integer stage only */
} hq_dtype;

/* Static, NUL-terminated description of a status code. */
const char *hq_status_string(hq_status s);

/*
 * Offline weight preparation.  (Method, "Matrix Multiplication" for the
 * block-diagonal H; "Single Hadamard Transformation" for the offline
 * quantisation of the transformed weights.)
 *
 *   w        [n_out, taps, k_in] of w_dtype (HQ_F16 | HQ_F32); taps = 1 for a
 *            linear layer y = x W^T with W [n_out, k_in], taps = R*S for a
 *            convolution stored [Cout, R, S, Cin].
 *   had_block power of two in 1..128 dividing k_in; the transform runs along
 *            k_in inside every (n_out, tap) row; 1 means H = I.
 *   w_bits   4 (codes in [-8, 7]), 3, 2 (codes in [-2, 1]; both in the 4-bit container), or 8
 *            (codes in [-128, 127], ONE int8 code per byte:
 *            wq is then [n_out, taps, k_in] bytes; see the 8-bit section below).
 *   wq       out, [n_out, taps, k_in / 2] packed codes.
 *   w_scale  out, [n_out] fp32: max |transformed row over all taps| / (2^(w_bits-1) - 1),
 *            1.0 for an all-zero channel.
 */
hq_status hq_quantize_weights(const void *w, hq_dtype w_dtype, int n_out, int taps, int k_in,
                              int had_block, int w_bits, uint8_t *wq, float *w_scale,
                              void *stream);

/*
 * Online activation path: block Hadamard over the channel axis fused with
 * per-token symmetric quantisation.  (Method, "Matrix Multiplication";
 * Background, "Model Quantization".)
 *
 *   x        [m, k] of x_dtype (HQ_F16 | HQ_F32).  NHWC activations are passed
 *            with m = N*H*W and k = C.
 *   had_block power of two in 1..128 dividing k; k must be a multiple of 8.
 *   a_bits   4 (codes in [-8, 7]), 3 (codes in [-4, 3]), 2 (codes in [-2, 1]), or 8 (codes in [-128, 127], ONE int8
 *            code per byte: xq is then [m, k] bytes; see the 8-bit section below).
 *   xq       out, [m, k / 2] packed codes.
 *   x_scale  out, [m] fp32: max |transformed token| / (2^(a_bits-1) - 1), 1.0 for an
 *            all-zero token.
 */
hq_status hq_act_hadamard_quant(const void *x, hq_dtype x_dtype, int64_t m, int k,
                                int had_block, int a_bits, uint8_t *xq, float *x_scale,
                                void *stream);

/*
 * Integer linear layer with dequantising epilogue.  (Method, linear-layer
 * equation: only an integer matrix product between the quantised operands,
 * then the product of scales.)
 *
 *   acc[i, j] = sum_c xq[i, c] * wq[j, c]                       (int32)
 *   y[i, j]   = acc[i, j] * x_scale[i] * w_scale[j] + bias[j]   (fp32, cast to y_dtype)
 *
 *   xq [m, k/2], x_scale [m], wq [n, k/2], w_scale [n]; bias [n] of y_dtype or
 *   NULL; k a multiple of 8 (multiples of 64 take the fast kernels; any other multiple of 8, e.g.
 *   the few channels of a layer that keeps H = I, takes a small general kernel), k < 131072; y [m, n].
 *   y_dtype == HQ_I32 writes acc itself (bias and scales ignored; they may be NULL).
 */
hq_status hq_int_linear(const uint8_t *xq, const float *x_scale, const uint8_t *wq,
                        const float *w_scale, const void *bias, int64_t m, int n, int k,
                        void *y, hq_dtype y_dtype, void *stream);

/*
 * Integer NHWC convolution (implicit GEMM) with dequantising epilogue.
 * (Method, "Convolution": integer convolution of the quantised operands, then
 * the product of scales.)  Every input pixel carries its own scale, so the
 * integer sum is kept per kernel tap t = (r, s) and the taps are combined in
 * fp32, in the order t = 0 .. R*S-1:
 *
 *   acc_t[b, p, q, co] = sum_ci xq[b, stride p + r - pad, stride q + s - pad, ci] * wq[co, r, s, ci]
 *   y[b, p, q, co]     = w_scale[co] * sum_t x_scale[b, stride p + r - pad, stride q + s - pad] * acc_t
 *                        + bias[co]
 *
 *   A tap outside the image contributes 0.
 *   xq [nb, h, w, c_in/2], x_scale [nb, h, w], wq [c_out, R, S, c_in/2],
 *   w_scale [c_out], bias [c_out] of y_dtype or NULL, y [nb, h_out, w_out, c_out].
 *   Built: R = S in {1, 3}, stride 1, pad (R-1)/2 (h_out = h, w_out = w), and the
 *   downsampling form R = S = 3, stride 2, pad 1 (h_out = (h-1)/2 + 1,
 *   w_out = (w-1)/2 + 1); anything else returns HQ_ERR_UNSUPPORTED.
 *   c_in a multiple of 8 at stride 1 (multiples of 64 take the fast kernels), a multiple of 64 at stride 2.
 *   y_dtype == HQ_I32 writes the per-tap accumulators [nb, h_out, w_out, R*S, c_out].
 */
hq_status hq_int_conv2d(const uint8_t *xq, const float *x_scale, const uint8_t *wq,
                        const float *w_scale, const void *bias, int nb, int h, int w,
                        int c_in, int c_out, int r, int s, int stride, int pad,
                        void *y, hq_dtype y_dtype, void *stream);

/*
 * The whole layer in one launch (3x3 convolution): hq_act_hadamard_quant followed by
 * hq_int_conv2d, with the activation codes kept on chip.  (Method, "Matrix Multiplication": the
 * transformed activations X H are only ever consumed by the integer product; Method,
 * "Convolution".)  Every workgroup transforms and quantises the rows of its own pixel tile and of
 * the pixels one image row and one pixel either side of it, with the arithmetic of
 * hq_act_hadamard_quant, so codes, scales and results are those of the two calls in sequence.
 *
 *   x        [nb, h, w, c_in] of x_dtype; wq [c_out, 3, 3, c_in/2], w_scale [c_out], bias [c_out] of
 *            y_dtype or NULL, y [nb, h, w, c_out] (y_dtype == HQ_I32: per-tap sums [nb, h, w, 9, c_out]).
 *   xq_out   NULL, or out [nb, h, w, c_in/2]: the activation codes the kernel used (for inspection).
 *   x_scale_out  NULL, or out [nb, h, w] fp32: the scales it used.
 *   Built: x_dtype HQ_F16, had_block 64, a_bits 2..4, R = S = 3, stride 1, pad 1, c_in a multiple of
 *   192 and small enough for a tile's activations to fit on chip (c_in <= 576 for 16-pixel-wide images,
 *   fewer channels for wider ones); anything else returns HQ_ERR_UNSUPPORTED (use the two calls).
 */
hq_status hq_act_quant_int_conv2d(const void *x, hq_dtype x_dtype, const uint8_t *wq,
                                  const float *w_scale, const void *bias, int nb, int h, int w,
                                  int c_in, int c_out, int r, int s, int stride, int pad,
                                  int had_block, int a_bits, void *y, hq_dtype y_dtype,
                                  uint8_t *xq_out, float *x_scale_out, void *stream);

/*
 * The same for a linear layer / 1x1 convolution (m = N*H*W rows): hq_act_hadamard_quant followed by
 * hq_int_linear in one launch, codes and scales identical to those of the two calls.  (Method,
 * "Matrix Multiplication".)  Such layers are bound by reading their input and writing their output;
 * the single launch saves the round trip of the codes and one launch.
 *
 *   x [m, k] of x_dtype; wq [n, k/2], w_scale [n], bias [n] of y_dtype or NULL; y [m, n]
 *   (y_dtype == HQ_I32: the int32 sums).  xq_out NULL or out [m, k/2]; x_scale_out NULL or out [m].
 *   Built: x_dtype HQ_F16, had_block 64, a_bits 2..4, k a multiple of 64 up to 1024; anything else
 *   returns HQ_ERR_UNSUPPORTED (use the two calls).
 */
hq_status hq_act_quant_int_linear(const void *x, hq_dtype x_dtype, const uint8_t *wq,
                                  const float *w_scale, const void *bias, int64_t m, int n, int k,
                                  int had_block, int a_bits, void *y, hq_dtype y_dtype,
                                  uint8_t *xq_out, float *x_scale_out, void *stream);

/*
 * Diagnostic: the kernel family that hq_int_conv2d (static_scale = 0) or hq_int_conv2d_static
 * (static_scale = 1) runs for a convolution of this geometry on the current device, for 4-bit
 * (bits = 4) or 8-bit (bits = 8, hq_int_conv2d_i8) codes.  The choice depends on the geometry
 * only, never on y_dtype: the HQ_I32 outputs (raw integer sums) come from the same kernel as the
 * floating-point outputs.  Host logic only; returns a static string: "tile", "tile (stride 2)",
 * "wave-split", "activation-resident", "activation-resident-int8 (P pixels)" with P = 256, 128 or 64
 * (the pixel tile of a workgroup; "128 pixels, 4 waves" for the four-wave form), "small-channel-count"
 * (c_in not a multiple of 64), or "unsupported".
 */
const char *hq_int_conv2d_kernel_name(int nb, int h, int w, int c_in, int c_out, int r, int s,
                                      int stride, int pad, int static_scale, int bits);

/*
 * ---- Static activation scale -------------------------------------------------
 *
 * The paper's own quantiser uses a learned scale S that is a property of the
 * tensor, one per denoising timestep (Background, "Model Quantization"; Method,
 * timestep-indexed quantisation parameters), not a value derived from the data.
 * The three calls below are the layer with such a scale: x_scale is a DEVICE
 * pointer to ONE positive fp32 (4-byte aligned) that the caller selects per
 * timestep; it is read when the kernel runs, so a captured launch can be replayed
 * with another value in that memory.  Everything else is as in the dynamic calls.
 */

/*
 * Block Hadamard over the channel axis, then xq = clamp(rne((x H) / x_scale[0]),
 * -2^(a_bits-1), 2^(a_bits-1) - 1).  With a given scale the clamp is active and
 * the most negative code is reachable.  Writes xq [m, k/2] only.
 */
hq_status hq_act_hadamard_quant_static(const void *x, hq_dtype x_dtype, int64_t m, int k,
                                       int had_block, int a_bits, const float *x_scale,
                                       uint8_t *xq, void *stream);

/*
 * y[i, j] = acc[i, j] * x_scale[0] * w_scale[j] + bias[j], acc as in hq_int_linear.
 */
hq_status hq_int_linear_static(const uint8_t *xq, const float *x_scale, const uint8_t *wq,
                               const float *w_scale, const void *bias, int64_t m, int n, int k,
                               void *y, hq_dtype y_dtype, void *stream);

/*
 * With one scale for the whole activation tensor a convolution is the paper's
 * form (Method, "Convolution"): ONE integer sum over all taps and input channels,
 * then one product of scales:
 *
 *   acc[b, p, q, co] = sum_{r, s, ci} xq[b, p + r - pad, q + s - pad, ci] * wq[co, r, s, ci]
 *   y[b, p, q, co]   = acc * x_scale[0] * w_scale[co] + bias[co]
 *
 * A tap outside the image contributes 0.  Shapes and the built geometries are
 * those of hq_int_conv2d (p, q and the output size follow the stride in the same
 * way); c_in * R * S < 131072.  y_dtype == HQ_I32 writes acc, [nb, h_out, w_out, c_out].
 */
hq_status hq_int_conv2d_static(const uint8_t *xq, const float *x_scale, const uint8_t *wq,
                               const float *w_scale, const void *bias, int nb, int h, int w,
                               int c_in, int c_out, int r, int s, int stride, int pad,
                               void *y, hq_dtype y_dtype, void *stream);

/*
 * ---- Single Hadamard scheme (linear layers) ------------------------------------
 *
 * The paper's own linear layer (Method, linear-layer equation; "Single Hadamard
 * Transformation") quantises the weights WITHOUT the transform and keeps the
 * transform of the contracted axis in the integer domain, between the two
 * quantised operands:
 *
 *   Y ~ S_XH S_W 2^(-k/2) ( (XH)_int  H_raw  W_int^T ),   H_raw = BlockDiag of +-1 blocks.
 *
 * The activation side is hq_act_hadamard_quant unchanged.  The two calls below are
 * the weight side and the integer stage.  A 1x1 convolution is this linear layer
 * with m = N*H*W.
 */

/*
 * Offline: W_int = clamp(rne(W / w_scale)) with w_scale[j] = max |W[j, :]| / (2^(w_bits-1) - 1)
 * (1.0 for an all-zero row), then B = W_int * BlockDiag(H_raw) in exact integers
 * (|B| <= 2^(w_bits-1) * had_block), stored as three signed base-16 digit planes:
 * B = d0 + 16 d1 + 256 d2, every digit in [-8, 7], each plane in the packed-nibble format.
 *
 *   w        [n_out, k_in] of w_dtype (HQ_F16 | HQ_F32), k_in even.
 *   had_block power of two in 1..128 dividing k_in (the block size the activations use).
 *   w_bits   4, 3 or 2.
 *   wq3      out, [n_out, 3, k_in / 2] packed digits, plane p at [:, p, :].
 *   w_scale  out, [n_out] fp32.
 */
hq_status hq_quantize_weights_single(const void *w, hq_dtype w_dtype, int n_out, int k_in,
                                     int had_block, int w_bits, uint8_t *wq3, float *w_scale,
                                     void *stream);

/*
 * Integer stage and dequantisation of the Single scheme:
 *
 *   acc_p[i, j] = sum_c xq[i, c] * d_p[j, c]                      (int32, p = 0, 1, 2)
 *   y[i, j]     = (acc_0 + 16 acc_1 + 256 acc_2) * x_scale[i] * w_scale[j] / sqrt(had_block) + bias[j]
 *
 * acc_0 + 16 acc_1 + 256 acc_2 is the integer (XH)_int H_raw W_int^T of the paper's equation;
 * the three sums are combined in fp32.  Shapes as in hq_int_linear, with wq3 [n, 3, k/2].
 * y_dtype == HQ_I32 writes the three sums, [m, 3, n] (bias and scales ignored).  For floating-point
 * outputs and had_block <= 8 the third plane (zero by construction: |W_int H_raw| <= 64) is not read.
 */
hq_status hq_int_linear_single(const uint8_t *xq, const float *x_scale, const uint8_t *wq3,
                               const float *w_scale, const void *bias, int64_t m, int n, int k,
                               int had_block, void *y, hq_dtype y_dtype, void *stream);

/*
 * ---- Width-axis convolution ----------------------------------------------------
 *
 * The paper's own convolution (Method, "Convolution") reshapes the activations to
 * rows of one image line each, X~ of shape (B C_in h) x w, transforms them along the
 * WIDTH axis with H_c = BlockDiag(H_k) (w x w), quantises with one scale S for the
 * tensor, leaves the weights un-transformed, and convolves in integers:
 *
 *   Y ~ S S_W 2^(-k/2) Conv( (X~ H_c)_int H_c,raw , W_int ).
 *
 * The weight side is hq_quantize_weights with had_block = 1 (no transform).
 */

/*
 * q = clamp(rne((X~ H_c) / x_scale[0]), -2^(a_bits-1), 2^(a_bits-1) - 1), then, in exact
 * integers, u = q * BlockDiag(H_raw) along the width axis (|u| <= 2^(a_bits-1) * had_block),
 * stored as three signed base-16 digit planes, u = d0 + 16 d1 + 256 d2, digits in [-8, 7].
 *
 *   x        [nb, h, w, c] (NHWC) of x_dtype (HQ_F16 | HQ_F32), c even.
 *   had_block power of two in 1..64 dividing w.
 *   x_scale  DEVICE pointer to one positive fp32, read when the kernel runs.
 *   xu3      out, [3, nb, h, w, c / 2] packed digits: plane p is an NHWC tensor of packed nibbles.
 */
hq_status hq_act_hadamard_quant_width(const void *x, hq_dtype x_dtype, int nb, int h, int w, int c,
                                      int had_block, int a_bits, const float *x_scale,
                                      uint8_t *xu3, void *stream);

/*
 *   acc[b, p, q, co] = sum_{r, s, ci} u[b, p + r - pad, q + s - pad, ci] * wq[co, r, s, ci]   (int32, exact)
 *   y[b, p, q, co]   = acc * x_scale[0] * w_scale[co] / sqrt(had_block) + bias[co]
 *
 * with u the integers held by the three planes of xu3 (one integer sum per plane, combined
 * as acc_0 + 16 acc_1 + 256 acc_2).  A tap outside the image contributes 0.
 *   xu3 [3, nb, h, w, c_in/2], wq [c_out, 3, 3, c_in/2] (codes of the un-transformed weights),
 *   w_scale [c_out], bias [c_out] of y_dtype or NULL, y [nb, h, w, c_out].
 * Built: R = S = 3, pad 1, stride 1 (y [nb, h, w, c_out]) or stride 2 (y [nb, (h-1)/2 + 1, (w-1)/2 + 1, c_out],
 * the window of output (p, q) centred on input (2p, 2q)); c_in a multiple of 64, 9 c_in < 131072.
 * Up to had_block = 8 the third digit plane is zero by construction and is not read.
 * y_dtype == HQ_I32 writes acc, [nb, h_out, w_out, c_out].
 */
hq_status hq_int_conv2d_width(const uint8_t *xu3, const float *x_scale, const uint8_t *wq,
                              const float *w_scale, const void *bias, int nb, int h, int w,
                              int c_in, int c_out, int r, int s, int stride, int pad,
                              int had_block, void *y, hq_dtype y_dtype, void *stream);

/*
 * ---- 8-bit codes (W8A8) ---------------------------------------------------------
 *
 * The same layer at 8 bits for both operands (the paper's higher-precision setting;
 * Background, "Model Quantization" with N = 8): hq_act_hadamard_quant and
 * hq_quantize_weights with a_bits = w_bits = 8 write one int8 code per byte (xq [m, k],
 * wq [n_out, taps, k_in]); the two calls below take such codes.  The codes feed the int8
 * matrix instruction as they are.  Everything else (scales, per-tap sums of a convolution,
 * bias, HQ_I32 outputs, error behaviour) is as in hq_int_linear / hq_int_conv2d, including the
 * built geometries of the convolution (R = S in {1, 3} at stride 1, pad (R-1)/2; R = S = 3 at
 * stride 2, pad 1); k (c_in) a multiple of 64.
 */
/*
 * Mixed widths (the paper also reports W8A4): the activation path of hq_act_hadamard_quant with
 * codes of a_bits in {3, 4, 8} written one per byte, xq [m, k], whatever a_bits is; such codes
 * go with 8-bit weight codes into the two calls below.
 */
hq_status hq_act_hadamard_quant_i8(const void *x, hq_dtype x_dtype, int64_t m, int k, int had_block,
                                   int a_bits, int8_t *xq, float *x_scale, void *stream);

hq_status hq_int_linear_i8(const int8_t *xq, const float *x_scale, const int8_t *wq,
                           const float *w_scale, const void *bias, int64_t m, int n, int k,
                           void *y, hq_dtype y_dtype, void *stream);

hq_status hq_int_conv2d_i8(const int8_t *xq, const float *x_scale, const int8_t *wq,
                           const float *w_scale, const void *bias, int nb, int h, int w,
                           int c_in, int c_out, int r, int s, int stride, int pad,
                           void *y, hq_dtype y_dtype, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* HQ_H */
