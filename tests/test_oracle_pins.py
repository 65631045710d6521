"""Pins for the CPU oracle: identities, the paper's worked examples, library
routines and brute force that the oracle must agree with.  None of these
re-states the oracle's own formulas; a dropped term, a wrong sign or index, or a
transposed operand in the oracle fails at least one of them.  CPU only."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def sylvester_closed_form(n):
    """Entry (i, j) of the natural-order +-1 matrix is (-1)^popcount(i & j)."""
    i = np.arange(n)
    pc = np.vectorize(lambda v: bin(v).count("1"))(i[:, None] & i[None, :])
    return np.where(pc % 2 == 0, 1.0, -1.0)


# ---- H itself (Background, "Hadamard Transformation") -------------------------------------

@pytest.mark.parametrize("n", [1, 2, 4, 8, 64, 128])
def test_hraw_orthogonal_symmetric_natural_order(n):
    h = oracle.hadamard_raw(n)
    assert set(np.unique(h)) <= {-1.0, 1.0}
    assert np.array_equal(h @ h.T, n * np.eye(n))          # H_raw H_raw^T = n I, exactly
    assert np.array_equal(h, h.T)
    assert np.array_equal(h, sylvester_closed_form(n))      # Sylvester (natural) ordering


@pytest.mark.parametrize("k", [64, 192, 256, 384, 576, 960])
def test_block_diag_orthonormal(k):
    """H H^T = I and H = H^T for the block-diagonal embedding (Method, "Matrix Multiplication")."""
    h = oracle.block_hadamard(np.eye(k), 64)                # rows of the embedded H
    assert np.allclose(h @ h.T, np.eye(k), atol=1e-15)
    assert np.array_equal(h, h.T)
    off = h.copy()
    for b in range(0, k, 64):
        off[b:b + 64, b:b + 64] = 0
    assert not off.any()                                    # nothing leaks across blocks


def test_involution_and_norm():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((37, 384))
    xt = oracle.block_hadamard(x, 64)
    assert np.allclose(oracle.block_hadamard(xt, 64), x, atol=1e-12)     # X H H = X
    assert np.allclose(np.linalg.norm(xt, axis=1), np.linalg.norm(x, axis=1), rtol=1e-13)


def test_golden_worked_examples():
    with open(os.path.join(GOLDEN, "hadamard_worked_examples.json")) as f:
        gold = json.load(f)

    def vec(spec, n):
        if spec["kind"] == "one_hot":
            v = np.zeros(n)
            v[spec["index"]] = spec["value"]
            return v
        return np.full(n, spec["value"])

    for ex in gold["examples"]:
        n = 2 ** ex["k"]
        got = oracle.block_hadamard(vec(ex["input"], n)[None, :], n)[0]
        assert np.allclose(got, vec(ex["expected"], n), atol=1e-14), ex["cite"]


@pytest.mark.parametrize("bits,qmax", [(4, 7), (3, 3), (8, 127)])
def test_one_hot_codes(bits, qmax):
    """a e_i in one block -> x' = (a/8) Hraw[i, :], so s = |a| / (8 qmax) and every
    code is +-qmax with the sign pattern of row i."""
    hcf = sylvester_closed_form(64)
    for i, a in [(0, 3.0), (5, -2.5), (63, 0.75)]:
        x = np.zeros((1, 192))
        x[0, 64 + i] = a
        q, s, _ = oracle.act_hadamard_quant(x, 64, bits)
        assert s[0] == pytest.approx(abs(a) / (8 * qmax), rel=1e-15)
        assert np.array_equal(q[0, 64:128], (np.sign(a) * qmax * hcf[i]).astype(np.int8))
        assert not q[0, :64].any() and not q[0, 128:].any()


@pytest.mark.parametrize("bits,qmax", [(4, 7), (3, 3), (8, 127)])
def test_constant_vector_codes(bits, qmax):
    """c 1_64 -> (8c, 0, ..., 0): one spike, the paper's own counter-example."""
    c = -0.3
    q, s, _ = oracle.act_hadamard_quant(np.full((1, 64), c), 64, bits)
    assert s[0] == pytest.approx(8 * abs(c) / qmax, rel=1e-15)
    assert q[0, 0] == -qmax and not q[0, 1:].any()


# ---- quantiser (Background, "Model Quantization") ----------------------------------------

def test_round_half_to_even_and_range():
    # abs-max 7 gives scale exactly 1, so the codes are the rounded inputs themselves
    x = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 6.5, -6.5, 3.49, -3.51, 0.0]])
    q, s, t = oracle.quantize_rows(x, 4)
    assert s[0] == 1.0 and np.array_equal(t, x)
    assert q[0].tolist() == [7, 0, 2, 2, 0, -2, -2, 6, -6, 3, -4, 0]
    x3 = np.array([[3.0, 0.5, 1.5, 2.5, -2.5, -0.5]])     # abs-max 3 -> scale 1 at 3 bits
    q3, s3, _ = oracle.quantize_rows(x3, 3)
    assert s3[0] == 1.0 and q3[0].tolist() == [3, 0, 2, 2, -2, 0]


def test_zero_row_scale_is_one():
    q, s, _ = oracle.act_hadamard_quant(np.zeros((2, 64)), 64, 4)
    assert np.array_equal(s, [1.0, 1.0]) and not q.any()


@pytest.mark.parametrize("bits", [3, 4, 8])
def test_error_bound_half_step(bits):
    """No clipping with an abs-max scale, so |x' - s q| <= s / 2 everywhere."""
    layer = workloads.tiny_layers()[0]
    x = workloads.make_x(layer)
    xt = oracle.block_hadamard(x, 64)
    q, s, _ = oracle.quantize_rows(xt, bits)
    qmax = 2 ** (bits - 1) - 1
    assert np.abs(q).max() == qmax and q.min() >= -qmax
    assert np.all(np.abs(xt - s[:, None] * q) <= s[:, None] * (0.5 + 1e-12))
    # and the scale is the abs-max one: some element of every row sits exactly at +-qmax
    assert np.all(np.abs(q).max(axis=1) == qmax)


def test_scaling_and_permutation_invariance():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((16, 128))
    q, s, _ = oracle.act_hadamard_quant(x, 64, 4)
    q2, s2, _ = oracle.act_hadamard_quant(x * 8.0, 64, 4)    # power of two: exact
    assert np.array_equal(q, q2) and np.array_equal(s2, s * 8.0)
    perm = rng.permutation(16)
    qp, sp, _ = oracle.act_hadamard_quant(x[perm], 64, 4)
    assert np.array_equal(qp, q[perm]) and np.array_equal(sp, s[perm])


# ---- weights ------------------------------------------------------------------------------

def test_weight_scale_is_per_output_channel_over_all_taps():
    rng = np.random.default_rng(4)
    w = rng.standard_normal((5, 9, 128)) * 0.02
    wq, sw, _ = oracle.quantize_weights(w, 64, 4)
    wt = oracle.block_hadamard(w, 64)                        # pinned above
    assert np.allclose(sw, np.abs(wt).reshape(5, -1).max(axis=1) / 7, rtol=1e-15)
    assert np.all(np.abs(wt - sw[:, None, None] * wq) <= sw[:, None, None] * (0.5 + 1e-12))
    assert np.all(np.abs(wq).reshape(5, -1).max(axis=1) == 7)


# ---- the layer as a whole -----------------------------------------------------------------

def test_pre_quantisation_identity():
    """(X H)(W H)^T = X W^T: H acts on the contracted axis (Method, linear-layer identity)."""
    rng = np.random.default_rng(5)
    x, w = rng.standard_normal((33, 192)), rng.standard_normal((21, 192))
    lhs = oracle.block_hadamard(x, 64) @ oracle.block_hadamard(w, 64).T
    assert np.allclose(lhs, x @ w.T, rtol=1e-10, atol=1e-10)


def test_lossless_case_reduces_to_plain_matmul():
    """Choose X' = s Qx and W' = sw Qw with integer Q (and |Q| reaching qmax in every
    row) so that quantisation loses nothing; the whole chain must then equal the
    fp64 product X W^T of the un-transformed tensors."""
    rng = np.random.default_rng(6)
    m, k, n = 19, 192, 23
    qx = rng.integers(-7, 8, (m, k)); qx[:, 0] = 7
    qw = rng.integers(-7, 8, (n, k)); qw[:, 1] = -7
    sxp = 2.0 ** rng.integers(-6, 3, m)
    swp = 2.0 ** rng.integers(-8, -2, n)
    h = np.kron(np.eye(k // 64), sylvester_closed_form(64) / 8.0)
    x = (sxp[:, None] * qx) @ h                              # exact: power-of-two scales
    w = (swp[:, None] * qw) @ h
    bias = rng.standard_normal(n)
    xq, sx, _ = oracle.act_hadamard_quant(x, 64, 4)
    wq, sw, _ = oracle.quantize_weights(w[:, None, :], 64, 4)
    assert np.array_equal(xq, qx) and np.array_equal(wq[:, 0, :], qw)
    acc, y = oracle.int_linear(xq, sx, wq[:, 0, :], sw, bias)
    assert np.array_equal(acc, qx @ qw.T)
    assert np.allclose(y, x @ w.T + bias, rtol=1e-12, atol=1e-12)


def test_bypass_block_1_is_plain_absmax_quantised_matmul():
    rng = np.random.default_rng(7)
    x, w = rng.standard_normal((12, 40)), rng.standard_normal((9, 40))
    xq, sx, _ = oracle.act_hadamard_quant(x, 1, 4)
    wq, sw, _ = oracle.quantize_weights(w[:, None, :], 1, 4)
    _, y = oracle.int_linear(xq, sx, wq[:, 0, :], sw)
    ax, aw = np.abs(x).max(1, keepdims=True) / 7, np.abs(w).max(1, keepdims=True) / 7
    ref = (np.rint(x / ax) * ax) @ (np.rint(w / aw) * aw).T
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-14)


def test_linear_equals_matmul_of_dequantised_tensors():
    layer = workloads.tiny_layers()[0]
    x, w, b = workloads.make_x(layer), workloads.make_w(layer), workloads.make_bias(layer)
    xq, sx, _ = oracle.act_hadamard_quant(x, 64, 4)
    wq, sw, _ = oracle.quantize_weights(w, 64, 4)
    acc, y = oracle.int_linear(xq, sx, wq[:, 0, :], sw, b)
    assert acc.shape == (layer.m, layer.n_out)               # non-square: catches a transpose
    xh, wh = sx[:, None] * xq, sw[:, None] * wq[:, 0, :]
    assert np.allclose(y, xh @ wh.T + b.astype(np.float64), rtol=1e-12, atol=1e-12)


def direct_conv_taps(xq, wq, stride, pad):
    """Seven nested loops, integer, one accumulator per tap."""
    nb, h, w, cin = xq.shape
    cout, r, s, _ = wq.shape
    ho, wo = (h + 2 * pad - r) // stride + 1, (w + 2 * pad - s) // stride + 1
    acc = np.zeros((nb, ho, wo, r * s, cout), dtype=np.int64)
    for b in range(nb):
        for p in range(ho):
            for q in range(wo):
                for co in range(cout):
                    for i in range(r):
                        for j in range(s):
                            ih, iw = p * stride + i - pad, q * stride + j - pad
                            if 0 <= ih < h and 0 <= iw < w:
                                for c in range(cin):
                                    acc[b, p, q, i * s + j, co] += int(xq[b, ih, iw, c]) * int(wq[co, i, j, c])
    return acc


@pytest.mark.parametrize("ksize,stride,pad", [(3, 1, 1), (3, 2, 1), (3, 1, 0), (1, 1, 0), (3, 2, 0)])
def test_conv_vs_brute_force_and_library(ksize, stride, pad):
    rng = np.random.default_rng(8 + ksize + 10 * stride + 100 * pad)
    nb, h, w, cin, cout = 2, 5, 6, 64, 3
    x = rng.standard_normal((nb, h, w, cin))
    x[..., 7] *= 20
    wt = rng.standard_normal((cout, ksize * ksize, cin)) * 0.02
    bias = rng.standard_normal(cout) * 0.01
    xq, sx, _ = oracle.act_hadamard_quant(x, 64, 4)
    wq, sw, _ = oracle.quantize_weights(wt, 64, 4)
    wq4 = wq.reshape(cout, ksize, ksize, cin)
    acc, y = oracle.int_conv2d(xq, sx, wq4, sw, bias, stride=stride, pad=pad)
    # integer stage, tap by tap, against the brute-force loops
    assert np.array_equal(acc, direct_conv_taps(xq, wq4, stride, pad))
    # the dequantised result is the ordinary convolution of the dequantised tensors
    xh = torch.from_numpy(sx[..., None] * xq).permute(0, 3, 1, 2)
    wh = torch.from_numpy(sw[:, None, None, None] * wq4).permute(0, 3, 1, 2)
    ref = torch.nn.functional.conv2d(xh, wh, torch.from_numpy(bias), stride=stride, padding=pad)
    assert np.allclose(y, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-13)


def test_conv_pre_quantisation_identity_per_tap():
    """Transforming x over Cin and every tap of w over Cin leaves the convolution
    unchanged, for any stride / padding (H acts on the contracted axis, 0 H = 0)."""
    rng = np.random.default_rng(9)
    x = torch.from_numpy(rng.standard_normal((1, 6, 7, 128)))
    w = torch.from_numpy(rng.standard_normal((4, 3, 3, 128)))
    xt = torch.from_numpy(oracle.block_hadamard(x.numpy(), 64))
    wt = torch.from_numpy(oracle.block_hadamard(w.numpy(), 64))
    f = lambda a, b: torch.nn.functional.conv2d(a.permute(0, 3, 1, 2), b.permute(0, 3, 1, 2),
                                                stride=2, padding=1)
    assert torch.allclose(f(xt, wt), f(x, w), rtol=1e-10, atol=1e-10)


# ---- the paper's qualitative claims on the synthetic stand-in data -------------------------

def test_outlier_spread_shrinks_after_transform():
    """max|x| / RMS(x) per token drops after H on activations with a few heavy
    channels (the claim of the Method section's opening and of the outlier figure)."""
    layer = workloads.config_layers(1)[0]
    x = workloads.make_x(layer).astype(np.float64)
    xt = oracle.block_hadamard(x, 64)
    spread = lambda a: np.abs(a).max(axis=1) / np.sqrt((a * a).mean(axis=1))
    assert spread(xt).mean() < 0.5 * spread(x).mean()


@pytest.mark.parametrize("cfg", [1])
def test_transform_improves_sqnr(cfg):
    """W4A4 output error against the fp64 layer is smaller with the block-64
    transform than with H = I on outlier-heavy activations."""
    layer = workloads.config_layers(cfg)[0]
    x = workloads.make_x(layer).astype(np.float64)
    w = workloads.make_w(layer).astype(np.float64)
    ref = x @ w[:, 0, :].T

    def sqnr(block):
        xq, sx, _ = oracle.act_hadamard_quant(x, block, 4)
        wq, sw, _ = oracle.quantize_weights(w, block, 4)
        _, y = oracle.int_linear(xq, sx, wq[:, 0, :], sw)
        return 10 * np.log10((ref ** 2).sum() / ((y - ref) ** 2).sum())

    assert sqnr(64) > sqnr(1) + 3.0


# ---- the input recipe ---------------------------------------------------------------------

def test_workload_recipe_counts_and_determinism():
    want = {192: 2, 384: 4, 576: 6, 960: 10}
    for layer in workloads.config_layers(5):
        assert layer.n_outlier_channels() == want[layer.k_in]
    c4 = workloads.config_layers(4)
    assert [l.n_outlier_channels() for l in c4] == [5, 5] and c4[0].a_bits == 3
    assert workloads.config_layers(1)[0].n_outlier_channels() == 4
    assert sum(l.ops for l in workloads.config_layers(5)) == pytest.approx(150.9e9, rel=2e-3)
    t = workloads.tiny_layers()[3]
    assert np.array_equal(workloads.make_x(t), workloads.make_x(t))
    x = workloads.make_x(t).astype(np.float64)
    rms = np.sqrt((x.reshape(-1, t.k_in) ** 2).mean(axis=0))
    assert (rms > 10).sum() == t.n_outlier_channels()


# ---- static mode: one caller-supplied activation scale (the paper's learned, per-timestep S) ----

def test_static_quantiser_clamps_and_rounds_to_even():
    # Background, "Model Quantization": x_int = clamp(round(x / S), min, max)
    s = 0.25
    xt = np.array([0.0, 0.125, 0.375, -0.125, -0.375, 0.625, 1.74, 1.76, 5.0, -1.99, -2.2, -50.0, 1e9]) 
    q, t = oracle.quantize_static(xt, 4, s)
    #   t =     0    0.5    1.5    -0.5   -1.5    2.5   6.96  7.04   20    -7.96  -8.8   -200   4e9
    assert q.tolist() == [0, 0, 2, 0, -2, 2, 7, 7, 7, -8, -8, -8, 7]
    assert np.allclose(t, xt / s)
    q3, _ = oracle.quantize_static(xt, 3, s)
    assert q3.min() == -4 and q3.max() == 3
    with pytest.raises(ValueError):
        oracle.quantize_static(xt, 4, 0.0)


def test_static_equals_dynamic_when_given_the_dynamic_scale():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((1, 128)).astype(np.float32)
    q_dyn, s_dyn, t_dyn = oracle.act_hadamard_quant(x, 64, 4)
    q_st, t_st = oracle.act_hadamard_quant_static(x, 64, 4, float(s_dyn[0]))
    assert np.array_equal(q_dyn, q_st) and np.array_equal(t_dyn, t_st)


def test_static_one_hot_saturates_at_both_ends():
    # e_i H = row i of H, entries +-1/8 for block 64: with S = 1/64 every |t| is 8, so the codes
    # are +7 (clamped) where H is positive and -8 (reachable only with a static scale) elsewhere
    x = np.zeros((1, 64)); x[0, 5] = 1.0
    q, t = oracle.act_hadamard_quant_static(x, 64, 4, 1.0 / 64)
    h = oracle.hadamard_raw(64)[5]
    assert np.allclose(np.abs(t), 8.0)
    assert np.array_equal(q[0], np.where(h > 0, 7, -8))


def test_static_linear_is_matmul_of_dequantised_tensors():
    rng = np.random.default_rng(12)
    x = rng.standard_normal((9, 128)); w = rng.standard_normal((5, 1, 128)) * 0.02
    bias = rng.standard_normal(5) * 0.01
    sx = 0.05
    xq, _ = oracle.act_hadamard_quant_static(x, 64, 4, sx)
    wq, sw, _ = oracle.quantize_weights(w, 64, 4)
    acc, y = oracle.int_linear_static(xq, sx, wq[:, 0, :], sw, bias)
    assert np.array_equal(acc, xq.astype(np.int64) @ wq[:, 0, :].astype(np.int64).T)
    ref = (sx * xq.astype(np.float64)) @ (sw[:, None] * wq[:, 0, :]).T + bias
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("ksize,stride,pad", [(3, 1, 1), (3, 2, 1), (3, 1, 0), (1, 1, 0)])
def test_static_conv_vs_brute_force_and_library(ksize, stride, pad):
    rng = np.random.default_rng(13 + ksize + stride + pad)
    nb, h, w, cin, cout = 2, 5, 6, 8, 3
    xq = rng.integers(-8, 8, (nb, h, w, cin)).astype(np.int8)
    wq = rng.integers(-8, 8, (cout, ksize, ksize, cin)).astype(np.int8)
    sw = rng.uniform(0.5, 1.5, cout); bias = rng.standard_normal(cout); sx = 0.37
    acc, y = oracle.int_conv2d_static(xq, sx, wq, sw, bias, stride=stride, pad=pad)
    ho, wo = acc.shape[1], acc.shape[2]
    brute = np.zeros((nb, ho, wo, cout), dtype=np.int64)
    for b in range(nb):
        for p in range(ho):
            for q in range(wo):
                for co in range(cout):
                    for kr in range(ksize):
                        for ks in range(ksize):
                            ih, iw = p * stride + kr - pad, q * stride + ks - pad
                            if 0 <= ih < h and 0 <= iw < w:
                                for c in range(cin):
                                    brute[b, p, q, co] += int(xq[b, ih, iw, c]) * int(wq[co, kr, ks, c])
    assert np.array_equal(acc, brute)
    # one sum over taps and channels = the per-tap sums of the dynamic-scale oracle added up
    acc_t, _ = oracle.int_conv2d(xq, np.full((nb, h, w), sx), wq, sw, bias, stride=stride, pad=pad)
    assert np.array_equal(acc, acc_t.sum(axis=3))
    xh = torch.from_numpy(sx * xq.astype(np.float64)).permute(0, 3, 1, 2)
    wh = torch.from_numpy(sw[:, None, None, None] * wq).permute(0, 3, 1, 2)
    ref = torch.nn.functional.conv2d(xh, wh, torch.from_numpy(bias), stride=stride, padding=pad)
    assert np.allclose(y, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)


# ---- Single scheme: un-transformed quantised weights, integer H between the operands ----------

def test_single_integer_stage_against_library_hadamard():
    """(XH)_int H_raw W_int^T against SciPy's Sylvester-ordered Hadamard matrix and NumPy integer
    products, non-square so that a transposed operand or a wrong block offset shows."""
    from scipy.linalg import hadamard
    rng = np.random.default_rng(21)
    m, k, n = 11, 192, 7
    xq = rng.integers(-8, 8, (m, k)).astype(np.int8)
    wq = rng.integers(-8, 8, (n, k)).astype(np.int8)
    for block in (1, 2, 16, 64):
        hb = np.kron(np.eye(k // block, dtype=np.int64), hadamard(block).astype(np.int64))
        want = (xq.astype(np.int64) @ hb) @ wq.astype(np.int64).T
        assert np.array_equal(oracle.int_gemm_single(xq, wq, block), want)
    with pytest.raises(ValueError):
        oracle.int_gemm_single(xq, wq, 128)   # 128 does not divide 192


def test_single_block_1_is_the_plain_quantised_linear():
    rng = np.random.default_rng(22)
    x, w, b = rng.standard_normal((12, 40)), rng.standard_normal((9, 40)), rng.standard_normal(9)
    xq, sx, _ = oracle.act_hadamard_quant(x, 1, 4)
    wq, sw, _ = oracle.quantize_weights_single(w, 4)
    acc1, y1 = oracle.int_linear_single(xq, sx, wq, sw, 1, b)
    acc0, y0 = oracle.int_linear(xq, sx, wq, sw, b)
    assert np.array_equal(acc1, acc0) and np.array_equal(y1, y0)


def test_single_is_matmul_of_dequantised_tensors_through_h():
    """y = (S_x X_int) H (S_w W_int)^T with the orthonormal H: the plain definition of the scheme."""
    layer = workloads.tiny_layers()[0]
    x, w, b = workloads.make_x(layer), workloads.make_w(layer)[:, 0, :], workloads.make_bias(layer)
    xq, sx, _ = oracle.act_hadamard_quant(x, 64, 4)
    wq, sw, _ = oracle.quantize_weights_single(w, 4)
    assert np.array_equal(sw, np.abs(w.astype(np.float64)).max(axis=1) / 7)   # scale of the UN-transformed rows
    acc, y = oracle.int_linear_single(xq, sx, wq, sw, 64, b)
    assert acc.shape == (layer.m, layer.n_out)
    hn = np.kron(np.eye(layer.k_in // 64), sylvester_closed_form(64) / 8.0)
    ref = ((sx[:, None] * xq) @ hn) @ (sw[:, None] * wq).T + b.astype(np.float64)
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_single_lossless_case_reduces_to_plain_matmul():
    """Integer-valued W (times a power of two) and X = (s Qx) H quantise without loss; the scheme
    must then return the fp64 product X W^T of the original tensors."""
    rng = np.random.default_rng(23)
    m, k, n = 17, 128, 21
    qx = rng.integers(-7, 8, (m, k)); qx[:, 3] = -7
    qw = rng.integers(-7, 8, (n, k)); qw[:, 5] = 7
    sxp = 2.0 ** rng.integers(-5, 3, m)
    swp = 2.0 ** rng.integers(-7, -1, n)
    hn = np.kron(np.eye(k // 64), sylvester_closed_form(64) / 8.0)
    x = (sxp[:, None] * qx) @ hn
    w = swp[:, None] * qw
    xq, sx, _ = oracle.act_hadamard_quant(x, 64, 4)
    wq, sw, _ = oracle.quantize_weights_single(w, 4)
    assert np.array_equal(xq, qx) and np.array_equal(wq, qw)
    _, y = oracle.int_linear_single(xq, sx, wq, sw, 64)
    assert np.allclose(y, x @ w.T, rtol=1e-12, atol=1e-12)


def test_single_integer_range_and_transform_helps():
    """|(XH)_int H_raw| <= 8 * block, so the integer sums stay far inside int32; and on data with
    outlier channels the scheme is closer to the fp64 product than quantising without H."""
    layer = workloads.config_layers(2)[0]
    x = workloads.make_x(layer)[:256]
    w = workloads.make_w(layer)[:, 0, :]
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    wq, sw, _ = oracle.quantize_weights_single(w, 4)
    err = {}
    for block in (1, 64):
        xq, sx, _ = oracle.act_hadamard_quant(x, block, 4)
        acc, y = oracle.int_linear_single(xq, sx, wq, sw, block)
        assert np.abs(acc).max() <= 8 * block * 8 * layer.k_in
        err[block] = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert err[64] < 0.8 * err[1]


# ---- width-axis convolution: the paper's own convolution ---------------------------------------

def width_hadamard(w, block, raw):
    """BlockDiag of the Sylvester matrix over an axis of length w, from SciPy."""
    from scipy.linalg import hadamard
    h = hadamard(block).astype(np.float64)
    return np.kron(np.eye(w // block), h if raw else h / np.sqrt(block))


def test_width_quantiser_transforms_along_the_width_axis():
    """x [N, H, W, C]: every (image, line, channel) is one row of X~; the transform mixes pixels of
    a line only, never channels or lines, and the codes are those of the static quantiser."""
    rng = np.random.default_rng(31)
    x = rng.standard_normal((2, 3, 16, 5))
    for block in (1, 4, 16):
        q, t = oracle.act_width_quant_static(x, block, 4, 0.3)
        want_t = np.einsum("nhwc,wv->nhvc", x, width_hadamard(16, block, raw=False)) / 0.3
        assert np.allclose(t, want_t, rtol=1e-12, atol=1e-12)
        assert np.array_equal(q, np.clip(np.rint(want_t), -8, 7).astype(np.int8))
    # a one-hot line becomes a flat +-1 pattern along the width, in its own channel only
    x = np.zeros((1, 1, 8, 3)); x[0, 0, 5, 1] = 8.0
    q, _ = oracle.act_width_quant_static(x, 8, 4, 8.0 / np.sqrt(8) / 7)
    assert np.array_equal(np.abs(q[0, 0, :, 1]), np.full(8, 7)) and not q[..., 0].any() and not q[..., 2].any()


@pytest.mark.parametrize("ksize,stride,pad,block", [(3, 1, 1, 8), (3, 2, 1, 4), (3, 1, 0, 8), (1, 1, 0, 2), (3, 1, 1, 1)])
def test_width_conv_vs_brute_force_and_library(ksize, stride, pad, block):
    """Integer stage against seven nested loops over u = q H_raw (SciPy's matrix), result against
    conv2d of the dequantised tensors S (q H) and S_W W_int."""
    rng = np.random.default_rng(40 + ksize + stride + pad + block)
    nb, h, w, cin, cout = 2, 5, 8, 6, 3
    xq = rng.integers(-8, 8, (nb, h, w, cin)).astype(np.int8)
    wq = rng.integers(-8, 8, (cout, ksize, ksize, cin)).astype(np.int8)
    sw = rng.uniform(0.5, 1.5, cout); bias = rng.standard_normal(cout); sx = 0.21
    acc, y = oracle.int_conv2d_width(xq, sx, wq, sw, block, bias, stride=stride, pad=pad)
    u = np.rint(np.einsum("nhwc,wv->nhvc", xq.astype(np.float64), width_hadamard(w, block, raw=True))).astype(np.int64)
    assert np.abs(u).max() <= 8 * block
    ho, wo = acc.shape[1], acc.shape[2]
    brute = np.zeros((nb, ho, wo, cout), dtype=np.int64)
    for b in range(nb):
        for p in range(ho):
            for q in range(wo):
                for co in range(cout):
                    for kr in range(ksize):
                        for ks in range(ksize):
                            ih, iw = p * stride + kr - pad, q * stride + ks - pad
                            if 0 <= ih < h and 0 <= iw < w:
                                for c in range(cin):
                                    brute[b, p, q, co] += int(u[b, ih, iw, c]) * int(wq[co, kr, ks, c])
    assert np.array_equal(acc, brute)
    xhat = sx * np.einsum("nhwc,wv->nhvc", xq.astype(np.float64), width_hadamard(w, block, raw=False))
    ref = torch.nn.functional.conv2d(torch.from_numpy(xhat).permute(0, 3, 1, 2),
                                     torch.from_numpy(sw[:, None, None, None] * wq).permute(0, 3, 1, 2),
                                     torch.from_numpy(bias), stride=stride, padding=pad)
    assert np.allclose(y, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)


def test_width_conv_block_1_is_the_static_convolution():
    rng = np.random.default_rng(45)
    xq = rng.integers(-8, 8, (2, 4, 6, 8)).astype(np.int8)
    wq = rng.integers(-8, 8, (5, 3, 3, 8)).astype(np.int8)
    sw = rng.uniform(0.5, 1.5, 5)
    a1, y1 = oracle.int_conv2d_width(xq, 0.4, wq, sw, 1, None, stride=1, pad=1)
    a0, y0 = oracle.int_conv2d_static(xq, 0.4, wq, sw, None, stride=1, pad=1)
    assert np.array_equal(a1, a0) and np.array_equal(y1, y0)


def test_width_conv_lossless_case_reduces_to_plain_convolution():
    """X~ H = s Q exactly and integer-valued weights: nothing is lost, so the scheme must return the
    fp64 convolution of the original tensors (strided and padded: H never meets the weights)."""
    rng = np.random.default_rng(46)
    nb, h, w, cin, cout, block = 2, 6, 16, 4, 3, 16
    q = rng.integers(-8, 8, (nb, h, w, cin)).astype(np.float64)
    s = 2.0 ** -3
    x = np.einsum("nhwc,wv->nhvc", s * q, width_hadamard(w, block, raw=False))     # exact: entries +-1/4
    qw = rng.integers(-7, 8, (cout, 3, 3, cin)); qw[:, 0, 0, 0] = 7
    swp = 2.0 ** rng.integers(-6, -1, cout)
    wgt = swp[:, None, None, None] * qw
    xq, _ = oracle.act_width_quant_static(x, block, 4, s)
    assert np.array_equal(xq, q.astype(np.int8))
    wq, sw, _ = oracle.quantize_weights(wgt.reshape(cout, 9, cin), 1, 4)           # block 1: no transform
    assert np.array_equal(wq.reshape(cout, 3, 3, cin), qw)
    for stride, pad in ((1, 1), (2, 1), (1, 0)):
        _, y = oracle.int_conv2d_width(xq, s, wq.reshape(cout, 3, 3, cin), sw, block, None, stride=stride, pad=pad)
        ref = torch.nn.functional.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2),
                                         torch.from_numpy(wgt).permute(0, 3, 1, 2), None, stride=stride, padding=pad)
        assert np.allclose(y, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)
