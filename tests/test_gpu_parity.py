"""Parity of the HIP library against the CPU oracle, element by element, on the
same seeded stored tensors.  Every call goes through the C ABI (via the ctypes
binding).  Three layers of checks per layer of a workload:

  (i)   codes and scales of both quantisers against the oracle's: scales to
        1e-6 relative, codes identical except where the oracle's pre-rounding
        value is within 1e-5 of a tie (then off by at most one);
  (ii)  the integer stage fed the ORACLE's codes: int32 sums bit-equal to the
        oracle's int64 sums (per tap for a convolution);
  (iii) the whole chain on the GPU against the oracle's fp64 result within
        max|y - ref| / max|ref| <= 2e-3.  If (i) found codes that legitimately
        differ at a tie, the oracle's integer + dequantisation stages are re-run
        on the validated GPU codes (with the oracle's own fp64 scales), since a
        single flipped code moves a whole output row by more than the tolerance.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from parity_util import (check_codes, check_scales, check_y, pack_codes, unpack_codes)

pytestmark = pytest.mark.gpu

TORCH_DT = {"f16": torch.float16, "f32": torch.float32}


@pytest.fixture(scope="module")
def hq():
    import paper_2512_05746_amd as lib
    lib.load_library()
    return lib


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def run_layer(hq, layer, block=workloads.HAD_BLOCK):
    print("layer", layer.name, layer.kind, layer.x_shape, "->", layer.n_out, flush=True)
    x, w, bias = workloads.make_x(layer), workloads.make_w(layer), workloads.make_bias(layer)
    ydt = TORCH_DT[layer.dtype]

    # oracle, stages S0..S3
    xq_o, sx_o, tx = oracle.act_hadamard_quant(x, block, layer.a_bits)
    wq_o, sw_o, tw = oracle.quantize_weights(w, block, layer.w_bits)

    # (i) quantisers
    xq_g, sx_g = hq.hq_act_hadamard_quant(dev(x), block, layer.a_bits)
    wq_g, sw_g = hq.hq_quantize_weights(dev(w), block, layer.w_bits)
    xq_gc, wq_gc = unpack_codes(host(xq_g)), unpack_codes(host(wq_g))
    check_scales(layer.name + " x_scale", host(sx_g), sx_o)
    check_scales(layer.name + " w_scale", host(sw_g), sw_o)
    flips = check_codes(layer.name + " xq", xq_gc, xq_o, tx, layer.a_bits)
    flips += check_codes(layer.name + " wq", wq_gc, wq_o, tw, layer.w_bits)

    # (ii) integer stage on the oracle's codes, (iii) whole chain
    xq_od, wq_od = dev(pack_codes(xq_o)), dev(pack_codes(wq_o))
    bias_d = dev(bias) if bias is not None else None
    if layer.kind == "linear":
        acc_o, y_o = oracle.int_linear(xq_o, sx_o, wq_o[:, 0, :], sw_o, bias)
        acc_g = host(hq.hq_int_linear(xq_od, None, wq_od, None, None, y_dtype=torch.int32))
        assert np.array_equal(acc_g, acc_o), layer.name + " int32 sums"
        del acc_g, acc_o
        if flips:
            _, y_o = oracle.int_linear(xq_gc, sx_o, wq_gc[:, 0, :], sw_o, bias)
        y_g = host(hq.hq_int_linear(xq_g, sx_g, wq_g, sw_g, bias_d, y_dtype=ydt))
    else:
        ks = layer.ksize
        wq4 = lambda c: c.reshape(layer.n_out, ks, ks, layer.k_in)
        # the integer output comes from the same kernel as the fp output (the choice has no dtype argument)
        print("   kernel:", hq.hq_int_conv2d_kernel_name(*layer.x_shape, layer.n_out, ksize=ks), flush=True)
        acc_o, y_o = oracle.int_conv2d(xq_o, sx_o, wq4(wq_o), sw_o, bias, stride=1, pad=layer.pad)
        acc_g = host(hq.hq_int_conv2d(xq_od, None, wq_od, None, None, ksize=ks, y_dtype=torch.int32))
        assert np.array_equal(acc_g, acc_o), layer.name + " per-tap int32 sums"
        del acc_g, acc_o
        if flips:
            _, y_o = oracle.int_conv2d(xq_gc, sx_o, wq4(wq_gc), sw_o, bias, stride=1, pad=layer.pad,
                                       want_acc=False)
        y_g = host(hq.hq_int_conv2d(xq_g, sx_g, wq_g, sw_g, bias_d, ksize=ks, y_dtype=ydt))
    err = check_y(layer.name + " y", y_g.reshape(y_o.shape), y_o)
    print("   ok: tie flips %d, y err %.2e" % (flips, err), flush=True)
    return flips, err


def run_layer_static(hq, layer, block=workloads.HAD_BLOCK):
    """The same three layers of checks with ONE caller-supplied activation scale (the paper's
    learned per-timestep scale): active clamp, no scale output, and for a 3x3 convolution one
    integer sum over all taps."""
    print("layer (static scale)", layer.name, layer.kind, layer.x_shape, "->", layer.n_out, flush=True)
    x, w, bias = workloads.make_x(layer), workloads.make_w(layer), workloads.make_bias(layer)
    ydt = TORCH_DT[layer.dtype]
    qmax = 2 ** (layer.a_bits - 1) - 1
    # a scale below most tokens' own abs-max scale, so that the clamp is at work
    _, sx_dyn, _ = oracle.act_hadamard_quant(x, block, layer.a_bits)
    s = float(np.float32(0.7 * np.median(sx_dyn)))
    s_d = torch.tensor([s], dtype=torch.float32, device="cuda")

    xq_o, tx = oracle.act_hadamard_quant_static(x, block, layer.a_bits, s)
    assert (tx > qmax + 0.5).any() and (tx < -qmax - 1.5).any(), "the test scale does not clamp"
    wq_o, sw_o, tw = oracle.quantize_weights(w, block, layer.w_bits)

    # (i) the activation quantiser (the weight path is that of the dynamic mode)
    xq_g = hq.hq_act_hadamard_quant_static(dev(x), s_d, block, layer.a_bits)
    xq_gc = unpack_codes(host(xq_g))
    flips = check_codes(layer.name + " xq (static)", xq_gc, xq_o, tx, layer.a_bits)
    assert xq_gc.min() == -qmax - 1 and xq_gc.max() == qmax
    wq_g, sw_g = hq.hq_quantize_weights(dev(w), block, layer.w_bits)
    wq_gc = unpack_codes(host(wq_g))
    check_scales(layer.name + " w_scale", host(sw_g), sw_o)
    flips += check_codes(layer.name + " wq", wq_gc, wq_o, tw, layer.w_bits)

    # (ii) integer stage on the oracle's codes, (iii) whole chain against the oracle's own result
    # (its codes and scales; the GPU's codes only where (i) found legitimate flips at ties)
    xq_od, wq_od = dev(pack_codes(xq_o)), dev(pack_codes(wq_o))
    bias_d = dev(bias) if bias is not None else None
    xq_r, wq_r = (xq_gc, wq_gc) if flips else (xq_o, wq_o)
    if layer.kind == "linear":
        acc_o, _ = oracle.int_linear_static(xq_o, s, wq_o[:, 0, :], sw_o, bias)
        acc_g = host(hq.hq_int_linear_static(xq_od, None, wq_od, None, None, y_dtype=torch.int32))
        assert np.array_equal(acc_g, acc_o), layer.name + " int32 sums (static)"
        _, y_o = oracle.int_linear_static(xq_r, s, wq_r[:, 0, :], sw_o, bias)
        y_g = host(hq.hq_int_linear_static(xq_g, s_d, wq_g, sw_g, bias_d, y_dtype=ydt))
    else:
        ks = layer.ksize
        wq4 = lambda c: c.reshape(layer.n_out, ks, ks, layer.k_in)
        print("   kernel:", hq.hq_int_conv2d_kernel_name(*layer.x_shape, layer.n_out, ksize=ks, static_scale=True),
              flush=True)
        acc_o, _ = oracle.int_conv2d_static(xq_o, s, wq4(wq_o), sw_o, bias, stride=1, pad=layer.pad,
                                            want_y=False)
        acc_g = host(hq.hq_int_conv2d_static(xq_od, None, wq_od, None, None, ksize=ks, y_dtype=torch.int32))
        assert np.array_equal(acc_g, acc_o), layer.name + " int32 sums over all taps (static)"
        _, y_o = oracle.int_conv2d_static(xq_r, s, wq4(wq_r), sw_o, bias, stride=1, pad=layer.pad,
                                          want_acc=False)
        y_g = host(hq.hq_int_conv2d_static(xq_g, s_d, wq_g, sw_g, bias_d, ksize=ks, y_dtype=ydt))
    err = check_y(layer.name + " y (static)", y_g.reshape(y_o.shape), y_o)
    print("   ok: tie flips %d, y err %.2e" % (flips, err), flush=True)
    return flips, err


def digit_planes_to_int(planes):
    """uint8 [n, 3, k/2] signed base-16 digit planes -> int64 [n, k] = d0 + 16 d1 + 256 d2."""
    d = unpack_codes(planes).astype(np.int64)
    return d[:, 0] + 16 * d[:, 1] + 256 * d[:, 2]


def int_to_digit_planes(b):
    """int64 [n, k] -> uint8 [n, 3, k/2]: digits in [-8, 7], least significant plane first."""
    b = b.astype(np.int64)
    d0 = ((b + 8) % 16) - 8
    r = (b - d0) // 16
    d1 = ((r + 8) % 16) - 8
    d2 = (r - d1) // 16
    assert np.abs(d2).max(initial=0) <= 7
    return pack_codes(np.stack([d0, d1, d2], axis=1).astype(np.int8))


def run_linear_single(hq, layer, block=workloads.HAD_BLOCK):
    """The paper's Single scheme on a linear layer: weights quantised without the transform, the
    integer H_raw folded into three digit planes; the same three layers of checks."""
    print("layer (single scheme)", layer.name, layer.x_shape, "->", layer.n_out, "block", block, flush=True)
    x, w, bias = workloads.make_x(layer), workloads.make_w(layer)[:, 0, :], workloads.make_bias(layer)
    x = x.reshape(-1, layer.k_in)
    ydt = TORCH_DT[layer.dtype]
    hb = np.kron(np.eye(layer.k_in // block, dtype=np.int64), np.rint(oracle.hadamard_raw(block)).astype(np.int64))

    xq_o, sx_o, tx = oracle.act_hadamard_quant(x, block, layer.a_bits)
    wq_o, sw_o, tw = oracle.quantize_weights_single(w, layer.w_bits)

    # (i) quantisers: the digit planes must decode to W_int H_raw for a W_int that matches the oracle's
    xq_g, sx_g = hq.hq_act_hadamard_quant(dev(x), block, layer.a_bits)
    wq3_g, sw_g = hq.hq_quantize_weights_single(dev(w), block, layer.w_bits)
    b_g = digit_planes_to_int(host(wq3_g))
    back = b_g @ hb                                          # = block * W_int, H_raw H_raw = block I
    assert (back % block == 0).all(), layer.name + ": planes are not W_int H_raw for any integer W_int"
    wq_gc = (back // block).astype(np.int8)
    xq_gc = unpack_codes(host(xq_g))
    check_scales(layer.name + " x_scale", host(sx_g), sx_o)
    check_scales(layer.name + " w_scale", host(sw_g), sw_o)
    flips = check_codes(layer.name + " xq", xq_gc, xq_o, tx, layer.a_bits)
    flips += check_codes(layer.name + " wq (un-transformed)", wq_gc, wq_o, tw, layer.w_bits)

    # (ii) integer stage on the oracle's codes: the three sums, combined exactly, are the paper's integer
    acc_o, y_o = oracle.int_linear_single(xq_o, sx_o, wq_o, sw_o, block, bias)
    planes_o = dev(int_to_digit_planes(wq_o.astype(np.int64) @ hb))
    acc3 = host(hq.hq_int_linear_single(dev(pack_codes(xq_o)), None, planes_o, None, None, block,
                                        y_dtype=torch.int32)).astype(np.int64)
    assert acc3.shape == (x.shape[0], 3, layer.n_out)
    assert np.array_equal(acc3[:, 0] + 16 * acc3[:, 1] + 256 * acc3[:, 2], acc_o), layer.name + " integer sums"
    del acc3, acc_o

    # (iii) whole chain
    if flips:
        _, y_o = oracle.int_linear_single(xq_gc, sx_o, wq_gc, sw_o, block, bias)
    bias_d = dev(bias) if bias is not None else None
    y_g = host(hq.hq_int_linear_single(xq_g, sx_g, wq3_g, sw_g, bias_d, block, y_dtype=ydt))
    err = check_y(layer.name + " y (single)", y_g, y_o)
    print("   ok: tie flips %d, y err %.2e" % (flips, err), flush=True)
    return flips, err


@pytest.mark.parametrize("idx", [0, 1, 2])
def test_single_scheme_tiny_linears(hq, idx):
    run_linear_single(hq, workloads.tiny_layers()[idx])


@pytest.mark.parametrize("block", [1, 4, 8, 16, 128])
def test_single_scheme_other_block_sizes(hq, block):
    """H = I (all higher digits zero), blocks up to 8 (third digit plane zero: its pass is skipped),
    a block just above that, and the largest block (sums up to 8 * 128)."""
    layer = workloads.tiny_layers()[1]          # k = 128, fp32 input
    run_linear_single(hq, layer, block)


def test_single_scheme_extreme_codes(hq):
    """Weight rows of constant sign drive W_int H_raw to +-8 * 64 (third digit +-2); the sums of
    every plane and their combination stay exact."""
    m, n, k = 70, 40, 192
    rng = np.random.default_rng(77)
    xq = rng.integers(-8, 8, (m, k)).astype(np.int8)
    xq[0], xq[1] = 7, -8
    wq = rng.integers(-8, 8, (n, k)).astype(np.int8)
    wq[0], wq[1], wq[2, :64] = -8, 7, -8
    hb = np.kron(np.eye(k // 64, dtype=np.int64), np.rint(oracle.hadamard_raw(64)).astype(np.int64))
    b = wq.astype(np.int64) @ hb
    assert b.min() == -512 and b.max() == 448
    acc3 = host(hq.hq_int_linear_single(dev(pack_codes(xq)), None, dev(int_to_digit_planes(b)), None, None, 64,
                                        y_dtype=torch.int32)).astype(np.int64)
    assert np.array_equal(acc3[:, 0] + 16 * acc3[:, 1] + 256 * acc3[:, 2], oracle.int_gemm_single(xq, wq, 64))


@pytest.mark.parametrize("config", [1, 2])
def test_single_scheme_benchmark_linears_full_size(hq, config):
    for layer in workloads.config_layers(config):
        run_linear_single(hq, layer)


def run_conv_width(hq, layer, block):
    """The paper's width-axis convolution on a 3x3 layer: activations transformed along the width
    axis and quantised with one scale, the codes taken back with the integer H_raw (three digit
    planes), weights quantised without a transform; the same three layers of checks."""
    print("layer (width axis)", layer.name, layer.x_shape, "->", layer.n_out, "block", block, flush=True)
    x, w, bias = workloads.make_x(layer), workloads.make_w(layer), workloads.make_bias(layer)
    nb, h, wd, cin = x.shape
    ydt = TORCH_DT[layer.dtype]
    qmax = 2 ** (layer.a_bits - 1) - 1
    hb = np.kron(np.eye(wd // block, dtype=np.int64), np.rint(oracle.hadamard_raw(block)).astype(np.int64))
    along_w = lambda a: np.einsum("nhwc,wv->nhvc", a, hb)
    # one scale for the tensor, small enough for the clamp to be at work
    xt = oracle.block_hadamard(np.moveaxis(x.astype(np.float64), 2, 3), block)
    s = float(np.float32(np.percentile(np.abs(xt), 99.5) / qmax))
    s_d = torch.tensor([s], dtype=torch.float32, device="cuda")
    wq4 = lambda c: c.reshape(layer.n_out, 3, 3, cin)

    xq_o, tx = oracle.act_width_quant_static(x, block, layer.a_bits, s)
    assert (tx > qmax + 0.5).any() and (tx < -qmax - 1.5).any(), "the test scale does not clamp"
    wq_o, sw_o, tw = oracle.quantize_weights(w, 1, layer.w_bits)

    # (i) quantisers: the planes must decode to q H_raw (along the width) for codes q matching the oracle's
    xu3_g = hq.hq_act_hadamard_quant_width(dev(x), s_d, block, layer.a_bits)
    d = unpack_codes(host(xu3_g)).astype(np.int64)                    # [3, N, H, W, C]
    back = along_w(d[0] + 16 * d[1] + 256 * d[2])                      # = block * q
    assert (back % block == 0).all(), layer.name + ": planes are not q H_raw for any integer q"
    xq_gc = (back // block).astype(np.int8)
    flips = check_codes(layer.name + " xq (width)", xq_gc, xq_o, tx, layer.a_bits)
    wq_g, sw_g = hq.hq_quantize_weights(dev(w), 1, layer.w_bits)
    wq_gc = unpack_codes(host(wq_g))
    check_scales(layer.name + " w_scale", host(sw_g), sw_o)
    flips += check_codes(layer.name + " wq (un-transformed)", wq_gc, wq_o, tw, layer.w_bits)

    # (ii) integer stage on the oracle's codes
    acc_o, y_o = oracle.int_conv2d_width(xq_o, s, wq4(wq_o), sw_o, block, bias, stride=1, pad=1)
    u = along_w(xq_o.astype(np.int64))
    d0 = ((u + 8) % 16) - 8
    r1 = (u - d0) // 16
    d1 = ((r1 + 8) % 16) - 8
    planes_o = dev(pack_codes(np.stack([d0, d1, (r1 - d1) // 16]).astype(np.int8)))
    acc_g = host(hq.hq_int_conv2d_width(planes_o, None, dev(pack_codes(wq_o)), None, None, block, y_dtype=torch.int32))
    assert np.array_equal(acc_g, acc_o), layer.name + " integer sums (width)"
    del acc_g, acc_o, u, d0, d1, r1, d

    # (iii) whole chain
    if flips:
        _, y_o = oracle.int_conv2d_width(xq_gc, s, wq4(wq_gc), sw_o, block, bias, stride=1, pad=1, want_acc=False)
    bias_d = dev(bias) if bias is not None else None
    y_g = host(hq.hq_int_conv2d_width(xu3_g, s_d, wq_g, sw_g, bias_d, block, y_dtype=ydt))
    err = check_y(layer.name + " y (width)", y_g, y_o)
    print("   ok: tie flips %d, y err %.2e" % (flips, err), flush=True)
    return flips, err


@pytest.mark.parametrize("idx,block", [(3, 1), (4, 4), (6, 1), (7, 16), (7, 2), (7, 8)])
def test_width_conv_tiny_layers(hq, idx, block):
    run_conv_width(hq, workloads.tiny_layers()[idx], block)


@pytest.mark.parametrize("config,index,block", [(3, 0, 32), (5, 0, 64), (5, 1, 32), (5, 3, 8)])
def test_width_conv_benchmark_layers_full_size(hq, config, index, block):
    run_conv_width(hq, workloads.config_layers(config)[index], block)


def run_layer_w8a8(hq, layer, block=workloads.HAD_BLOCK):
    """The layer with 8-bit codes for both operands (one int8 code per byte): the same three layers
    of checks as run_layer."""
    print("layer (W8A8)", layer.name, layer.kind, layer.x_shape, "->", layer.n_out, flush=True)
    x, w, bias = workloads.make_x(layer), workloads.make_w(layer), workloads.make_bias(layer)
    ydt = TORCH_DT[layer.dtype]
    xq_o, sx_o, tx = oracle.act_hadamard_quant(x, block, 8)
    wq_o, sw_o, tw = oracle.quantize_weights(w, block, 8)

    xq_g, sx_g = hq.hq_act_hadamard_quant(dev(x), block, 8)
    wq_g, sw_g = hq.hq_quantize_weights(dev(w), block, 8)
    assert xq_g.dtype == torch.int8 and xq_g.shape == x.shape and wq_g.shape == w.shape
    xq_gc, wq_gc = host(xq_g), host(wq_g)
    check_scales(layer.name + " x_scale", host(sx_g), sx_o)
    check_scales(layer.name + " w_scale", host(sw_g), sw_o)
    flips = check_codes(layer.name + " xq", xq_gc, xq_o, tx, 8)
    flips += check_codes(layer.name + " wq", wq_gc, wq_o, tw, 8)

    xq_od, wq_od = dev(xq_o), dev(wq_o)
    bias_d = dev(bias) if bias is not None else None
    if layer.kind == "linear":
        acc_o, y_o = oracle.int_linear(xq_o, sx_o, wq_o[:, 0, :], sw_o, bias)
        acc_g = host(hq.hq_int_linear_i8(xq_od, None, wq_od, None, None, y_dtype=torch.int32))
        assert np.array_equal(acc_g, acc_o), layer.name + " int32 sums (W8A8)"
        del acc_g, acc_o
        if flips:
            _, y_o = oracle.int_linear(xq_gc, sx_o, wq_gc[:, 0, :], sw_o, bias)
        y_g = host(hq.hq_int_linear_i8(xq_g, sx_g, wq_g, sw_g, bias_d, y_dtype=ydt))
    else:
        ks = layer.ksize
        wq4 = lambda c: c.reshape(layer.n_out, ks, ks, layer.k_in)
        acc_o, y_o = oracle.int_conv2d(xq_o, sx_o, wq4(wq_o), sw_o, bias, stride=1, pad=layer.pad)
        acc_g = host(hq.hq_int_conv2d_i8(xq_od, None, wq_od, None, None, ksize=ks, y_dtype=torch.int32))
        assert np.array_equal(acc_g.reshape(acc_o.shape), acc_o), layer.name + " per-tap int32 sums (W8A8)"
        del acc_g, acc_o
        if flips:
            _, y_o = oracle.int_conv2d(xq_gc, sx_o, wq4(wq_gc), sw_o, bias, stride=1, pad=layer.pad, want_acc=False)
        y_g = host(hq.hq_int_conv2d_i8(xq_g, sx_g, wq_g, sw_g, bias_d, ksize=ks, y_dtype=ydt))
    err = check_y(layer.name + " y (W8A8)", y_g.reshape(y_o.shape), y_o)
    print("   ok: tie flips %d, y err %.2e" % (flips, err), flush=True)
    return flips, err


@pytest.mark.parametrize("layer", workloads.tiny_layers(), ids=lambda l: l.name)
def test_w8a8_tiny_layers(hq, layer):
    run_layer_w8a8(hq, layer)


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_w8a8_benchmark_configs_full_size(hq, config):
    for layer in workloads.config_layers(config):
        run_layer_w8a8(hq, layer)


@pytest.mark.parametrize("a_bits", [3, 4])
def test_w8a4_mixed_widths(hq, a_bits):
    """8-bit weights with 4- or 3-bit activation codes stored one per byte (the paper's W8A4)."""
    for layer in (workloads.tiny_layers()[0], workloads.tiny_layers()[4], workloads.config_layers(2)[0]):
        x, w, bias = workloads.make_x(layer), workloads.make_w(layer), workloads.make_bias(layer)
        xq_o, sx_o, tx = oracle.act_hadamard_quant(x, 64, a_bits)
        wq_o, sw_o, tw = oracle.quantize_weights(w, 64, 8)
        xq_g, sx_g = hq.hq_act_hadamard_quant_i8(dev(x), 64, a_bits)
        wq_g, sw_g = hq.hq_quantize_weights(dev(w), 64, 8)
        xq_gc, wq_gc = host(xq_g), host(wq_g)
        check_scales(layer.name + " x_scale", host(sx_g), sx_o)
        flips = check_codes(layer.name + " xq", xq_gc, xq_o, tx, a_bits)
        flips += check_codes(layer.name + " wq", wq_gc, wq_o, tw, 8)
        bias_d = dev(bias) if bias is not None else None
        if layer.kind == "linear":
            _, y_o = oracle.int_linear(xq_gc if flips else xq_o, sx_o, (wq_gc if flips else wq_o)[:, 0, :], sw_o, bias)
            y_g = host(hq.hq_int_linear_i8(xq_g, sx_g, wq_g, sw_g, bias_d, y_dtype=TORCH_DT[layer.dtype]))
        else:
            wq4 = lambda c: c.reshape(layer.n_out, 3, 3, layer.k_in)
            _, y_o = oracle.int_conv2d(xq_gc if flips else xq_o, sx_o, wq4(wq_gc if flips else wq_o), sw_o, bias,
                                       stride=1, pad=1, want_acc=False)
            y_g = host(hq.hq_int_conv2d_i8(xq_g, sx_g, wq_g, sw_g, bias_d, ksize=3, y_dtype=TORCH_DT[layer.dtype]))
        check_y(layer.name + " y (W8A%d)" % a_bits, y_g.reshape(y_o.shape), y_o)


def test_w8a8_extreme_codes(hq):
    """All codes at -128 / 127: the largest sums the int8 path can meet stay exact."""
    m, n, k = 65, 130, 1024
    xq = np.full((m, k), -128, dtype=np.int8); xq[1::2] = 127
    wq = np.full((n, k), -128, dtype=np.int8); wq[::3] = 127
    acc = host(hq.hq_int_linear_i8(dev(xq), None, dev(wq), None, None, y_dtype=torch.int32))
    assert np.array_equal(acc, oracle.int_gemm(xq, wq))


@pytest.mark.parametrize("layer", workloads.tiny_layers(), ids=lambda l: l.name)
def test_tiny_layers(hq, layer):
    run_layer(hq, layer)


@pytest.mark.parametrize("layer", workloads.tiny_layers(), ids=lambda l: l.name)
def test_tiny_layers_static_scale(hq, layer):
    run_layer_static(hq, layer)


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_benchmark_configs_full_size_static_scale(hq, config):
    for layer in workloads.config_layers(config):
        run_layer_static(hq, layer)


@pytest.mark.parametrize("block,dtype,k", [(1, np.float32, 64), (8, np.float16, 264), (32, np.float32, 384),
                                           (64, np.float32, 960), (128, np.float16, 256),
                                           (64, np.float16, 2112), (64, np.float16, 16384)])
def test_act_quant_static_paths(hq, block, dtype, k):
    """Every kernel family of the quantiser with a given scale: butterfly (short and long rows,
    fp32 and fp16, all block sizes) and the matrix-core kernel."""
    rng = np.random.default_rng(300 + block + k)
    x = rng.standard_normal((37, k))
    x[:, 3] *= 20
    x = x.astype(dtype)
    for bits in (3, 4):
        s = 0.4
        q_o, t = oracle.act_hadamard_quant_static(x, block, bits, s)
        q_g = hq.hq_act_hadamard_quant_static(dev(x), torch.tensor([s], dtype=torch.float32, device="cuda"),
                                              block, bits)
        check_codes("codes", unpack_codes(host(q_g)), q_o, t, bits)


def test_static_scale_is_read_at_run_time(hq):
    """The scale lives in device memory: the same call with another value there gives other codes."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((64, 192)).astype(np.float16)
    s_d = torch.tensor([0.5], dtype=torch.float32, device="cuda")
    xd = dev(x)
    for s in (0.5, 0.125):
        s_d.fill_(s)
        q_o, t = oracle.act_hadamard_quant_static(x, 64, 4, s)
        check_codes("codes", unpack_codes(host(hq.hq_act_hadamard_quant_static(xd, s_d, 64, 4))), q_o, t, 4)


@pytest.mark.parametrize("a_bits,w_bits", [(4, 2), (2, 4), (2, 2), (3, 3)])
def test_lower_bit_widths(hq, a_bits, w_bits):
    """2- and 3-bit codes (in the 4-bit container) for either operand, linear and 3x3."""
    import dataclasses
    for idx in (0, 3, 4):
        run_layer(hq, dataclasses.replace(workloads.tiny_layers()[idx], a_bits=a_bits, w_bits=w_bits))


@pytest.mark.parametrize("config", [1, 2, 3, 4, 5])
def test_benchmark_configs_full_size(hq, config):
    """All five configurations at their full sizes, every output element compared."""
    for layer in workloads.config_layers(config):
        run_layer(hq, layer)


# ---- quantiser edge cases --------------------------------------------------------------------

@pytest.mark.parametrize("block", [1, 2, 4, 8, 16, 32, 64, 128])
@pytest.mark.parametrize("dtype", [np.float16, np.float32])
def test_act_quant_block_sizes(hq, block, dtype):
    rng = np.random.default_rng(100 + block)
    k = 384 if block <= 64 else 256
    x = rng.standard_normal((77, k))
    x[:, 5] *= 20
    x = x.astype(dtype)
    for bits in (3, 4):
        q_o, s_o, t = oracle.act_hadamard_quant(x, block, bits)
        q_g, s_g = hq.hq_act_hadamard_quant(dev(x), block, bits)
        check_scales("scale", host(s_g), s_o)
        check_codes("codes", unpack_codes(host(q_g)), q_o, t, bits)


@pytest.mark.parametrize("m,k", [(1, 64), (1, 8640), (3, 9600), (5, 8), (1025, 8), (300, 2048),
                                 (7, 2112), (4099, 192), (2, 16384)])
def test_act_quant_shapes(hq, m, k):
    """One row, rows longer than a workgroup holds, the shortest legal row, ragged last workgroup."""
    rng = np.random.default_rng(m * 7 + k)
    x = rng.standard_normal((m, k)).astype(np.float16)
    block = 64 if k % 64 == 0 else 8
    q_o, s_o, t = oracle.act_hadamard_quant(x, block, 4)
    q_g, s_g = hq.hq_act_hadamard_quant(dev(x), block, 4)
    check_scales("scale", host(s_g), s_o)
    check_codes("codes", unpack_codes(host(q_g)), q_o, t, 4)


@pytest.mark.parametrize("k", [64, 192, 320, 1024])
def test_act_quant_many_tokens(hq, k):
    """Enough tokens for the matrix-core kernel that gives a wave 16 whole tokens (values kept in
    registers up to four blocks per row, recomputed beyond), ragged last group; both scale modes."""
    m = 16 * 8 * 256 + 16 * 3 + 5
    rng = np.random.default_rng(900 + k)
    x = rng.standard_normal((m, k))
    x[:, 7] *= 20
    x[11] = 0.0
    x = x.astype(np.float16)
    xd = dev(x)
    bits = 3 if k == 320 else 4
    q_o, s_o, t = oracle.act_hadamard_quant(x, 64, bits)
    q_g, s_g = hq.hq_act_hadamard_quant(xd, 64, bits)
    check_scales("scale", host(s_g), s_o)
    check_codes("codes", unpack_codes(host(q_g)), q_o, t, bits)
    s = float(np.median(s_o)) * 0.7
    q_o, t = oracle.act_hadamard_quant_static(x, 64, bits, s)
    q_g = hq.hq_act_hadamard_quant_static(xd, torch.tensor([s], dtype=torch.float32, device="cuda"), 64, bits)
    check_codes("static codes", unpack_codes(host(q_g)), q_o, t, bits)


def test_act_quant_degenerate_rows(hq):
    """All-zero tokens (scale 1, codes 0), the paper's two worked examples, and exact ties."""
    x = np.zeros((5, 192), dtype=np.float16)
    x[1, 64 + 5] = -2.5                      # one-hot -> flat +-qmax pattern
    x[2, 128:] = 0.75                        # constant block -> single spike
    x[4, :] = 1.0
    q_o, s_o, _ = oracle.act_hadamard_quant(x, 64, 4)
    q_g, s_g = hq.hq_act_hadamard_quant(dev(x), 64, 4)
    assert np.array_equal(unpack_codes(host(q_g)), q_o)      # all values exact in fp32: no slack
    assert np.array_equal(host(s_g).astype(np.float64), s_o.astype(np.float32).astype(np.float64))
    assert host(s_g)[0] == 1.0 and host(s_g)[3] == 1.0
    # ties: abs-max 7 gives scale 1 with H = I, so t is exactly the input
    xt = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 6.5]], dtype=np.float32)
    q_g, s_g = hq.hq_act_hadamard_quant(dev(xt), 1, 4)
    assert unpack_codes(host(q_g))[0].tolist() == [7, 0, 2, 2, 0, -2, -2, 6]
    assert host(s_g)[0] == 1.0


def test_results_are_deterministic(hq):
    layer = workloads.tiny_layers()[3]
    x, w = dev(workloads.make_x(layer)), dev(workloads.make_w(layer))
    outs = []
    for _ in range(2):
        xq, sx = hq.hq_act_hadamard_quant(x, 64, 4)
        wq, sw = hq.hq_quantize_weights(w, 64, 4)
        y = hq.hq_int_conv2d(xq, sx, wq, sw, None, ksize=3, y_dtype=torch.float16)
        outs.append([host(t).copy() for t in (xq, sx, wq, sw, y)])
    for a, b in zip(*outs):
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8))


# ---- integer stage edge cases ----------------------------------------------------------------

@pytest.mark.parametrize("m,n,k", [(1, 1, 64), (31, 17, 64), (129, 129, 128), (128, 256, 1024),
                                   (1000, 40, 4096), (64, 520, 64)])
def test_int_linear_extreme_codes(hq, m, n, k):
    """Random full-range codes including -8, ragged tiles, long K: sums bit-exact."""
    rng = np.random.default_rng(m + n + k)
    xq = rng.integers(-8, 8, (m, k)).astype(np.int8)
    wq = rng.integers(-8, 8, (n, k)).astype(np.int8)
    xq[0, :], wq[0, :] = -8, -8              # the largest possible sum, 64 k
    acc_o = oracle.int_gemm(xq, wq)
    acc_g = host(hq.hq_int_linear(dev(pack_codes(xq)), None, dev(pack_codes(wq)), None, None,
                                  y_dtype=torch.int32))
    assert np.array_equal(acc_g, acc_o)
    sx = rng.uniform(0.01, 1.0, m)
    sw = rng.uniform(0.001, 0.1, n)
    bias = rng.standard_normal(n).astype(np.float32)
    _, y_o = oracle.int_linear(xq, sx.astype(np.float32), wq, sw.astype(np.float32), bias)
    y_g = host(hq.hq_int_linear(dev(pack_codes(xq)), dev(sx.astype(np.float32)), dev(pack_codes(wq)),
                                dev(sw.astype(np.float32)), dev(bias), y_dtype=torch.float32))
    check_y("y", y_g, y_o, rtol=1e-5)


@pytest.mark.parametrize("nb,h,w,cin,cout,ks", [(1, 1, 1, 64, 8, 3), (1, 3, 5, 64, 16, 3),
                                                 (2, 8, 8, 128, 32, 3), (1, 20, 7, 64, 24, 3),
                                                 (3, 5, 5, 64, 8, 1)])
def test_int_conv_geometry(hq, nb, h, w, cin, cout, ks):
    """Images smaller than a tile, tiles spanning several images, one-pixel images."""
    rng = np.random.default_rng(nb * 1000 + h * 100 + w * 10 + ks)
    xq = rng.integers(-8, 8, (nb, h, w, cin)).astype(np.int8)
    wq = rng.integers(-8, 8, (cout, ks, ks, cin)).astype(np.int8)
    sx = rng.uniform(0.01, 1.0, (nb, h, w)).astype(np.float32)
    sw = rng.uniform(0.001, 0.1, cout).astype(np.float32)
    bias = rng.standard_normal(cout).astype(np.float32)
    acc_o, y_o = oracle.int_conv2d(xq, sx, wq, sw, bias, stride=1, pad=(ks - 1) // 2)
    wq_d = dev(pack_codes(wq.reshape(cout, ks * ks, cin)))
    acc_g = host(hq.hq_int_conv2d(dev(pack_codes(xq)), None, wq_d, None, None, ksize=ks,
                                  y_dtype=torch.int32))
    assert np.array_equal(acc_g, acc_o)
    y_g = host(hq.hq_int_conv2d(dev(pack_codes(xq)), dev(sx), wq_d, dev(sw), dev(bias), ksize=ks,
                                y_dtype=torch.float32))
    check_y("y", y_g, y_o, rtol=1e-5)


@pytest.mark.parametrize("nb,h,w,cin,cout", [(8, 41, 50, 192, 250), (5, 60, 71, 384, 200), (3, 79, 70, 192, 330)])
def test_activation_resident_conv_odd_geometry(hq, nb, h, w, cin, cout):
    """Shapes that take the kernel with the activation tile resident in LDS (at least one 64 x 256
    tile per CU), with image sizes that are not powers of two, tiles that span image rows and
    images, a ragged last pixel tile and a ragged last channel tile; per-pixel scales (one or two
    192-channel slices) and one scale for the tensor (zeros must be loaded outside the image)."""
    rng = np.random.default_rng(nb * 1000 + h * 100 + w + cin + cout)
    xq = rng.integers(-8, 8, (nb, h, w, cin)).astype(np.int8)
    wq = rng.integers(-8, 8, (cout, 3, 3, cin)).astype(np.int8)
    sx = rng.uniform(0.01, 1.0, (nb, h, w)).astype(np.float32)
    sw = rng.uniform(0.001, 0.1, cout).astype(np.float32)
    bias = rng.standard_normal(cout).astype(np.float32)
    xq_d, wq_d = dev(pack_codes(xq)), dev(pack_codes(wq.reshape(cout, 9, cin)))
    assert hq.hq_int_conv2d_kernel_name(nb, h, w, cin, cout, static_scale=True) == "activation-resident"
    if cin == 192:
        assert hq.hq_int_conv2d_kernel_name(nb, h, w, cin, cout) == "activation-resident"
    acc_o, y_o = oracle.int_conv2d(xq, sx, wq, sw, bias, stride=1, pad=1)
    acc_g = host(hq.hq_int_conv2d(xq_d, None, wq_d, None, None, ksize=3, y_dtype=torch.int32))
    assert np.array_equal(acc_g, acc_o), "per-tap int32 sums"
    del acc_g
    y_g = host(hq.hq_int_conv2d(xq_d, dev(sx), wq_d, dev(sw), dev(bias), ksize=3, y_dtype=torch.float32))
    check_y("y", y_g, y_o, rtol=2e-4)     # sums are folded per (slice, tap) from a biased accumulator
    s1 = torch.tensor([0.37], dtype=torch.float32, device="cuda")
    _, y_o = oracle.int_conv2d_static(xq, 0.37, wq, sw, bias, stride=1, pad=1, want_acc=False)
    acc_g = host(hq.hq_int_conv2d_static(xq_d, None, wq_d, None, None, ksize=3, y_dtype=torch.int32))
    assert np.array_equal(acc_g, acc_o.sum(axis=3)), "int32 sums over all taps"
    del acc_g, acc_o
    y_g = host(hq.hq_int_conv2d_static(xq_d, s1, wq_d, dev(sw), dev(bias), ksize=3, y_dtype=torch.float32))
    check_y("y (static)", y_g, y_o, rtol=1e-5)


@pytest.mark.parametrize("nb,h,w,cin,cout,px", [(20, 50, 50, 192, 64, "128 pixels, 4 waves"), (6, 70, 75, 192, 330, 256),
                                                (4, 80, 60, 192, 100, 128),
                                                (3, 40, 40, 192, 500, 64), (20, 30, 33, 384, 150, 128),
                                                (17, 32, 20, 384, 390, 128), (33, 16, 16, 192, 200, 128),
                                                (19, 15, 15, 576, 300, 64), (8, 32, 32, 384, 384, 64)])
def test_int8_resident_conv_odd_geometry(hq, nb, h, w, cin, cout, px):
    """Shapes that take the kernel with the int8 activation tile resident in LDS, for each of its
    three pixel-tile sizes with eight waves (K ranges split over 1+2, 2+4 and 4+8 waves, partial sums
    exchanged through LDS) and for its four-wave form, one to three 192-channel slices, image sizes that are not powers of
    two, tiles that span image rows and images, ragged last pixel and channel tiles.  Per-tap int32
    sums bit for bit (twice: the call zeroes its output), fp32 output to 2e-4 (sums are folded per
    slice and tap from a biased accumulator)."""
    rng = np.random.default_rng(nb * 1000 + h * 100 + w + cin + cout)
    xq = rng.integers(-8, 8, (nb, h, w, cin)).astype(np.int8)
    wq = rng.integers(-8, 8, (cout, 3, 3, cin)).astype(np.int8)
    xq[0, 0, 0, :], wq[0, :, :, :] = -8, -8
    sx = rng.uniform(0.01, 1.0, (nb, h, w)).astype(np.float32)
    sw = rng.uniform(0.001, 0.1, cout).astype(np.float32)
    bias = rng.standard_normal(cout).astype(np.float32)
    xq_d, wq_d = dev(pack_codes(xq)), dev(pack_codes(wq.reshape(cout, 9, cin)))
    want = "activation-resident-int8 (%s)" % (px if isinstance(px, str) else "%d pixels" % px)
    assert hq.hq_int_conv2d_kernel_name(nb, h, w, cin, cout) == want
    acc_o, y_o = oracle.int_conv2d(xq, sx, wq, sw, bias, stride=1, pad=1)
    for rep in range(2):
        acc_g = host(hq.hq_int_conv2d(xq_d, None, wq_d, None, None, ksize=3, y_dtype=torch.int32))
        assert np.array_equal(acc_g, acc_o), "per-tap int32 sums, call %d" % rep
        del acc_g
    del acc_o
    y_g = host(hq.hq_int_conv2d(xq_d, dev(sx), wq_d, dev(sw), dev(bias), ksize=3, y_dtype=torch.float32))
    check_y("y", y_g, y_o, rtol=2e-4)
    y_h = host(hq.hq_int_conv2d(xq_d, dev(sx), wq_d, dev(sw), dev(bias.astype(np.float16)), ksize=3,
                                y_dtype=torch.float16))
    _, y_o = oracle.int_conv2d(xq, sx, wq, sw, bias.astype(np.float16), stride=1, pad=1, want_acc=False)
    check_y("y (fp16)", y_h, y_o, rtol=1e-3)


@pytest.mark.parametrize("nb,h,w,cin,cout", [(1, 16, 16, 192, 100), (3, 9, 6, 384, 24), (5, 7, 9, 576, 130),
                                             (2, 8, 8, 960, 960), (1, 1, 1, 192, 8), (4, 16, 16, 192, 320)])
def test_wave_split_conv_odd_geometry(hq, nb, h, w, cin, cout):
    """Shapes that take the kernel which splits a tile's K range over the waves of a workgroup
    (few 64 x 64 tiles): 1, 2 and 4 waves per tile, ragged pixel and channel tiles, tiles spanning
    images.  Per-tap int32 sums and the one sum over all taps bit for bit (every wave adds its
    share with integer atomics), fp32 outputs of both scale modes to 1e-5."""
    rng = np.random.default_rng(nb * 1000 + h * 100 + w + cin + cout)
    xq = rng.integers(-8, 8, (nb, h, w, cin)).astype(np.int8)
    wq = rng.integers(-8, 8, (cout, 3, 3, cin)).astype(np.int8)
    xq[0, 0, 0, :], wq[0, :, :, :] = -8, -8
    sx = rng.uniform(0.01, 1.0, (nb, h, w)).astype(np.float32)
    sw = rng.uniform(0.001, 0.1, cout).astype(np.float32)
    bias = rng.standard_normal(cout).astype(np.float32)
    xq_d, wq_d = dev(pack_codes(xq)), dev(pack_codes(wq.reshape(cout, 9, cin)))
    assert hq.hq_int_conv2d_kernel_name(nb, h, w, cin, cout) == "wave-split"
    assert hq.hq_int_conv2d_kernel_name(nb, h, w, cin, cout, static_scale=True) == "wave-split"
    acc_o, y_o = oracle.int_conv2d(xq, sx, wq, sw, bias, stride=1, pad=1)
    for rep in range(2):     # twice: the output buffer is zeroed by the call itself
        acc_g = host(hq.hq_int_conv2d(xq_d, None, wq_d, None, None, ksize=3, y_dtype=torch.int32))
        assert np.array_equal(acc_g, acc_o), "per-tap int32 sums, call %d" % rep
    acc_g = host(hq.hq_int_conv2d_static(xq_d, None, wq_d, None, None, ksize=3, y_dtype=torch.int32))
    assert np.array_equal(acc_g, acc_o.sum(axis=3)), "int32 sums over all taps"
    y_g = host(hq.hq_int_conv2d(xq_d, dev(sx), wq_d, dev(sw), dev(bias), ksize=3, y_dtype=torch.float32))
    check_y("y", y_g, y_o, rtol=1e-5)
    s1 = torch.tensor([0.37], dtype=torch.float32, device="cuda")
    _, y_o = oracle.int_conv2d_static(xq, 0.37, wq, sw, bias, stride=1, pad=1, want_acc=False)
    y_g = host(hq.hq_int_conv2d_static(xq_d, s1, wq_d, dev(sw), dev(bias), ksize=3, y_dtype=torch.float32))
    check_y("y (static)", y_g, y_o, rtol=1e-5)


@pytest.mark.parametrize("nb,h,w,cin,cout", [(1, 1, 1, 64, 8), (1, 2, 2, 64, 8), (2, 5, 7, 64, 16), (1, 8, 8, 128, 32),
                                             (3, 9, 6, 192, 24), (2, 16, 16, 192, 70), (1, 33, 31, 64, 130),
                                             (5, 12, 20, 384, 64)])
def test_int_conv_stride_2(hq, nb, h, w, cin, cout):
    """The downsampling convolution (3x3, stride 2, pad 1): odd and even image sizes (the last
    window row / column hangs over the edge for even sizes), one-pixel images, tiles spanning
    images, channel counts with 64- and 192-code chunks; per-tap int32 sums and the sum over all
    taps bit for bit, fp32 outputs of both scale modes."""
    rng = np.random.default_rng(nb * 1000 + h * 100 + w * 10 + cin + cout)
    xq = rng.integers(-8, 8, (nb, h, w, cin)).astype(np.int8)
    wq = rng.integers(-8, 8, (cout, 3, 3, cin)).astype(np.int8)
    sx = rng.uniform(0.01, 1.0, (nb, h, w)).astype(np.float32)
    sw = rng.uniform(0.001, 0.1, cout).astype(np.float32)
    bias = rng.standard_normal(cout).astype(np.float32)
    xq_d, wq_d = dev(pack_codes(xq)), dev(pack_codes(wq.reshape(cout, 9, cin)))
    acc_o, y_o = oracle.int_conv2d(xq, sx, wq, sw, bias, stride=2, pad=1)
    assert acc_o.shape[1:3] == ((h - 1) // 2 + 1, (w - 1) // 2 + 1)
    acc_g = host(hq.hq_int_conv2d(xq_d, None, wq_d, None, None, ksize=3, stride=2, y_dtype=torch.int32))
    assert acc_g.shape == acc_o.shape and np.array_equal(acc_g, acc_o)
    y_g = host(hq.hq_int_conv2d(xq_d, dev(sx), wq_d, dev(sw), dev(bias), ksize=3, stride=2, y_dtype=torch.float32))
    check_y("y", y_g, y_o, rtol=1e-5)
    s1 = torch.tensor([0.37], dtype=torch.float32, device="cuda")
    acc_o, y_o = oracle.int_conv2d_static(xq, 0.37, wq, sw, bias, stride=2, pad=1)
    acc_g = host(hq.hq_int_conv2d_static(xq_d, None, wq_d, None, None, ksize=3, stride=2, y_dtype=torch.int32))
    assert np.array_equal(acc_g, acc_o)
    y_g = host(hq.hq_int_conv2d_static(xq_d, s1, wq_d, dev(sw), dev(bias), ksize=3, stride=2, y_dtype=torch.float32))
    check_y("y (static)", y_g, y_o, rtol=1e-5)


@pytest.mark.parametrize("nb,h,w,cin,cout", [(1, 1, 1, 64, 8), (2, 5, 7, 64, 16), (3, 9, 6, 192, 24), (1, 33, 31, 64, 130),
                                             (5, 12, 20, 384, 64)])
def test_int8_conv_stride_2(hq, nb, h, w, cin, cout):
    """The downsampling convolution with 8-bit codes: per-tap int32 sums bit for bit, fp32 output."""
    rng = np.random.default_rng(nb * 1000 + h * 100 + w * 10 + cin + cout + 8)
    xq = rng.integers(-128, 128, (nb, h, w, cin)).astype(np.int8)
    wq = rng.integers(-128, 128, (cout, 3, 3, cin)).astype(np.int8)
    sx = rng.uniform(0.01, 1.0, (nb, h, w)).astype(np.float32)
    sw = rng.uniform(0.001, 0.1, cout).astype(np.float32)
    bias = rng.standard_normal(cout).astype(np.float32)
    xq_d, wq_d = dev(xq), dev(wq.reshape(cout, 9, cin))
    acc_o, y_o = oracle.int_conv2d(xq, sx, wq, sw, bias, stride=2, pad=1)
    acc_g = host(hq.hq_int_conv2d_i8(xq_d, None, wq_d, None, None, ksize=3, stride=2, y_dtype=torch.int32))
    assert acc_g.shape == acc_o.shape and np.array_equal(acc_g, acc_o)
    y_g = host(hq.hq_int_conv2d_i8(xq_d, dev(sx), wq_d, dev(sw), dev(bias), ksize=3, stride=2, y_dtype=torch.float32))
    check_y("y", y_g, y_o, rtol=1e-5)


@pytest.mark.parametrize("nb,h,w,cin,cout,block", [(2, 5, 8, 64, 16, 8), (1, 9, 16, 192, 24, 16), (3, 12, 32, 128, 70, 32),
                                                   (2, 7, 4, 64, 8, 1), (1, 16, 64, 64, 40, 64)])
def test_width_conv_stride_2(hq, nb, h, w, cin, cout, block):
    """The paper's width-axis convolution at stride 2 (two and three digit planes): the exact integer
    sums on the oracle's codes, bit for bit, and the fp32 output."""
    rng = np.random.default_rng(nb * 1000 + h * 100 + w * 10 + cin + cout + block)
    q = rng.integers(-8, 8, (nb, h, w, cin)).astype(np.int8)
    wq = rng.integers(-8, 8, (cout, 3, 3, cin)).astype(np.int8)
    sw = rng.uniform(0.001, 0.1, cout).astype(np.float32)
    bias = rng.standard_normal(cout).astype(np.float32)
    hb = np.kron(np.eye(w // block, dtype=np.int64), np.rint(oracle.hadamard_raw(block)).astype(np.int64))
    u = np.einsum("nhwc,wv->nhvc", q.astype(np.int64), hb)
    d0 = ((u + 8) % 16) - 8
    r1 = (u - d0) // 16
    d1 = ((r1 + 8) % 16) - 8
    planes = dev(pack_codes(np.stack([d0, d1, (r1 - d1) // 16]).astype(np.int8)))
    acc_o, y_o = oracle.int_conv2d_width(q, 0.3, wq, sw, block, bias, stride=2, pad=1)
    wq_d = dev(pack_codes(wq.reshape(cout, 9, cin)))
    acc_g = host(hq.hq_int_conv2d_width(planes, None, wq_d, None, None, block, y_dtype=torch.int32, stride=2))
    assert acc_g.shape == acc_o.shape and np.array_equal(acc_g, acc_o)
    s1 = torch.tensor([0.3], dtype=torch.float32, device="cuda")
    y_g = host(hq.hq_int_conv2d_width(planes, s1, wq_d, dev(sw), dev(bias), block, y_dtype=torch.float32, stride=2))
    check_y("y", y_g, y_o, rtol=1e-5)


@pytest.mark.parametrize("hw,c", [(64, 192), (32, 384), (16, 576)])
def test_stride_2_downsampling_layers_full_size(hq, hw, c):
    """The three downsampling convolutions of an LDM-4-shaped UNet at batch 16, fp16 output with
    per-pixel scales, every output against the oracle; per-tap int32 sums on the first two images."""
    rng = np.random.default_rng(hw + c)
    nb = 16
    xq = rng.integers(-8, 8, (nb, hw, hw, c)).astype(np.int8)
    wq = rng.integers(-8, 8, (c, 3, 3, c)).astype(np.int8)
    sx = rng.uniform(0.01, 1.0, (nb, hw, hw)).astype(np.float32)
    sw = rng.uniform(0.001, 0.1, c).astype(np.float32)
    bias = rng.standard_normal(c).astype(np.float16)
    xq_d, wq_d = dev(pack_codes(xq)), dev(pack_codes(wq.reshape(c, 9, c)))
    _, y_o = oracle.int_conv2d(xq, sx, wq, sw, bias, stride=2, pad=1, want_acc=False)
    y_g = host(hq.hq_int_conv2d(xq_d, dev(sx), wq_d, dev(sw), dev(bias), ksize=3, stride=2, y_dtype=torch.float16))
    check_y("y", y_g, y_o)
    acc_o, _ = oracle.int_conv2d(xq[:2], sx[:2], wq, sw, None, stride=2, pad=1, want_y=False)
    acc_g = host(hq.hq_int_conv2d(xq_d[:2].contiguous(), None, wq_d, None, None, ksize=3, stride=2,
                                  y_dtype=torch.int32))
    assert np.array_equal(acc_g, acc_o)


@pytest.mark.parametrize("k", [8, 40, 72, 200, 264])
def test_channel_counts_that_are_not_multiples_of_64(hq, k):
    """The integer stage for k a multiple of 8 but not of 64 (a layer with fewer channels than the
    transform's order keeps H = I): linear, 1x1 and 3x3, ragged tiles, full-range codes; int32 sums
    bit for bit (per tap, and the one sum of the static-scale calls), fp32 outputs to 1e-5."""
    rng = np.random.default_rng(k)
    m, n = 200 + k, 70
    xq = rng.integers(-8, 8, (m, k)).astype(np.int8)
    wq = rng.integers(-8, 8, (n, k)).astype(np.int8)
    xq[0], wq[0] = -8, -8
    sx = rng.uniform(0.01, 1.0, m).astype(np.float32)
    sw = rng.uniform(0.001, 0.1, n).astype(np.float32)
    bias = rng.standard_normal(n).astype(np.float32)
    xq_d, wq_d = dev(pack_codes(xq)), dev(pack_codes(wq))
    acc_o, y_o = oracle.int_linear(xq, sx, wq, sw, bias)
    assert np.array_equal(host(hq.hq_int_linear(xq_d, None, wq_d, None, None, y_dtype=torch.int32)), acc_o)
    check_y("y", host(hq.hq_int_linear(xq_d, dev(sx), wq_d, dev(sw), dev(bias), y_dtype=torch.float32)), y_o, rtol=1e-5)
    s1 = torch.tensor([0.37], dtype=torch.float32, device="cuda")
    _, y_o = oracle.int_linear_static(xq, 0.37, wq, sw, bias)
    check_y("y (static)", host(hq.hq_int_linear_static(xq_d, s1, wq_d, dev(sw), dev(bias), y_dtype=torch.float32)),
            y_o, rtol=1e-5)
    for ks, (nb, h, w, cout) in ((3, (2, 9, 11, 70)), (1, (3, 5, 7, 33)), (3, (1, 1, 1, 8))):
        xc = rng.integers(-8, 8, (nb, h, w, k)).astype(np.int8)
        wc = rng.integers(-8, 8, (cout, ks, ks, k)).astype(np.int8)
        sxc = rng.uniform(0.01, 1.0, (nb, h, w)).astype(np.float32)
        swc = rng.uniform(0.001, 0.1, cout).astype(np.float32)
        bc = rng.standard_normal(cout).astype(np.float32)
        assert hq.hq_int_conv2d_kernel_name(nb, h, w, k, cout, ksize=ks) == "small-channel-count"
        xc_d, wc_d = dev(pack_codes(xc)), dev(pack_codes(wc.reshape(cout, ks * ks, k)))
        acc_o, y_o = oracle.int_conv2d(xc, sxc, wc, swc, bc, stride=1, pad=(ks - 1) // 2)
        acc_g = host(hq.hq_int_conv2d(xc_d, None, wc_d, None, None, ksize=ks, y_dtype=torch.int32))
        assert np.array_equal(acc_g, acc_o), "per-tap sums, %dx%d" % (ks, ks)
        y_g = host(hq.hq_int_conv2d(xc_d, dev(sxc), wc_d, dev(swc), dev(bc), ksize=ks, y_dtype=torch.float32))
        check_y("y conv", y_g, y_o, rtol=1e-5)
        acc_g = host(hq.hq_int_conv2d_static(xc_d, None, wc_d, None, None, ksize=ks, y_dtype=torch.int32))
        assert np.array_equal(acc_g, acc_o.sum(axis=3)), "one sum, %dx%d" % (ks, ks)
        _, y_o = oracle.int_conv2d_static(xc, 0.37, wc, swc, bc, stride=1, pad=(ks - 1) // 2, want_acc=False)
        y_g = host(hq.hq_int_conv2d_static(xc_d, s1, wc_d, dev(swc), dev(bc), ksize=ks, y_dtype=torch.float32))
        check_y("y conv (static)", y_g, y_o, rtol=1e-5)


def test_bypass_layer_end_to_end(hq):
    """A convolution on an 8-channel input (fewer channels than the transform's order: H = I,
    had_block = 1) through both calls of the layer, with the three layers of checks."""
    import dataclasses
    layer = dataclasses.replace(workloads.tiny_layers()[3], name="t_conv3_8ch", x_shape=(2, 19, 23, 8), n_out=200)
    run_layer(hq, layer, block=1)
    run_layer_static(hq, layer, block=1)
    layer = dataclasses.replace(workloads.tiny_layers()[0], name="t_lin_40", x_shape=(301, 40), n_out=96)
    run_layer(hq, layer, block=8)


def run_layer_fused(hq, layer):
    """A 3x3 layer through the one-launch call that transforms and quantises its own activation
    tile: (i) the codes and scales it used against the oracle's (tie rule) AND bit for bit against
    the stand-alone transform-quantise call; (ii) its per-tap int32 sums against the oracle's integer
    convolution of those (validated) codes, bit for bit; (iii) its result against the oracle's chain."""
    print("layer (fused)", layer.name, layer.x_shape, "->", layer.n_out, flush=True)
    x, w, bias = workloads.make_x(layer), workloads.make_w(layer), workloads.make_bias(layer)
    ydt = TORCH_DT[layer.dtype]
    xq_o, sx_o, tx = oracle.act_hadamard_quant(x, 64, layer.a_bits)
    wq_o, sw_o, tw = oracle.quantize_weights(w, 64, layer.w_bits)
    wq4 = lambda c: c.reshape(layer.n_out, 3, 3, layer.k_in)
    xd = dev(x)
    wq_g, sw_g = hq.hq_quantize_weights(dev(w), 64, layer.w_bits)
    wq_gc = unpack_codes(host(wq_g))
    flips = check_codes(layer.name + " wq", wq_gc, wq_o, tw, layer.w_bits)
    bias_d = dev(bias) if bias is not None else None
    xq_f = torch.zeros(x.shape[:-1] + (layer.k_in // 2,), dtype=torch.uint8, device="cuda")
    sx_f = torch.zeros(x.shape[:-1], dtype=torch.float32, device="cuda")
    y_g = host(hq.hq_act_quant_int_conv2d(xd, wq_g, sw_g, bias_d, a_bits=layer.a_bits, y_dtype=ydt,
                                          codes_out=(xq_f, sx_f)))
    # (i)
    xq_s, sx_s = hq.hq_act_hadamard_quant(xd, 64, layer.a_bits)
    assert np.array_equal(host(xq_f), host(xq_s)), layer.name + ": codes differ from the stand-alone call's"
    assert np.array_equal(host(sx_f), host(sx_s)), layer.name + ": scales differ from the stand-alone call's"
    xq_gc = unpack_codes(host(xq_f))
    check_scales(layer.name + " x_scale", host(sx_f), sx_o)
    flips += check_codes(layer.name + " xq", xq_gc, xq_o, tx, layer.a_bits)
    # (ii) integer sums of the fused call (its own codes, the oracle's weight codes)
    acc_g = host(hq.hq_act_quant_int_conv2d(xd, dev(pack_codes(wq_o)), None, None, a_bits=layer.a_bits,
                                            y_dtype=torch.int32))
    acc_o, y_o = oracle.int_conv2d(xq_gc, sx_o, wq4(wq_o), sw_o, bias, stride=1, pad=1)
    assert np.array_equal(acc_g, acc_o), layer.name + " per-tap int32 sums (fused)"
    del acc_g, acc_o
    # (iii)
    if flips:
        _, y_o = oracle.int_conv2d(xq_gc, sx_o, wq4(wq_gc), sw_o, bias, stride=1, pad=1, want_acc=False)
    else:
        _, y_o = oracle.int_conv2d(xq_o, sx_o, wq4(wq_o), sw_o, bias, stride=1, pad=1, want_acc=False)
    err = check_y(layer.name + " y (fused)", y_g.reshape(y_o.shape), y_o)
    print("   ok: tie flips %d, y err %.2e" % (flips, err), flush=True)


@pytest.mark.parametrize("idx", [4, 7])
def test_fused_conv_tiny_layers(hq, idx):
    run_layer_fused(hq, workloads.tiny_layers()[idx])


@pytest.mark.parametrize("nb,h,w,cin,cout,a_bits", [(8, 41, 50, 192, 250, 4), (3, 79, 70, 192, 330, 3),
                                                     (20, 30, 33, 384, 150, 4), (19, 15, 15, 576, 300, 4),
                                                     (1, 1, 1, 192, 8, 4), (2, 5, 3, 384, 200, 2)])
def test_fused_conv_odd_geometry(hq, nb, h, w, cin, cout, a_bits):
    """The one-launch layer on image sizes that are not powers of two, tiles that span images, ragged
    pixel and channel tiles, one to three channel slices, every tile configuration of the kernel."""
    import dataclasses
    layer = dataclasses.replace(workloads.tiny_layers()[4], name="fused_%dx%dx%dx%d_%d" % (nb, h, w, cin, cout),
                                x_shape=(nb, h, w, cin), n_out=cout, a_bits=a_bits, bias_std=0.01)
    run_layer_fused(hq, layer)


@pytest.mark.parametrize("config,index", [(3, 0), (5, 0), (5, 1), (5, 2)])
def test_fused_conv_benchmark_layers_full_size(hq, config, index):
    run_layer_fused(hq, workloads.config_layers(config)[index])


def run_linear_fused(hq, layer):
    """A linear layer / 1x1 convolution through the one-launch call: codes and scales against the
    oracle (tie rule) and bit for bit against the stand-alone call, int32 sums of those codes bit for
    bit, the result against the oracle's chain."""
    print("layer (fused linear)", layer.name, layer.x_shape, "->", layer.n_out, flush=True)
    x, w, bias = workloads.make_x(layer), workloads.make_w(layer)[:, 0, :], workloads.make_bias(layer)
    ydt = TORCH_DT[layer.dtype]
    x2 = x.reshape(-1, layer.k_in)
    xq_o, sx_o, tx = oracle.act_hadamard_quant(x2, 64, layer.a_bits)
    wq_o, sw_o, tw = oracle.quantize_weights(w[:, None, :], 64, layer.w_bits)
    wq_o = wq_o[:, 0, :]
    xd = dev(x2)
    wq_g, sw_g = hq.hq_quantize_weights(dev(w[:, None, :]), 64, layer.w_bits)
    wq_gc = unpack_codes(host(wq_g))[:, 0, :]
    flips = check_codes(layer.name + " wq", wq_gc, wq_o, tw[:, 0, :], layer.w_bits)
    bias_d = dev(bias) if bias is not None else None
    xq_f = torch.zeros((x2.shape[0], layer.k_in // 2), dtype=torch.uint8, device="cuda")
    sx_f = torch.zeros((x2.shape[0],), dtype=torch.float32, device="cuda")
    y_g = host(hq.hq_act_quant_int_linear(xd, wq_g, sw_g, bias_d, a_bits=layer.a_bits, y_dtype=ydt,
                                          codes_out=(xq_f, sx_f)))
    xq_s, sx_s = hq.hq_act_hadamard_quant(xd, 64, layer.a_bits)
    assert np.array_equal(host(xq_f), host(xq_s)), layer.name + ": codes differ from the stand-alone call's"
    assert np.array_equal(host(sx_f), host(sx_s)), layer.name + ": scales differ from the stand-alone call's"
    xq_gc = unpack_codes(host(xq_f))
    check_scales(layer.name + " x_scale", host(sx_f), sx_o)
    flips += check_codes(layer.name + " xq", xq_gc, xq_o, tx, layer.a_bits)
    acc_g = host(hq.hq_act_quant_int_linear(xd, dev(pack_codes(wq_o)), None, None, a_bits=layer.a_bits,
                                            y_dtype=torch.int32))
    acc_o, y_o = oracle.int_linear(xq_gc, sx_o, wq_o, sw_o, bias)
    assert np.array_equal(acc_g, acc_o), layer.name + " int32 sums (fused linear)"
    if flips:
        _, y_o = oracle.int_linear(xq_gc, sx_o, wq_gc, sw_o, bias)
    else:
        _, y_o = oracle.int_linear(xq_o, sx_o, wq_o, sw_o, bias)
    err = check_y(layer.name + " y (fused linear)", y_g.reshape(y_o.shape), y_o)
    print("   ok: tie flips %d, y err %.2e" % (flips, err), flush=True)


@pytest.mark.parametrize("idx", [0, 2, 5])
def test_fused_linear_tiny_layers(hq, idx):
    run_linear_fused(hq, workloads.tiny_layers()[idx])


@pytest.mark.parametrize("m,k,n,a_bits", [(1, 64, 1, 4), (65, 128, 40, 3), (333, 1024, 200, 4), (700, 960, 1000, 4),
                                          (5000, 192, 72, 2)])
def test_fused_linear_shapes(hq, m, k, n, a_bits):
    """One row, ragged row and column tiles, the longest row, several column groups per row tile."""
    import dataclasses
    layer = dataclasses.replace(workloads.tiny_layers()[0], name="fl_%d_%d_%d" % (m, k, n), x_shape=(m, k),
                                n_out=n, a_bits=a_bits)
    run_linear_fused(hq, layer)


@pytest.mark.parametrize("config,index", [(2, 0), (4, 1), (5, 4), (5, 5), (5, 6), (5, 7), (5, 8)])
def test_fused_linear_benchmark_layers_full_size(hq, config, index):
    run_linear_fused(hq, workloads.config_layers(config)[index])


def test_fused_conv_refuses_what_is_not_built(hq):
    x = torch.zeros((1, 8, 8, 960), dtype=torch.float16, device="cuda")
    wq = torch.zeros((8, 9, 480), dtype=torch.uint8, device="cuda")
    with pytest.raises(hq.HqError):   # five slices of an 8-pixel-wide image do not fit on chip
        hq.hq_act_quant_int_conv2d(x, wq, torch.ones(8, device="cuda"))
    with pytest.raises(hq.HqError):
        hq.hq_act_quant_int_conv2d(x[..., :128].contiguous(), wq[..., :64].contiguous(), torch.ones(8, device="cuda"))


def _random_bytes(shape, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randint(0, 256, shape, dtype=torch.uint8, device="cuda", generator=g)


def test_int_linear_at_the_largest_token_count(hq):
    """The packed operands are addressed with 32-bit byte offsets: the largest token count the
    linear call accepts for K = 256 (4 GiB of codes) must give the oracle's sums on its first,
    middle and LAST rows, and one token more must be refused, not wrapped."""
    k, n = 256, 24
    m = (2 ** 32 - 1) // (k // 2) - 3
    print("linear at m =", m, flush=True)
    xq = _random_bytes((m, k // 2), 1)
    sx = torch.rand(m, device="cuda") * 0.5 + 0.01
    rng = np.random.default_rng(5)
    wq = rng.integers(-8, 8, (n, k)).astype(np.int8)
    sw = rng.uniform(0.001, 0.1, n).astype(np.float32)
    bias = rng.standard_normal(n).astype(np.float32)
    wq_d = dev(pack_codes(wq))
    rows = np.unique(np.concatenate([np.arange(130), m // 2 + np.arange(-64, 64), np.arange(m - 300, m),
                                     rng.integers(0, m, 500)]))
    rows_d = torch.from_numpy(rows).cuda()
    xq_s = unpack_codes(host(xq[rows_d]))
    acc_o, y_o = oracle.int_linear(xq_s, host(sx[rows_d]), wq, sw, bias)
    acc_g = hq.hq_int_linear(xq, None, wq_d, None, None, y_dtype=torch.int32)
    assert np.array_equal(host(acc_g[rows_d]), acc_o)
    del acc_g
    y_g = hq.hq_int_linear(xq, sx, wq_d, dev(sw), dev(bias), y_dtype=torch.float32)
    check_y("y", host(y_g[rows_d]), y_o, rtol=1e-5)
    del y_g
    # one row more: the offsets of the last rows would pass 2^32 (the buffer below is big enough,
    # and is never read: the call is refused before any launch)
    xq1 = torch.empty((m + 1, k // 2), dtype=torch.uint8, device="cuda")
    with pytest.raises(hq.HqError):
        hq.hq_int_linear(xq1, None, wq_d, None, None, y_dtype=torch.int32)


@pytest.mark.parametrize("cin,cout,hw,static", [(64, 8, 128, False), (192, 64, 64, False), (192, 64, 64, True)])
def test_int_conv_at_the_largest_pixel_count(hq, cin, cout, hw, static):
    """The same for the 3x3 convolution (tile kernel with 64-code chunks; kernel with the activation
    tile resident in LDS, per-pixel scales and one scale): the largest batch whose activation
    offsets, shifted by a tap, stay below 2^32.  Whole images - the first, a middle one, the last
    two - against the oracle; one image more is refused."""
    kb = cin // 2
    nb = ((2 ** 32 - 1) // kb - hw - 2) // (hw * hw)
    print("conv at", (nb, hw, hw, cin), "->", cout, "static" if static else "dynamic", flush=True)
    xq = _random_bytes((nb, hw, hw, kb), 2)
    sx = torch.rand((nb, hw, hw), device="cuda") * 0.5 + 0.01
    rng = np.random.default_rng(cin + cout)
    wq = rng.integers(-8, 8, (cout, 3, 3, cin)).astype(np.int8)
    sw = rng.uniform(0.001, 0.1, cout).astype(np.float32)
    bias = rng.standard_normal(cout).astype(np.float32)
    wq_d = dev(pack_codes(wq.reshape(cout, 9, cin)))
    images = [0, nb // 2, nb - 2, nb - 1]
    if static:
        s1 = torch.tensor([0.37], dtype=torch.float32, device="cuda")
        y_g = hq.hq_int_conv2d_static(xq, s1, wq_d, dev(sw), dev(bias), ksize=3, y_dtype=torch.float32)
    else:
        y_g = hq.hq_int_conv2d(xq, sx, wq_d, dev(sw), dev(bias), ksize=3, y_dtype=torch.float32)
    for i in images:
        xq_i = unpack_codes(host(xq[i:i + 1]))
        if static:
            _, y_o = oracle.int_conv2d_static(xq_i, 0.37, wq, sw, bias, stride=1, pad=1, want_acc=False)
        else:
            _, y_o = oracle.int_conv2d(xq_i, host(sx[i:i + 1]), wq, sw, bias, stride=1, pad=1, want_acc=False)
        check_y("y of image %d" % i, host(y_g[i:i + 1]).reshape(y_o.shape), y_o, rtol=2e-4)
    del y_g
    if cout <= 8 and not static:   # per-tap int32 sums (9 x the output volume): the small layer only
        acc_g = hq.hq_int_conv2d(xq, None, wq_d, None, None, ksize=3, y_dtype=torch.int32)
        for i in images:
            acc_o, _ = oracle.int_conv2d(unpack_codes(host(xq[i:i + 1])), host(sx[i:i + 1]), wq, sw, None,
                                         stride=1, pad=1)
            assert np.array_equal(host(acc_g[i:i + 1]).reshape(acc_o.shape), acc_o), "image %d" % i
        del acc_g
    xq1 = torch.empty((nb + 1, hw, hw, kb), dtype=torch.uint8, device="cuda")   # never read: refused before any launch
    sx1 = torch.empty((nb + 1, hw, hw), dtype=torch.float32, device="cuda")
    with pytest.raises(hq.HqError):
        hq.hq_int_conv2d(xq1, sx1, wq_d, dev(sw), None, ksize=3, y_dtype=torch.float16)


def test_act_quant_beyond_4gi_elements(hq):
    """More than 2^32 elements (8.6 GB of fp16) through the transform-quantise call: sampled
    tokens, the last ones included, against the oracle."""
    k = 256
    m = 2 ** 24 + 5
    print("act quant at m =", m, flush=True)
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    x = torch.randn((m, k), dtype=torch.float16, device="cuda", generator=g)
    rng = np.random.default_rng(9)
    rows = np.unique(np.concatenate([np.arange(70), np.arange(m - 70, m), rng.integers(0, m, 400)]))
    rows_d = torch.from_numpy(rows).cuda()
    xq_o, sx_o, t = oracle.act_hadamard_quant(host(x[rows_d]), 64, 4)
    xq_g, sx_g = hq.hq_act_hadamard_quant(x, 64, 4)
    check_scales("x_scale", host(sx_g[rows_d]), sx_o)
    check_codes("xq", unpack_codes(host(xq_g[rows_d])), xq_o, t, 4)
    del xq_g, sx_g
    s1 = torch.tensor([0.2], dtype=torch.float32, device="cuda")
    xq_o, t = oracle.act_hadamard_quant_static(host(x[rows_d]), 64, 4, float(np.float32(0.2)))
    xq_g = hq.hq_act_hadamard_quant_static(x, s1, 64, 4)
    check_codes("xq (static)", unpack_codes(host(xq_g[rows_d])), xq_o, t, 4)


def test_random_small_shapes(hq):
    """A seeded sweep of small ragged shapes through every integer-stage entry point: int32 sums bit
    for bit on random full-range codes."""
    rng = np.random.default_rng(20251205)
    for case in range(24):
        m, n = int(rng.integers(1, 300)), int(rng.integers(1, 200))
        k = 64 * int(rng.integers(1, 7))
        xq = rng.integers(-8, 8, (m, k)).astype(np.int8)
        wq = rng.integers(-8, 8, (n, k)).astype(np.int8)
        tag = "case %d: m %d n %d k %d" % (case, m, n, k)
        acc = host(hq.hq_int_linear(dev(pack_codes(xq)), None, dev(pack_codes(wq)), None, None, y_dtype=torch.int32))
        assert np.array_equal(acc, oracle.int_gemm(xq, wq)), tag
        x8 = rng.integers(-128, 128, (m, k)).astype(np.int8)
        w8 = rng.integers(-128, 128, (n, k)).astype(np.int8)
        acc = host(hq.hq_int_linear_i8(dev(x8), None, dev(w8), None, None, y_dtype=torch.int32))
        assert np.array_equal(acc, oracle.int_gemm(x8, w8)), tag + " (int8)"
        nb, h, w = int(rng.integers(1, 4)), int(rng.integers(1, 14)), int(rng.integers(1, 14))
        cout = int(rng.integers(1, 100))
        xc = rng.integers(-8, 8, (nb, h, w, k)).astype(np.int8)
        wc = rng.integers(-8, 8, (cout, 3, 3, k)).astype(np.int8)
        tag = "case %d: %dx%dx%d cin %d cout %d" % (case, nb, h, w, k, cout)
        xc_d, wc_d = dev(pack_codes(xc)), dev(pack_codes(wc.reshape(cout, 9, k)))
        ones_x, ones_w = np.ones((nb, h, w)), np.ones(cout)
        acc_t, _ = oracle.int_conv2d(xc, ones_x, wc, ones_w, None, stride=1, pad=1, want_y=False)
        acc = host(hq.hq_int_conv2d(xc_d, None, wc_d, None, None, ksize=3, y_dtype=torch.int32))
        assert np.array_equal(acc, acc_t), tag
        acc = host(hq.hq_int_conv2d_static(xc_d, None, wc_d, None, None, ksize=3, y_dtype=torch.int32))
        assert np.array_equal(acc, acc_t.sum(axis=3)), tag + " (one sum)"


def test_errors_raise(hq):
    x = torch.zeros((4, 96), dtype=torch.float16, device="cuda")
    with pytest.raises(hq.HqError):
        hq.hq_act_hadamard_quant(x, 64, 4)
    with pytest.raises(hq.HqError):
        hq.hq_act_hadamard_quant(x[:, :64].contiguous(), 64, 5)


def test_binding_refuses_buffers_of_the_wrong_size(hq):
    """Output buffers, scales and bias handed to the binding must have exactly the size the call
    writes or reads, and codes the dtype of their format; anything else is refused before the
    library is called."""
    xq = torch.zeros((8, 32), dtype=torch.uint8, device="cuda")
    wq = torch.zeros((16, 32), dtype=torch.uint8, device="cuda")
    sx = torch.ones(8, device="cuda")
    sw = torch.ones(16, device="cuda")
    ok = hq.hq_int_linear(xq, sx, wq, sw, None, y_dtype=torch.float16)
    assert ok.shape == (8, 16)
    bad = [
        lambda: hq.hq_int_linear(xq, sx, wq, sw, None, y_dtype=torch.float16, out=torch.empty((8, 15), dtype=torch.float16, device="cuda")),
        lambda: hq.hq_int_linear(xq, sx, wq, sw, None, y_dtype=torch.float16, out=torch.empty((8, 16), dtype=torch.float32, device="cuda")),
        lambda: hq.hq_int_linear(xq, sx[:7], wq, sw, None, y_dtype=torch.float16),
        lambda: hq.hq_int_linear(xq, sx, wq, sw[:15], None, y_dtype=torch.float16),
        lambda: hq.hq_int_linear(xq, sx, wq, sw, torch.zeros(15, dtype=torch.float16, device="cuda"), y_dtype=torch.float16),
        lambda: hq.hq_int_linear(xq, sx, wq, sw, torch.zeros(16, dtype=torch.float32, device="cuda"), y_dtype=torch.float16),
        lambda: hq.hq_int_linear(xq.view(torch.int8), sx, wq, sw, None, y_dtype=torch.float16),
        lambda: hq.hq_int_linear_i8(xq, sx, wq, sw, None, y_dtype=torch.float16),
        lambda: hq.hq_int_linear_static(xq, sx, wq, sw, None, y_dtype=torch.float16),      # the scale must be ONE value
        lambda: hq.hq_int_conv2d(xq.view(1, 2, 4, 32), sx, wq.new_zeros((16, 9, 32)), sw, None, ksize=3,
                                 out=torch.empty((1, 2, 4, 15), dtype=torch.float16, device="cuda")),
        lambda: hq.hq_act_hadamard_quant(torch.zeros((8, 64), dtype=torch.float16, device="cuda"), 64, 4,
                                         out=(xq, torch.empty(7, device="cuda"))),
        lambda: hq.hq_act_hadamard_quant_static(torch.zeros((8, 64), dtype=torch.float16, device="cuda"),
                                                torch.ones(1, device="cuda"), 64, 4, out=xq[:7]),
    ]
    for i, call in enumerate(bad):
        with pytest.raises(ValueError):
            call()
            pytest.fail("case %d was accepted" % i)


def test_hip_graph_replay_matches_eager(hq):
    """The whole layer captured into a HIP graph: every replay (with eager work and
    synchronisations in between) must reproduce the eager result bit for bit."""
    layer = workloads.tiny_layers()[4]
    x = dev(workloads.make_x(layer))
    wq, sw = hq.hq_quantize_weights(dev(workloads.make_w(layer)), 64, 4)
    xq = torch.empty(x.shape[:-1] + (layer.k_in // 2,), dtype=torch.uint8, device="cuda")
    sx = torch.empty(x.shape[:-1], dtype=torch.float32, device="cuda")
    y = torch.empty(x.shape[:-1] + (layer.n_out,), dtype=torch.float16, device="cuda")

    def run():
        hq.hq_act_hadamard_quant(x, 64, 4, out=(xq, sx))
        hq.hq_int_conv2d(xq, sx, wq, sw, None, ksize=3, y_dtype=torch.float16, out=y)

    run()
    want = host(y).copy()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for i in range(4):
        y.zero_()
        xq.zero_()
        torch.cuda.synchronize()
        graph.replay()
        assert np.array_equal(host(y).view(np.uint16), want.view(np.uint16)), "replay %d" % i
        run()   # eager work between replays
        torch.cuda.synchronize()


def test_hip_graph_replay_of_the_other_schemes(hq):
    """Static-scale, Single-scheme, width-axis and 8-bit calls captured into one HIP graph; the
    static scale is changed between replays in device memory and the replay must follow it."""
    layer = workloads.tiny_layers()[7]                      # 13 x 16 x 16, 192 -> 320, 3x3
    x = dev(workloads.make_x(layer))
    w = dev(workloads.make_w(layer))
    wq, sw = hq.hq_quantize_weights(w, 64, 4)
    wq1, sw1 = hq.hq_quantize_weights(w, 1, 4)
    wq8, sw8 = hq.hq_quantize_weights(w, 64, 8)
    wq3, sw3 = hq.hq_quantize_weights_single(w[:, 4, :].contiguous(), 64, 4)
    s_d = torch.tensor([0.3], dtype=torch.float32, device="cuda")
    shape = tuple(x.shape[:-1])
    xq = torch.empty(shape + (layer.k_in // 2,), dtype=torch.uint8, device="cuda")
    xd = torch.empty(shape + (layer.k_in // 2,), dtype=torch.uint8, device="cuda")
    sxd = torch.empty(shape, dtype=torch.float32, device="cuda")
    xu3 = torch.empty((3,) + shape + (layer.k_in // 2,), dtype=torch.uint8, device="cuda")
    x8 = torch.empty(shape + (layer.k_in,), dtype=torch.int8, device="cuda")
    sx8 = torch.empty(shape, dtype=torch.float32, device="cuda")
    ys = [torch.empty(shape + (layer.n_out,), dtype=torch.float16, device="cuda") for _ in range(4)]
    m = x.numel() // layer.k_in

    def run():
        hq.hq_act_hadamard_quant_static(x, s_d, 64, 4, out=xq)
        hq.hq_int_conv2d_static(xq, s_d, wq, sw, None, ksize=3, y_dtype=torch.float16, out=ys[0])
        hq.hq_act_hadamard_quant(x, 64, 4, out=(xd, sxd))
        hq.hq_int_linear_single(xd.reshape(m, -1), sxd.reshape(-1), wq3, sw3, None, 64, y_dtype=torch.float16,
                                out=ys[1].reshape(m, -1))
        hq.hq_act_hadamard_quant_width(x, s_d, 16, 4, out=xu3)
        hq.hq_int_conv2d_width(xu3, s_d, wq1, sw1, None, 16, y_dtype=torch.float16, out=ys[2])
        hq.hq_act_hadamard_quant(x, 64, 8, out=(x8, sx8))
        hq.hq_int_conv2d_i8(x8, sx8, wq8, sw8, None, ksize=3, y_dtype=torch.float16, out=ys[3])

    want = {}
    for s in (0.3, 0.11):
        s_d.fill_(s)
        run()
        want[s] = [host(y).copy() for y in ys]
    assert not np.array_equal(want[0.3][0], want[0.11][0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for i, s in enumerate((0.11, 0.3, 0.3, 0.11)):
        for y in ys:
            y.zero_()
        s_d.fill_(s)
        torch.cuda.synchronize()
        graph.replay()
        for j, y in enumerate(ys):
            assert np.array_equal(host(y).view(np.uint16), want[s][j].view(np.uint16)), "replay %d output %d" % (i, j)
        run()   # eager work between replays
        torch.cuda.synchronize()


def test_hip_graph_replay_of_the_one_launch_layers_and_integer_outputs(hq):
    """The one-launch 3x3 and linear layers, the int8-resident convolution and the integer outputs that
    are accumulated with atomics (their output is zeroed by a kernel inside the call, not by a memset
    node) captured into one HIP graph: every replay must reproduce the eager results bit for bit."""
    rng = np.random.default_rng(11)
    nb, h, w, cin, cout = 8, 41, 50, 192, 250
    x = dev((rng.standard_normal((nb, h, w, cin)) * 2).astype(np.float16))
    wc = dev(rng.integers(-8, 8, (cout, 9, cin // 2 * 2)).astype(np.int8))
    wq = dev(pack_codes(rng.integers(-8, 8, (cout, 9, cin)).astype(np.int8)))
    sw = dev(rng.uniform(0.001, 0.1, cout).astype(np.float32))
    wl = dev(pack_codes(rng.integers(-8, 8, (cout, cin)).astype(np.int8)))
    xq = torch.empty((nb, h, w, cin // 2), dtype=torch.uint8, device="cuda")
    sx = torch.empty((nb, h, w), dtype=torch.float32, device="cuda")
    xs = dev(rng.integers(-8, 8, (1, 16, 16, 192)).astype(np.int8))      # a shape of the wave-split kernel
    xs_q = dev(pack_codes(host(xs)))
    ws_q = dev(pack_codes(rng.integers(-8, 8, (100, 9, 192)).astype(np.int8)))
    ys = [torch.empty((nb, h, w, cout), dtype=torch.float16, device="cuda") for _ in range(3)]
    yi = torch.empty((nb, h, w, 9, cout), dtype=torch.int32, device="cuda")
    yw = torch.empty((1, 16, 16, 9, 100), dtype=torch.int32, device="cuda")
    del wc
    assert hq.hq_int_conv2d_kernel_name(nb, h, w, cin, cout) == "activation-resident"
    assert hq.hq_int_conv2d_kernel_name(1, 16, 16, 192, 100) == "wave-split"

    def run():
        hq.hq_act_quant_int_conv2d(x, wq, sw, None, y_dtype=torch.float16, out=ys[0])
        hq.hq_act_quant_int_linear(x, wl, sw, None, y_dtype=torch.float16, out=ys[1])
        hq.hq_act_hadamard_quant(x, 64, 4, out=(xq, sx))
        hq.hq_int_conv2d(xq, sx, wq, sw, None, ksize=3, y_dtype=torch.float16, out=ys[2])
        hq.hq_int_conv2d(xq, None, wq, None, None, ksize=3, y_dtype=torch.int32, out=yi)
        hq.hq_int_conv2d(xs_q, None, ws_q, None, None, ksize=3, y_dtype=torch.int32, out=yw)

    outs = ys + [yi, yw]
    run()
    want = [host(t).copy() for t in outs]
    # (the two calls take another kernel for this shape: the same integers, fp32 sums in another order)
    check_y("one-launch layer against the two calls", want[0], want[2].astype(np.float64), rtol=1e-3)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for i in range(4):
        for t in outs:
            t.fill_(7)
        torch.cuda.synchronize()
        graph.replay()
        for j, t in enumerate(outs):
            assert np.array_equal(host(t), want[j]), "replay %d output %d" % (i, j)
        run()   # eager work between replays
        torch.cuda.synchronize()


def test_two_streams_at_once(hq):
    """The library keeps no state: two layers run on two streams at the same time and both results
    equal those of running them one after the other."""
    la, lb = workloads.tiny_layers()[4], workloads.tiny_layers()[0]
    xa, xb = dev(workloads.make_x(la)), dev(workloads.make_x(lb))
    wa, swa = hq.hq_quantize_weights(dev(workloads.make_w(la)), 64, 4)
    wb, swb = hq.hq_quantize_weights(dev(workloads.make_w(lb)), 64, 4)

    def layer_a():
        q, s = hq.hq_act_hadamard_quant(xa, 64, 4)
        return hq.hq_int_conv2d(q, s, wa, swa, None, ksize=3, y_dtype=torch.float16)

    def layer_b():
        q, s = hq.hq_act_hadamard_quant(xb, 64, 4)
        return hq.hq_int_linear(q, s, wb, swb, None, y_dtype=torch.float16)

    ya, yb = host(layer_a()).copy(), host(layer_b()).copy()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    outs = []
    for _ in range(8):
        with torch.cuda.stream(s1):
            oa = layer_a()
        with torch.cuda.stream(s2):
            ob = layer_b()
        outs.append((oa, ob))
    torch.cuda.synchronize()
    for oa, ob in outs:
        assert np.array_equal(host(oa).view(np.uint16), ya.view(np.uint16))
        assert np.array_equal(host(ob).view(np.uint16), yb.view(np.uint16))
