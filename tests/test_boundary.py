"""The C-ABI library: it loads, exports what include/hq.h declares, and rejects
bad arguments on the host before anything is launched.  No GPU needed."""
import ctypes
import os
import re

import pytest

import paper_2512_05746_amd as hq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
OK, NULL, SHAPE, DTYPE, BITS, ALIGN, UNSUPPORTED = range(7)
P = 4096  # any non-null, 16-byte-aligned fake device address: validation never dereferences it


@pytest.fixture(scope="module")
def lib():
    return hq.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hq_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(hq.binding.SYMBOLS) | set(hq.binding.INFO_SYMBOLS)
    for name in names:
        assert getattr(lib, name) is not None


def test_conv_kernel_choice_is_a_function_of_the_geometry(lib):
    """The kernel family is reported per geometry (no output type among the arguments): the three
    3x3 families are each reachable, and geometries that are not built say so."""
    name = hq.hq_int_conv2d_kernel_name
    assert name(16, 64, 64, 192, 192) == "activation-resident"
    assert name(20, 50, 50, 192, 64) == "activation-resident-int8 (128 pixels, 4 waves)"
    assert name(6, 70, 75, 192, 330) == "activation-resident-int8 (256 pixels)"
    assert name(16, 32, 32, 384, 384) == "activation-resident-int8 (128 pixels)"
    assert name(16, 16, 16, 576, 576) == "activation-resident-int8 (64 pixels)"
    assert name(16, 8, 8, 960, 960) == "wave-split"
    assert name(16, 64, 64, 192, 192, static_scale=True) == "activation-resident"
    assert name(16, 32, 32, 384, 384, static_scale=True) == "activation-resident"
    assert name(2, 9, 9, 64, 8) == "tile"
    assert name(2, 9, 9, 64, 8, ksize=1) == "tile"
    assert name(2, 9, 9, 64, 8, stride=2) == "tile (stride 2)"
    assert name(2, 9, 9, 64, 8, ksize=5) == "unsupported"
    assert name(16, 64, 64, 192, 192, bits=8) == "tile"
    assert name(2, 32, 32, 8, 320) == "small-channel-count"
    assert name(2, 32, 32, 200, 64, ksize=1) == "small-channel-count"
    assert name(2, 32, 32, 12, 64) == "unsupported"
    assert name(2, 32, 32, 72, 64, bits=8) == "unsupported"


def test_fused_conv_argument_errors(lib):
    f = lib.hq_act_quant_int_conv2d
    args = lambda **kw: [kw.get(k, d) for k, d in [
        ("x", P), ("xdt", 0), ("wq", P), ("sw", P), ("bias", None), ("nb", 1), ("h", 4), ("w", 4), ("cin", 192),
        ("cout", 8), ("r", 3), ("s", 3), ("stride", 1), ("pad", 1), ("block", 64), ("bits", 4), ("y", P),
        ("dt", 0), ("xq", None), ("sx", None), ("stream", None)]]
    assert f(*args(x=None)) == NULL
    assert f(*args(sw=None)) == NULL
    assert f(*args(dt=7)) == DTYPE
    assert f(*args(xdt=2)) == DTYPE
    assert f(*args(bits=5)) == BITS
    assert f(*args(h=0)) == SHAPE
    assert f(*args(cin=100)) == SHAPE            # not a multiple of the block
    assert f(*args(y=P + 4)) == ALIGN
    assert f(*args(xq=P + 8)) == ALIGN
    assert f(*args(xdt=1)) == UNSUPPORTED        # fp32 activations: use the two calls
    assert f(*args(block=32)) == UNSUPPORTED
    assert f(*args(cin=128)) == UNSUPPORTED      # channel slices of 192 only
    assert f(*args(r=1, s=1, pad=0)) == UNSUPPORTED
    assert f(*args(stride=2)) == UNSUPPORTED
    assert f(*args(cin=192 * 12, w=64)) == UNSUPPORTED   # the tile's activations do not fit on chip


def test_fused_linear_argument_errors(lib):
    f = lib.hq_act_quant_int_linear
    args = lambda **kw: [kw.get(k, d) for k, d in [
        ("x", P), ("xdt", 0), ("wq", P), ("sw", P), ("bias", None), ("m", 8), ("n", 8), ("k", 64), ("block", 64),
        ("bits", 4), ("y", P), ("dt", 0), ("xq", None), ("sx", None), ("stream", None)]]
    assert f(*args(x=None)) == NULL
    assert f(*args(sw=None)) == NULL
    assert f(*args(dt=7)) == DTYPE
    assert f(*args(bits=5)) == BITS
    assert f(*args(m=0)) == SHAPE
    assert f(*args(k=100)) == SHAPE
    assert f(*args(y=P + 4)) == ALIGN
    assert f(*args(xdt=1)) == UNSUPPORTED
    assert f(*args(block=32, k=96)) == UNSUPPORTED
    assert f(*args(k=2048)) == UNSUPPORTED


def test_status_strings(lib):
    texts = [hq.status_string(i) for i in range(8)]
    assert texts[0] == "ok" and len(set(texts)) == 8
    assert hq.status_string(99) == "unknown status"


def test_act_quant_argument_errors(lib):
    f = lib.hq_act_hadamard_quant
    assert f(None, 0, 8, 64, 64, 4, P, P, None) == NULL
    assert f(P, 0, 8, 64, 64, 4, None, P, None) == NULL
    assert f(P, 0, 8, 64, 64, 4, P, None, None) == NULL
    assert f(P, 2, 8, 64, 64, 4, P, P, None) == DTYPE      # int32 is not an input dtype
    assert f(P, 0, 8, 64, 64, 6, P, P, None) == BITS
    assert f(P, 0, 8, 64, 64, 1, P, P, None) == BITS
    assert f(P, 0, 0, 64, 64, 4, P, P, None) == SHAPE      # no rows
    assert f(P, 0, 8, 96, 64, 4, P, P, None) == SHAPE      # k not a multiple of the block
    assert f(P, 0, 8, 64, 48, 4, P, P, None) == SHAPE      # block not a power of two
    assert f(P, 0, 8, 256, 256, 4, P, P, None) == SHAPE    # block above 128
    assert f(P, 0, 8, 4, 4, 4, P, P, None) == SHAPE        # k not a multiple of 8
    assert f(P + 8, 0, 8, 64, 64, 4, P, P, None) == ALIGN
    assert f(P, 0, 8, 64, 64, 4, P + 4, P, None) == ALIGN
    assert f(P, 0, 8, 64, 64, 4, P, P + 2, None) == ALIGN


def test_weight_quant_argument_errors(lib):
    f = lib.hq_quantize_weights
    assert f(None, 0, 8, 1, 64, 64, 4, P, P, None) == NULL
    assert f(P, 0, 8, 0, 64, 64, 4, P, P, None) == SHAPE
    assert f(P, 0, 0, 1, 64, 64, 4, P, P, None) == SHAPE
    assert f(P, 0, 8, 9, 96, 64, 4, P, P, None) == SHAPE
    assert f(P, 7, 8, 9, 64, 64, 4, P, P, None) == DTYPE
    assert f(P, 0, 8, 9, 64, 64, 5, P, P, None) == BITS


def test_linear_argument_errors(lib):
    f = lib.hq_int_linear
    assert f(None, P, P, P, None, 8, 8, 64, P, 0, None) == NULL
    assert f(P, None, P, P, None, 8, 8, 64, P, 0, None) == NULL    # scales needed for fp output
    assert f(P, P, P, P, None, 8, 8, 64, None, 0, None) == NULL
    assert f(P, P, P, P, None, 8, 8, 64, P, 5, None) == DTYPE
    assert f(P, P, P, P, None, 8, 8, 36, P, 0, None) == SHAPE       # k not a multiple of 8
    assert f(P, P, P, P, None, 8, 8, 4, P, 0, None) == SHAPE
    assert f(P, P, P, P, None, 8, 0, 64, P, 0, None) == SHAPE
    assert f(P, P, P, P, None, 0, 8, 64, P, 0, None) == SHAPE
    assert f(P, P, P, P, None, 8, 8, 131072, P, 0, None) == SHAPE   # 256 * acc would overflow
    assert f(P + 4, P, P, P, None, 8, 8, 64, P, 0, None) == ALIGN
    assert f(P, P, P, P, P + 1, 8, 8, 64, P, 0, None) == ALIGN


def test_conv_argument_errors(lib):
    f = lib.hq_int_conv2d
    args = lambda **kw: [kw.get(k, d) for k, d in [
        ("xq", P), ("sx", P), ("wq", P), ("sw", P), ("bias", None), ("nb", 1), ("h", 4), ("w", 4),
        ("cin", 64), ("cout", 8), ("r", 3), ("s", 3), ("stride", 1), ("pad", 1), ("y", P),
        ("dt", 0), ("stream", None)]]
    assert f(*args(xq=None)) == NULL
    assert f(*args(h=0)) == SHAPE
    assert f(*args(cin=20)) == SHAPE                          # not a multiple of 8
    assert f(*args(cin=96, stride=2)) == SHAPE               # the stride-2 form needs whole 64-code chunks
    assert f(*args(stride=3)) == UNSUPPORTED
    assert f(*args(stride=2, pad=0)) == UNSUPPORTED          # stride 2 is built for 3x3, pad 1 only
    assert f(*args(stride=2, r=1, s=1, pad=0)) == UNSUPPORTED
    assert f(*args(pad=0)) == UNSUPPORTED
    assert f(*args(r=5, s=5, pad=2)) == UNSUPPORTED
    assert f(*args(r=3, s=1)) == UNSUPPORTED
    assert f(*args(dt=9)) == DTYPE
    assert f(*args(y=P + 2)) == ALIGN


def test_static_scale_argument_errors(lib):
    q = lib.hq_act_hadamard_quant_static
    assert q(P, 0, 8, 64, 64, 4, None, P, None) == NULL     # the scale is an input here
    assert q(P, 0, 8, 64, 64, 4, P, None, None) == NULL
    assert q(P, 0, 8, 64, 64, 4, P + 2, P, None) == ALIGN
    assert q(P, 0, 8, 96, 64, 4, P, P, None) == SHAPE
    assert q(P, 0, 8, 64, 64, 5, P, P, None) == BITS
    lin = lib.hq_int_linear_static
    assert lin(P, None, P, P, None, 8, 8, 64, P, 0, None) == NULL
    assert lin(P, P, P, P, None, 8, 8, 12, P, 0, None) == SHAPE
    conv = lib.hq_int_conv2d_static
    args = lambda **kw: [kw.get(k, d) for k, d in [
        ("xq", P), ("sx", P), ("wq", P), ("sw", P), ("bias", None), ("nb", 1), ("h", 4), ("w", 4),
        ("cin", 64), ("cout", 8), ("r", 3), ("s", 3), ("stride", 1), ("pad", 1), ("y", P),
        ("dt", 0), ("stream", None)]]
    assert conv(*args(sx=None)) == NULL
    assert conv(*args(stride=3)) == UNSUPPORTED
    assert conv(*args(stride=2, pad=0)) == UNSUPPORTED
    assert conv(*args(cin=14592)) == SHAPE      # 9 * 14592 codes in one sum: 256 * acc would overflow
    assert conv(*args(cin=20)) == SHAPE          # not a multiple of 8


def test_single_scheme_argument_errors(lib):
    wq = lib.hq_quantize_weights_single
    assert wq(None, 0, 8, 64, 64, 4, P, P, None) == NULL
    assert wq(P, 2, 8, 64, 64, 4, P, P, None) == DTYPE
    assert wq(P, 0, 8, 64, 64, 8, P, P, None) == BITS
    assert wq(P, 0, 0, 64, 64, 4, P, P, None) == SHAPE
    assert wq(P, 0, 8, 63, 1, 4, P, P, None) == SHAPE        # odd row length
    assert wq(P, 0, 8, 96, 64, 4, P, P, None) == SHAPE       # block does not divide the row
    assert wq(P, 0, 8, 768, 256, 4, P, P, None) == SHAPE     # block above 128
    assert wq(P + 2, 0, 8, 64, 64, 4, P, P, None) == ALIGN
    lin = lib.hq_int_linear_single
    assert lin(P, P, None, P, None, 8, 8, 64, 64, P, 0, None) == NULL
    assert lin(P, None, P, P, None, 8, 8, 64, 64, P, 0, None) == NULL     # scales needed for fp output
    assert lin(P, P, P, P, None, 8, 8, 96, 32, P, 0, None) == SHAPE       # k not a multiple of 64
    assert lin(P, P, P, P, None, 8, 8, 192, 128, P, 0, None) == SHAPE     # block does not divide k
    assert lin(P, P, P, P, None, 8, 8, 64, 64, P, 3, None) == DTYPE
    assert lin(P, P, P, P, None, 8, 8, 64, 64, P + 4, 0, None) == ALIGN


def test_width_axis_argument_errors(lib):
    q = lib.hq_act_hadamard_quant_width
    assert q(P, 0, 1, 4, 8, 64, 8, 4, None, P, None) == NULL
    assert q(P, 2, 1, 4, 8, 64, 8, 4, P, P, None) == DTYPE
    assert q(P, 0, 1, 4, 8, 64, 8, 5, P, P, None) == BITS
    assert q(P, 0, 1, 4, 8, 63, 8, 4, P, P, None) == SHAPE       # odd channel count
    assert q(P, 0, 1, 4, 12, 64, 8, 4, P, P, None) == SHAPE      # block does not divide the width
    assert q(P, 0, 1, 4, 128, 64, 128, 4, P, P, None) == SHAPE   # block above 64
    assert q(P, 0, 1, 4, 8, 64, 8, 4, P + 2, P, None) == ALIGN
    conv = lib.hq_int_conv2d_width
    args = lambda **kw: [kw.get(k, d) for k, d in [
        ("xu3", P), ("sx", P), ("wq", P), ("sw", P), ("bias", None), ("nb", 1), ("h", 4), ("w", 8),
        ("cin", 64), ("cout", 8), ("r", 3), ("s", 3), ("stride", 1), ("pad", 1), ("block", 8), ("y", P),
        ("dt", 0), ("stream", None)]]
    assert conv(*args(xu3=None)) == NULL
    assert conv(*args(sx=None)) == NULL
    assert conv(*args(block=16)) == SHAPE
    assert conv(*args(cin=20)) == SHAPE          # not a multiple of 8
    assert conv(*args(r=1, s=1, pad=0)) == UNSUPPORTED
    assert conv(*args(stride=3)) == UNSUPPORTED


def test_int8_code_argument_errors(lib):
    lin = lib.hq_int_linear_i8
    assert lin(None, P, P, P, None, 8, 8, 64, P, 0, None) == NULL
    assert lin(P, P, P, P, None, 8, 8, 96, P, 0, None) == SHAPE
    assert lin(P, P, P, P, None, 8, 8, 64, P, 5, None) == DTYPE
    conv = lib.hq_int_conv2d_i8
    assert conv(P, P, P, P, None, 1, 4, 4, 64, 8, 3, 3, 3, 1, P, 0, None) == UNSUPPORTED
    assert conv(P, None, P, P, None, 1, 4, 4, 64, 8, 3, 3, 1, 1, P, 0, None) == NULL
    q8 = lib.hq_act_hadamard_quant_i8
    assert q8(P, 0, 8, 64, 64, 4, None, P, None) == NULL
    assert q8(P, 0, 8, 64, 64, 5, P, P, None) == BITS
    assert q8(P, 0, 8, 96, 64, 4, P, P, None) == SHAPE
    # 8-bit codes are a legal width for both quantisers, 5 bits are not
    assert lib.hq_act_hadamard_quant(None, 0, 8, 64, 64, 8, P, P, None) == NULL
    assert lib.hq_act_hadamard_quant(P, 0, 8, 64, 64, 5, P, P, None) == BITS


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2512_05746_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text, os.path.join(dirpath, fn)


def test_binding_rejects_host_tensors_before_any_call():
    """The Python face takes device tensors only; a host tensor is refused by the binding itself,
    before the library is asked anything (so this needs no GPU)."""
    import torch
    import paper_2512_05746_amd as hq
    codes = torch.zeros((4, 32), dtype=torch.uint8)
    with pytest.raises(ValueError):
        hq.hq_int_linear(codes, None, codes, None, None, y_dtype=torch.int32)
    with pytest.raises(ValueError):
        hq.hq_act_hadamard_quant(torch.zeros((4, 64), dtype=torch.float16), 64, 4)
    with pytest.raises(ValueError):
        hq.hq_int_conv2d(torch.zeros((1, 2, 2, 32), dtype=torch.uint8), None, torch.zeros((8, 9, 32), dtype=torch.uint8),
                         None, None, ksize=3, y_dtype=torch.int32)
