"""NumPy face of the CPU oracle (``hq_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Nothing in the product imports this module; only the
tests, the smoke check and the CPU-baseline leg of the benchmark may.  It
shares no code with the HIP library.

Every function takes the *stored* tensors (fp16 / fp32 NumPy arrays), widens
them exactly to fp64 and runs the plain C routines.  The steps follow the
paper's Method section: block-diagonal Hadamard transform over the contracted
axis ("Matrix Multiplication"), the symmetric quantiser of Background "Model
Quantization", an integer product, and dequantisation by the product of scales.
The header of ``hq_oracle.c`` states which variant of each open point is taken.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hq_oracle.c")
_LIB = os.path.join(_HERE, "libhq_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile hq_oracle.c with gcc (plain -O2, OpenMP over rows)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_dp = ctypes.POINTER(ctypes.c_double)
        c_i8p = ctypes.POINTER(ctypes.c_int8)
        c_i64p = ctypes.POINTER(ctypes.c_int64)
        i64, i32 = ctypes.c_int64, ctypes.c_int
        lib.hqo_hadamard_raw.argtypes = [i32, c_dp]
        lib.hqo_hadamard_raw.restype = None
        lib.hqo_block_hadamard.argtypes = [c_dp, i64, i32, i32, c_dp]
        lib.hqo_block_hadamard.restype = i32
        lib.hqo_quantize_rows.argtypes = [c_dp, i64, i32, i32, c_i8p, c_dp, c_dp]
        lib.hqo_quantize_rows.restype = i32
        lib.hqo_int_gemm.argtypes = [c_i8p, c_i8p, i64, i32, i32, c_i64p]
        lib.hqo_int_gemm.restype = None
        lib.hqo_dequant_linear.argtypes = [c_i64p, c_dp, c_dp, c_dp, i64, i32, c_dp]
        lib.hqo_dequant_linear.restype = None
        lib.hqo_int_conv2d.argtypes = [c_i8p, c_dp, c_i8p, c_dp, c_dp] + [i32] * 9 + [c_i64p, c_dp]
        lib.hqo_int_conv2d.restype = i32
        lib.hqo_quantize_static.argtypes = [c_dp, i64, i32, ctypes.c_double, c_i8p, c_dp]
        lib.hqo_quantize_static.restype = i32
        lib.hqo_int_conv2d_static.argtypes = ([c_i8p, ctypes.c_double, c_i8p, c_dp, c_dp] + [i32] * 9
                                              + [c_i64p, c_dp])
        lib.hqo_int_conv2d_static.restype = i32
        lib.hqo_int_gemm_single.argtypes = [c_i8p, c_i8p, i64, i32, i32, i32, c_i64p]
        lib.hqo_int_gemm_single.restype = i32
        lib.hqo_int_conv2d_width.argtypes = ([c_i8p, ctypes.c_double, c_i8p, c_dp, c_dp] + [i32] * 10
                                             + [c_i64p, c_dp])
        lib.hqo_int_conv2d_width.restype = i32
        lib.hqo_max_threads.argtypes = []
        lib.hqo_max_threads.restype = i32
        _lib = lib
    return _lib


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if a is not None else None


def _i8p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int8))


def _i64p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def max_threads() -> int:
    """Threads the oracle's row loops use."""
    return int(_load().hqo_max_threads())


def hadamard_raw(n: int) -> np.ndarray:
    """Unnormalised Sylvester matrix of order n (entries +-1)."""
    h = np.empty((n, n), dtype=np.float64)
    _load().hqo_hadamard_raw(n, _dp(h))
    return h


def block_hadamard(x, block: int) -> np.ndarray:
    """X * BlockDiag(H_k) over the last axis, dense fp64 product."""
    x64 = _f64(x)
    k = x64.shape[-1]
    m = x64.size // k if k else 0
    out = np.empty_like(x64)
    rc = _load().hqo_block_hadamard(_dp(x64), m, k, block, _dp(out))
    if rc != 0:
        raise ValueError("bad Hadamard shape: k=%d block=%d" % (k, block))
    return out


def quantize_rows(xt, bits: int):
    """Per-row abs-max symmetric quantiser.  Returns (codes int8, scale fp64, t fp64)."""
    x64 = _f64(xt)
    k = x64.shape[-1]
    m = x64.size // k if k else 0
    q = np.empty(x64.shape, dtype=np.int8)
    s = np.empty(x64.shape[:-1], dtype=np.float64)
    t = np.empty_like(x64)
    rc = _load().hqo_quantize_rows(_dp(x64), m, k, bits, _i8p(q), _dp(s), _dp(t))
    if rc != 0:
        raise ValueError("bad bit width %d" % bits)
    return q, s, t


def act_hadamard_quant(x, block: int, bits: int):
    """Activation side: transform over the last axis, one scale per token / pixel.

    x: [..., K] -> (codes [..., K] int8, scale [...] fp64, t [..., K] fp64)."""
    return quantize_rows(block_hadamard(x, block), bits)


def quantize_weights(w, block: int, bits: int):
    """Weight side, offline: w [n_out, taps, k_in] (taps = 1 for a linear layer,
    R*S for a convolution stored [Cout, R, S, Cin]).  The transform runs along
    k_in for every (n_out, tap) row; the scale is one per output channel, taken
    over all taps and input channels.

    Returns (codes [n_out, taps, k_in] int8, scale [n_out] fp64, t fp64)."""
    w64 = _f64(w)
    n_out, taps, k_in = w64.shape
    wt = block_hadamard(w64, block)
    q, s, t = quantize_rows(wt.reshape(n_out, taps * k_in), bits)
    return q.reshape(n_out, taps, k_in), s, t.reshape(n_out, taps, k_in)


def int_gemm(xq, wq) -> np.ndarray:
    """acc[m, n] = sum_k xq[m, k] wq[n, k] in int64."""
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    m, k = xq.shape
    n, k2 = wq.shape
    assert k == k2
    acc = np.empty((m, n), dtype=np.int64)
    _load().hqo_int_gemm(_i8p(xq), _i8p(wq), m, n, k, _i64p(acc))
    return acc


def int_linear(xq, sx, wq, sw, bias=None):
    """Integer product then dequantisation.  Returns (acc int64 [m, n], y fp64 [m, n])."""
    acc = int_gemm(xq, wq)
    m, n = acc.shape
    sx64, sw64 = _f64(sx).reshape(m), _f64(sw).reshape(n)
    b64 = _f64(bias).reshape(n) if bias is not None else None
    y = np.empty((m, n), dtype=np.float64)
    _load().hqo_dequant_linear(_i64p(acc), _dp(sx64), _dp(sw64), _dp(b64), m, n, _dp(y))
    assert np.abs(acc).max(initial=0) < 2**31
    return acc, y


def int_conv2d(xq, sx, wq, sw, bias=None, stride: int = 1, pad: int = 0,
               want_acc: bool = True, want_y: bool = True):
    """NHWC integer convolution with per-tap accumulators.

    xq [N, H, W, Cin] int8, sx [N, H, W], wq [Cout, R, S, Cin] int8, sw [Cout].
    Returns (acc_t int64 [N, Ho, Wo, R*S, Cout] or None, y fp64 [N, Ho, Wo, Cout] or None)."""
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    nb, h, w, cin = xq.shape
    cout, r, s, cin2 = wq.shape
    assert cin == cin2
    ho = (h + 2 * pad - r) // stride + 1
    wo = (w + 2 * pad - s) // stride + 1
    sx64, sw64 = _f64(sx).reshape(nb, h, w), _f64(sw).reshape(cout)
    b64 = _f64(bias).reshape(cout) if bias is not None else None
    acc = np.empty((nb, ho, wo, r * s, cout), dtype=np.int64) if want_acc else None
    y = np.empty((nb, ho, wo, cout), dtype=np.float64) if want_y else None
    rc = _load().hqo_int_conv2d(_i8p(xq), _dp(sx64), _i8p(wq), _dp(sw64), _dp(b64),
                                nb, h, w, cin, cout, r, s, stride, pad, _i64p(acc), _dp(y))
    if rc != 0:
        raise ValueError("bad convolution shape")
    if acc is not None:
        assert np.abs(acc).max(initial=0) < 2**31
    return acc, y


# ---- static mode: one caller-supplied activation scale per tensor -----------------------------

def quantize_static(xt, bits: int, scale: float):
    """Symmetric quantiser with a given scale for the whole tensor; the clamp is active.
    Returns (codes int8, t fp64)."""
    x64 = _f64(xt)
    q = np.empty(x64.shape, dtype=np.int8)
    t = np.empty_like(x64)
    rc = _load().hqo_quantize_static(_dp(x64), x64.size, bits, float(scale), _i8p(q), _dp(t))
    if rc != 0:
        raise ValueError("bad bit width %d or scale %r" % (bits, scale))
    return q, t


def act_hadamard_quant_static(x, block: int, bits: int, scale: float):
    """Activation side with a static scale: x [..., K] -> (codes [..., K] int8, t fp64)."""
    return quantize_static(block_hadamard(x, block), bits, scale)


def int_linear_static(xq, sx: float, wq, sw, bias=None):
    """Integer product, then y = sx * sw[n] * acc + bias.  Returns (acc int64, y fp64)."""
    acc = int_gemm(xq, wq)
    assert np.abs(acc).max(initial=0) < 2**31
    y = float(sx) * _f64(sw).reshape(1, -1) * acc.astype(np.float64)
    if bias is not None:
        y = y + _f64(bias).reshape(1, -1)
    return acc, y


def int_conv2d_static(xq, sx: float, wq, sw, bias=None, stride: int = 1, pad: int = 0,
                      want_acc: bool = True, want_y: bool = True):
    """NHWC integer convolution with one sum over all taps and input channels.

    Returns (acc int64 [N, Ho, Wo, Cout] or None, y fp64 [N, Ho, Wo, Cout] or None)."""
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    nb, h, w, cin = xq.shape
    cout, r, s, cin2 = wq.shape
    assert cin == cin2
    ho = (h + 2 * pad - r) // stride + 1
    wo = (w + 2 * pad - s) // stride + 1
    sw64 = _f64(sw).reshape(cout)
    b64 = _f64(bias).reshape(cout) if bias is not None else None
    acc = np.empty((nb, ho, wo, cout), dtype=np.int64) if want_acc else None
    y = np.empty((nb, ho, wo, cout), dtype=np.float64) if want_y else None
    rc = _load().hqo_int_conv2d_static(_i8p(xq), float(sx), _i8p(wq), _dp(sw64), _dp(b64),
                                       nb, h, w, cin, cout, r, s, stride, pad, _i64p(acc), _dp(y))
    if rc != 0:
        raise ValueError("bad convolution shape")
    if acc is not None:
        assert np.abs(acc).max(initial=0) < 2**31
    return acc, y


# ---- Single scheme: weights quantised without the transform, integer H between the operands ----

def quantize_weights_single(w, bits: int):
    """Weights of the paper's own linear layer (Method, "Single Hadamard Transformation"): quantised
    as they are, one abs-max scale per output channel.  w [n_out, k_in].
    Returns (codes [n_out, k_in] int8, scale [n_out] fp64, t fp64)."""
    w64 = _f64(w)
    assert w64.ndim == 2
    return quantize_rows(w64, bits)


def int_gemm_single(xq, wq, block: int) -> np.ndarray:
    """acc = (xq BlockDiag(H_raw)) wq^T in int64 (Method, linear-layer equation)."""
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    m, k = xq.shape
    n, k2 = wq.shape
    assert k == k2
    acc = np.empty((m, n), dtype=np.int64)
    rc = _load().hqo_int_gemm_single(_i8p(xq), _i8p(wq), m, n, k, int(block), _i64p(acc))
    if rc != 0:
        raise ValueError("block %d does not fit k = %d" % (block, k))
    return acc


def int_linear_single(xq, sx, wq, sw, block: int, bias=None):
    """y = S_XH S_W 2^(-log2(block)/2) ((XH)_int H_raw W_int^T) + bias.
    Returns (acc int64 [m, n], y fp64 [m, n])."""
    acc = int_gemm_single(xq, wq, block)
    assert np.abs(acc).max(initial=0) < 2**31
    m, n = acc.shape
    y = acc.astype(np.float64) * _f64(sx).reshape(m, 1) * _f64(sw).reshape(1, n) / np.sqrt(float(block))
    if bias is not None:
        y = y + _f64(bias).reshape(1, n)
    return acc, y


# ---- width-axis convolution: the paper's own convolution ---------------------------------------

def act_width_quant_static(x, block: int, bits: int, scale: float):
    """Activation side of the paper's convolution (Method, "Convolution"): x [N, H, W, C] is
    transformed along the WIDTH axis (every image line of every channel is one row of X~) and
    quantised with one scale for the tensor.  Returns (codes [N, H, W, C] int8, t fp64)."""
    x64 = _f64(x)
    assert x64.ndim == 4
    lines = np.ascontiguousarray(np.moveaxis(x64, 2, 3))          # [N, H, C, W]: rows of X~
    q, t = quantize_static(block_hadamard(lines, block), bits, scale)
    return (np.ascontiguousarray(np.moveaxis(q, 3, 2)), np.ascontiguousarray(np.moveaxis(t, 3, 2)))


def int_conv2d_width(xq, sx: float, wq, sw, block: int, bias=None, stride: int = 1, pad: int = 0,
                     want_acc: bool = True, want_y: bool = True):
    """Conv((X~ H_c)_int H_c,raw, W_int), then y = sx * sw[co] * acc / sqrt(block) + bias.
    xq [N, H, W, Cin] codes of the width-transformed activations, wq [Cout, R, S, Cin] codes of the
    un-transformed weights.  Returns (acc int64 or None, y fp64 or None), [N, Ho, Wo, Cout]."""
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    wq = np.ascontiguousarray(wq, dtype=np.int8)
    nb, h, w, cin = xq.shape
    cout, r, s, cin2 = wq.shape
    assert cin == cin2
    ho = (h + 2 * pad - r) // stride + 1
    wo = (w + 2 * pad - s) // stride + 1
    sw64 = _f64(sw).reshape(cout)
    b64 = _f64(bias).reshape(cout) if bias is not None else None
    acc = np.empty((nb, ho, wo, cout), dtype=np.int64) if want_acc else None
    y = np.empty((nb, ho, wo, cout), dtype=np.float64) if want_y else None
    rc = _load().hqo_int_conv2d_width(_i8p(xq), float(sx), _i8p(wq), _dp(sw64), _dp(b64), nb, h, w, cin, cout,
                                      r, s, stride, pad, int(block), _i64p(acc), _dp(y))
    if rc != 0:
        raise ValueError("bad geometry or block for the width-axis convolution")
    if acc is not None:
        assert np.abs(acc).max(initial=0) < 2**31
    return acc, y
