"""ctypes binding of libhq.so: argument marshalling only.

Every function here has the name and meaning of the C entry point declared in
``include/hq.h``; tensors are PyTorch tensors used purely as device buffers, and
the work is enqueued on PyTorch's current HIP stream.  There is no fallback: if
the library cannot be loaded or a call is refused, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

from . import build as _build

HQ_F16, HQ_F32, HQ_I32 = 0, 1, 2
_DTYPES = {torch.float16: HQ_F16, torch.float32: HQ_F32, torch.int32: HQ_I32}

SYMBOLS = ("hq_status_string", "hq_quantize_weights", "hq_act_hadamard_quant",
           "hq_int_linear", "hq_int_conv2d", "hq_act_hadamard_quant_static",
           "hq_int_linear_static", "hq_int_conv2d_static",
           "hq_quantize_weights_single", "hq_int_linear_single",
           "hq_act_hadamard_quant_width", "hq_int_conv2d_width",
           "hq_int_linear_i8", "hq_int_conv2d_i8", "hq_act_hadamard_quant_i8",
           "hq_act_quant_int_conv2d", "hq_act_quant_int_linear")
# entry points that do not return a status
INFO_SYMBOLS = ("hq_int_conv2d_kernel_name",)


class HqError(RuntimeError):
    def __init__(self, fn: str, code: int, text: str):
        super().__init__("%s failed: %s (status %d)" % (fn, text, code))
        self.code = code


_lib = None


def load_library(path: Optional[str] = None) -> ctypes.CDLL:
    """Loads libhq.so.  The in-tree library is built first if it is missing or older than one of
    its sources (a child-process compile; nothing here touches the GPU before that)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    if path is None:
        path = _build.LIB
        if _build.is_stale():
            _build.build_lib()
    lib = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.hq_status_string.argtypes = [i32]
    lib.hq_status_string.restype = ctypes.c_char_p
    lib.hq_quantize_weights.argtypes = [vp, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.hq_act_hadamard_quant.argtypes = [vp, i32, i64, i32, i32, i32, vp, vp, vp]
    lib.hq_int_linear.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, vp, i32, vp]
    lib.hq_int_conv2d.argtypes = [vp] * 5 + [i32] * 9 + [vp, i32, vp]
    lib.hq_act_hadamard_quant_static.argtypes = [vp, i32, i64, i32, i32, i32, vp, vp, vp]
    lib.hq_int_linear_static.argtypes = lib.hq_int_linear.argtypes
    lib.hq_int_conv2d_static.argtypes = lib.hq_int_conv2d.argtypes
    lib.hq_quantize_weights_single.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.hq_int_linear_single.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, i32, vp, i32, vp]
    lib.hq_act_hadamard_quant_width.argtypes = [vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp]
    lib.hq_int_conv2d_width.argtypes = [vp] * 5 + [i32] * 10 + [vp, i32, vp]
    lib.hq_int_linear_i8.argtypes = lib.hq_int_linear.argtypes
    lib.hq_act_hadamard_quant_i8.argtypes = lib.hq_act_hadamard_quant.argtypes
    lib.hq_int_conv2d_i8.argtypes = lib.hq_int_conv2d.argtypes
    lib.hq_act_quant_int_conv2d.argtypes = [vp, i32, vp, vp, vp] + [i32] * 11 + [vp, i32, vp, vp, vp]
    lib.hq_act_quant_int_linear.argtypes = [vp, i32, vp, vp, vp, i64, i32, i32, i32, i32, vp, i32, vp, vp, vp]
    for name in SYMBOLS[1:]:
        getattr(lib, name).restype = i32
    lib.hq_int_conv2d_kernel_name.argtypes = [i32] * 11
    lib.hq_int_conv2d_kernel_name.restype = ctypes.c_char_p
    _lib = lib
    return lib


def hq_int_conv2d_kernel_name(nb: int, h: int, w: int, c_in: int, c_out: int, ksize: int = 3, stride: int = 1,
                              pad: Optional[int] = None, static_scale: bool = False, bits: int = 4) -> str:
    """Name of the kernel family the convolution calls run for this geometry (host logic only)."""
    pad = (ksize - 1) // 2 if pad is None else pad
    return load_library().hq_int_conv2d_kernel_name(nb, h, w, c_in, c_out, ksize, ksize, stride, pad,
                                                    1 if static_scale else 0, bits).decode()


def status_string(code: int) -> str:
    return load_library().hq_status_string(code).decode()


def _check(fn: str, code: int) -> None:
    if code != 0:
        raise HqError(fn, code, status_string(code))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _dev(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous device tensor" % name)
    return t


def _conv_out(h: int, w: int, ksize: int, stride: int, pad: int):
    if stride < 1 or pad < 0 or ksize < 1:
        raise ValueError("bad convolution geometry")
    return (h + 2 * pad - ksize) // stride + 1, (w + 2 * pad - ksize) // stride + 1


def _out(out: Optional[torch.Tensor], shape, dtype: torch.dtype, device) -> torch.Tensor:
    """A caller's output buffer (must hold exactly the result) or a new one."""
    if out is None:
        return torch.empty(shape, dtype=dtype, device=device)
    n = 1
    for d in shape:
        n *= d
    if not out.is_cuda or out.dtype != dtype or out.numel() != n or not out.is_contiguous():
        raise ValueError("out must be a contiguous device tensor of %s with %d elements" % (dtype, n))
    return out


def _vec(t: Optional[torch.Tensor], n: int, dtype: torch.dtype, name: str) -> Optional[torch.Tensor]:
    """An optional per-row / per-channel device vector: exactly n elements of dtype."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype or t.numel() != n:
        raise ValueError("%s must be a contiguous device tensor of %s with %d elements" % (name, dtype, n))
    return t


def _codes(t: torch.Tensor, dtype: torch.dtype, name: str) -> torch.Tensor:
    _dev(t, name)
    if t.dtype != dtype:
        raise ValueError("%s must hold %s codes" % (name, dtype))
    return t


def hq_quantize_weights(w: torch.Tensor, had_block: int = 64, w_bits: int = 4
                        ) -> Tuple[torch.Tensor, torch.Tensor]:
    """w [n_out, taps, k_in] fp16/fp32 -> (wq uint8 [n_out, taps, k_in/2], w_scale fp32 [n_out]);
    w_bits = 8: wq int8 [n_out, taps, k_in], one code per byte."""
    _dev(w, "w")
    n_out, taps, k_in = w.shape
    if w_bits == 8:
        wq = torch.empty((n_out, taps, k_in), dtype=torch.int8, device=w.device)
    else:
        wq = torch.empty((n_out, taps, k_in // 2), dtype=torch.uint8, device=w.device)
    ws = torch.empty((n_out,), dtype=torch.float32, device=w.device)
    _check("hq_quantize_weights", load_library().hq_quantize_weights(
        _ptr(w), _DTYPES[w.dtype], n_out, taps, k_in, had_block, w_bits, _ptr(wq), _ptr(ws), _stream()))
    return wq, ws


def hq_act_hadamard_quant(x: torch.Tensor, had_block: int = 64, a_bits: int = 4,
                          out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None
                          ) -> Tuple[torch.Tensor, torch.Tensor]:
    """x [..., k] fp16/fp32 -> (xq uint8 [..., k/2], x_scale fp32 [...]); a_bits = 8: xq int8 [..., k]."""
    _dev(x, "x")
    k = x.shape[-1]
    m = x.numel() // k
    if out is None:
        if a_bits == 8:
            xq = torch.empty(x.shape[:-1] + (k,), dtype=torch.int8, device=x.device)
        else:
            xq = torch.empty(x.shape[:-1] + (k // 2,), dtype=torch.uint8, device=x.device)
        xs = torch.empty(x.shape[:-1], dtype=torch.float32, device=x.device)
    else:
        xq = _out(out[0], x.shape[:-1] + ((k,) if a_bits == 8 else (k // 2,)),
                  torch.int8 if a_bits == 8 else torch.uint8, x.device)
        xs = _out(out[1], x.shape[:-1], torch.float32, x.device)
    _check("hq_act_hadamard_quant", load_library().hq_act_hadamard_quant(
        _ptr(x), _DTYPES[x.dtype], m, k, had_block, a_bits, _ptr(xq), _ptr(xs), _stream()))
    return xq, xs


def hq_int_linear(xq: torch.Tensor, x_scale: Optional[torch.Tensor], wq: torch.Tensor,
                  w_scale: Optional[torch.Tensor], bias: Optional[torch.Tensor] = None,
                  y_dtype: torch.dtype = torch.float16, out: Optional[torch.Tensor] = None
                  ) -> torch.Tensor:
    """xq [m, k/2], wq [n, k/2] (or [n, 1, k/2]) -> y [m, n]; y_dtype int32 returns the raw sums."""
    _codes(xq, torch.uint8, "xq"), _codes(wq, torch.uint8, "wq")
    m, kb = xq.shape
    n = wq.shape[0]
    if wq.numel() != n * kb:
        raise ValueError("wq does not match xq in k")
    _vec(x_scale, m, torch.float32, "x_scale"), _vec(w_scale, n, torch.float32, "w_scale")
    _vec(bias, n, y_dtype, "bias")
    y = _out(out, (m, n), y_dtype, xq.device)
    _check("hq_int_linear", load_library().hq_int_linear(
        _ptr(xq), _ptr(x_scale), _ptr(wq), _ptr(w_scale), _ptr(bias), m, n, kb * 2,
        _ptr(y), _DTYPES[y_dtype], _stream()))
    return y


def hq_int_conv2d(xq: torch.Tensor, x_scale: Optional[torch.Tensor], wq: torch.Tensor,
                  w_scale: Optional[torch.Tensor], bias: Optional[torch.Tensor] = None,
                  ksize: int = 3, stride: int = 1, pad: Optional[int] = None,
                  y_dtype: torch.dtype = torch.float16, out: Optional[torch.Tensor] = None
                  ) -> torch.Tensor:
    """xq [nb, h, w, cin/2], wq [cout, ksize*ksize, cin/2] -> y [nb, ho, wo, cout] (same size for
    stride 1; ksize 3, stride 2, pad 1 halves it, rounding up); y_dtype int32 returns the per-tap
    sums [nb, ho, wo, ksize*ksize, cout]."""
    _codes(xq, torch.uint8, "xq"), _codes(wq, torch.uint8, "wq")
    nb, h, w, cb = xq.shape
    cout = wq.shape[0]
    if wq.numel() != cout * ksize * ksize * cb:
        raise ValueError("wq does not match xq / ksize")
    _vec(x_scale, nb * h * w, torch.float32, "x_scale"), _vec(w_scale, cout, torch.float32, "w_scale")
    _vec(bias, cout, y_dtype, "bias")
    pad = (ksize - 1) // 2 if pad is None else pad
    ho, wo = _conv_out(h, w, ksize, stride, pad)
    if y_dtype == torch.int32:
        y = _out(out, (nb, ho, wo, ksize * ksize, cout), y_dtype, xq.device)
    else:
        y = _out(out, (nb, ho, wo, cout), y_dtype, xq.device)
    _check("hq_int_conv2d", load_library().hq_int_conv2d(
        _ptr(xq), _ptr(x_scale), _ptr(wq), _ptr(w_scale), _ptr(bias), nb, h, w, cb * 2, cout,
        ksize, ksize, stride, pad, _ptr(y), _DTYPES[y_dtype], _stream()))
    return y


def hq_act_quant_int_conv2d(x: torch.Tensor, wq: torch.Tensor, w_scale: Optional[torch.Tensor],
                            bias: Optional[torch.Tensor] = None, had_block: int = 64, a_bits: int = 4,
                            ksize: int = 3, stride: int = 1, pad: Optional[int] = None,
                            y_dtype: torch.dtype = torch.float16, out: Optional[torch.Tensor] = None,
                            codes_out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None) -> torch.Tensor:
    """The whole 3x3 layer in one launch: x [nb, h, w, cin] fp16, wq [cout, 9, cin/2] -> y [nb, h, w, cout]
    (y_dtype int32: per-tap sums [nb, h, w, 9, cout]).  codes_out = (xq uint8 [nb, h, w, cin/2],
    x_scale fp32 [nb, h, w]) receives the codes and scales the kernel used."""
    _dev(x, "x"), _codes(wq, torch.uint8, "wq")
    nb, h, w, cin = x.shape
    cout = wq.shape[0]
    if wq.numel() != cout * ksize * ksize * (cin // 2):
        raise ValueError("wq does not match x / ksize")
    _vec(w_scale, cout, torch.float32, "w_scale"), _vec(bias, cout, y_dtype, "bias")
    pad = (ksize - 1) // 2 if pad is None else pad
    ho, wo = _conv_out(h, w, ksize, stride, pad)
    if y_dtype == torch.int32:
        y = _out(out, (nb, ho, wo, ksize * ksize, cout), y_dtype, x.device)
    else:
        y = _out(out, (nb, ho, wo, cout), y_dtype, x.device)
    xq = sx = None
    if codes_out is not None:
        xq = _out(codes_out[0], (nb, h, w, cin // 2), torch.uint8, x.device)
        sx = _out(codes_out[1], (nb, h, w), torch.float32, x.device)
    _check("hq_act_quant_int_conv2d", load_library().hq_act_quant_int_conv2d(
        _ptr(x), _DTYPES[x.dtype], _ptr(wq), _ptr(w_scale), _ptr(bias), nb, h, w, cin, cout, ksize, ksize,
        stride, pad, had_block, a_bits, _ptr(y), _DTYPES[y_dtype], _ptr(xq), _ptr(sx), _stream()))
    return y


def hq_act_quant_int_linear(x: torch.Tensor, wq: torch.Tensor, w_scale: Optional[torch.Tensor],
                            bias: Optional[torch.Tensor] = None, had_block: int = 64, a_bits: int = 4,
                            y_dtype: torch.dtype = torch.float16, out: Optional[torch.Tensor] = None,
                            codes_out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None) -> torch.Tensor:
    """A linear layer / 1x1 convolution in one launch: x [..., k] fp16, wq [n, k/2] (or [n, 1, k/2]) ->
    y [..., n] (y_dtype int32: the integer sums).  codes_out = (xq uint8 [..., k/2], x_scale fp32 [...])
    receives the codes and scales the kernel used."""
    _dev(x, "x"), _codes(wq, torch.uint8, "wq")
    k = x.shape[-1]
    m = x.numel() // k
    n = wq.shape[0]
    if wq.numel() != n * (k // 2):
        raise ValueError("wq does not match x")
    _vec(w_scale, n, torch.float32, "w_scale"), _vec(bias, n, y_dtype, "bias")
    y = _out(out, tuple(x.shape[:-1]) + (n,), y_dtype, x.device)
    xq = sx = None
    if codes_out is not None:
        xq = _out(codes_out[0], tuple(x.shape[:-1]) + (k // 2,), torch.uint8, x.device)
        sx = _out(codes_out[1], tuple(x.shape[:-1]), torch.float32, x.device)
    _check("hq_act_quant_int_linear", load_library().hq_act_quant_int_linear(
        _ptr(x), _DTYPES[x.dtype], _ptr(wq), _ptr(w_scale), _ptr(bias), m, n, k, had_block, a_bits,
        _ptr(y), _DTYPES[y_dtype], _ptr(xq), _ptr(sx), _stream()))
    return y


def _scalar(x_scale: torch.Tensor) -> torch.Tensor:
    if x_scale is None or not x_scale.is_cuda or x_scale.dtype != torch.float32 or x_scale.numel() != 1:
        raise ValueError("x_scale must be a device tensor holding one float32")
    return x_scale


def hq_act_hadamard_quant_static(x: torch.Tensor, x_scale: torch.Tensor, had_block: int = 64,
                                 a_bits: int = 4, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """x [..., k] fp16/fp32, x_scale one fp32 on the device -> xq uint8 [..., k/2]."""
    _dev(x, "x")
    k = x.shape[-1]
    m = x.numel() // k
    xq = _out(out, x.shape[:-1] + (k // 2,), torch.uint8, x.device)
    _check("hq_act_hadamard_quant_static", load_library().hq_act_hadamard_quant_static(
        _ptr(x), _DTYPES[x.dtype], m, k, had_block, a_bits, _ptr(_scalar(x_scale)), _ptr(xq), _stream()))
    return xq


def hq_int_linear_static(xq: torch.Tensor, x_scale: Optional[torch.Tensor], wq: torch.Tensor,
                         w_scale: Optional[torch.Tensor], bias: Optional[torch.Tensor] = None,
                         y_dtype: torch.dtype = torch.float16, out: Optional[torch.Tensor] = None
                         ) -> torch.Tensor:
    """As hq_int_linear with one activation scale (a device tensor holding one float32)."""
    _codes(xq, torch.uint8, "xq"), _codes(wq, torch.uint8, "wq")
    m, kb = xq.shape
    n = wq.shape[0]
    if wq.numel() != n * kb:
        raise ValueError("wq does not match xq in k")
    _vec(x_scale, 1, torch.float32, "x_scale"), _vec(w_scale, n, torch.float32, "w_scale")
    _vec(bias, n, y_dtype, "bias")
    y = _out(out, (m, n), y_dtype, xq.device)
    _check("hq_int_linear_static", load_library().hq_int_linear_static(
        _ptr(xq), _ptr(x_scale), _ptr(wq), _ptr(w_scale), _ptr(bias), m, n, kb * 2,
        _ptr(y), _DTYPES[y_dtype], _stream()))
    return y


def hq_int_conv2d_static(xq: torch.Tensor, x_scale: Optional[torch.Tensor], wq: torch.Tensor,
                         w_scale: Optional[torch.Tensor], bias: Optional[torch.Tensor] = None,
                         ksize: int = 3, stride: int = 1, pad: Optional[int] = None,
                         y_dtype: torch.dtype = torch.float16, out: Optional[torch.Tensor] = None
                         ) -> torch.Tensor:
    """As hq_int_conv2d with one activation scale; y_dtype int32 returns the sums over all
    taps and input channels, [nb, h, w, cout]."""
    _codes(xq, torch.uint8, "xq"), _codes(wq, torch.uint8, "wq")
    nb, h, w, cb = xq.shape
    cout = wq.shape[0]
    if wq.numel() != cout * ksize * ksize * cb:
        raise ValueError("wq does not match xq / ksize")
    _vec(x_scale, 1, torch.float32, "x_scale"), _vec(w_scale, cout, torch.float32, "w_scale")
    _vec(bias, cout, y_dtype, "bias")
    pad = (ksize - 1) // 2 if pad is None else pad
    ho, wo = _conv_out(h, w, ksize, stride, pad)
    y = _out(out, (nb, ho, wo, cout), y_dtype, xq.device)
    _check("hq_int_conv2d_static", load_library().hq_int_conv2d_static(
        _ptr(xq), _ptr(x_scale), _ptr(wq), _ptr(w_scale), _ptr(bias), nb, h, w, cb * 2, cout,
        ksize, ksize, stride, pad, _ptr(y), _DTYPES[y_dtype], _stream()))
    return y


# ---- Single scheme: un-transformed quantised weights, integer H folded into digit planes -------

def hq_quantize_weights_single(w: torch.Tensor, had_block: int = 64, w_bits: int = 4
                               ) -> Tuple[torch.Tensor, torch.Tensor]:
    """w [n_out, k_in] fp16/fp32 -> (wq3 uint8 [n_out, 3, k_in/2] digit planes, w_scale fp32 [n_out])."""
    _dev(w, "w")
    if w.dim() != 2:
        raise ValueError("w must be [n_out, k_in]")
    n_out, k_in = w.shape
    wq3 = torch.empty((n_out, 3, k_in // 2), dtype=torch.uint8, device=w.device)
    ws = torch.empty((n_out,), dtype=torch.float32, device=w.device)
    _check("hq_quantize_weights_single", load_library().hq_quantize_weights_single(
        _ptr(w), _DTYPES[w.dtype], n_out, k_in, had_block, w_bits, _ptr(wq3), _ptr(ws), _stream()))
    return wq3, ws


def hq_int_linear_single(xq: torch.Tensor, x_scale: Optional[torch.Tensor], wq3: torch.Tensor,
                         w_scale: Optional[torch.Tensor], bias: Optional[torch.Tensor] = None,
                         had_block: int = 64, y_dtype: torch.dtype = torch.float16,
                         out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """xq [m, k/2], wq3 [n, 3, k/2] -> y [m, n]; y_dtype int32 returns the three sums [m, 3, n]."""
    _codes(xq, torch.uint8, "xq"), _codes(wq3, torch.uint8, "wq3")
    m, kb = xq.shape
    n = wq3.shape[0]
    if wq3.numel() != n * 3 * kb:
        raise ValueError("wq3 does not match xq in k")
    _vec(x_scale, m, torch.float32, "x_scale"), _vec(w_scale, n, torch.float32, "w_scale")
    _vec(bias, n, y_dtype, "bias")
    shape = (m, 3, n) if y_dtype == torch.int32 else (m, n)
    y = _out(out, shape, y_dtype, xq.device)
    _check("hq_int_linear_single", load_library().hq_int_linear_single(
        _ptr(xq), _ptr(x_scale), _ptr(wq3), _ptr(w_scale), _ptr(bias), m, n, kb * 2, had_block,
        _ptr(y), _DTYPES[y_dtype], _stream()))
    return y


# ---- width-axis convolution: the paper's own convolution ---------------------------------------

def hq_act_hadamard_quant_width(x: torch.Tensor, x_scale: torch.Tensor, had_block: int, a_bits: int = 4,
                                out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """x [N, H, W, C] fp16/fp32, x_scale one fp32 on the device -> xu3 uint8 [3, N, H, W, C/2]
    (digit planes of the codes taken back along the width axis with the +-1 matrix)."""
    _dev(x, "x")
    _scalar(x_scale)
    if x.dim() != 4:
        raise ValueError("x must be [N, H, W, C]")
    nb, h, w, c = x.shape
    xu3 = _out(out, (3, nb, h, w, c // 2), torch.uint8, x.device)
    _check("hq_act_hadamard_quant_width", load_library().hq_act_hadamard_quant_width(
        _ptr(x), _DTYPES[x.dtype], nb, h, w, c, had_block, a_bits, _ptr(x_scale), _ptr(xu3), _stream()))
    return xu3


def hq_int_conv2d_width(xu3: torch.Tensor, x_scale: Optional[torch.Tensor], wq: torch.Tensor,
                        w_scale: Optional[torch.Tensor], bias: Optional[torch.Tensor] = None,
                        had_block: int = 64, y_dtype: torch.dtype = torch.float16,
                        out: Optional[torch.Tensor] = None, stride: int = 1) -> torch.Tensor:
    """xu3 [3, N, H, W, Cin/2], wq [Cout, 9, Cin/2] (or [Cout, 3, 3, Cin/2]) -> y [N, Ho, Wo, Cout]
    (same size for stride 1; stride 2 halves it, rounding up); y_dtype int32 returns the exact integer sums."""
    _codes(xu3, torch.uint8, "xu3"), _codes(wq, torch.uint8, "wq")
    if xu3.dim() != 5 or xu3.shape[0] != 3:
        raise ValueError("xu3 must be [3, N, H, W, Cin/2]")
    _, nb, h, w, kb = xu3.shape
    c_out = wq.shape[0]
    if wq.numel() != c_out * 9 * kb:
        raise ValueError("wq does not match xu3 in Cin or is not a 3x3 kernel")
    _vec(x_scale, 1, torch.float32, "x_scale"), _vec(w_scale, c_out, torch.float32, "w_scale")
    _vec(bias, c_out, y_dtype, "bias")
    ho, wo = _conv_out(h, w, 3, stride, 1)
    y = _out(out, (nb, ho, wo, c_out), y_dtype, xu3.device)
    _check("hq_int_conv2d_width", load_library().hq_int_conv2d_width(
        _ptr(xu3), _ptr(x_scale), _ptr(wq), _ptr(w_scale), _ptr(bias), nb, h, w, kb * 2, c_out, 3, 3, stride, 1,
        had_block, _ptr(y), _DTYPES[y_dtype], _stream()))
    return y


# ---- 8-bit codes (W8A8): int8 operands, one code per byte ---------------------------------------

def hq_act_hadamard_quant_i8(x: torch.Tensor, had_block: int = 64, a_bits: int = 4
                             ) -> Tuple[torch.Tensor, torch.Tensor]:
    """x [..., k] fp16/fp32 -> (xq int8 [..., k] with codes of a_bits bits, x_scale fp32 [...])."""
    _dev(x, "x")
    k = x.shape[-1]
    m = x.numel() // k
    xq = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    xs = torch.empty(x.shape[:-1], dtype=torch.float32, device=x.device)
    _check("hq_act_hadamard_quant_i8", load_library().hq_act_hadamard_quant_i8(
        _ptr(x), _DTYPES[x.dtype], m, k, had_block, a_bits, _ptr(xq), _ptr(xs), _stream()))
    return xq, xs


def hq_int_linear_i8(xq: torch.Tensor, x_scale: Optional[torch.Tensor], wq: torch.Tensor,
                     w_scale: Optional[torch.Tensor], bias: Optional[torch.Tensor] = None,
                     y_dtype: torch.dtype = torch.float16, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """xq int8 [m, k], wq int8 [n, k] (or [n, 1, k]) -> y [m, n]; y_dtype int32 returns the raw sums."""
    _codes(xq, torch.int8, "xq"), _codes(wq, torch.int8, "wq")
    m, k = xq.shape
    n = wq.shape[0]
    if wq.numel() != n * k:
        raise ValueError("wq does not match xq in k")
    _vec(x_scale, m, torch.float32, "x_scale"), _vec(w_scale, n, torch.float32, "w_scale")
    _vec(bias, n, y_dtype, "bias")
    y = _out(out, (m, n), y_dtype, xq.device)
    _check("hq_int_linear_i8", load_library().hq_int_linear_i8(
        _ptr(xq), _ptr(x_scale), _ptr(wq), _ptr(w_scale), _ptr(bias), m, n, k, _ptr(y), _DTYPES[y_dtype], _stream()))
    return y


def hq_int_conv2d_i8(xq: torch.Tensor, x_scale: Optional[torch.Tensor], wq: torch.Tensor,
                     w_scale: Optional[torch.Tensor], bias: Optional[torch.Tensor] = None,
                     ksize: int = 3, y_dtype: torch.dtype = torch.float16,
                     out: Optional[torch.Tensor] = None, stride: int = 1) -> torch.Tensor:
    """xq int8 [N, H, W, Cin], wq int8 [Cout, ksize*ksize, Cin] -> y [N, Ho, Wo, Cout] (same size for
    stride 1; ksize 3 at stride 2 halves it, rounding up); y_dtype int32 returns the per-tap sums
    [N, Ho, Wo, ksize*ksize, Cout]."""
    _codes(xq, torch.int8, "xq"), _codes(wq, torch.int8, "wq")
    nb, h, w, c_in = xq.shape
    c_out = wq.shape[0]
    taps = ksize * ksize
    if wq.numel() != c_out * taps * c_in:
        raise ValueError("wq does not match xq in Cin or the kernel size")
    _vec(x_scale, nb * h * w, torch.float32, "x_scale"), _vec(w_scale, c_out, torch.float32, "w_scale")
    _vec(bias, c_out, y_dtype, "bias")
    ho, wo = _conv_out(h, w, ksize, stride, (ksize - 1) // 2)
    shape = (nb, ho, wo, taps, c_out) if (y_dtype == torch.int32 and taps > 1) else (nb, ho, wo, c_out)
    y = _out(out, shape, y_dtype, xq.device)
    _check("hq_int_conv2d_i8", load_library().hq_int_conv2d_i8(
        _ptr(xq), _ptr(x_scale), _ptr(wq), _ptr(w_scale), _ptr(bias), nb, h, w, c_in, c_out, ksize, ksize, stride,
        (ksize - 1) // 2, _ptr(y), _DTYPES[y_dtype], _stream()))
    return y
