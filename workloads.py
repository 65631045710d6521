"""Seeded synthetic inputs shaped like the layers of the LDM-4 UNet.

This module holds shapes and random-number recipes only: none of the method's
arithmetic (no transform, no quantiser, no product).  It is the one module the
tests, the benchmark and the oracle-side checks all share, so that both sides
see bit-identical stored tensors.

The tensors stand in for real LDM-4 activations and weights (the paper's
evaluation uses ImageNet / LSUN and trained checkpoints, which are not used
here).  Recipe: NumPy ``default_rng(seed)`` (PCG64) with
``seed = 251205746 + 1000 * config + tensor_index``; values drawn in fp64, a few
whole channels ("outlier channels", chosen by a seeded permutation, the same for
every token) multiplied by a factor, then cast to the stored dtype.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np

SEED_BASE = 251205746
HAD_BLOCK = 64


@dataclass(frozen=True)
class Layer:
    """One quantised layer.  kind = "linear" (x [M, K], w [N, 1, K]) or
    "conv" (x NHWC [nb, h, w, cin], w [cout, r, s, cin], stride 1, pad (r-1)/2)."""
    name: str
    config: int
    index: int                      # position inside the config (seeds)
    kind: str
    dtype: str                      # "f16" | "f32": storage of x, w, bias and y
    a_bits: int
    w_bits: int
    x_shape: Tuple[int, ...]
    n_out: int
    ksize: int = 1                  # r = s
    dist: str = "normal"            # "normal" N(0,1) | "laplace" scale 1
    outlier_frac: Optional[float] = None   # fraction of channels, or
    outlier_count: Optional[int] = None    # an explicit count
    outlier_factor: float = 20.0
    w_std: float = 0.02
    bias_std: Optional[float] = None

    @property
    def k_in(self) -> int:
        return self.x_shape[-1]

    @property
    def taps(self) -> int:
        return self.ksize * self.ksize

    @property
    def m(self) -> int:
        return int(np.prod(self.x_shape[:-1]))

    @property
    def ops(self) -> int:
        """Integer multiply + add count of the contraction, 2 M N K_total."""
        return 2 * self.m * self.n_out * self.taps * self.k_in

    @property
    def pad(self) -> int:
        return (self.ksize - 1) // 2

    def n_outlier_channels(self) -> int:
        if self.outlier_count is not None:
            return self.outlier_count
        return max(1, int(round(self.outlier_frac * self.k_in)))


def _np_dtype(name: str):
    return {"f16": np.float16, "f32": np.float32}[name]


def make_x(layer: Layer) -> np.ndarray:
    rng = np.random.default_rng(SEED_BASE + 1000 * layer.config + 10 * layer.index + 0)
    if layer.dist == "normal":
        x = rng.standard_normal(layer.x_shape)
    elif layer.dist == "laplace":
        x = rng.laplace(0.0, 1.0, layer.x_shape)
    else:
        raise ValueError(layer.dist)
    ch = rng.permutation(layer.k_in)[: layer.n_outlier_channels()]
    x[..., ch] *= layer.outlier_factor
    return x.astype(_np_dtype(layer.dtype))


def make_w(layer: Layer) -> np.ndarray:
    """[n_out, taps, k_in] (for a convolution this is [Cout, R, S, Cin] flattened over R, S)."""
    rng = np.random.default_rng(SEED_BASE + 1000 * layer.config + 10 * layer.index + 1)
    w = rng.standard_normal((layer.n_out, layer.taps, layer.k_in)) * layer.w_std
    return w.astype(_np_dtype(layer.dtype))


def make_bias(layer: Layer) -> Optional[np.ndarray]:
    if layer.bias_std is None:
        return None
    rng = np.random.default_rng(SEED_BASE + 1000 * layer.config + 10 * layer.index + 2)
    return (rng.standard_normal(layer.n_out) * layer.bias_std).astype(_np_dtype(layer.dtype))


def _conv(name, config, index, nb, hw, cin, cout, ksize, **kw) -> Layer:
    return Layer(name=name, config=config, index=index, kind="conv", dtype="f16",
                 x_shape=(nb, hw, hw, cin), n_out=cout, ksize=ksize, **kw)


def _lin(name, config, index, m, k, n, dtype="f16", **kw) -> Layer:
    return Layer(name=name, config=config, index=index, kind="linear", dtype=dtype,
                 x_shape=(m, k), n_out=n, **kw)


def config_layers(config: int) -> List[Layer]:
    """The five benchmark configurations (numbered 1..5)."""
    if config == 1:
        return [_lin("c1_linear_256", 1, 0, 256, 256, 256, dtype="f32", a_bits=4, w_bits=4,
                     outlier_count=4, outlier_factor=20.0, bias_std=0.01)]
    if config == 2:
        return [_lin("c2_qkv_384x1152", 2, 0, 8192, 384, 1152, a_bits=4, w_bits=4,
                     outlier_frac=0.01)]
    if config == 3:
        return [_conv("c3_conv3x3_32_384", 3, 0, 8, 32, 384, 384, 3, a_bits=4, w_bits=4,
                      outlier_frac=0.01)]
    if config == 4:
        kw = dict(a_bits=3, w_bits=4, dist="laplace", outlier_frac=0.005, outlier_factor=30.0)
        return [_conv("c4_conv3x3_16_960", 4, 0, 8, 16, 960, 960, 3, **kw),
                _lin("c4_ffn_960x3840", 4, 1, 2048, 960, 3840, **kw)]
    if config == 5:
        kw = dict(a_bits=4, w_bits=4, outlier_frac=0.01)
        sizes = [(64, 192), (32, 384), (16, 576), (8, 960)]
        out = []
        for i, (hw, c) in enumerate(sizes):
            out.append(_conv("c5_conv3x3_%d_%d" % (hw, c), 5, i, 16, hw, c, c, 3, **kw))
        for i, (hw, c) in enumerate(sizes):
            out.append(_conv("c5_conv1x1_%d_%d" % (hw, c), 5, 4 + i, 16, hw, c, c, 1, **kw))
        out.append(_lin("c5_attn_576x1728", 5, 8, 16 * 16 * 16, 576, 1728, **kw))
        return out
    raise ValueError("config must be 1..5")


def tiny_layers() -> List[Layer]:
    """Small cases that still span several tiles and ragged tails; the oracle
    finishes each in well under a second."""
    kw = dict(a_bits=4, w_bits=4, outlier_frac=0.02)
    return [
        _lin("t_lin_ragged", 0, 0, 333, 192, 200, bias_std=0.01, **kw),
        _lin("t_lin_f32", 0, 1, 130, 128, 72, dtype="f32", bias_std=0.01, **kw),
        _lin("t_lin_a3", 0, 2, 257, 320, 136, a_bits=3, w_bits=4, dist="laplace",
             outlier_frac=0.01, outlier_factor=30.0),
        _conv("t_conv3_ragged", 0, 3, 2, 9, 128, 72, 3, bias_std=0.01, **kw),
        _conv("t_conv3_wide", 0, 4, 3, 12, 192, 264, 3, **kw),
        _conv("t_conv1", 0, 5, 2, 7, 64, 40, 1, **kw),
        _conv("t_conv3_a3", 0, 6, 1, 17, 64, 130, 3, a_bits=3, w_bits=4, dist="laplace",
              outlier_frac=0.02, outlier_factor=30.0, bias_std=0.01),
        # 52 x 5 = 260 output tiles of 64 x 64: between one tile per CU and 1.25 (a K range in two shares)
        _conv("t_conv3_split2", 0, 7, 13, 16, 192, 320, 3, bias_std=0.01, **kw),
    ]
