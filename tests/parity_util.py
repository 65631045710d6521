"""Helpers of the GPU parity tests: code (un)packing in the documented nibble
format, the comparison rules, and one function that runs a whole layer through
the HIP library and the oracle side by side."""
from __future__ import annotations

import numpy as np

BOUNDARY_EPS = 1e-5      # codes may differ only where the oracle's t is this close to a tie
SCALE_RTOL = 1e-6
Y_RTOL = 2e-3            # max |y - y_ref| / max |y_ref|


def unpack_codes(packed: np.ndarray) -> np.ndarray:
    """uint8 [..., k/2] -> int8 [..., k]; element 2j in bits 0..3, 2j+1 in bits 4..7."""
    b = packed.astype(np.uint8)
    lo = (b & 0xF).astype(np.int8)
    hi = (b >> 4).astype(np.int8)
    lo = np.where(lo > 7, lo - 16, lo).astype(np.int8)
    hi = np.where(hi > 7, hi - 16, hi).astype(np.int8)
    return np.stack([lo, hi], axis=-1).reshape(b.shape[:-1] + (b.shape[-1] * 2,))


def pack_codes(codes: np.ndarray) -> np.ndarray:
    c = codes.astype(np.int16) & 0xF
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def check_codes(name, got, want, t, bits):
    """Codes equal, except within BOUNDARY_EPS of a rounding tie where they may differ by one.
    Returns the number of (legitimately) differing codes."""
    qmax, qmin = 2 ** (bits - 1) - 1, -(2 ** (bits - 1))
    assert got.shape == want.shape, name
    assert got.min() >= qmin and got.max() <= qmax, "%s: code out of range" % name
    diff = got != want
    n = int(diff.sum())
    if n:
        td = t[diff]
        tie_dist = np.abs(np.abs(td - np.floor(td)) - 0.5)
        step = np.abs(got[diff].astype(np.int32) - want[diff].astype(np.int32))
        assert tie_dist.max() < BOUNDARY_EPS, "%s: %d codes differ away from a tie (worst %.3g)" % (
            name, int((tie_dist >= BOUNDARY_EPS).sum()), tie_dist.max())
        assert step.max() <= 1, "%s: a code differs by more than one" % name
    return n


def check_scales(name, got, want):
    rel = np.abs(got.astype(np.float64) - want) / np.abs(want)
    assert rel.max() <= SCALE_RTOL, "%s: scale rel err %.3g" % (name, rel.max())


def check_y(name, got, want, rtol=Y_RTOL):
    got = got.astype(np.float64)
    assert np.isfinite(got).all(), name
    denom = np.abs(want).max()
    err = np.abs(got - want).max() / denom
    assert err <= rtol, "%s: max|y - ref| / max|ref| = %.3g" % (name, err)
    return err
