"""Shard / unshard formatting and the float32 -> bfloat16 rounding (oracle side).

shard_format is the pad fused into the dynamic-slice of Section 4.1: it reads
only replica r's piece of each variable and fills the slots past the
variable's end with +0.0.  unshard_format is the reverse formatting that
follows the all-gather (Section 4.2): row r of the gathered [N, S] array is
replica r's packed shard.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from .plan import Plan


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round to nearest, ties to even); returns the 16-bit patterns.

    NaN inputs keep their sign and upper payload bits and get the quiet bit set.
    """
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) & 0xFFFF
    is_nan = ((bits & 0x7F800000) == 0x7F800000) & ((bits & 0x007FFFFF) != 0)
    quiet = ((bits >> 16) | 0x0040) & 0xFFFF
    return np.where(is_nan, quiet, rounded).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _convert(x: np.ndarray, dst: str) -> np.ndarray:
    """x is float32 data or uint16 bfloat16 bit patterns; dst is 'f32' or 'bf16'."""
    src_is_bf16 = x.dtype == np.uint16
    if dst == "bf16":
        return x if src_is_bf16 else f32_to_bf16_bits(x)
    if dst == "f32":
        return bf16_bits_to_f32(x) if src_is_bf16 else x
    raise ValueError(dst)


def shard_format(plan: Plan, r: int, flats: Sequence[np.ndarray], dst: str = None) -> np.ndarray:
    """Replica r's packed shard [S] of the given variables (1-D arrays of n_i elements each)."""
    if not (0 <= r < plan.N):
        raise ValueError("replica id out of range")
    src_is_bf16 = len(flats) > 0 and flats[0].dtype == np.uint16
    if dst is None:
        dst = "bf16" if src_is_bf16 else "f32"
    out = np.zeros(plan.S, dtype=np.uint16 if dst == "bf16" else np.uint32)   # all-zero bits == +0.0
    for i, flat in enumerate(flats):
        assert flat.ndim == 1 and flat.size == plan.numel[i]
        start = r * plan.stride[i]
        real = plan.real_count(i, r)
        if real > 0:
            piece = _convert(flat[start:start + real], dst)
            out[plan.off[i]:plan.off[i] + real] = piece.view(out.dtype)
    return out if dst == "bf16" else out.view(np.float32)


def unshard_format(plan: Plan, gathered: np.ndarray, dst: str = None) -> List[np.ndarray]:
    """Full flat variables from the gathered shards [N, S]; padding is dropped."""
    assert gathered.shape == (plan.N, plan.S)
    src_is_bf16 = gathered.dtype == np.uint16
    if dst is None:
        dst = "bf16" if src_is_bf16 else "f32"
    flats = []
    for i in range(plan.V):
        flat = np.empty(plan.numel[i], dtype=np.uint16 if dst == "bf16" else np.float32)
        for r in range(plan.N):
            start = r * plan.stride[i]
            real = plan.real_count(i, r)
            if real > 0:
                flat[start:start + real] = _convert(gathered[r, plan.off[i]:plan.off[i] + real], dst)
        flats.append(flat)
    return flats
