"""Shared plumbing of the GPU parity tests: moving arrays, tolerances, oracle-side state.

Nothing here computes expected values except by calling oracle/; nothing here is used by the
library.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np
import torch

import oracle
from workloads import normal_f32

DEV = "cuda"


def f32_hp(hp: Dict[str, float]) -> Dict[str, float]:
    """Hyper-parameters as the float32 values the C ABI carries, so both sides use the same constants."""
    return {k: float(np.float32(v)) for k, v in hp.items()}


def to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    return a.shape == b.shape and a.dtype == b.dtype and np.array_equal(a.view(np.uint8), b.view(np.uint8))


def gen_weights_grads(cfg_seed: int, numel: Sequence[int], wstd: float, gstd: float, step: int = 0):
    ws = [normal_f32(cfg_seed, i, "w", n, wstd) for i, n in enumerate(numel)]
    gs = [normal_f32(cfg_seed, i, "g", n, gstd, step) for i, n in enumerate(numel)]
    return ws, gs


def shards_of(plan: oracle.Plan, flats: List[np.ndarray]) -> np.ndarray:
    """[N, S] array of every replica's packed shard, built by the oracle."""
    return np.stack([oracle.shard_format(plan, r, flats) for r in range(plan.N)])


# ---- tolerances -------------------------------------------------------------------------------
# Weights: the bound the task fixes, |d| <= 1e-6 (1 + |w|).
# Moments: both sides round m and v to float32 once per step; the GPU also rounds each product.
# One step perturbs m by at most a few 2^-24 of (|m| + |g|) and v (no cancellation, all terms
# >= 0) by a few 2^-24 of v; k steps add up at most linearly.

def assert_weights_close(got: np.ndarray, ref: np.ndarray, what: str = "w"):
    d = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = 1e-6 * (1.0 + np.abs(ref.astype(np.float64)))
    worst = float(np.max(d / bound)) if d.size else 0.0
    assert worst <= 1.0, "%s: |d| exceeds 1e-6(1+|w|) by factor %.3g" % (what, worst)
    return float(d.max()) if d.size else 0.0


def assert_first_moment_close(got, ref, g_scale: float, steps: int = 1, what: str = "m"):
    d = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = steps * 4e-7 * (np.abs(ref.astype(np.float64)) + g_scale)
    assert np.all(d <= bound), "%s: max excess %.3g" % (what, float(np.max(d / np.maximum(bound, 1e-300))))


def assert_second_moment_close(got, ref, steps: int = 1, what: str = "v"):
    d = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = steps * 4e-7 * np.abs(ref.astype(np.float64)) + 1e-37
    assert np.all(d <= bound), "%s: max excess %.3g" % (what, float(np.max(d / bound)))


def assert_sumsq_close(got, ref, numel: Sequence[int], what: str = "sums"):
    """Per-variable [sum w^2, sum u^2] tables.  Sums of squares have no cancellation of their own: relative 3e-6
    against the float64 sums.  An element of u can be the small difference of larger terms, though (LAMB's first
    moment beta1 m + (1 - beta1) g, LARS's g + wd w), and float32 then leaves it an absolute error of a few 1e-7 of
    its uncancelled size (at most about 1 for these optimizers' normalised updates) however small u itself is; by
    Cauchy-Schwarz the sum over n elements moves by at most 2 sqrt(n sum u^2) x that.  Only variables of a handful
    of elements can have this term exceed the relative one."""
    got = np.asarray(got, dtype=np.float64).reshape(-1, 2)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, 2)
    n = np.asarray(numel, dtype=np.float64)
    assert got.shape == ref.shape == (n.size, 2), (got.shape, ref.shape, n.size)
    tol_w = 3e-6 * ref[:, 0] + 1e-30
    tol_u = 3e-6 * ref[:, 1] + 2.0 * np.sqrt(n * ref[:, 1]) * 5e-7 + 1e-30
    bad_w = np.abs(got[:, 0] - ref[:, 0]) > tol_w
    bad_u = np.abs(got[:, 1] - ref[:, 1]) > tol_u
    assert not bad_w.any(), (what, "sum w^2", np.nonzero(bad_w)[0], got[bad_w, 0], ref[bad_w, 0])
    assert not bad_u.any(), (what, "sum u^2", np.nonzero(bad_u)[0], got[bad_u, 1], ref[bad_u, 1])


def pads_are_zero(plan: oracle.Plan, r: int, shard: np.ndarray) -> bool:
    # real_count counts from the piece start in both plan kinds (row plans pad inside the piece too)
    bits = shard.view(np.uint32 if shard.dtype == np.float32 else np.uint16)
    for i in range(plan.V):
        real = plan.real_count(i, r)
        if bits[plan.off[i] + real: plan.off[i] + plan.L[i]].any():
            return False
    return True


# ---- guard bands -----------------------------------------------------------------------------------
CANARY = 0x5A
BAND = 256           # bytes before and after the payload; keeps the payload 16-byte aligned


class Guarded:
    """A device tensor of `n` elements of `dtype` carved out of a byte buffer with canary bands on both
    sides: a kernel that stores outside its output shows up in `intact()`."""

    def __init__(self, n: int, dtype=torch.float32, init=None):
        self.nbytes = n * torch.empty((), dtype=dtype).element_size()
        self.buf = torch.full((self.nbytes + 2 * BAND,), CANARY, dtype=torch.uint8, device=DEV)
        self.t = self.buf[BAND:BAND + self.nbytes].view(dtype)
        if init is None:
            self.t.zero_()
        else:
            self.t.copy_(init if isinstance(init, torch.Tensor) else to_dev(np.ascontiguousarray(init)))

    def intact(self) -> bool:
        return bool((self.buf[:BAND] == CANARY).all()) and bool((self.buf[BAND + self.nbytes:] == CANARY).all())
