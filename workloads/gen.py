"""Seeded, counter-based input generators.

Every tensor is drawn from its own Philox stream keyed by (seed, variable
index, tensor kind), so any variable can be regenerated on its own, in any
order, on any machine: the oracle and the GPU path see identical bits
without either producing inputs for the other.
"""
from __future__ import annotations

from typing import Dict

import numpy as np

_KIND = {"w": 0, "g": 1, "m": 2, "v": 3, "bits": 4}


def _rng(seed: int, var: int, kind: str, step: int = 0) -> np.random.Generator:
    key = (int(seed) & 0xFFFFFFFF) | ((int(var) & 0xFFFFF) << 32) | (_KIND[kind] << 52) | ((int(step) & 0xFF) << 56)
    return np.random.Generator(np.random.Philox(key=key))


def normal_f32(seed: int, var: int, kind: str, n: int, std: float, step: int = 0) -> np.ndarray:
    """n i.i.d. N(0, std^2) samples as float32 (std is a standard deviation)."""
    x = _rng(seed, var, kind, step).standard_normal(int(n), dtype=np.float32)
    x *= np.float32(std)
    return x


def random_bits_u32(seed: int, var: int, n: int) -> np.ndarray:
    """n arbitrary 32-bit patterns (as float32 they include NaN payloads, infinities, -0.0, denormals)."""
    return _rng(seed, var, "bits").integers(0, 2**32, size=int(n), dtype=np.uint32)


def variable_inputs(seed: int, var: int, n: int, weight_std: float, grad_std: float, step: int = 0) -> Dict[str, np.ndarray]:
    """Weights and gradient of one variable; the gradient stream depends on the step."""
    return {
        "w": normal_f32(seed, var, "w", n, weight_std),
        "g": normal_f32(seed, var, "g", n, grad_std, step),
    }
