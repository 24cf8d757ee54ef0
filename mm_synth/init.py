"""Seeded initial parameter values for one module's flat parameter vector.

The caller supplies the tensor table (role, offset, size) it obtained from whichever
implementation it is feeding; this module only draws numbers:
matrices and embedding tables ~ N(0, 0.02^2), biases 0, LayerNorm gain 1 / shift 0.
`perturbed=True` also randomises biases, gains and shifts so tests exercise those paths.
"""
from __future__ import annotations

from typing import Iterable, Tuple

import numpy as np

ROLES = ("matrix", "embed", "bias", "gamma", "beta")


def fill_params(tensors: Iterable[Tuple[str, int, int]], total: int, seed: int,
                perturbed: bool = False, std: float = 0.02) -> np.ndarray:
    """Returns float32[total]; gaps between tensors stay zero."""
    rng = np.random.Generator(np.random.Philox(key=int(seed)))
    flat = np.zeros(int(total), dtype=np.float32)
    for role, off, size in tensors:
        off, size = int(off), int(size)
        if role in ("matrix", "embed"):
            flat[off:off + size] = rng.standard_normal(size, dtype=np.float32) * np.float32(std)
        elif role == "bias" or role == "beta":
            if perturbed:
                flat[off:off + size] = rng.standard_normal(size, dtype=np.float32) * np.float32(std)
        elif role == "gamma":
            flat[off:off + size] = 1.0
            if perturbed:
                flat[off:off + size] += rng.standard_normal(size, dtype=np.float32) * np.float32(std)
        else:
            raise ValueError(f"unknown tensor role {role!r}")
    return flat
