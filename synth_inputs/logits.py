"""Seeded synthetic logits."""

from __future__ import annotations

import numpy as np


def make_logits(batch: int, vocab: int, seed: int, sigma: float = 1.0) -> np.ndarray:
    """float32 array [batch, vocab] drawn from N(0, sigma^2).

    The caller converts to bf16/fp16 (one rounding on the host) when the
    workload asks for a 16-bit type.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_normal((batch, vocab), dtype=np.float32) * np.float32(sigma))
