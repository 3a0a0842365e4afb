"""Seeded synthetic tensors shaped like the paper's workloads.

Only input generation lives here -- none of the NVFP4 arithmetic.  Both the CPU
oracle (through the tests) and the HIP library are fed from these generators so
that they see identical bits.  Every tensor is returned as a ``uint16`` numpy
array holding bf16 bit patterns, row-major ``[rows, cols]``.

The paper's activations, weights and gradients are not available; the recipes
below stand in for them: Gaussian activations with a sprinkle of large outliers
(the "block-level outliers" of Sec. 4.2), small Gaussian weights at an
initialisation-like std, and heavy-tailed Student-t(3) gradients.  Shapes come
from the 12B model (App. A.1: model dimension 5120, FFN dimension 20480,
sequence length 8192).
"""
from __future__ import annotations

import numpy as np

_CHUNK_ROWS = 512


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round binary32 to bf16 (nearest, ties to even); returns the 16-bit patterns."""
    w = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (w >> np.uint32(16)) & np.uint32(1)
    r = (w + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=int(seed)))


def normal(rows: int, cols: int, std: float, seed: int) -> np.ndarray:
    """N(0, std^2)."""
    rng = _rng(seed)
    out = np.empty((rows, cols), dtype=np.uint16)
    for r0 in range(0, rows, _CHUNK_ROWS):
        r1 = min(rows, r0 + _CHUNK_ROWS)
        z = rng.standard_normal((r1 - r0, cols), dtype=np.float32) * np.float32(std)
        out[r0:r1] = f32_to_bf16_bits(z)
    return out


def normal_with_outliers(rows: int, cols: int, std: float, seed: int,
                         frac: float = 1e-3, mult: float = 50.0) -> np.ndarray:
    """N(0, std^2) with a seeded Bernoulli(frac) subset of entries multiplied by ``mult``."""
    rng = _rng(seed)
    out = np.empty((rows, cols), dtype=np.uint16)
    for r0 in range(0, rows, _CHUNK_ROWS):
        r1 = min(rows, r0 + _CHUNK_ROWS)
        z = rng.standard_normal((r1 - r0, cols), dtype=np.float32) * np.float32(std)
        hit = rng.random((r1 - r0, cols), dtype=np.float32) < np.float32(frac)
        z = np.where(hit, z * np.float32(mult), z)
        out[r0:r1] = f32_to_bf16_bits(z)
    return out


def student_t3(rows: int, cols: int, scale: float, seed: int) -> np.ndarray:
    """scale * t(nu=3): t = Z0 / sqrt((Z1^2 + Z2^2 + Z3^2) / 3)."""
    rng = _rng(seed)
    out = np.empty((rows, cols), dtype=np.uint16)
    for r0 in range(0, rows, _CHUNK_ROWS):
        r1 = min(rows, r0 + _CHUNK_ROWS)
        z = rng.standard_normal((4, r1 - r0, cols), dtype=np.float32)
        chi = np.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / np.float32(3.0))
        t = z[0] / np.maximum(chi, np.float32(1e-12)) * np.float32(scale)
        out[r0:r1] = f32_to_bf16_bits(t)
    return out


# The five workloads named in the benchmark spec, by index 1..5.  Each entry lists the
# tensors as (name, generator, rows, cols, parameter, seed).
def config_tensors(cfg: int) -> dict:
    if cfg == 1:
        return {"X": normal_with_outliers(256, 512, 1.0, 101),
                "W": normal(512, 256, 0.02, 102)}
    if cfg == 2:
        return {"dY": student_t3(4096, 5120, 1e-3, 201),
                "X": normal_with_outliers(4096, 5120, 1.0, 202)}
    if cfg == 3:
        return {"X": normal_with_outliers(8192, 5120, 1.0, 301),
                "W": normal(5120, 20480, 0.02, 302)}
    if cfg == 4:
        return {"dY": student_t3(8192, 20480, 1e-3, 401),
                "W": normal(5120, 20480, 0.02, 302)}
    if cfg == 5:
        return {"T1": student_t3(8192, 5120, 0.02, 501),
                "T2": student_t3(8192, 20480, 0.02, 502),
                "T3": student_t3(5120, 20480, 0.02, 503)}
    raise ValueError(f"unknown config {cfg}")
