"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds none of the quantisation method's arithmetic: it only draws random tensors
with the shapes and value distributions of the workloads and casts them to the storage type.
Both the GPU library and the CPU oracle are fed the same bytes produced here.

The tensors stand in for the paper's workloads: i.i.d. normal blocks of the numerical study
(Results, "Numerical Study") and the MLP weights / activations of 7B-14B language models
(Results, "Downstream LLM Perplexity"),
whose real weights and evaluation corpus are not available.  Weights are heavy-tailed
(Student-t, 4 degrees of freedom, scale 0.02); activations are N(0,1) with 1 % outlier
channels multiplied by 50.

bf16 tensors are returned as ``numpy.uint16`` bit patterns (numpy has no bf16 type).
"""
from __future__ import annotations

import numpy as np

# Shapes of the synthetic 8B-class decoder layer (rows x cols, row-major, blocks along cols).
LAYER_SHAPES = {
    "q": (4096, 4096), "k": (1024, 4096), "v": (1024, 4096), "o": (4096, 4096),
    "gate": (14336, 4096), "up": (14336, 4096), "down": (4096, 14336),
}
N_LAYERS = 32


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even cast of finite fp32 values to bf16 bit patterns."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_f32(rows: int, cols: int, seed: int, sigma: float = 1.0) -> np.ndarray:
    """fp32 matrix, entries i.i.d. N(0, sigma^2)."""
    return (_rng(seed).standard_normal((rows, cols), dtype=np.float32) * np.float32(sigma))


def student_t_weights(rows: int, cols: int, seed: int, df: float = 4.0,
                      scale: float = 0.02) -> np.ndarray:
    """bf16 weight matrix: scale * Student-t(df), drawn in row chunks to bound memory."""
    rng = _rng(seed)
    out = np.empty((rows, cols), np.uint16)
    step = max(1, (1 << 22) // max(cols, 1))
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        t = rng.standard_t(df, size=(step, cols)) * scale      # whole chunk: prefix-stable
        out[r0:r1] = f32_to_bf16_bits(t[: r1 - r0].astype(np.float32))
    return out


def outlier_activations(rows: int, cols: int, seed: int, frac: float = 0.01,
                        mult: float = 50.0) -> np.ndarray:
    """bf16 activations: N(0,1); round(frac*cols) seeded distinct channels multiplied by mult."""
    rng = _rng(seed)
    n_out = int(round(frac * cols))
    ch = rng.choice(cols, size=n_out, replace=False)       # channels first: prefix-stable rows
    x = rng.standard_normal((rows, cols), dtype=np.float32)
    x[:, ch] *= np.float32(mult)
    return f32_to_bf16_bits(x)


def layer_matrix(layer: int, name: str, rows: int | None = None) -> np.ndarray:
    """One matrix of the synthetic 32-layer model; ``rows`` draws only the first rows."""
    r, c = LAYER_SHAPES[name]
    if rows is not None:
        r = min(r, rows)
    seed = 50_000 + 16 * layer + list(LAYER_SHAPES).index(name)
    return student_t_weights(r, c, seed)


def normal_blocks_f32(sigma: float, n_blocks: int, block: int, seed: int) -> np.ndarray:
    """The numerical study's sample: n_blocks x block values from N(0, sigma^2), fp32."""
    return normal_f32(n_blocks, block, seed, sigma)


# The five benchmark configurations, by name.
def config1() -> np.ndarray:
    return normal_f32(1024, 4096, seed=1001)


def config2(rows: int = 4096) -> np.ndarray:
    return student_t_weights(rows, 14336, seed=1002)


def config3(rows: int = 8192) -> np.ndarray:
    return outlier_activations(rows, 4096, seed=1003)
