"""Seeded synthetic inputs for the Dion step (weights, gradients, initial right factor).

This module holds no arithmetic of the optimizer itself: it only draws numbers and
handles the bf16 storage format.  Both the CPU oracle's tests and the GPU harness draw
their inputs from here, so the two sides always see bit-identical tensors.

Streams are keyed by (seed, tensor id, step, matrix index): every tensor of every
step of every matrix of a batch can be regenerated independently of all the others.

Recipe (shapes follow the paper's Figure 1 micro-benchmark and its model table; values
are i.i.d. Gaussian because the paper's gradient streams need its training data):
  X  ~ N(0, 0.02^2)        fp32         tensor id 1
  Q0 ~ N(0, 1)             fp32         tensor id 2   (column-normalised by the init call)
  G_t ~ 1e-2 * N(0, 1)     fp32 / bf16  tensor id 0, step t
  structured G_t = A diag(k^-1) C^T * scale + noise   (power-law spectrum, parity only)
"""
from __future__ import annotations

import numpy as np

TENSOR_G = 0
TENSOR_X = 1
TENSOR_Q = 2
TENSOR_AUX = 3

X_STD = 0.02
G_STD = 1e-2


def _rng(seed: int, tensor: int, step: int = 0, index: int = 0) -> np.random.Generator:
    key = (int(seed) & 0xFFFFFFFF) | ((int(tensor) & 0xFFFF) << 32) | ((int(index) & 0xFFFF) << 48)
    return np.random.Generator(np.random.Philox(key=key, counter=[0, 0, 0, int(step)]))


def gaussian(shape, std: float, seed: int, tensor: int, step: int = 0, index: int = 0) -> np.ndarray:
    """fp32 array of i.i.d. N(0, std^2) values from the stream (seed, tensor, step, index)."""
    a = _rng(seed, tensor, step, index).standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact upcast of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def weight(m: int, n: int, seed: int = 1, index: int = 0) -> np.ndarray:
    return gaussian((m, n), X_STD, seed, TENSOR_X, 0, index)


def right_factor_raw(n: int, r: int, seed: int = 2, index: int = 0) -> np.ndarray:
    """Un-normalised N(0,1) start for Q; the init call column-normalises it."""
    return gaussian((n, r), 1.0, seed, TENSOR_Q, 0, index)


def gradient(m: int, n: int, step: int, seed: int = 0, index: int = 0, bf16: bool = False,
             std: float = G_STD):
    """Gradient of step `step`: fp32 array, or (bf16 bit patterns as uint16) when bf16=True."""
    g = gaussian((m, n), std, seed, TENSOR_G, step, index)
    return f32_to_bf16_bits(g) if bf16 else g


def structured_gradient(m: int, n: int, step: int, k: int, seed: int = 0, index: int = 0,
                        bf16: bool = False, noise: float = 1e-3, decay: float = 1.0,
                        std: float = G_STD):
    """Gradient with a power-law spectrum: A diag(j^-decay) C^T plus Gaussian noise.

    Real momentum buffers are far from i.i.d.: a few directions dominate.  This input has k
    dominant directions with singular values ~ j^-decay, so B*Q is markedly worse conditioned
    than for the flat-spectrum Gaussian input.  Used for parity and robustness, never timing.
    """
    rng = _rng(seed, TENSOR_AUX, step, index)
    a = rng.standard_normal(size=(m, k), dtype=np.float32) / np.float32(np.sqrt(m))
    c = rng.standard_normal(size=(n, k), dtype=np.float32) / np.float32(np.sqrt(n))
    w = (np.arange(1, k + 1, dtype=np.float32) ** np.float32(-decay))
    g = (a * w) @ c.T
    g *= np.float32(std * np.sqrt(m * n) / np.sqrt(np.sum(w.astype(np.float64) ** 2)))
    g += gaussian((m, n), std * noise, seed, TENSOR_G, step, index)
    g = np.ascontiguousarray(g, dtype=np.float32)
    return f32_to_bf16_bits(g) if bf16 else g


# The five benchmark configurations (shapes, ranks, dtypes, step counts).
CONFIGS = {
    "C1": dict(shapes=[(256, 256, 64)], g_bf16=False, math="f32", steps=10),
    "C2": dict(shapes=[(2048, 2048, 512)], g_bf16=True, math="f32", steps=20),
    "C2b": dict(shapes=[(2048, 2048, 512)], g_bf16=True, math="bf16", steps=20),
    "C3a": dict(shapes=[(8192, 8192, 2048)], g_bf16=True, math="bf16", steps=10),
    "C3b": dict(shapes=[(8192, 8192, 512)], g_bf16=True, math="bf16", steps=10),
    "C4a": dict(shapes=[(16384, 53248, 1024)], g_bf16=True, math="bf16", steps=5),
    "C4b": dict(shapes=[(16384, 53248, 4096)], g_bf16=True, math="bf16", steps=5),
    "C5": dict(shapes=([(3072, 3072, 768)] * 4 + [(3072, 8192, 768)] * 2 + [(8192, 3072, 768)]) * 28,
               g_bf16=True, math="bf16", steps=1),
}
MU = 0.95
ETA = 0.01
