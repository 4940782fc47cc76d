"""Seeded synthetic inputs with the shapes and value distributions of the
Llama-3.1-8B linear layers the paper trains (Sec. 2.2).

This module draws random tensors and nothing else: it contains none of the
method's arithmetic (no rotation, no scaling rule, no FP4 cast), so both the
GPU tests and the CPU checks may take their inputs from it.

Every tensor is drawn on the host from numpy's Philox counter generator keyed by
(seed, stream), cast once to bf16 (round to nearest even, torch's cast) and
returned as a CPU ``torch.bfloat16`` tensor.  ``as_u16`` gives the bit patterns.
"""
from __future__ import annotations

import numpy as np
import torch

# one stream id per tensor role, so X, W and dY of a layer are independent
STREAM_X, STREAM_W, STREAM_DY, STREAM_AUX = 1, 2, 3, 4


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed & (2**64 - 1), stream]))


def _to_bf16(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)


def as_u16(t: torch.Tensor) -> np.ndarray:
    """bf16 CPU tensor -> uint16 numpy view of the same memory."""
    assert t.dtype == torch.bfloat16 and t.device.type == "cpu"
    return t.view(torch.int16).numpy().view(np.uint16)


def normal(rows: int, cols: int, std: float, seed: int, stream: int) -> torch.Tensor:
    """N(0, std^2) entries."""
    a = _rng(seed, stream).standard_normal((rows, cols), dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return _to_bf16(a)


def normal_with_outlier_channels(rows: int, cols: int, seed: int, stream: int,
                                 fraction: float = 0.001, gain: float = 100.0) -> torch.Tensor:
    """N(0,1) activations in which round(fraction*cols) seeded channels (columns)
    are multiplied by ``gain``: the activation-outlier pattern of LLM hidden states."""
    a = _rng(seed, stream).standard_normal((rows, cols), dtype=np.float32)
    n_out = int(round(fraction * cols))
    if n_out > 0:
        ch = _rng(seed, STREAM_AUX + 16 * stream).choice(cols, size=n_out, replace=False)
        a[:, np.sort(ch)] *= np.float32(gain)
    return _to_bf16(a)


def student_t3(rows: int, cols: int, scale: float, seed: int, stream: int) -> torch.Tensor:
    """scale * t_3, with t_3 = Z / sqrt(chi2_3 / 3): heavy-tailed gradients."""
    g = _rng(seed, stream)
    z = g.standard_normal((rows, cols), dtype=np.float32)
    chi = np.zeros((rows, cols), dtype=np.float32)
    for _ in range(3):
        n = g.standard_normal((rows, cols), dtype=np.float32)
        chi += n * n
    z /= np.sqrt(chi / np.float32(3.0))
    z *= np.float32(scale)
    return _to_bf16(z)


def small_integers(rows: int, cols: int, lo: int, hi: int, seed: int, stream: int) -> torch.Tensor:
    """Integer-valued entries in [lo, hi] (exactly representable in bf16 when |v| <= 256)."""
    a = _rng(seed, stream).integers(lo, hi + 1, size=(rows, cols)).astype(np.float32)
    return _to_bf16(a)


def from_bits(bits: np.ndarray) -> torch.Tensor:
    """uint16 bit patterns -> bf16 CPU tensor (for edge-case tensors built by hand)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return torch.from_numpy(b.view(np.int16)).view(torch.bfloat16)
