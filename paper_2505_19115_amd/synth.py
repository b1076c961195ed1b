"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Only random draws and casts live here -- none of the quantization arithmetic.
Shapes are the Llama2-7B linear layers the paper trains (Sec. 5, Setup); the
value distributions stand in for its activations, weights and gradients, which
come from a training run that is not available: Gaussian activations/weights,
heavy-tailed tensors with sparse large outliers for the quantizer sweep, and
tiny Gaussian gradients with rarer outliers.
All tensors are CPU torch tensors; the caller moves them to the device.
"""
from __future__ import annotations

import numpy as np
import torch


def _finish(a: np.ndarray, dtype: torch.dtype) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(dtype) if dtype != torch.float32 else t


def normal(rows: int, cols: int, std: float, seed: int, dtype=torch.bfloat16) -> torch.Tensor:
    """N(0, std^2) entries."""
    rng = np.random.default_rng(seed)
    return _finish(rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(std), dtype)


def student_t_outliers(rows: int, cols: int, seed: int, nu: float = 3.0, scale: float = 0.02,
                       p_outlier: float = 1e-3, outlier_gain: float = 100.0,
                       dtype=torch.bfloat16) -> torch.Tensor:
    """Student-t(nu) * scale with a Bernoulli(p_outlier) subset multiplied by outlier_gain."""
    rng = np.random.default_rng(seed)
    a = rng.standard_t(nu, size=(rows, cols)).astype(np.float32) * np.float32(scale)
    mask = rng.random((rows, cols), dtype=np.float32) < p_outlier
    a[mask] *= np.float32(outlier_gain)
    return _finish(a, dtype)


def gradient_like(rows: int, cols: int, seed: int, std: float = 1e-3, p_outlier: float = 5e-4,
                  outlier_gain: float = 50.0, dtype=torch.bfloat16) -> torch.Tensor:
    """N(0, std^2) upstream gradient with sparse outliers."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(std)
    mask = rng.random((rows, cols), dtype=np.float32) < p_outlier
    a[mask] *= np.float32(outlier_gain)
    return _finish(a, dtype)


# Llama2-7B linear layers as (name, out_features N, in_features K); tokens M = batch * seq.
LLAMA2_7B_LINEARS = (
    ("qkv", 12288, 4096),
    ("out_proj", 4096, 4096),
    ("gate", 11008, 4096),
    ("up", 11008, 4096),
    ("down", 4096, 11008),
)
