"""Seeded synthetic inputs shaped like the paper's workloads.

This module holds no arithmetic of the method: only tensor shapes and random draws.  It is
the one module both the GPU tests/benchmark and the CPU oracle's tests may share.

The paper trains OPT / GPT-2 / LLaMA checkpoints on text corpora (Sec. 6.1, Table 11); neither
the checkpoints nor the corpora are used here.  What is kept is the shape of every linear
weight of those models ([out_features, in_features], groups of M along in_features, Eq. 3)
with Gaussian values: weights ~ N(0, std 0.02), gradients ~ N(0, std 1e-3).
"""
from __future__ import annotations

import numpy as np
import torch

# (name, rows = out_features, cols = in_features) of one decoder block's linear layers


def opt125m_block():
    return [("q", 768, 768), ("k", 768, 768), ("v", 768, 768), ("o", 768, 768),
            ("fc1", 3072, 768), ("fc2", 768, 3072)]


def llama2_7b_block():
    return [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
            ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]


def llama2_13b_block():
    return [("q", 5120, 5120), ("k", 5120, 5120), ("v", 5120, 5120), ("o", 5120, 5120),
            ("gate", 13824, 5120), ("up", 13824, 5120), ("down", 5120, 13824)]


def llama3_8b_block():
    # grouped-query attention: 8 key/value heads of 128, so k and v are 1024 x 4096
    return [("q", 4096, 4096), ("k", 1024, 4096), ("v", 1024, 4096), ("o", 4096, 4096),
            ("gate", 14336, 4096), ("up", 14336, 4096), ("down", 4096, 14336)]


WEIGHT_SETS = {
    "opt125m": (12, opt125m_block),
    "llama2_7b": (32, llama2_7b_block),
    "llama2_13b": (40, llama2_13b_block),
    "llama3_8b": (32, llama3_8b_block),
}


def weight_set(name: str, layers: int | None = None):
    """List of (tensor_name, rows, cols) for every linear weight of the named model."""
    n_layers, block = WEIGHT_SETS[name]
    if layers is not None:
        n_layers = layers
    return [(f"layer{l}.{nm}", r, c) for l in range(n_layers) for (nm, r, c) in block()]


def set_params(shapes) -> int:
    return sum(r * c for _, r, c in shapes)


def _rng(seed: int, tensor_id: int, step: int, stream: int) -> np.random.Generator:
    # counter-based generator keyed by (seed, tensor, step, purpose): any tensor can be
    # regenerated alone, so a whole model never has to sit on the host
    return np.random.Generator(np.random.Philox(key=[(seed << 32) | tensor_id, (step << 8) | stream]))


def weights(seed: int, tensor_id: int, rows: int, cols: int, std: float = 0.02) -> np.ndarray:
    return (_rng(seed, tensor_id, 0, 0).standard_normal((rows, cols), np.float32) * np.float32(std))


def grads_f32(seed: int, tensor_id: int, step: int, rows: int, cols: int, std: float = 1e-3) -> np.ndarray:
    return (_rng(seed, tensor_id, step, 1).standard_normal((rows, cols), np.float32) * np.float32(std))


def grads_bf16(seed: int, tensor_id: int, step: int, rows: int, cols: int, std: float = 1e-3) -> torch.Tensor:
    """bf16 gradient tensor (CPU).  The rounding is the tensor library's own conversion."""
    g = grads_f32(seed, tensor_id, step, rows, cols, std)
    return torch.from_numpy(g).to(torch.bfloat16)


def widen_bf16(g: torch.Tensor) -> np.ndarray:
    """Exact bf16 -> fp32 widening of a CPU tensor, as a numpy array."""
    return g.to(torch.float32).numpy()


def tie_outlier_weights(seed: int, tensor_id: int, rows: int, cols: int, std: float = 0.02,
                        outlier_frac: float = 1e-3, zero_group_frac: float = 0.05,
                        zero_granule: int = 8) -> np.ndarray:
    """Stress input for selection and packing: values rounded to bf16 (many exact magnitude
    ties), a small fraction of N(0, 1) outliers, and a fraction of aligned granules of
    ``zero_granule`` consecutive entries set to zero (so the same tensor has all-zero
    groups for M = 2, 4 and 8)."""
    assert cols % zero_granule == 0
    rng = _rng(seed, tensor_id, 0, 2)
    w = rng.standard_normal((rows, cols), np.float32) * np.float32(std)
    w = torch.from_numpy(w).to(torch.bfloat16).to(torch.float32).numpy()
    outlier = rng.random((rows, cols)) < outlier_frac
    w[outlier] = rng.standard_normal(int(outlier.sum()), np.float32)
    zero = rng.random((rows, cols // zero_granule)) < zero_group_frac
    w.reshape(rows, cols // zero_granule, zero_granule)[zero] = 0.0
    return w


def device_gaussian(shape, std: float, dtype: torch.dtype, seed: int, device="cuda:0") -> torch.Tensor:
    """Gaussian tensor drawn directly in device memory (for weight sets too large to stage
    through the host)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(0.0, std, generator=gen)
    return t if dtype == torch.float32 else t.to(dtype)
