"""Seeded synthetic inputs shared by the GPU tests, the oracle tests and the benchmark.

This module holds input recipes only: none of the method's arithmetic lives here, and it
imports neither the GPU binding nor the oracle.

The paper's runtime benchmark draws every row i.i.d. from a unit normal (Appendix B.1,
"Runtime benchmarks", steps 2a/3a), so `normal_rows` is that workload itself.
`attention_scores` stands in for the SparQ attention-score rows of Section 4.2 /
Appendix B.2 (which need a trained model): scores q.K^T / sqrt(d) with q, K i.i.d.
unit normal, rounded to bf16, which gives near-normal rows with many exact ties.
All tensors are produced on the CPU with a seeded torch.Generator, so every machine
sees the same bits.
"""
from __future__ import annotations

import math

import numpy as np
import torch

# The five benchmark configurations.  `cases` lists (k, b, k_b) triples.
CONFIGS = {
    "cfg1": dict(m=4, n=4096, dtype="f32", seed=0, cases=[(64, 64, 1)]),
    "cfg2": dict(m=128, n=65536, dtype="f32", seed=0,
                 cases=[(64, 64, 1), (64, 128, 1), (64, 256, 1), (64, 512, 1), (64, 1024, 1)]),
    "cfg3": dict(m=128, n=65536, dtype="f32", seed=0,
                 cases=[(16384, 16384, 1), (16384, 8192, 2), (16384, 4096, 4), (16384, 2048, 8),
                        (16384, 1024, 16)]),
    "cfg4": dict(m=128, n=1 << 20, dtype="f32", seed=0,
                 cases=[(64, 64, 1), (64, 1024, 1), (64, 8, 8), (64, 128, 8),
                        (1 << 18, 1 << 18, 1), (1 << 18, 1 << 15, 8)]),
    "cfg5": dict(m=2048, n=8192, dtype="bf16", seed=0, cases=[(512, 512, 1)]),
    # Shapes of the paper's two small-k downstream tasks (Section 4.2, Figure 4), as synthetic
    # stand-ins: the Llama 3 logits and the PharMeBINet scores themselves are not available.
    # n is not a power of two and most b do not divide it.
    "vocab": dict(m=64, n=128256, dtype="bf16", seed=0,
                  cases=[(256, 256, 1), (256, 512, 1), (256, 1024, 1), (256, 256, 2), (256, 512, 2)]),
    "kg": dict(m=128, n=2653751, dtype="bf16", seed=0,
               cases=[(100, 100, 1), (100, 256, 1), (100, 1024, 1), (100, 128, 2), (100, 512, 2)]),
}


def normal_rows(m: int, n: int, seed: int = 0, dtype: str = "f32") -> torch.Tensor:
    """m x n i.i.d. N(0, 1); f32, or f32 rounded to nearest-even bf16."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    x = torch.randn((m, n), generator=g, dtype=torch.float32)
    return x if dtype == "f32" else x.to(torch.bfloat16)


def correlated_rows(m: int, n: int, rho: float, seed: int = 0, shuffle: bool = False) -> torch.Tensor:
    """m x n f32 rows of N(0, Sigma) with Sigma_ij = rho^|i-j| (Appendix A.1's correlated-sequence
    simulation), drawn as the stationary AR(1) sequence x_0 = z_0, x_i = rho*x_{i-1} +
    sqrt(1-rho^2)*z_i, which has exactly that covariance.  shuffle=True applies one random
    permutation per row afterwards (the figure's right panel)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    z = torch.randn((m, n), generator=g, dtype=torch.float64)
    x = torch.empty_like(z)
    x[:, 0] = z[:, 0]
    c = math.sqrt(1.0 - rho * rho)
    for i in range(1, n):
        x[:, i] = rho * x[:, i - 1] + c * z[:, i]
    if shuffle:
        for r in range(m):
            x[r] = x[r, torch.randperm(n, generator=g)]
    return x.to(torch.float32)


def attention_scores(heads: int = 32, queries: int = 64, keys: int = 8192, d: int = 128,
                     seed: int = 0) -> torch.Tensor:
    """(heads*queries) x keys bf16 score rows: (q . K^T) / sqrt(d), f32 matmul, then bf16."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    q = torch.randn((heads, queries, d), generator=g, dtype=torch.float32)
    kmat = torch.randn((heads, keys, d), generator=g, dtype=torch.float32)
    s = torch.matmul(q, kmat.transpose(1, 2)) / math.sqrt(d)
    return s.reshape(heads * queries, keys).to(torch.bfloat16)


def config_input(name: str) -> torch.Tensor:
    c = CONFIGS[name]
    if name == "cfg5":
        return attention_scores(seed=c["seed"])
    return normal_rows(c["m"], c["n"], c["seed"], c["dtype"])


def few_levels(m: int, n: int, levels: int, seed: int = 0, dtype: str = "f32") -> torch.Tensor:
    """Rows drawn from `levels` distinct values: almost every comparison is a tie."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    table = torch.randn((levels,), generator=g, dtype=torch.float32)
    pick = torch.randint(0, levels, (m, n), generator=g)
    x = table[pick]
    return x if dtype == "f32" else x.to(torch.bfloat16)


def special_values(m: int, n: int, seed: int = 0, dtype: str = "f32") -> torch.Tensor:
    """N(0,1) rows salted with +0, -0, +inf, -inf, denormals and the largest finite values."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    x = torch.randn((m, n), generator=g, dtype=torch.float32)
    if dtype == "f32":
        specials = torch.tensor([0.0, -0.0, float("inf"), float("-inf"), 1e-45, -1e-45, 1e-40, -1e-40,
                                 3.4028234e38, -3.4028234e38, 1.17549435e-38, -1.17549435e-38],
                                dtype=torch.float32)
    else:
        # bf16 denormals are f32 values below 2^-126 whose low 16 bits are zero
        specials = torch.tensor([0.0, -0.0, float("inf"), float("-inf"), 9.18355e-41, -9.18355e-41,
                                 1.8367e-40, -1.8367e-40, 3.3895314e38, -3.3895314e38,
                                 1.17549435e-38, -1.17549435e-38], dtype=torch.float32)
    where = torch.rand((m, n), generator=g) < 0.3
    pick = torch.randint(0, specials.numel(), (m, n), generator=g)
    x = torch.where(where, specials[pick], x)
    return x if dtype == "f32" else x.to(torch.bfloat16)


def as_numpy_bits(t: torch.Tensor) -> np.ndarray:
    """CPU view for the oracle: float32 array, or uint16 bit patterns for bf16."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    raise TypeError("expected float32 or bfloat16")
