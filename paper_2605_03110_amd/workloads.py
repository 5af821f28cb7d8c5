"""Seeded synthetic activations shaped like the paper's workloads.

This module only DRAWS inputs; it holds none of the selection arithmetic, so both
the GPU library's tests and the CPU oracle's tests may take their inputs from it.

The paper measures on real GPT-2 / GPT-J / OPT activations (Section 6.1), which
need weights and text that are not available; clustered synthetic activations
stand in for them.  A layer sequence is built as

    C_0[k]   = g_k / ||g_k||,  g_k ~ N(0, I_d)              K unit-norm centres
    a_0[t]   ~ Uniform{0..K-1}                               token -> centre
    X_l[t]   = C_l[a_l[t]] + s_n * eps,  eps ~ N(0, I_d)     redrawn every layer
    C_{l+1}  = C_l + s_c * N(0, I)                           centre drift
    a_{l+1}  = a_l with round(p*T) tokens (uniform, no replacement) re-drawn

with s_n = sigma_n / sqrt(d) and s_c = sigma_c / sqrt(d) under the default
"relative" scale (sigma is relative to the per-dimension RMS 1/sqrt(d) of a
unit-norm centre, which is what makes tokens of one centre redundant at
tau = 0.1), or s_n = sigma_n, s_c = sigma_c under scale="literal" (every token
then stays representative: a stress case with r = T).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Iterator, List, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    T: int
    d: int
    L: int
    dtype: str          # "f32" or "bf16"
    tau: float
    K: int              # number of centres
    sigma_n: float      # token noise
    sigma_c: float      # centre drift per layer
    p: float            # fraction of tokens re-assigned per layer
    batch: int = 1
    scale: str = "relative"

    def seed(self, sequence: int = 0) -> int:
        return 1000 * self.config_id + sequence


CONFIGS: Tuple[Workload, ...] = (
    Workload("c0_gpt2_small_T512", 0, 512, 768, 12, "f32", 0.1, 100, 0.004, 0.01, 0.05),
    Workload("c1_gpt2_T2048", 1, 2048, 768, 12, "bf16", 0.1, 400, 0.004, 0.01, 0.05),
    Workload("c2_gptj_T2048", 2, 2048, 4096, 28, "bf16", 0.1, 400, 0.004, 0.01, 0.03),
    Workload("c3_opt_T2048_lowcoh", 3, 2048, 4096, 32, "bf16", 0.1, 1000, 0.004, 0.02, 0.12),
    Workload("c4_long_T8192", 4, 8192, 4096, 32, "bf16", 0.1, 400, 0.004, 0.01, 0.05, batch=4),
)


def config(i: int, **overrides) -> Workload:
    w = CONFIGS[i]
    return replace(w, **overrides) if overrides else w


def to_dtype(x32: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 host array -> CPU tensor in the workload's dtype (bf16: round-to-nearest-even)."""
    t = torch.from_numpy(np.ascontiguousarray(x32))
    if dtype == "bf16":
        return t.to(torch.bfloat16)
    if dtype == "f32":
        return t
    raise ValueError("dtype must be 'f32' or 'bf16'")


def as_f64(x: torch.Tensor) -> np.ndarray:
    """Exact widening of the values a device kernel would see, for a float64 checker."""
    return x.to(torch.float64).numpy()


def layers(w: Workload, sequence: int = 0, n_layers: int | None = None) -> Iterator[torch.Tensor]:
    """Yield X_0, X_1, ... (CPU tensors, T x d, in w.dtype) for one sequence."""
    rng = np.random.default_rng(w.seed(sequence))
    T, d, K = w.T, w.d, w.K
    L = w.L if n_layers is None else n_layers
    unit = 1.0 / np.sqrt(d) if w.scale == "relative" else 1.0
    if w.scale not in ("relative", "literal"):
        raise ValueError("scale must be 'relative' or 'literal'")
    s_n = np.float32(w.sigma_n * unit)
    s_c = np.float32(w.sigma_c * unit)
    C = rng.standard_normal((K, d), dtype=np.float32)
    C /= np.linalg.norm(C, axis=1, keepdims=True)
    a = rng.integers(0, K, size=T)
    n_move = int(round(w.p * T))
    for _ in range(L):
        X = C[a] + s_n * rng.standard_normal((T, d), dtype=np.float32)
        yield to_dtype(X, w.dtype)
        C = C + s_c * rng.standard_normal((K, d), dtype=np.float32)
        moved = rng.choice(T, size=n_move, replace=False)
        a = a.copy()
        a[moved] = rng.integers(0, K, size=n_move)


def layer_list(w: Workload, sequence: int = 0, n_layers: int | None = None) -> List[torch.Tensor]:
    return list(layers(w, sequence, n_layers))


def small(T: int, d: int, K: int, L: int, dtype: str = "bf16", seed: int = 7, p: float = 0.05,
          sigma_c: float = 0.01, tau: float = 0.1, scale: str = "relative") -> Workload:
    """A reduced workload of the same recipe for tests (ragged T and d allowed)."""
    return Workload("small_T%d_d%d" % (T, d), seed, T, d, L, dtype, tau, K, 0.004, sigma_c, p, scale=scale)


def qkv(w: Workload, H: int, sequence: int = 0, layer: int = 0):
    """Seeded stand-ins for one layer's query / key / value activations, T x d with H heads side by side (the paper's
    are projections of real activations, which are not available): i.i.d. N(0, 1) entries, so that scores divided by
    sqrt(d_h) have unit variance.  Returns three CPU tensors in w.dtype."""
    if w.d % H != 0:
        raise ValueError("d must be a multiple of the head count")
    rng = np.random.default_rng(7_000_000 + 1000 * w.seed(sequence) + layer)
    return tuple(to_dtype(rng.standard_normal((w.T, w.d), dtype=np.float32), w.dtype) for _ in range(3))
