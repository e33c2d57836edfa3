"""Seeded synthetic workloads shared by the tests, the benchmark and the smoke check.

This module only draws random tensors and measures distances between outputs;
it holds none of the method's arithmetic (no quantiser, no softmax) and is
imported neither by the GPU library nor by the CPU oracle.

The five configurations are the ones the benchmark definition names: shapes of
an LLM prefill (causal, d=128), of a video diffusion transformer (N not a tile
multiple, d=64) and an outlier stress case.  They stand in for the real model
activations the paper measured on (Section 4.1), which are not available.

Recipe: numpy ``Generator(PCG64(SEED0 + index))``, drawn in float32 in the order
Q, K, K-bias, (outlier channel choice), V, then rounded to nearest-even to the
16-bit dtype of the configuration.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import torch

SEED0 = 250521136


@dataclass(frozen=True)
class Workload:
    name: str
    index: int
    B: int
    H: int
    N: int
    d: int
    causal: bool
    dtype: str          # "fp16" | "bf16"
    q_dist: str = "normal"      # "normal" | "student_t3"
    k_outlier_channels: int = 0  # channels per (b, h) multiplied by 20 before the bias
    k_bias_std: float = 3.0

    @property
    def sm_scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def ops(self) -> float:
        """Attention operation count 4*B*H*N^2*d, halved under a causal mask."""
        full = 4.0 * self.B * self.H * float(self.N) ** 2 * self.d
        return full / 2 if self.causal else full

    def scaled(self, *, B=None, H=None, N=None, name=None) -> "Workload":
        """Same distributions and dtype at a smaller size (CPU tests, smoke)."""
        return Workload(name or f"{self.name}-small", self.index, B or self.B, H or self.H,
                        N or self.N, self.d, self.causal, self.dtype, self.q_dist,
                        self.k_outlier_channels, self.k_bias_std)


CONFIGS = [
    Workload("cfg1", 1, 1, 2, 1024, 128, False, "fp16"),
    Workload("cfg2", 2, 4, 32, 4096, 128, True, "fp16"),
    Workload("cfg3", 3, 2, 32, 8192, 64, False, "bf16"),
    Workload("cfg4", 4, 1, 48, 17776, 64, False, "bf16"),
    Workload("cfg5", 5, 1, 24, 32768, 128, False, "bf16", q_dist="student_t3", k_outlier_channels=4),
]


def torch_dtype(name: str) -> torch.dtype:
    return {"fp16": torch.float16, "bf16": torch.bfloat16}[name]


def generate(wl: Workload, seed: int | None = None):
    """Return (q, k, v) as CPU torch tensors [B, H, N, d] of the workload's 16-bit dtype."""
    rng = np.random.Generator(np.random.PCG64(SEED0 + wl.index if seed is None else seed))
    shape = (wl.B, wl.H, wl.N, wl.d)
    if wl.q_dist == "student_t3":
        q = rng.standard_t(3.0, size=shape).astype(np.float32)
    else:
        q = rng.standard_normal(shape, dtype=np.float32)
    k = rng.standard_normal(shape, dtype=np.float32)
    bias = rng.standard_normal((wl.B, wl.H, 1, wl.d), dtype=np.float32) * np.float32(wl.k_bias_std)
    if wl.k_outlier_channels:
        for b in range(wl.B):
            for h in range(wl.H):
                ch = rng.choice(wl.d, size=wl.k_outlier_channels, replace=False)
                k[b, h][:, ch] *= np.float32(20.0)
    k += bias
    v = rng.standard_normal(shape, dtype=np.float32)
    dt = torch_dtype(wl.dtype)
    return tuple(torch.from_numpy(x).to(dt) for x in (q, k, v))


def as_f32(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a 16-bit tensor to a float32 numpy array."""
    return t.detach().to("cpu", torch.float32).numpy()


# --------------------------------------------------------------------------
# accuracy metrics (paper, Appendix "Accuracy metrics"): outputs are flattened
# --------------------------------------------------------------------------
def cos_sim(o_ref, o) -> float:
    a = np.asarray(o_ref, dtype=np.float64).ravel()
    b = np.asarray(o, dtype=np.float64).ravel()
    return float(np.dot(a, b) / (np.sqrt(np.dot(a, a)) * np.sqrt(np.dot(b, b))))


def rel_l1(o_ref, o) -> float:
    a = np.asarray(o_ref, dtype=np.float64).ravel()
    b = np.asarray(o, dtype=np.float64).ravel()
    return float(np.abs(a - b).sum() / np.abs(a).sum())


def rmse(o_ref, o) -> float:
    a = np.asarray(o_ref, dtype=np.float64).ravel()
    b = np.asarray(o, dtype=np.float64).ravel()
    return float(np.sqrt(np.mean((a - b) ** 2)))
