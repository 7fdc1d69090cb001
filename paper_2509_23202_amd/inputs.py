"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds NO arithmetic of the method (no Hadamard, no scales, no FP4 rounding): it only draws
random matrices with the value distributions and shapes of the workloads and rounds them to bf16 so that
the CPU oracle and the HIP library see identical bits.  Everything is host-side NumPy.

Stand-in statement: the paper times single linear layers taken from Llama-3.3-70B / Qwen3-32B checkpoints
(Section 5 item 4, Appendix on QuTLASS performance).  Those weights are not available here; the tensors
below take the layers' shapes and a stylised version of LLM statistics (heavy tails, a few outlier
channels; Section 3 "Modeling Distributions") instead.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 2509_23202 * 10  # + config number


# ---------------------------------------------------------------- bf16 bit helpers (storage only)
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------- generators
def _rng(seed: int, stream: int) -> np.random.Generator:
    ss = np.random.SeedSequence(seed).spawn(stream + 1)[stream]
    return np.random.Generator(np.random.Philox(ss))


def _draw(rng: np.random.Generator, dist: str, shape) -> np.ndarray:
    if dist == "normal":
        return rng.standard_normal(shape, dtype=np.float32)
    if dist == "laplace":  # Laplace(0, 1): scale 1, variance 2
        return rng.laplace(0.0, 1.0, shape).astype(np.float32)
    if dist == "student_t3":  # Student-t, nu = 3, scaled to unit variance (var = nu/(nu-2) = 3)
        return (rng.standard_t(3.0, shape) / np.sqrt(3.0)).astype(np.float32)
    raise ValueError(f"unknown distribution {dist!r}")


def activations(M: int, K: int, *, dist: str = "normal", outlier_frac: float = 0.005,
                outlier_mult: float = 50.0, seed: int = BASE_SEED, chunk_rows: int = 1024) -> np.ndarray:
    """bf16 bit patterns [M,K]: i.i.d. ``dist`` with round(outlier_frac*K) channels (columns, chosen
    without replacement from a separate stream) multiplied by ``outlier_mult``."""
    rng_x = _rng(seed, 0)
    rng_o = _rng(seed, 2)
    n_out = int(round(outlier_frac * K))
    cols = rng_o.choice(K, size=n_out, replace=False) if n_out > 0 else np.zeros(0, dtype=np.int64)
    out = np.empty((M, K), dtype=np.uint16)
    for r0 in range(0, M, chunk_rows):
        r1 = min(M, r0 + chunk_rows)
        x = _draw(rng_x, dist, (r1 - r0, K))
        if n_out:
            x[:, cols] *= np.float32(outlier_mult)
        out[r0:r1] = f32_to_bf16_bits(x)
    return out


def weights(N: int, K: int, *, sigma: float = 0.02, seed: int = BASE_SEED, chunk_rows: int = 1024) -> np.ndarray:
    """bf16 bit patterns [N,K] ~ Normal(0, sigma) (sigma is the standard deviation)."""
    rng_w = _rng(seed, 1)
    out = np.empty((N, K), dtype=np.uint16)
    for r0 in range(0, N, chunk_rows):
        r1 = min(N, r0 + chunk_rows)
        w = rng_w.standard_normal((r1 - r0, K), dtype=np.float32) * np.float32(sigma)
        out[r0:r1] = f32_to_bf16_bits(w)
    return out


# ---------------------------------------------------------------- workload recipes
@dataclass(frozen=True)
class Layer:
    name: str
    K: int
    N: int


LLAMA3_8B_LAYERS = (Layer("qkv", 4096, 6144), Layer("o_proj", 4096, 4096),
                    Layer("gate_up", 4096, 28672), Layer("down", 14336, 4096))
LLAMA3_70B_LAYERS = (Layer("qkv", 8192, 10240), Layer("gate_up", 8192, 57344), Layer("down", 28672, 8192))


@dataclass(frozen=True)
class Recipe:
    """Value distributions of one benchmark configuration."""
    cfg: int
    fmt: str            # "mxfp4" | "nvfp4"
    had_block: int
    x_dist: str
    outlier_frac: float
    outlier_mult: float
    w_sigma: float

    @property
    def seed(self) -> int:
        return BASE_SEED + self.cfg

    def x(self, M: int, K: int, salt: int = 0) -> np.ndarray:
        return activations(M, K, dist=self.x_dist, outlier_frac=self.outlier_frac,
                           outlier_mult=self.outlier_mult, seed=self.seed + 1000 * salt)

    def w(self, N: int, K: int, salt: int = 0) -> np.ndarray:
        return weights(N, K, sigma=self.w_sigma, seed=self.seed + 1000 * salt)


RECIPES = {
    1: Recipe(1, "mxfp4", 32, "normal", 0.005, 50.0, 0.02),       # M=64, K=N=4096
    2: Recipe(2, "mxfp4", 32, "normal", 0.005, 50.0, 0.02),       # decode, M in {1,16}
    3: Recipe(3, "mxfp4", 32, "normal", 0.005, 50.0, 0.02),       # prefill, M=4096
    4: Recipe(4, "nvfp4", 16, "student_t3", 0.0, 1.0, 0.015),     # 70B shapes
    5: Recipe(5, "mxfp4", 32, "normal", 0.005, 50.0, 0.02),       # 5a: block sweep, M=2048, K=N=8192
    6: Recipe(6, "mxfp4", 32, "laplace", 0.01, 100.0, 0.02),      # 5b: standalone rotate+quantize
}
