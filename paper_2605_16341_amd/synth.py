"""Seeded synthetic inputs for the Orth-Dion optimizer step.

This module only *draws inputs*: gradients with a prescribed spectrum plus
isotropic noise, initial parameters, momentum buffers and warm-start right
factors, and the bf16 bit patterns both consumers read.  It holds none of the
method's arithmetic (no buffer accumulation, projection, orthogonalisation of
the method's factors, error feedback or update), so the CPU oracle and the HIP
path can both take their inputs from here without sharing any step of the
algorithm.

The paper trains on language-model gradients (Sec. 7.1, App. K); those data are
not available, so the matrix *shapes*, storage types (bf16 parameters and
gradients, fp32 state; App. K tables) and rank fractions (r = d/4, App. K.2)
are kept and the values are synthetic: a fixed low-dimensional signal with a
power-law spectrum and fresh Gaussian noise at every step, which mimics a
stable gradient subspace under mini-batch noise (the stochastic regime of
Sec. 6').
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 20260516


# --------------------------------------------------------------------------
# bf16 bit patterns (storage format of X and G in the bf16 configurations)
# --------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round-to-nearest-even), as uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# random factors
# --------------------------------------------------------------------------

def rng_for(seed: int) -> np.random.Generator:
    """Counter-based generator (Philox) keyed by ``seed``."""
    return np.random.Generator(np.random.Philox(key=int(seed)))


def random_orthonormal(rows: int, cols: int, rng: np.random.Generator) -> np.ndarray:
    """``rows x cols`` matrix with orthonormal columns: the Q factor of a Gaussian
    matrix, with the signs chosen so that the triangular factor has a positive
    diagonal (which makes the draw a deterministic function of the Gaussian)."""
    a = rng.standard_normal((rows, cols))
    q, t = np.linalg.qr(a)
    return q * np.where(np.diag(t) < 0.0, -1.0, 1.0)[None, :]


def gaussian_factor(rows: int, cols: int, rng: np.random.Generator) -> np.ndarray:
    """Cheap stand-in for a random orthonormal factor at large shapes: i.i.d.
    N(0, 1/rows) entries (columns have unit norm and are orthogonal in expectation)."""
    return (rng.standard_normal((rows, cols), dtype=np.float32) / np.float32(np.sqrt(rows)))


# --------------------------------------------------------------------------
# gradient streams
# --------------------------------------------------------------------------

@dataclasses.dataclass
class GradientStream:
    """A fixed signal ``left @ diag(spectrum) @ right.T`` plus fresh noise each step.

    ``gradient(step)`` is a deterministic function of ``(seed, step)``; the noise
    generator of step ``t`` is keyed by ``seed + t`` so steps can be drawn in any order.
    """

    m: int
    n: int
    seed: int
    signal: np.ndarray          # m x n, float64 or float32
    noise_std: float
    out_dtype: str              # "f32" or "bf16"
    persistence: float = 0.0    # lag-1 correlation of the noise terms, in [-0.5, 0.5]

    def _draw(self, step: int) -> np.ndarray:
        rng = rng_for(self.seed + 1 + int(step))
        return rng.standard_normal((self.m, self.n), dtype=np.float32)

    def gradient_f32(self, step: int) -> np.ndarray:
        noise = self._draw(step)
        if self.persistence != 0.0:
            # moving average of two independent draws: unit variance, lag-1 correlation
            # phi * sqrt(1 - phi^2) = persistence, zero correlation beyond lag 1
            rho = float(self.persistence)
            if abs(rho) > 0.5:
                raise ValueError("persistence must lie in [-0.5, 0.5]")
            phi = np.sign(rho) * np.sqrt((1.0 - np.sqrt(1.0 - 4.0 * rho * rho)) / 2.0)
            noise = (np.float32(phi) * self._draw(step - 1) + np.float32(np.sqrt(1.0 - phi * phi)) * noise)
        g = (self.signal + np.float32(self.noise_std) * noise).astype(np.float32)
        return g

    def gradient(self, step: int) -> np.ndarray:
        """The gradient as stored: float32 array, or uint16 bf16 bit patterns."""
        g = self.gradient_f32(step)
        if self.out_dtype == "bf16":
            return f32_to_bf16_bits(g)
        return g


def inverse_index_stream(m: int, n: int, seed: int, noise_std: float = 0.01,
                         out_dtype: str = "f32") -> GradientStream:
    """Gradients ``U diag(1/i) V^T + noise_std * N(0,1)`` with random orthogonal U, V
    (the small all-fp32 configuration)."""
    rng = rng_for(seed)
    k = min(m, n)
    u = random_orthonormal(m, k, rng)
    v = random_orthonormal(n, k, rng)
    s = 1.0 / np.arange(1, k + 1, dtype=np.float64)
    signal = (u * s[None, :]) @ v.T
    return GradientStream(m, n, seed, signal.astype(np.float32), noise_std, out_dtype)


def power_law_stream(m: int, n: int, seed: int, exponent: float = 0.5,
                     noise_energy: float = 0.05, rms: float = 1e-2,
                     out_dtype: str = "bf16", orthonormal: bool = True,
                     components: Optional[int] = None, persistence: float = 0.0) -> GradientStream:
    """Gradients whose signal has singular values ``i^-exponent`` and whose isotropic
    Gaussian noise carries ``noise_energy`` of the squared Frobenius norm.

    ``rms`` is the root-mean-square entry of the whole gradient.  With
    ``orthonormal=False`` the singular-vector factors are Gaussian/sqrt(dim)
    stand-ins (used for the largest shapes, where an exact orthonormal factor
    would cost more than the test itself).  ``components`` limits the number of
    spectral terms (default ``min(m, n)``).  ``persistence`` correlates the noise of
    consecutive steps (the coherent / stochastic / anti-correlated regimes of the
    error-feedback analysis, Sec. 6.3 of the paper).
    """
    rng = rng_for(seed)
    k = min(m, n) if components is None else int(components)
    s = np.arange(1, k + 1, dtype=np.float64) ** (-float(exponent))
    total = float(m) * float(n) * rms * rms
    c_s = np.sqrt((1.0 - noise_energy) * total / float(np.sum(s * s)))
    c_n = np.sqrt(noise_energy * total / (float(m) * float(n)))
    if orthonormal:
        a = random_orthonormal(m, k, rng)
        c = random_orthonormal(n, k, rng)
        signal = ((a * (c_s * s)[None, :]) @ c.T).astype(np.float32)
    else:
        a = gaussian_factor(m, k, rng)
        c = gaussian_factor(n, k, rng)
        signal = (a * (c_s * s).astype(np.float32)[None, :]) @ c.T
    return GradientStream(m, n, seed, signal, float(c_n), out_dtype, float(persistence))


# --------------------------------------------------------------------------
# initial state
# --------------------------------------------------------------------------

@dataclasses.dataclass
class MatrixState:
    """Initial buffers of one parameter matrix, in their storage formats."""

    X: np.ndarray   # float32, or uint16 bf16 bits
    M: np.ndarray   # float32
    Q: np.ndarray   # float32, n x r


def initial_state(m: int, n: int, r: int, seed: int, x_dtype: str = "bf16",
                  momentum_std: float = 0.0, param_std: float = 0.02) -> MatrixState:
    """X ~ N(0, param_std^2) rounded to its storage type; M ~ N(0, momentum_std^2)
    (zero when ``momentum_std`` is 0); Q a random ``n x r`` orthonormal matrix."""
    rng = rng_for(seed + 500_000)
    x = (param_std * rng.standard_normal((m, n))).astype(np.float32)
    if momentum_std > 0.0:
        mom = (momentum_std * rng.standard_normal((m, n))).astype(np.float32)
    else:
        mom = np.zeros((m, n), dtype=np.float32)
    q = random_orthonormal(n, r, rng).astype(np.float32)
    if x_dtype == "bf16":
        x = f32_to_bf16_bits(x)
    return MatrixState(x, mom, q)


# --------------------------------------------------------------------------
# workloads (shapes of the five benchmark configurations)
# --------------------------------------------------------------------------

@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    shapes: Tuple[Tuple[int, int], ...]   # (m, n) per matrix, in order
    r: int
    x_dtype: str                          # "f32" | "bf16"  (X and G share it)
    mu: float = 0.95
    lr: float = 0.01
    steps: int = 10
    spectrum: str = "power_law"           # "inverse_index" | "power_law"
    momentum_std: float = 0.0

    @property
    def elements(self) -> int:
        return sum(m * n for m, n in self.shapes)


def _layers(n_layers: int, per_layer: List[Tuple[int, int]]) -> Tuple[Tuple[int, int], ...]:
    out: List[Tuple[int, int]] = []
    for _ in range(n_layers):
        out.extend(per_layer)
    return tuple(out)


WORKLOADS: Dict[str, Workload] = {
    # single small all-fp32 matrix
    "C1": Workload("C1", ((256, 256),), r=16, x_dtype="f32", steps=5,
                   spectrum="inverse_index", momentum_std=0.02),
    # one square matrix, bf16 parameters/gradients, fp32 state
    "C2": Workload("C2", ((4096, 4096),), r=256, x_dtype="bf16", steps=20),
    # 1.3B-style decoder: 24 layers x {Wqkv, Wo, W_up, W_down}
    "C3": Workload("C3", _layers(24, [(2048, 6144), (2048, 2048), (2048, 8192), (8192, 2048)]),
                   r=512, x_dtype="bf16", steps=10),
    # 8B-style single layer at real shape
    "C4": Workload("C4", ((4096, 6144), (4096, 4096), (4096, 14336), (4096, 14336), (14336, 4096)),
                   r=1024, x_dtype="bf16", steps=10),
}
for _r in (16, 64, 256, 1024, 2048):
    WORKLOADS[f"C5-r{_r}"] = Workload(f"C5-r{_r}", ((8192, 8192),), r=_r, x_dtype="bf16", steps=10)


def matrix_seed(workload: str, index: int) -> int:
    """Seed of matrix ``index`` of a workload: base + 1000 * index, offset per workload
    so that different workloads never share a stream."""
    tag = sum((i + 1) * ord(c) for i, c in enumerate(workload)) % 9973
    return BASE_SEED + 1_000_000 * tag + 1000 * int(index)


def make_stream(w: Workload, index: int, orthonormal: Optional[bool] = None) -> GradientStream:
    m, n = w.shapes[index]
    seed = matrix_seed(w.name, index)
    if w.spectrum == "inverse_index":
        return inverse_index_stream(m, n, seed, 0.01, w.x_dtype)
    if orthonormal is None:
        orthonormal = max(m, n) <= 4096
    return power_law_stream(m, n, seed, out_dtype=w.x_dtype, orthonormal=orthonormal)


def make_state(w: Workload, index: int) -> MatrixState:
    m, n = w.shapes[index]
    return initial_state(m, n, w.r, matrix_seed(w.name, index), w.x_dtype, w.momentum_std)
