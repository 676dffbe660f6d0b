"""Helpers shared by the GPU parity tests: upload seeded inputs, step the HIP path through
the C ABI, fetch results, and step the fp64 oracle on the same inputs."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

from oracle.orthdion_oracle import OrthDionOracle, bf16_bits_to_f64, rel_fro
from paper_2605_16341_amd import binding, synth
from paper_2605_16341_amd.device_inputs import to_device, to_host


class GpuRun:
    """State of a set of matrices on the GPU, stepped by the library."""

    def __init__(self, shapes, r, x_dtype, states: Sequence[synth.MatrixState], variant="qr", ef="dion",
                 precision="auto", mu=0.95, lr=0.01, groups=0):
        import torch
        self.torch = torch
        self.opt = binding.OrthDion(shapes, r, x_dtype=x_dtype, variant=variant, ef=ef, precision=precision,
                                    mu=mu, lr=lr, groups=groups)
        self.X = [to_device(s.X, torch) for s in states]
        self.M = [to_device(s.M, torch) for s in states]
        self.Q = [to_device(s.Q, torch) for s in states]

    def step(self, grads: Sequence[np.ndarray]):
        G = [to_device(g, self.torch) for g in grads]
        self.opt.step(self.X, G, self.M, self.Q)
        self.torch.cuda.synchronize()
        return self.opt.info()

    def fetch(self, index: int, with_factors=True) -> Dict[str, np.ndarray]:
        t = self.torch
        out = {"X": to_host(self.X[index], t), "M": to_host(self.M[index], t), "Q": to_host(self.Q[index], t)}
        if with_factors:
            for k, v in self.opt.debug_factors(index).items():
                out[k] = v.cpu().numpy()
        return out


def x_as_f64(x: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f64(x) if x.dtype == np.uint16 else x.astype(np.float64)


def bf16_ulp_distance(a_bits: np.ndarray, b_bits: np.ndarray) -> np.ndarray:
    """Distance in units of the last place between two bf16 bit patterns (sign-magnitude
    mapped onto a monotone integer line)."""
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def bf16_gap_beyond(a_bits: np.ndarray, b_bits: np.ndarray, spacings: float, slack: float) -> float:
    """Fraction of entries whose two bf16 values lie further apart than `spacings` bf16
    spacings (2^-7 of the larger magnitude) plus `slack`.  The distance in ulps alone says
    little where |x| is tiny: there one spacing is far below the update itself, so two correct
    updates that differ within the direction's tolerance are many ulps apart; `slack` is that
    tolerance times the largest update entry."""
    a, b = bf16_bits_to_f64(a_bits), bf16_bits_to_f64(b_bits)
    spacing = np.maximum(np.abs(a), np.abs(b)) * 2.0 ** -7
    return float(np.mean(np.abs(a - b) > spacings * spacing + slack))


def compare_step(gpu: Dict[str, np.ndarray], orc: Dict[str, np.ndarray], x_prev: np.ndarray, lr: float) -> Dict[str, float]:
    """Relative Frobenius errors of the GPU results against the oracle's.  The parameter is
    compared through the applied update (X_prev - X_new) / lr, because ||X_new - X_prev||
    is tiny next to ||X||; for bf16 parameters also the fraction of entries whose stored
    bits differ from the oracle's rounding, and the largest distance in ulps."""
    res = {"M": rel_fro(gpu["M"], orc["M"]), "Q": rel_fro(gpu["Q"], orc["Q"])}
    if "P" in gpu:
        res["P"] = rel_fro(gpu["P"], orc["P"])
        res["R"] = rel_fro(gpu["R"], orc["R"])
        res["D"] = rel_fro(gpu["P"].astype(np.float64) @ gpu["Q"].astype(np.float64).T, orc["D"])
    xg = x_as_f64(gpu["X"])
    res["X"] = rel_fro(xg, orc["X"])
    if gpu["X"].dtype == np.uint16:
        dist = bf16_ulp_distance(gpu["X"], orc["X_bits"])
        res["X_bits_mismatch"] = float(np.mean(dist != 0))
        res["X_max_ulp"] = float(dist.max())
        slack = 2e-2 * lr * float(np.max(np.abs(orc["D"])))
        res["X_beyond_one_spacing"] = bf16_gap_beyond(gpu["X"], orc["X_bits"], 1.0, slack)
    else:
        res["update"] = rel_fro((x_as_f64(x_prev) - xg) / lr, orc["D"])
    return res


def oracle_for(w: synth.Workload, variant="qr", ef="dion", mu=None, lr=None) -> OrthDionOracle:
    return OrthDionOracle(mu=w.mu if mu is None else mu, lr=w.lr if lr is None else lr, variant=variant, ef=ef,
                          x_bf16=(w.x_dtype == "bf16"))
