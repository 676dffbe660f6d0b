"""Seeded synthetic inputs placed in device memory (torch is used for memory only).

Two routes, both free of the method's arithmetic:
  * ``to_device`` / ``to_host`` move the numpy arrays of ``synth`` (float32, or uint16 bf16 bit
    patterns) to and from the GPU unchanged;
  * ``device_state`` / ``device_gradients`` draw the same recipe directly on the device for
    matrix sets too large to generate on the host in reasonable time: a power-law signal
    with Gaussian stand-ins for the singular-vector factors plus fresh noise per pool entry
    (the recipe of ``synth.power_law_stream(orthonormal=False)``, drawn with torch's
    generator).
"""
from __future__ import annotations

import numpy as np

from . import synth


def to_device(arr: np.ndarray, torch, device="cuda:0"):
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16).copy()).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr)).to(device)


def to_host(t, torch) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def device_gradients(torch, w: synth.Workload, index: int, pool: int, dev):
    """`pool` gradients of matrix `index` of workload `w`, generated on the device."""
    m, n = w.shapes[index]
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.matrix_seed(w.name, index))
    k = min(m, n)
    s = torch.arange(1, k + 1, device=dev, dtype=torch.float32) ** -0.5
    rms, noise_energy = 1e-2, 0.05
    total = float(m) * float(n) * rms * rms
    c_s = ((1.0 - noise_energy) * total / float((s * s).sum())) ** 0.5
    c_n = (noise_energy * total / (float(m) * float(n))) ** 0.5
    a = torch.randn(m, k, device=dev, generator=gen) / m ** 0.5
    c = torch.randn(n, k, device=dev, generator=gen) / n ** 0.5
    signal = (a * (c_s * s)[None, :]) @ c.T
    del a, c
    out = []
    for _ in range(pool):
        g = signal + c_n * torch.randn(m, n, device=dev, generator=gen)
        out.append(g.to(torch.bfloat16) if w.x_dtype == "bf16" else g)
    del signal
    return out


def device_state(torch, w: synth.Workload, index: int, dev):
    """Initial X, M and an orthonormal warm-start factor Q0 of matrix `index`, on the device."""
    m, n = w.shapes[index]
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.matrix_seed(w.name, index) + 500_000)
    x = 0.02 * torch.randn(m, n, device=dev, generator=gen)
    x = x.to(torch.bfloat16) if w.x_dtype == "bf16" else x
    if w.momentum_std == 0:
        mom = torch.zeros(m, n, device=dev)
    else:
        mom = w.momentum_std * torch.randn(m, n, device=dev, generator=gen)
    return x, mom, _orthonormal_columns(torch, torch.randn(n, w.r, device=dev, generator=gen))


def _orthonormal_columns(torch, a):
    """Orthonormal basis of the columns of the Gaussian matrix `a` (well conditioned) by two
    rounds of Cholesky QR in fp64: products on the device, the r x r factorisation on the host.
    (The device QR of the solver library is avoided: under rocprofv3 counter collection it
    aborts for some of the benchmark shapes.)"""
    q = a.double()
    for _ in range(2):
        gram = (q.T @ q).cpu()
        lower = torch.linalg.cholesky(gram)
        w = torch.linalg.solve_triangular(lower, torch.eye(gram.shape[0], dtype=torch.float64), upper=False).T
        q = q @ w.to(a.device)
    return q.float().contiguous()
