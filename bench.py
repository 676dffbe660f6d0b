#!/usr/bin/env python3
"""Benchmark of the Orth-Dion optimizer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--variant qr]

One "step" is one orthdion_step over the whole matrix set of the workload (all phases of
the method: buffer, projection, left orthogonalisation, back-projection, right
orthogonalisation or column normalisation, error feedback and parameter update).  Inputs
are synthetic, seeded, and resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense fp16 / bf16 matrix cores, published

# HBM traffic per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE scaled by a
# copy kernel of known size); see profiles/.  Keyed by (workload, phase); bytes per launch.
MEASURED_TRAFFIC = {
    # profiles/orthdion_step_C2_hbm_counters.txt: 2.000 * FETCH_SIZE + 1.000 * WRITE_SIZE, bytes
    ("C2", "efx"): 272795008,
    ("C2", "back"): 186232466,
    ("C2", "proj"): 155187017,
    # profiles/orthdion_step_C5-r16_hbm_counters.txt
    ("C5-r16", "efx"): 944195895,
    ("C5-r16", "back"): 409127991,
    ("C5-r16", "proj"): 419819959,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C2")
    ap.add_argument("--variant", default="qr", choices=["qr", "colnorm"])
    ap.add_argument("--precision", default="auto", choices=["auto", "fast", "exact"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--pool", type=int, default=4, help="distinct gradients per matrix cycled through")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="accepted for older command lines: the plain 1 GiB device copy that a counter run is "
                         "scaled by now always runs (its bandwidth is reported as copy_GBps)")
    return ap.parse_args()


def device_gradients(torch, w, index, pool, dev):
    """Gradients of one matrix generated on the device: power-law signal with Gaussian
    stand-ins for the singular-vector factors plus fresh noise per pool entry (the same
    recipe as synth.power_law_stream(orthonormal=False), drawn with torch's generator)."""
    m, n = w.shapes[index]
    from paper_2605_16341_amd import synth
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


def device_state(torch, w, index, dev):
    from paper_2605_16341_amd import synth
    m, n = w.shapes[index]
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.matrix_seed(w.name, index) + 500_000)
    x = 0.02 * torch.randn(m, n, device=dev, generator=gen)
    x = x.to(torch.bfloat16) if w.x_dtype == "bf16" else x
    mom = torch.zeros(m, n, device=dev) if w.momentum_std == 0 else w.momentum_std * torch.randn(m, n, device=dev, generator=gen)
    q, _ = torch.linalg.qr(torch.randn(n, w.r, device=dev, generator=gen))
    return x, mom, q.contiguous()


def algorithmic_work(w, phase):
    """Algorithmic HBM bytes and flops of one step's launches of a phase, summed over the
    matrix set.  Matrix traffic follows the 20 B/element floor for bf16 (28 for fp32):
    M and G are read by the projection and again by the back-projection (a grid-wide
    dependency separates them), M is written once and X read and written once (both
    booked on the fused error-feedback/update kernel); factor traffic is added per kernel."""
    e = 2 if w.x_dtype == "bf16" else 4
    r = w.r
    nbytes = flops = 0
    for m, n in w.shapes:
        mn = m * n
        if phase == "proj":
            nbytes += mn * (4 + e) + 4 * r * (n + m)
            flops += 2 * mn * r
        elif phase == "back":
            nbytes += mn * (4 + e) + 4 * r * (n + m)
            flops += 2 * mn * r
        elif phase == "efx":
            nbytes += mn * (4 + 2 * e) + 4 * r * (m + 2 * n)
            flops += 4 * mn * r
    return nbytes, flops


def cpu_baseline(w, variant, seconds):
    """The fp64 oracle, as it stands, timed on the host cores on the first matrix of the
    workload (whole steps until `seconds` have passed, after one untimed step)."""
    import numpy as np
    from oracle.orthdion_oracle import OrthDionOracle
    from paper_2605_16341_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    m, n = w.shapes[0]
    stream = synth.make_stream(w, 0, orthonormal=False) if w.spectrum == "power_law" else synth.make_stream(w, 0)
    st = synth.make_state(w, 0)
    orc = OrthDionOracle(mu=w.mu, lr=w.lr, variant=variant, ef="dion", x_bf16=(w.x_dtype == "bf16"))
    x, mom, q = st.X, st.M.astype(np.float64), st.Q.astype(np.float64)
    grads = [stream.gradient(t) for t in range(2)]
    o = orc.step(x, grads[0], mom, q)
    x = o["X_bits"] if w.x_dtype == "bf16" else o["X"]
    mom, q = o["M"], o["Q"]
    done, t0 = 0, time.perf_counter()
    while True:
        o = orc.step(x, grads[done % 2], mom, q)
        x = o["X_bits"] if w.x_dtype == "bf16" else o["X"]
        mom, q = o["M"], o["Q"]
        done += 1
        el = time.perf_counter() - t0
        if el >= seconds or done >= 200:
            break
    frac = (m * n) / float(w.elements)
    per_set = el / done / frac
    return {"value": 1.0 / per_set, "unit": "steps/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{done} oracle step(s) on matrix 0 ({m}x{n}, r={w.r}) of {w.name} in {el:.1f} s"
                      + ("" if len(w.shapes) == 1 else f", scaled by its share {frac:.4f} of the set's elements")}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2605_16341_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    binding.load()
    dev = torch.device("cuda:0")
    w = synth.WORKLOADS[args.workload]
    nmat = len(w.shapes)

    # ---------------- inputs, resident in HBM
    X, M, Q, Gpool = [], [], [], []
    if w.name in ("C1", "C2"):
        # the exact seeded recipe the parity tests use
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        from gpu_harness import to_device
        for i in range(nmat):
            stream = synth.make_stream(w, i)
            st = synth.make_state(w, i)
            X.append(to_device(st.X, torch)); M.append(to_device(st.M, torch)); Q.append(to_device(st.Q, torch))
            Gpool.append([to_device(stream.gradient(t), torch) for t in range(args.pool)])
        data = "synthetic (seeded numpy recipe of the parity tests)"
    else:
        for i in range(nmat):
            x, mom, q = device_state(torch, w, i, dev)
            X.append(x); M.append(mom); Q.append(q)
            Gpool.append(device_gradients(torch, w, i, args.pool, dev))
        data = "synthetic (seeded, generated on device; Gaussian stand-ins for the singular-vector factors)"
    torch.cuda.synchronize()

    opt = binding.OrthDion(w.shapes, w.r, x_dtype=w.x_dtype, variant=args.variant, precision=args.precision,
                           mu=w.mu, lr=w.lr)
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    xs = [t.data_ptr() for t in X]; ms = [t.data_ptr() for t in M]; qs = [t.data_ptr() for t in Q]
    gs = [[Gpool[i][p].data_ptr() for i in range(nmat)] for p in range(args.pool)]
    wsp, wsb = opt.workspace.data_ptr(), opt.workspace_bytes

    def one_step(t):
        binding.orthdion_step(opt.handle, xs, gs[t % args.pool], ms, qs, wsp, wsb, sh)

    # ---------------- warmup, with all phases bracketed to find the dominant kernel
    nw = max(args.warmup, 1)
    one_step(0)
    torch.cuda.synchronize()
    binding.orthdion_profile_begin(opt.handle, (1 << binding.ORTHDION_NPHASE) - 1, nw)
    for t in range(nw):
        one_step(t)
    torch.cuda.synchronize()
    phases = binding.orthdion_profile_end(opt.handle)
    batches = max(c for _, c in phases.values()) // nw
    phase_ms = {k: v[0] / nw for k, v in phases.items()}          # per step, summed over batches
    kernel_phases = {k: phase_ms[k] for k in ("proj", "back", "efx")}
    dominant = max(kernel_phases, key=kernel_phases.get)
    info = opt.info()
    if any(info):
        print(f"bench.py: numerical breakdown flagged during warmup: {info}", file=sys.stderr)
        sys.exit(3)

    # A plain 1 GiB device copy (256 Mi floats read + 256 Mi written, four times the Infinity
    # Cache): the bandwidth this chip sustains for mixed traffic, reported beside the 8 TB/s peak;
    # with --calibrate-copy it is also the known-size kernel the HBM counters are scaled by.
    src = torch.ones(256 * 1024 * 1024, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(3):
        dst.copy_(src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbps = 3 * 2 * src.numel() * 4 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    del src, dst

    # ---------------- timed region: K steps, dominant kernel bracketed by HIP events
    K = args.steps
    binding.orthdion_profile_begin(opt.handle, 1 << binding.PHASES.index(dominant), K)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(K):
        one_step(t)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom = binding.orthdion_profile_end(opt.handle)[dominant]
    elapsed = t1 - t0
    ms_per_step = 1e3 * elapsed / K
    steps_per_s = K / elapsed
    info = opt.info()
    if any(info):
        print(f"bench.py: numerical breakdown flagged: {info}", file=sys.stderr)
        sys.exit(3)

    fast_path = args.precision == "fast" or (args.precision == "auto" and w.x_dtype == "bf16")
    dom_ms_per_step = dom[0] / K                   # all launches of the kernel in one step
    launches_per_step = dom[1] // K
    nbytes, flops = algorithmic_work(w, dominant)
    # which roofline binds the kernel: its arithmetic intensity against the ridge of the two peaks
    hbm_frac_k = nbytes / (dom_ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS
    mfma_frac_k = flops / (dom_ms_per_step * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS
    hbm_bound = flops / nbytes < MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    if hbm_bound:
        achieved = nbytes / (dom_ms_per_step * 1e-3) / 1e9
        peak, unit = HBM_PEAK_GBS, "GB/s"
    else:
        achieved = flops / (dom_ms_per_step * 1e-3) / 1e12
        peak, unit = MFMA_PEAK_TFLOPS, "TFLOP/s"
    traffic = MEASURED_TRAFFIC.get((w.name, dominant))
    step_bytes = sum(algorithmic_work(w, p)[0] for p in ("proj", "back", "efx"))
    step_flops = sum(algorithmic_work(w, p)[1] for p in ("proj", "back", "efx"))

    # counter-measured traffic of the three streaming kernels over the whole step, where profiled
    meas = [MEASURED_TRAFFIC.get((w.name, p)) for p in ("proj", "back", "efx")]
    step_measured = sum(meas) if all(meas) and args.variant == "qr" else None

    out = {
        "metric": "Orth-Dion optimizer steps/sec over model matrix set; achieved HBM GB/s vs peak",
        "value": steps_per_s, "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if (w.x_dtype == "bf16" and args.precision != "exact") else "bf16",
        "data": data,
        "config": {"workload": w.name, "matrices": nmat, "shapes": sorted({f"{m}x{n}" for m, n in w.shapes}),
                   "r": w.r, "x_g_dtype": w.x_dtype, "state_dtype": "f32", "variant": args.variant,
                   "ef": "dion", "mu": w.mu, "lr": w.lr, "precision": args.precision,
                   "elements": w.elements},
        "roofline": {"bound": "hbm" if hbm_bound else "mfma", "achieved": achieved, "peak": peak, "unit": unit,
                     "frac": achieved / peak, "traffic": traffic, "kernel": {"proj": "k_proj", "back": "k_back",
                                                                              "efx": "k_efx_h" if fast_path else "k_efx"}[dominant],
                     "kernel_ms_per_launch": dom_ms_per_step / max(launches_per_step, 1),
                     "launches_per_step": launches_per_step,
                     "algorithmic_bytes_per_step": nbytes, "algorithmic_flops_per_step": flops,
                     "hbm_frac": hbm_frac_k, "mfma_frac": mfma_frac_k,
                     "measured_GBps": (traffic / (dom_ms_per_step / max(launches_per_step, 1) * 1e-3) / 1e9) if traffic else None,
                     "copy_GBps": copy_gbps},
        "whole_step": {"algorithmic_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
                       "algorithmic_TFLOPs": step_flops / (ms_per_step * 1e-3) / 1e12,
                       "hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                       "mfma_frac": step_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
                       "hbm_frac_of_copy": step_bytes / (ms_per_step * 1e-3) / 1e9 / copy_gbps,
                       "measured_GBps": (step_measured / (ms_per_step * 1e-3) / 1e9) if step_measured else None,
                       "measured_hbm_frac": (step_measured / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS) if step_measured else None},
        "phase_ms_per_step_warmup": {k: round(v, 5) for k, v in phase_ms.items()},
        "batches": batches,
    }
    if not args.no_cpu_baseline:
        del Gpool
        out["cpu_baseline"] = cpu_baseline(w, args.variant, args.cpu_seconds)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
