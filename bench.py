#!/usr/bin/env python3
"""Benchmark of the Orth-Dion optimizer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--variant qr]

One "step" is one orthdion_step over the whole matrix set of the workload (all phases of
the method: buffer, projection, left orthogonalisation, back-projection, right
orthogonalisation or column normalisation, error feedback and parameter update).  Inputs
are synthetic, seeded, and resident in HBM before the timed region.  Prints ONE JSON line.

The headline workload is the model matrix set C3 (96 matrices of a 1.3B-style decoder,
r = 512).  The same line carries `sweep`: a few timed steps of C2, C4 and the rank sweep C5
(r = 16, 256, 1024, 2048), because the target is split by rank (HBM roofline up to r = 256,
matrix-core roofline from r = 1024).
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0      # MI355X dense fp16 / bf16 matrix cores, published
METRIC = "Orth-Dion optimizer steps/sec over model matrix set; achieved HBM GB/s vs peak"
SWEEP = [("C2", 30), ("C4", 10), ("C5-r16", 30), ("C5-r256", 20), ("C5-r1024", 10), ("C5-r2048", 6)]

# Kernel groups: the phases orthdion_profile_begin can bracket, gathered by the kernel that
# does their work, and the name prefixes of those kernels in a rocprofv3 counter summary.
GROUPS = {
    "k_proj": (["proj"], ["od::k_proj<", "od::k_stream_d<false"]),
    "k_back": (["back"], ["od::k_back<", "od::k_stream_d<true"]),
    "k_efx": (["efx"], ["od::k_efx_d<", "od::k_efx_h<", "od::k_efx<"]),
    "k_gram (first pass)": (["gram_left", "gram_right"], []),
    "cholesky chain (k_chol256, k_chol_ahead, k_sgemm_pair)": (["chol_left", "chol_right"], ["od::k_chol256", "od::k_chol_ahead", "od::k_sgemm", "od::k_zero_pair"]),
    "rest of orth (k_apply, k_gram, k_corr | ColNorm)": (["orth_left", "orth_right", "guard_left", "guard_right", "finish_left", "finish_right"],
                                                         ["od::k_apply<", "od::k_corr", "od::k_colsq", "od::k_colnorm"]),
    "k_reduce": (["proj_reduce", "back_reduce"], ["od::k_reduce"]),
    "k_prologue": (["stats"], ["od::k_prologue<"]),
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--variant", default="qr", choices=["qr", "colnorm"])
    ap.add_argument("--precision", default="auto", choices=["auto", "fast", "exact"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true")
    ap.add_argument("--groups", type=int, default=0, choices=[0, 1, 2], help="0: the library chooses")
    ap.add_argument("--pool", type=int, default=4, help="distinct gradients per matrix cycled through")
    return ap.parse_args()


def group_work(w, variant, group):
    """Algorithmic HBM bytes and flops per step of a kernel group, summed over the matrix set.
    Matrix traffic follows the 20 B/element floor for bf16 storage (28 for fp32): M and G are
    read by the projection and again by the back-projection (a grid-wide dependency separates
    them), M is written once and X read and written once (both booked on the fused
    error-feedback / update kernel); factor traffic is added per kernel.  Orthogonalisation:
    a Gram matrix costs rows r^2 flops (symmetric half), a triangular product rows r^2, the
    Cholesky factor and its inverse r^3 / 3 each."""
    e = 2 if w.x_dtype == "bf16" else 4
    r = w.r
    nbytes = flops = 0
    for m, n in w.shapes:
        mn = m * n
        sides = [m, n] if variant == "qr" else [m]
        if group in ("k_proj", "k_back"):
            nbytes += mn * (4 + e) + 4 * r * (n + m)
            flops += 2 * mn * r
        elif group == "k_efx":
            nbytes += mn * (4 + 2 * e) + 4 * r * (m + 2 * n)
            flops += 4 * mn * r
        elif group.startswith("k_gram"):
            for rows in sides:
                nbytes += 4 * rows * r + 4 * r * r
                flops += rows * r * r
        elif group.startswith("cholesky"):
            for _ in sides:
                nbytes += 3 * 4 * r * r
                flops += 2 * r * r * r // 3
        elif group.startswith("rest of orth"):
            for rows in sides:
                nbytes += 5 * 4 * rows * r
                flops += 3 * rows * r * r
            if variant != "qr":
                nbytes += 3 * 4 * n * r
        elif group == "k_reduce":
            nbytes += 2 * 4 * r * (m + n)
    return nbytes, flops


def step_work(w, variant):
    """Whole-step algorithmic bytes (the 20 / 28 B/element floor plus factor traffic) and
    flops: 8 m n r for the four contractions, and with the orthogonalisations counted
    (CholeskyQR2: 6 rows r^2 per side)."""
    nbytes = sum(group_work(w, variant, g)[0] for g in ("k_proj", "k_back", "k_efx"))
    flops = sum(group_work(w, variant, g)[1] for g in ("k_proj", "k_back", "k_efx"))
    qr = 0
    for m, n in w.shapes:
        qr += 6 * (m + (n if variant == "qr" else 0)) * w.r * w.r
    return nbytes, flops, flops + qr


def measured_traffic(workload, variant, prefixes):
    """HBM bytes per launch of the kernels whose names start with one of `prefixes`, from the
    committed rocprofv3 counter summary of this workload (FETCH_SIZE and WRITE_SIZE, each
    scaled by a copy kernel of known size); None when there is no summary.  Lines:
    kernel, dispatches, FETCH KiB, WRITE KiB, scaled bytes per launch."""
    if variant != "qr" or not prefixes:
        return None
    path = os.path.join(ROOT, "profiles", f"orthdion_step_{workload}_hbm_counters.txt")
    if not os.path.exists(path):
        return None
    total = launches = 0.0
    with open(path) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            cols = [c.strip() for c in line.rsplit(",", 4)]
            if len(cols) != 5:
                continue
            name = cols[0].replace("void ", "")
            if any(name.startswith(p) for p in prefixes):
                total += float(cols[4]) * float(cols[1])
                launches += float(cols[1])
    return total / launches if launches else None


def cpu_baseline(w, variant):
    """The fp64 oracle, as it stands, timed on the host cores: one step per distinct shape of
    the workload, weighted by how often the shape occurs, summed to the time of one step
    over the whole set."""
    import numpy as np
    from oracle.orthdion_oracle import OrthDionOracle
    from paper_2605_16341_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    first, count = {}, {}
    for i, shape in enumerate(w.shapes):
        first.setdefault(shape, i)
        count[shape] = count.get(shape, 0) + 1
    orc = OrthDionOracle(mu=w.mu, lr=w.lr, variant=variant, ef="dion", x_bf16=(w.x_dtype == "bf16"))
    per_set, timed, parts = 0.0, 0.0, []
    for shape, i in first.items():
        stream = synth.make_stream(w, i, orthonormal=False) if w.spectrum == "power_law" else synth.make_stream(w, i)
        st = synth.make_state(w, i)
        g = stream.gradient(0)
        t0 = time.perf_counter()
        orc.step(st.X, g, st.M.astype(np.float64), st.Q.astype(np.float64))
        el = time.perf_counter() - t0
        timed += el
        per_set += el * count[shape]
        parts.append(f"{shape[0]}x{shape[1]} ({count[shape]}x): {el:.1f} s")
        del stream, st, g
    return {"value": 1.0 / per_set, "unit": "steps/s", "cores": int(threads), "kind": "oracle",
            "sample": f"one oracle step per distinct shape of {w.name} (r={w.r}), {timed:.1f} s of CPU time, each weighted by "
                      f"its multiplicity: " + "; ".join(parts)}


def measure(torch, binding, synth, dev, name, variant, precision, steps, warmup, pool, groups=0):
    """Times `steps` steps of one workload; returns the fields of its bench record."""
    from paper_2605_16341_amd.device_inputs import device_gradients, device_state, to_device
    w = synth.WORKLOADS[name]
    nmat = len(w.shapes)
    X, M, Q, Gpool = [], [], [], []
    if w.name in ("C1", "C2"):
        # the exact seeded recipe the parity tests use
        for i in range(nmat):
            stream = synth.make_stream(w, i)
            st = synth.make_state(w, i)
            X.append(to_device(st.X, torch)); M.append(to_device(st.M, torch)); Q.append(to_device(st.Q, torch))
            Gpool.append([to_device(stream.gradient(t), torch) for t in range(pool)])
        data = "synthetic (seeded numpy recipe of the parity tests)"
    else:
        for i in range(nmat):
            x, mom, q = device_state(torch, w, i, dev)
            X.append(x); M.append(mom); Q.append(q)
            Gpool.append(device_gradients(torch, w, i, pool, dev))
        data = "synthetic (seeded, generated on device; Gaussian stand-ins for the singular-vector factors)"
    torch.cuda.synchronize()

    opt = binding.OrthDion(w.shapes, w.r, x_dtype=w.x_dtype, variant=variant, precision=precision, mu=w.mu, lr=w.lr, groups=groups)
    sh = torch.cuda.current_stream().cuda_stream
    xs = [t.data_ptr() for t in X]; ms = [t.data_ptr() for t in M]; qs = [t.data_ptr() for t in Q]
    gs = [[Gpool[i][p].data_ptr() for i in range(nmat)] for p in range(pool)]
    wsp, wsb = opt.workspace.data_ptr(), opt.workspace_bytes

    def one_step(t):
        binding.orthdion_step(opt.handle, xs, gs[t % pool], ms, qs, wsp, wsb, sh)

    # ---- warm-up with every phase bracketed: the kernel group that takes the most time
    nw = max(warmup, 1)
    one_step(0)
    torch.cuda.synchronize()
    binding.orthdion_profile_begin(opt.handle, (1 << binding.ORTHDION_NPHASE) - 1, nw)
    for t in range(nw):
        one_step(t)
    torch.cuda.synchronize()
    phases = binding.orthdion_profile_end(opt.handle)
    phase_ms = {k: v[0] / nw for k, v in phases.items()}          # per step, summed over batches
    group_ms = {g: sum(phase_ms.get(p, 0.0) for p in ph) for g, (ph, _) in GROUPS.items()}
    dominant = max(group_ms, key=group_ms.get)
    info = opt.info()
    if any(info):
        raise RuntimeError(f"numerical breakdown flagged during warm-up of {name}: {info}")

    # ---- timed region: K steps; only the dominant group's phases carry events
    mask = 0
    for p in GROUPS[dominant][0]:
        mask |= 1 << binding.PHASES.index(p)
    binding.orthdion_profile_begin(opt.handle, mask, steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(steps):
        one_step(t)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = binding.orthdion_profile_end(opt.handle)
    info = opt.info()
    if any(info):
        raise RuntimeError(f"numerical breakdown flagged in {name}: {info}")
    elapsed = t1 - t0
    ms_per_step = 1e3 * elapsed / steps
    # the same number of steps once more without any event on the stream: every recorded event
    # is a barrier packet between two kernels, which a step of a few hundred microseconds feels
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for t in range(steps):
        one_step(t)
    torch.cuda.synchronize()
    ms_per_step_plain = 1e3 * (time.perf_counter() - t2) / steps
    dom_ms = sum(prof[p][0] for p in GROUPS[dominant][0] if p in prof) / steps      # per step
    dom_launches = sum(prof[p][1] for p in GROUPS[dominant][0] if p in prof) // steps

    fast_path = precision == "fast" or (precision == "auto" and w.x_dtype == "bf16")
    # the kernel the library's launchers pick for this group (same rules as od_kernels.hip)
    kname = dominant
    if fast_path and dominant == "k_efx":
        kname = "k_efx_d" if (w.r % 32 == 0 and w.r >= 64) else "k_efx_h"
    if fast_path and dominant in ("k_proj", "k_back") and w.x_dtype == "bf16" and w.r >= 192:
        kname = "k_stream_d<%s>" % ("false" if dominant == "k_proj" else "true")
    nbytes, flops = group_work(w, variant, dominant)
    hbm_frac_k = nbytes / (dom_ms * 1e-3) / 1e9 / HBM_PEAK_GBS
    mfma_frac_k = flops / (dom_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS
    # which roofline binds the kernel: its arithmetic intensity against the ridge of the two peaks
    hbm_bound = flops / max(nbytes, 1) < MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    traffic = measured_traffic(w.name, variant, GROUPS[dominant][1])
    per_launch_ms = dom_ms / max(dom_launches, 1)
    step_bytes, step_flops, step_flops_qr = step_work(w, variant)
    rec = {
        "workload": w.name, "groups_used": opt.groups, "variant": variant, "steps": steps, "ms_per_step": ms_per_step, "steps_per_s": steps / elapsed,
        "ms_per_step_without_events": ms_per_step_plain,
        "data": data, "nmat": nmat, "r": w.r, "elements": w.elements, "x_dtype": w.x_dtype, "mu": w.mu, "lr": w.lr,
        "shapes": sorted({f"{m}x{n}" for m, n in w.shapes}), "fast_path": fast_path,
        "roofline": {
            "bound": "hbm" if hbm_bound else "mfma",
            "achieved": (nbytes / (dom_ms * 1e-3) / 1e9) if hbm_bound else (flops / (dom_ms * 1e-3) / 1e12),
            "peak": HBM_PEAK_GBS if hbm_bound else MFMA_PEAK_TFLOPS, "unit": "GB/s" if hbm_bound else "TFLOP/s",
            "frac": hbm_frac_k if hbm_bound else mfma_frac_k,
            "traffic": traffic, "kernel": kname, "kernel_ms_per_launch": per_launch_ms, "launches_per_step": dom_launches,
            "kernel_ms_per_step": dom_ms, "share_of_step": dom_ms / ms_per_step,
            "algorithmic_bytes_per_launch": nbytes / max(dom_launches, 1),
            "algorithmic_flops_per_launch": flops / max(dom_launches, 1),
            "hbm_frac": hbm_frac_k, "mfma_frac": mfma_frac_k,
            "measured_GBps": (traffic / (per_launch_ms * 1e-3) / 1e9) if traffic else None},
        "whole_step": {
            "algorithmic_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
            "algorithmic_TFLOPs": step_flops / (ms_per_step * 1e-3) / 1e12,
            "hbm_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "mfma_frac": step_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
            "mfma_frac_with_qr_flops": step_flops_qr / (ms_per_step * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS},
        "kernel_group_ms_per_step_warmup": {k: round(v, 5) for k, v in group_ms.items()},
        "phase_ms_per_step_warmup": {k: round(v, 5) for k, v in phase_ms.items()},
    }
    opt.close()
    del X, M, Q, Gpool, opt
    torch.cuda.empty_cache()
    return rec


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported. Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_16341_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    binding.load()
    dev = torch.device("cuda:0")
    try:
        head = measure(torch, binding, synth, dev, args.workload, args.variant, args.precision, args.steps, args.warmup, args.pool, args.groups)
    except RuntimeError as exc:
        print(f"bench.py: {exc}", file=sys.stderr)
        sys.exit(3)

    # a plain 1 GiB device copy (four times the Infinity Cache): what this chip sustains for
    # mixed read / write traffic, beside the 8 TB/s peak; also the known-size kernel that a
    # counter run of this command is scaled by
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
    torch.cuda.empty_cache()

    head["roofline"]["copy_GBps"] = copy_gbps
    head["whole_step"]["hbm_frac_of_copy"] = head["whole_step"]["algorithmic_GBps"] / copy_gbps
    out = {
        "metric": METRIC, "value": head["steps_per_s"], "unit": "steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "ms_per_step_without_events": head["ms_per_step_without_events"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16" if head["fast_path"] else "bf16",
        "data": head["data"],
        "config": {"workload": head["workload"], "matrices": head["nmat"], "shapes": head["shapes"], "r": head["r"],
                   "x_g_dtype": head["x_dtype"], "state_dtype": "f32", "variant": args.variant, "ef": "dion",
                   "mu": head["mu"], "lr": head["lr"], "precision": args.precision, "groups": head["groups_used"], "elements": head["elements"]},
        "roofline": head["roofline"], "whole_step": head["whole_step"],
        "kernel_group_ms_per_step_warmup": head["kernel_group_ms_per_step_warmup"],
        "phase_ms_per_step_warmup": head["phase_ms_per_step_warmup"],
    }
    if not args.no_sweep:
        sweep = []
        for name, k in SWEEP:
            if name == args.workload:
                continue
            try:
                rec = measure(torch, binding, synth, dev, name, args.variant, args.precision, k, 2, 2, args.groups)
            except RuntimeError as exc:
                sweep.append({"workload": name, "error": str(exc)})
                continue
            rf, ws = rec["roofline"], rec["whole_step"]
            sweep.append({"workload": name, "r": rec["r"], "groups": rec["groups_used"], "steps": k, "ms_per_step": rec["ms_per_step"],
                          "ms_per_step_without_events": rec["ms_per_step_without_events"],
                          "steps_per_s": rec["steps_per_s"], "dominant_kernel": rf["kernel"], "bound": rf["bound"],
                          "kernel_frac": rf["frac"], "kernel_hbm_frac": rf["hbm_frac"], "kernel_mfma_frac": rf["mfma_frac"],
                          "kernel_share_of_step": rf["share_of_step"], "traffic": rf["traffic"],
                          "whole_step_hbm_frac": ws["hbm_frac"], "whole_step_mfma_frac": ws["mfma_frac"],
                          "whole_step_mfma_frac_with_qr_flops": ws["mfma_frac_with_qr_flops"]})
        out["sweep"] = sweep
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(synth.WORKLOADS[args.workload], args.variant)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
