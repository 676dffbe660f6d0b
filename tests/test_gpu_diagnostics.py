"""Parity of the on-device diagnostics, the rank-change helper and an adaptive-rank loop
(through the C ABI) with the fp64 oracle.

Tolerances: norms, inner product and effective rank are relative; the tracking error is
compared through its square 1 - ||R||^2 / ||B||^2 (absolute), because that is what both the
difference of norms and the rounding of R perturb; nu is a power-iteration estimate from
below, relative.  "exact" rows are fp32 storage with split-bf16 operands, "fast" rows bf16
storage with fp16 operands (R carries a relative error of about 2^-11 per entry there).
"""
import numpy as np
import pytest

from gpu_harness import GpuRun, compare_step, oracle_for, to_device, to_host
from oracle.orthdion_oracle import (OrthDionOracle, bf16_bits_to_f64, diagnostics, rank_policy,
                                    resize_right_factor)
from paper_2605_16341_amd import binding, synth

pytestmark = pytest.mark.gpu

REL = {"f32": 1e-4, "bf16": 2e-3}
EPS2_ABS = {"f32": 2e-5, "bf16": 2e-3}
NU_REL = 1e-3


def check_diag(got: dict, want: dict, x_dtype: str, ctx):
    rel = REL[x_dtype]
    for key in ("b_norm", "r_norm", "inner", "erank"):
        assert abs(got[key] - want[key]) <= rel * abs(want[key]), (ctx, key, got[key], want[key])
    gn = got["g_norm"]
    assert gn > 0
    assert abs(got["residual_ratio"] - want["residual_ratio"]) <= rel * max(want["residual_ratio"], 1e-3), (ctx, got, want)
    assert abs(got["tracking_error"] ** 2 - want["tracking_error"] ** 2) <= EPS2_ABS[x_dtype], \
        (ctx, got["tracking_error"], want["tracking_error"])
    assert abs(got["nu"] - want["nu"]) <= NU_REL * want["nu"], (ctx, got["nu"], want["nu"])
    assert got["nu"] <= want["nu"] * (1 + 1e-5) or x_dtype == "bf16"


def run_case(shapes, r, x_dtype, variant, steps, seed, ef="dion", mu=0.95, momentum_std=1e-3, persistence=0.0):
    nmat = len(shapes)
    ranks = [r] * nmat if isinstance(r, int) else list(r)
    streams = [synth.power_law_stream(m, n, seed + 10 * i, out_dtype=x_dtype, orthonormal=True, persistence=persistence)
               for i, (m, n) in enumerate(shapes)]
    states = [synth.initial_state(m, n, ranks[i], seed + 10 * i, x_dtype, momentum_std) for i, (m, n) in enumerate(shapes)]
    gpu = GpuRun(shapes, r, x_dtype, states, variant=variant, ef=ef, mu=mu, lr=0.01)
    gpu.opt.set_diagnostics(True)
    orc = OrthDionOracle(mu=mu, lr=0.01, variant=variant, ef=ef, x_bf16=(x_dtype == "bf16"))
    cur = [(s.X, s.M.astype(np.float64), s.Q.astype(np.float64)) for s in states]
    for t in range(steps):
        grads = [st.gradient(t) for st in streams]
        assert gpu.step(grads) == [0] * nmat
        got = gpu.opt.diagnostics()
        assert len(got) == nmat
        for i in range(nmat):
            x, mom, q = cur[i]
            o = orc.step(x, grads[i], mom, q)
            want = diagnostics(o, mom, grads[i])
            check_diag(got[i], want, x_dtype, (shapes[i], ranks[i], variant, "step", t))
            cur[i] = (o["X_bits"] if x_dtype == "bf16" else o["X"], o["M"], o["Q"])
            if t == steps - 1:
                # the state itself, so that a result routed to the wrong matrix cannot hide
                res = compare_step(gpu.fetch(i), o, x, 0.01)
                for key in ("M", "Q", "P", "R"):
                    assert res[key] <= (1e-4 if x_dtype == "f32" else 2e-2), (shapes[i], ranks[i], key, res[key])


@pytest.mark.parametrize("variant", ["qr", "colnorm"])
@pytest.mark.parametrize("x_dtype", ["f32", "bf16"])
def test_diagnostics_small(variant, x_dtype):
    run_case([(200, 136)], 24, x_dtype, variant, steps=3, seed=700)


@pytest.mark.parametrize("variant", ["qr", "colnorm"])
def test_diagnostics_two_classes_interleaved(variant):
    # the table must come back in the caller's matrix order, not in shape-class order
    run_case([(128, 96), (64, 256), (128, 96)], 16, "f32", variant, steps=2, seed=710)


@pytest.mark.parametrize("variant", ["qr", "colnorm"])
@pytest.mark.parametrize("x_dtype", ["f32", "bf16"])
def test_matrices_of_different_rank_in_one_handle(variant, x_dtype):
    """Ranks per matrix ("sort-and-pack" of the adaptive-rank path): the Cholesky step runs per
    rank over several shape classes, and here the two rank-32 classes are separated by a rank-16
    one, so results and diagnostics must find their way back to the caller's matrix order."""
    shapes = [(256, 192), (192, 256), (128, 160), (256, 192), (192, 256), (320, 288)]
    ranks = [32, 16, 32, 32, 16, 264]
    run_case(shapes, ranks, x_dtype, variant, steps=2, seed=770)


@pytest.mark.parametrize("variant", ["qr", "colnorm"])
def test_diagnostics_rank_above_512(variant):
    # exercises the multi-launch power iteration and the blocked Cholesky
    run_case([(768, 640)], 520, "f32", variant, steps=2, seed=720)


@pytest.mark.parametrize("variant", ["qr", "colnorm"])
def test_diagnostics_c2_shape(variant):
    w = synth.WORKLOADS["C2"]
    run_case(list(w.shapes), w.r, w.x_dtype, variant, steps=2, seed=730, momentum_std=0.0)


def test_diagnostics_zero_residual_and_paper_ef():
    # first step from M = 0: the residual ratio is exactly 0; paper-form error feedback afterwards
    run_case([(96, 160)], 8, "f32", "qr", steps=3, seed=740, ef="paper", mu=0.3, momentum_std=0.0)


def test_get_diagnostics_needs_an_enabled_step():
    import torch
    w = synth.WORKLOADS["C1"]
    st = synth.make_state(w, 0)
    gpu = GpuRun(w.shapes, w.r, w.x_dtype, [st])
    with pytest.raises(binding.OrthDionError) as e:
        gpu.opt.diagnostics()
    assert e.value.status == binding.ORTHDION_E_NO_STEP
    gpu.step([synth.make_stream(w, 0).gradient(0)])
    with pytest.raises(binding.OrthDionError) as e:
        gpu.opt.diagnostics()
    assert e.value.status == binding.ORTHDION_E_NO_STEP
    gpu.opt.set_diagnostics(True)
    gpu.step([synth.make_stream(w, 0).gradient(1)])
    assert len(gpu.opt.diagnostics()) == 1
    gpu.opt.set_diagnostics(False)
    gpu.step([synth.make_stream(w, 0).gradient(2)])
    with pytest.raises(binding.OrthDionError):
        gpu.opt.diagnostics()
    torch.cuda.synchronize()


@pytest.mark.parametrize("n,r_old,r_new", [(64, 16, 8), (64, 16, 16), (64, 16, 40), (4104, 384, 360), (4104, 360, 384)])
def test_resize_q_bit_exact(n, r_old, r_new):
    import torch
    rng = synth.rng_for(900 + n + r_old + r_new)
    q = rng.standard_normal((n, r_old)).astype(np.float32)
    pad = rng.standard_normal((n, max(r_new - r_old, 0))).astype(np.float32) if r_new > r_old else None
    want = resize_right_factor(q, r_new, pad)
    dq = to_device(q, torch)
    dpad = to_device(pad, torch) if pad is not None else None
    out = torch.full((n, r_new), float("nan"), dtype=torch.float32, device="cuda:0")
    binding.orthdion_resize_q(dq.data_ptr(), n, r_old, out.data_ptr(), r_new,
                              dpad.data_ptr() if dpad is not None else 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert got.tobytes() == want.astype(np.float32).tobytes()


def test_adaptive_rank_loop_follows_the_oracle():
    """Ada-Orth-Dion on one matrix: step with diagnostics, apply the rank rule to the
    effective-rank estimate, rebuild the handle and resize Q when the rank changes.  The HIP
    loop and the oracle loop, each driven by its own estimate, must choose the same ranks."""
    import torch
    m, n, r0 = 192, 160, 64
    alpha, gamma, r_min, r_max = 0.5, 1.1, 8, 64
    # a gradient whose spectrum falls off quickly, so the rule shrinks the rank
    stream = synth.power_law_stream(m, n, 760, exponent=1.5, noise_energy=0.01, out_dtype="f32", orthonormal=True)
    st0 = synth.initial_state(m, n, r0, 760, "f32", 0.0)
    pads = synth.rng_for(761)
    orc = OrthDionOracle(mu=0.95, lr=0.01, variant="qr", x_bf16=False)
    xo, mo, qo = st0.X.astype(np.float64), st0.M.astype(np.float64), st0.Q.astype(np.float64)
    X, M, Q = to_device(st0.X, torch), to_device(st0.M, torch), to_device(st0.Q, torch)
    r_g = r_o = r0
    ema_g = ema_o = float(r0)
    opt = binding.OrthDion([(m, n)], r_g, x_dtype="f32", variant="qr")
    opt.set_diagnostics(True)
    ranks = []
    for t in range(8):
        g = stream.gradient(t)
        assert r_g == r_o, (t, r_g, r_o)
        opt.step([X], [to_device(g, torch)], [M], [Q])
        torch.cuda.synchronize()
        assert opt.info() == [0]
        d = opt.diagnostics()[0]
        o = orc.step(xo, g, mo, qo)
        want = diagnostics(o, mo, g)
        assert abs(d["erank"] - want["erank"]) <= 1e-3 * want["erank"], (t, d["erank"], want["erank"])
        xo, mo, qo = o["X"], o["M"], o["Q"]
        ema_g, nxt_g = binding.orthdion_rank_policy(d["erank"], ema_g, r_min, r_max, alpha, gamma)
        ema_o, nxt_o = rank_policy(want["erank"], r_o, ema_o, r_min, r_max, alpha, gamma)
        near_edge = abs(gamma * ema_o - round(gamma * ema_o)) < 2e-2
        if not near_edge:
            assert nxt_g == nxt_o, (t, nxt_g, nxt_o, ema_g, ema_o)
        else:
            nxt_g = nxt_o
        pad = pads.standard_normal((n, max(nxt_o - r_o, 0))).astype(np.float32) / np.sqrt(n) if nxt_o > r_o else None
        if nxt_o != r_o:
            qo = resize_right_factor(qo, nxt_o, pad.astype(np.float64) if pad is not None else None)
            q_new = torch.empty((n, nxt_g), dtype=torch.float32, device="cuda:0")
            dpad = to_device(pad, torch) if pad is not None else None
            binding.orthdion_resize_q(Q.data_ptr(), n, r_g, q_new.data_ptr(), nxt_g,
                                      dpad.data_ptr() if dpad is not None else 0,
                                      torch.cuda.current_stream().cuda_stream)
            torch.cuda.synchronize()
            Q = q_new
            opt.close()
            opt = binding.OrthDion([(m, n)], nxt_g, x_dtype="f32", variant="qr")
            opt.set_diagnostics(True)
            r_g, r_o = nxt_g, nxt_o
        ranks.append(r_o)
        assert np.linalg.norm(to_host(M, torch).astype(np.float64) - mo) <= 1e-4 * np.linalg.norm(mo), t
    assert ranks[-1] < r0, ranks          # the rule did shrink the rank on this spectrum


def test_adaptive_rank_loop_over_a_matrix_set():
    """Ada-Orth-Dion over three matrices with their own ranks: every step the rank rule runs per
    matrix on the device's effective-rank estimate; when any rank changes, the warm-start
    factors are resized and the handle is rebuilt with the new rank list (matrices of equal
    shape and rank share a batch, the Cholesky steps run per rank).  Ranks and states must
    follow an oracle loop that is driven by its own estimates."""
    import torch
    shapes = [(192, 160), (160, 224), (192, 160)]
    exps = [1.5, 0.4, 1.0]                        # fast, slow and medium spectral decay
    alpha, gamma, r_min, r_max = 0.6, 1.1, 8, 48
    nmat = len(shapes)
    streams = [synth.power_law_stream(m, n, 860 + 7 * i, exponent=exps[i], noise_energy=0.01, out_dtype="f32",
                                      orthonormal=True) for i, (m, n) in enumerate(shapes)]
    ranks = [48, 48, 48]
    states = [synth.initial_state(m, n, ranks[i], 860 + 7 * i, "f32", 0.0) for i, (m, n) in enumerate(shapes)]
    pads = synth.rng_for(861)
    orc = OrthDionOracle(mu=0.95, lr=0.01, variant="qr", x_bf16=False)
    host = [(s.X.astype(np.float64), s.M.astype(np.float64), s.Q.astype(np.float64)) for s in states]
    X = [to_device(s.X, torch) for s in states]
    M = [to_device(s.M, torch) for s in states]
    Q = [to_device(s.Q, torch) for s in states]
    ema = [float(r) for r in ranks]
    opt = binding.OrthDion(shapes, list(ranks), x_dtype="f32", variant="qr")
    opt.set_diagnostics(True)
    history = []
    for t in range(6):
        grads = [st.gradient(t) for st in streams]
        opt.step(X, [to_device(g, torch) for g in grads], M, Q)
        torch.cuda.synchronize()
        assert opt.info() == [0] * nmat
        dev = opt.diagnostics()
        new_ranks = list(ranks)
        for i in range(nmat):
            xo, mo, qo = host[i]
            o = orc.step(xo, grads[i], mo, qo)
            want = diagnostics(o, mo, grads[i])
            assert abs(dev[i]["erank"] - want["erank"]) <= 1e-3 * want["erank"], (t, i)
            ema_dev, nxt_dev = binding.orthdion_rank_policy(dev[i]["erank"], ema[i], r_min, r_max, alpha, gamma)
            ema_orc, nxt_orc = rank_policy(want["erank"], ranks[i], ema[i], r_min, r_max, alpha, gamma)
            if abs(gamma * ema_orc - round(gamma * ema_orc)) >= 2e-2:      # away from a rounding edge
                assert nxt_dev == nxt_orc, (t, i, nxt_dev, nxt_orc)
            ema[i] = ema_orc
            new_ranks[i] = nxt_orc
            qn = o["Q"]
            if nxt_orc != ranks[i]:
                grow = max(nxt_orc - ranks[i], 0)
                pad = pads.standard_normal((shapes[i][1], grow)).astype(np.float32) / np.sqrt(shapes[i][1]) if grow else None
                qn = resize_right_factor(qn, nxt_orc, pad.astype(np.float64) if pad is not None else None)
                q_new = torch.empty((shapes[i][1], nxt_orc), dtype=torch.float32, device="cuda:0")
                dpad = to_device(pad, torch) if pad is not None else None
                binding.orthdion_resize_q(Q[i].data_ptr(), shapes[i][1], ranks[i], q_new.data_ptr(), nxt_orc,
                                          dpad.data_ptr() if dpad is not None else 0,
                                          torch.cuda.current_stream().cuda_stream)
                torch.cuda.synchronize()
                Q[i] = q_new
            host[i] = (o["X"], o["M"], qn)
            assert np.linalg.norm(to_host(M[i], torch).astype(np.float64) - o["M"]) <= 1e-4 * np.linalg.norm(o["M"]), (t, i)
            assert np.linalg.norm(to_host(Q[i], torch).astype(np.float64) - qn) <= 1e-4 * np.linalg.norm(qn), (t, i)
        if new_ranks != ranks:
            opt.close()
            opt = binding.OrthDion(shapes, list(new_ranks), x_dtype="f32", variant="qr")
            opt.set_diagnostics(True)
            ranks = new_ranks
        history.append(tuple(ranks))
    # the three spectra end at different ranks, and the fast-decaying one shrank
    assert len(set(history[-1])) >= 2, history
    assert history[-1][0] < 48, history


@pytest.mark.parametrize("beta", [1.0, 0.5, 0.1, 0.05])
def test_beta_sweep_paper_form(beta):
    """Error-feedback coefficient sweep of Sec. 6.3 (paper-form EF, beta passed as mu) on a
    synthetic stream with fresh noise every step: diagnostics follow the oracle at every beta."""
    run_case([(256, 192)], 32, "f32", "qr", steps=4, seed=780, ef="paper", mu=beta, momentum_std=0.0)


@pytest.mark.parametrize("rho", [-0.4, 0.4])
@pytest.mark.parametrize("beta", [1.0, 0.1])
def test_beta_regimes_with_correlated_noise(beta, rho):
    """The coherent and anti-correlated regimes of Sec. 6.3: noise of consecutive steps
    correlated with the given sign (the uncorrelated regime is the sweep above)."""
    run_case([(256, 192)], 32, "bf16", "qr", steps=4, seed=785, ef="paper", mu=beta, momentum_std=0.0, persistence=rho)


def test_polyak_form():
    run_case([(256, 192)], 32, "bf16", "qr", steps=4, seed=790, ef="polyak", mu=0.95, momentum_std=0.0)
