"""Pins for the fp64 oracle: what the paper and the mathematics fix, independent of the
oracle's own code.  CPU only.

Each ``pin_*`` function takes a factory ``make(**kw) -> oracle`` and raises
AssertionError when the oracle it builds violates the pinned fact.  The real oracle must
pass all of them; each planted mistake (``MUTANTS``) must fail at least one.
"""
import math
import os

import numpy as np
import pytest

from oracle.orthdion_oracle import (OrthDionOracle, bf16_bits_to_f64, col_norm,
                                    f64_to_bf16_bits, rel_fro, thin_qr_library, thin_qr_positive)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- independent helpers

def jacobi_svd(a, sweeps=60):
    """Brute-force SVD by one-sided Jacobi rotations (tiny matrices only)."""
    a = np.array(a, dtype=np.float64)
    m, n = a.shape
    u = a.copy()
    v = np.eye(n)
    for _ in range(sweeps):
        off = 0.0
        for p in range(n - 1):
            for q in range(p + 1, n):
                alpha = float(u[:, p] @ u[:, p])
                beta = float(u[:, q] @ u[:, q])
                gamma = float(u[:, p] @ u[:, q])
                if gamma == 0.0:
                    continue
                off = max(off, abs(gamma) / math.sqrt(alpha * beta + 1e-300))
                zeta = (beta - alpha) / (2.0 * gamma)
                t = math.copysign(1.0, zeta) / (abs(zeta) + math.sqrt(1.0 + zeta * zeta))
                c = 1.0 / math.sqrt(1.0 + t * t)
                s = c * t
                up, uq = u[:, p].copy(), u[:, q].copy()
                u[:, p], u[:, q] = c * up - s * uq, s * up + c * uq
                vp, vq = v[:, p].copy(), v[:, q].copy()
                v[:, p], v[:, q] = c * vp - s * vq, s * vp + c * vq
        if off < 1e-15:
            break
    sig = np.sqrt(np.sum(u * u, axis=0))
    order = np.argsort(-sig)
    sig, u, v = sig[order], u[:, order], v[:, order]
    left = u / np.where(sig > 0, sig, 1.0)[None, :]
    return left, sig, v


def gram_schmidt_loops(a):
    """Thin QR by classical Gram-Schmidt in pure Python loops; positive diagonal by
    construction.  A different algorithm from the oracle's Householder QR; for full
    column rank both must give the same unique factor."""
    rows, cols = len(a), len(a[0])
    q = [[0.0] * cols for _ in range(rows)]
    t = [[0.0] * cols for _ in range(cols)]
    for j in range(cols):
        v = [a[i][j] for i in range(rows)]
        for _ in range(2):  # re-orthogonalise once for accuracy
            for k in range(j):
                dot = sum(q[i][k] * v[i] for i in range(rows))
                t[k][j] += dot
                for i in range(rows):
                    v[i] -= dot * q[i][k]
        nrm = math.sqrt(sum(x * x for x in v))
        t[j][j] = nrm
        for i in range(rows):
            q[i][j] = v[i] / nrm
    return q, t


def brute_step(x, g, m_prev, q_prev, lr, mu, variant, ef):
    """Alg. 1 in pure Python loops on lists (tiny inputs).  Written from the paper,
    not from the oracle: explicit index loops, Gram-Schmidt instead of Householder."""
    rows, cols, r = len(g), len(g[0]), len(q_prev[0])
    b = [[m_prev[i][j] + g[i][j] for j in range(cols)] for i in range(rows)]
    p_raw = [[sum(b[i][k] * q_prev[k][c] for k in range(cols)) for c in range(r)] for i in range(rows)]
    p, _ = gram_schmidt_loops(p_raw)
    rr = [[sum(b[i][j] * p[i][c] for i in range(rows)) for c in range(r)] for j in range(cols)]
    if variant == "qr":
        q, _ = gram_schmidt_loops(rr)
    else:
        lens = [math.sqrt(sum(rr[j][c] ** 2 for j in range(cols))) for c in range(r)]
        q = [[rr[j][c] / lens[c] for c in range(r)] for j in range(cols)]
    x_new = [[x[i][j] - lr * sum(p[i][c] * q[j][c] for c in range(r)) for j in range(cols)] for i in range(rows)]
    a_c, b_c = (1.0, 1.0 - mu) if ef == "dion" else (mu, mu)
    m_new = [[a_c * b[i][j] - b_c * sum(p[i][c] * rr[j][c] for c in range(r)) for j in range(cols)]
             for i in range(rows)]
    return {"X": np.array(x_new), "M": np.array(m_new), "Q": np.array(q), "P": np.array(p), "R": np.array(rr)}


def load_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, expr = line.split("=", 1)
            out[key.strip()] = np.array(eval(expr, {"__builtins__": {}}, {"sqrt": math.sqrt}), dtype=np.float64)
    return out


def rand_problem(seed, m, n, r, noise=1.0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((m, n))
    g = rng.standard_normal((m, n)) * noise
    mom = 0.3 * rng.standard_normal((m, n))
    q, _ = np.linalg.qr(rng.standard_normal((n, r)))
    return x, g, mom, q


def close(a, b, tol=1e-10):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, (a.shape, b.shape)
    scale = max(1.0, float(np.max(np.abs(b))))
    assert float(np.max(np.abs(a - b))) <= tol * scale, float(np.max(np.abs(a - b)))


# ----------------------------------------------------------------- the pins

def pin_golden_rotation(make):
    """Hand-worked 3x2 step (tests/golden/step_2x2_rotation.txt)."""
    gold = load_golden("step_2x2_rotation.txt")
    g = np.array([[2.0, 0.0], [0.0, 1.0], [0.0, 0.0]])
    qp = np.array([[1.0, -1.0], [1.0, 1.0]]) / math.sqrt(2.0)
    zero = np.zeros((3, 2))
    o = make(mu=0.95, lr=1.0, variant="qr", ef="dion").step(zero, g, zero, qp)
    close(o["P"], gold["P"]); close(o["T_P"], gold["T_P"]); close(o["R"], gold["R"])
    close(o["Q"], gold["Q_qr"]); close(o["T_Q"], gold["T_Q"]); close(o["D"], gold["D_qr"])
    close(o["X"], -gold["D_qr"]); close(o["M"], gold["M_dion"])
    o = make(mu=0.95, lr=1.0, variant="colnorm", ef="paper").step(zero, g, zero, qp)
    close(o["Q"], gold["Q_cn"]); close(o["D"], gold["D_cn"]); close(o["X"], -gold["D_cn"])
    close(o["M"], gold["M_paper"])


def pin_golden_345(make):
    """Hand-worked rank-1 step (tests/golden/step_3_4_5.txt)."""
    gold = load_golden("step_3_4_5.txt")
    mom = np.array([[1.0, 0.0], [1.0, 0.0]])
    g = np.array([[2.0, 1.0], [3.0, 0.0]])
    x = np.ones((2, 2))
    qp = np.array([[1.0], [0.0]])
    for variant in ("qr", "colnorm"):
        o = make(mu=0.9, lr=0.5, variant=variant, ef="dion").step(x, g, mom, qp)
        close(o["P"], gold["P"]); close(o["R"], gold["R"]); close(o["Q"], gold["Q_qr"])
        close(o["X"], gold["X_new"]); close(o["M"], gold["M_dion"])
    o = make(mu=0.9, lr=0.5, variant="qr", ef="paper").step(x, g, mom, qp)
    close(o["M"], gold["M_paper"]); close(o["T_P"], gold["T_P"]); close(o["T_Q"], gold["T_Q"])


def pin_brute_force(make):
    """Whole step against the pure-Python-loop transcription of Alg. 1 on tiny inputs,
    rectangular both ways, both variants, both error-feedback forms."""
    for seed, (m, n, r) in enumerate([(5, 4, 2), (4, 7, 3), (6, 6, 1), (3, 3, 3)]):
        x, g, mom, q = rand_problem(100 + seed, m, n, r)
        for variant in ("qr", "colnorm"):
            for ef in ("dion", "paper"):
                o = make(mu=0.8, lr=0.3, variant=variant, ef=ef).step(x, g, mom, q)
                ref = brute_step(x.tolist(), g.tolist(), mom.tolist(), q.tolist(), 0.3, 0.8, variant, ef)
                for k in ("X", "M", "Q", "P", "R"):
                    close(o[k], ref[k], 1e-9)


def pin_orthonormal_and_unit_singular_values(make):
    """Lemma 4.1: P and (QR variant) Q orthonormal, so all r singular values of P Q^T are 1."""
    x, g, mom, q = rand_problem(1, 24, 17, 5)
    o = make(variant="qr").step(x, g, mom, q)
    close(o["P"].T @ o["P"], np.eye(5), 1e-12)
    close(o["Q"].T @ o["Q"], np.eye(5), 1e-12)
    _, sig, _ = jacobi_svd(o["D"])
    close(sig[:5], np.ones(5), 1e-10)
    assert np.all(sig[5:] < 1e-10)
    assert np.all(np.diag(o["T_P"]) > 0) and np.all(np.diag(o["T_Q"]) > 0)
    close(np.tril(o["T_Q"], -1), np.zeros((5, 5)))
    close(o["Q"] @ o["T_Q"], o["R"], 1e-11)
    close(o["P"] @ o["T_P"], o["P_raw"], 1e-11)


def pin_colnorm_bounds(make):
    """Prop. 3.1: ColNorm gives unit diagonal Gram and an operator norm in [1, sqrt r]."""
    x, g, mom, q = rand_problem(2, 20, 30, 6)
    o = make(variant="colnorm").step(x, g, mom, q)
    close(np.diag(o["Q"].T @ o["Q"]), np.ones(6), 1e-12)
    _, sig, _ = jacobi_svd(o["Q"])
    assert 1.0 - 1e-12 <= sig[0] <= math.sqrt(6.0) + 1e-12
    assert sig[0] > 1.0 + 1e-6           # generic input: strictly inflated
    # the dual-norm factor of the update equals sigma_1(Q) because P is orthonormal
    _, sd, _ = jacobi_svd(o["D"])
    close(sd[0], sig[0], 1e-10)


def pin_polar_special_cases(make):
    """Sec. 2: the target is the rank-r polar factor U_r V_r^T.  One step reaches it
    exactly when (i) all r singular values of a rank-r B are equal, or (ii) the warm
    start already equals V_r."""
    rng = np.random.default_rng(3)
    m, n, r = 9, 7, 3
    u, _ = np.linalg.qr(rng.standard_normal((m, r)))
    v, _ = np.linalg.qr(rng.standard_normal((n, r)))
    q0, _ = np.linalg.qr(rng.standard_normal((n, r)))
    zero = np.zeros((m, n))
    # (i) equal singular values, generic warm start
    b = 2.5 * u @ v.T
    o = make(variant="qr").step(zero, b, zero, q0)
    close(o["D"], u @ v.T, 1e-10)
    # (ii) warm start = V_r of a full-rank B (brute-force SVD)
    bfull = rng.standard_normal((m, n))
    lu, sig, rv = jacobi_svd(bfull)
    o = make(variant="qr").step(zero, bfull, zero, rv[:, :r])
    close(o["D"], lu[:, :r] @ rv[:, :r].T, 1e-9)
    close(np.trace(o["T_Q"]), np.sum(sig[:r]), 1e-9)


def pin_fixed_point(make):
    """Repeating the step on a constant exactly-rank-r gradient converges to the polar
    factor; with the default error feedback the buffer stays a multiple of G
    (M_new = mu B because P P^T B = B), so B_t = G (1 + mu + ... + mu^t)."""
    rng = np.random.default_rng(4)
    m, n, r = 8, 10, 3
    u, _ = np.linalg.qr(rng.standard_normal((m, r)))
    v, _ = np.linalg.qr(rng.standard_normal((n, r)))
    s = np.array([5.0, 3.0, 1.0])
    g = (u * s) @ v.T
    orc = make(mu=0.5, lr=0.1, variant="qr", ef="dion")
    q, _ = np.linalg.qr(rng.standard_normal((n, r)))
    x = np.zeros((m, n)); mom = np.zeros((m, n))
    geo = 0.0
    errs = []
    for t in range(40):
        o = orc.step(x, g, mom, q)
        geo = 1.0 + 0.5 * geo
        close(o["B"], geo * g, 1e-10)
        close(o["M"], 0.5 * o["B"], 1e-9)
        errs.append(float(np.linalg.norm(o["D"] - u @ v.T)))
        x, mom, q = o["X"], o["M"], o["Q"]
    assert errs[0] > 1e-3 and errs[-1] < 1e-9 and errs[20] < errs[5] < errs[0]
    close(np.trace(o["T_Q"]), geo * np.sum(s), 1e-8)


def pin_variants_agree_on_orthogonal_columns(make):
    """Prop. 3.1 (equality case) and Lemma 4.3: when the columns of R are already
    orthogonal (warm start = V_r) QR and ColNorm give the same Q and X; for any input
    the two variants share P, R and the new momentum."""
    rng = np.random.default_rng(5)
    m, n, r = 7, 9, 4
    x = rng.standard_normal((m, n)); g = rng.standard_normal((m, n)); mom = rng.standard_normal((m, n))
    _, _, rv = jacobi_svd((mom + g).T)      # right singular vectors of B = left ones of B^T
    lu, _, _ = jacobi_svd((mom + g).T)
    vr = lu[:, :r]
    a = make(variant="qr").step(x, g, mom, vr)
    c = make(variant="colnorm").step(x, g, mom, vr)
    gram = a["R"].T @ a["R"]
    close(gram - np.diag(np.diag(gram)), np.zeros((r, r)), 1e-9)
    close(a["Q"], c["Q"], 1e-9); close(a["X"], c["X"], 1e-9)
    q0, _ = np.linalg.qr(rng.standard_normal((n, r)))
    a = make(variant="qr").step(x, g, mom, q0)
    c = make(variant="colnorm").step(x, g, mom, q0)
    close(a["P"], c["P"]); close(a["R"], c["R"]); close(a["M"], c["M"])
    assert float(np.max(np.abs(a["Q"] - c["Q"]))) > 1e-3      # generic: they differ
    # same column space (Lemma 4.3)
    proj_a = a["Q"] @ a["Q"].T
    qc, _ = np.linalg.qr(c["Q"])
    close(proj_a, qc @ qc.T, 1e-9)


def pin_error_feedback_identities(make):
    """Default form M_new = B - (1 - mu) P R^T:  P^T M_new = mu R^T, the part of B
    outside span(P) is kept whole, ||B - P R^T||^2 = ||B||^2 - ||R||^2.
    Paper form (Alg. 1 line 7): M_new = beta (I - P P^T) B, so P^T M_new = 0."""
    x, g, mom, q = rand_problem(6, 15, 11, 4)
    mu = 0.7
    o = make(mu=mu, ef="dion").step(x, g, mom, q)
    p, b, r = o["P"], o["B"], o["R"]
    close(b, mom + g)
    close(p.T @ o["M"], mu * r.T, 1e-11)
    perp = np.eye(15) - p @ p.T
    close(perp @ o["M"], perp @ b, 1e-11)
    close(np.linalg.norm(b - p @ r.T) ** 2, np.linalg.norm(b) ** 2 - np.linalg.norm(r) ** 2, 1e-10)
    close(o["M"], b - (1.0 - mu) * p @ (p.T @ b), 1e-11)
    o0 = make(mu=0.0, ef="dion").step(x, g, mom, q)
    close(o0["P"].T @ o0["M"], np.zeros((4, 11)), 1e-11)
    op = make(mu=mu, ef="paper").step(x, g, mom, q)
    close(op["M"], mu * perp @ b, 1e-11)
    o1 = make(mu=1.0, ef="paper").step(x, g, mom, q)
    od = make(mu=0.0, ef="dion").step(x, g, mom, q)
    close(o1["M"], od["M"], 1e-11)        # the two forms coincide at beta = 1 / mu = 0


def pin_trace_inequality(make):
    """Lemma 4.2 with the Hoelder identity of App. C: <B, P Q^T> = trace(T_Q) and it
    never exceeds the Ky Fan r-norm of B."""
    for seed in range(4):
        x, g, mom, q = rand_problem(20 + seed, 12, 10, 3)
        o = make(variant="qr").step(x, g, mom, q)
        _, sig, _ = jacobi_svd(o["B"])
        inner = float(np.sum(o["B"] * o["D"]))
        close(inner, np.trace(o["T_Q"]), 1e-10)
        assert inner <= np.sum(sig[:3]) + 1e-10
        assert inner > 0.0


def pin_update_direction_and_scale(make):
    """X moves by exactly lr along -P Q^T: ||X_new - X||_F = lr sqrt(r) for the QR
    variant, and <B, X - X_new> = lr trace(T_Q) > 0 (a descent direction for B)."""
    x, g, mom, q = rand_problem(7, 10, 14, 4)
    o = make(lr=0.25, variant="qr").step(x, g, mom, q)
    close(np.linalg.norm(o["X"] - x), 0.25 * 2.0, 1e-11)
    close(np.sum(o["B"] * (x - o["X"])), 0.25 * np.trace(o["T_Q"]), 1e-10)
    # rectangular orientation: Q is n x r, P is m x r
    assert o["P"].shape == (10, 4) and o["Q"].shape == (14, 4) and o["R"].shape == (14, 4)


def pin_multi_step_state(make):
    """run() carries X, M and Q forward (Alg. 1 line 8: warm start) and equals chained
    single steps; with bf16 parameters the stored bits are what the next step reads."""
    rng = np.random.default_rng(8)
    m, n, r = 6, 8, 2
    x0 = rng.standard_normal((m, n)); m0 = np.zeros((m, n))
    q0, _ = np.linalg.qr(rng.standard_normal((n, r)))
    grads = [rng.standard_normal((m, n)) for _ in range(3)]
    orc = make(mu=0.9, lr=0.05)
    outs = orc.run(x0, grads, m0, q0)
    x, mom, q = x0, m0, q0
    for t in range(3):
        o = orc.step(x, grads[t], mom, q)
        close(outs[t]["X"], o["X"]); close(outs[t]["M"], o["M"]); close(outs[t]["Q"], o["Q"])
        x, mom, q = o["X"], o["M"], o["Q"]
    # bf16 storage
    xb = f64_to_bf16_bits(x0)
    gb = [f64_to_bf16_bits(gr) for gr in grads]
    ob = make(mu=0.9, lr=0.05, x_bf16=True).run(xb, gb, m0, q0)
    first = make(mu=0.9, lr=0.05, x_bf16=True).step(xb, gb[0], m0, q0)
    assert np.array_equal(ob[0]["X_bits"], first["X_bits"])
    second = make(mu=0.9, lr=0.05, x_bf16=True).step(first["X_bits"], gb[1], first["M"], first["Q"])
    assert np.array_equal(ob[1]["X_bits"], second["X_bits"])
    close(first["B"], bf16_bits_to_f64(gb[0]))


PINS = [pin_golden_rotation, pin_golden_345, pin_brute_force,
        pin_orthonormal_and_unit_singular_values, pin_colnorm_bounds, pin_polar_special_cases,
        pin_fixed_point, pin_variants_agree_on_orthogonal_columns, pin_error_feedback_identities,
        pin_trace_inequality, pin_update_direction_and_scale, pin_multi_step_state]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_oracle_pin(pin):
    pin(lambda **kw: OrthDionOracle(**kw))


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_oracle_pin_library_qr_route(pin):
    """The route the largest parity cases take (numpy's QR with the signs fixed) is held to
    every pin of the default route: hand-worked goldens, the loop transcription, the lemmas."""
    pin(lambda **kw: OrthDionOracle(qr="library", **kw))


def test_library_qr_route_equals_written_out_reflections():
    rng = np.random.default_rng(21)
    for rows, cols in [(6, 6), (300, 40), (513, 128)]:
        a = rng.standard_normal((rows, cols)) @ np.diag(np.linspace(1.0, 1e-3, cols))
        a[:, ::3] *= -1.0
        q, t = thin_qr_positive(a)
        ql, tl = thin_qr_library(a)
        close(ql, q, 1e-10); close(tl, t, 1e-11)
        assert np.all(np.diag(tl) > 0) and np.all(np.tril(tl, -1) == 0)
    x, g, mom, q0 = rand_problem(5, 96, 160, 24)
    for variant in ("qr", "colnorm"):
        a = OrthDionOracle(variant=variant).step(x, g, mom, q0)
        b = OrthDionOracle(variant=variant, qr="library").step(x, g, mom, q0)
        for key in ("P", "R", "Q", "M", "X", "D"):
            close(b[key], a[key], 1e-10)


def test_rel_fro_is_the_relative_frobenius_distance():
    # 3-4-5: ||a - b||_F = 5 against ||b||_F = 10; the reference is the second argument
    b = np.array([[6.0, 0.0], [0.0, 8.0]])
    a = b + np.array([[3.0, 0.0], [0.0, -4.0]])
    assert rel_fro(a, b) == 0.5
    assert abs(rel_fro(b, a) - 5.0 / math.sqrt(81.0 + 16.0)) < 1e-15
    assert rel_fro(b, b) == 0.0
    assert rel_fro(np.array([3.0, 4.0]), np.zeros(2)) == 5.0      # zero reference: absolute distance
    assert rel_fro(np.array([1.0], dtype=np.float32), np.array([1.0 + 2.0 ** -30])) > 0.0   # compared in fp64


# ----------------------------------------------------------------- pieces against libraries

def test_thin_qr_matches_library_after_sign_fix():
    rng = np.random.default_rng(11)
    for rows, cols in [(7, 7), (40, 9), (130, 32), (5, 1)]:
        a = rng.standard_normal((rows, cols))
        a[:, 0] *= -1.0 if rows % 2 else 1.0
        q, t = thin_qr_positive(a)
        ql, tl = np.linalg.qr(a)
        s = np.where(np.diag(tl) < 0, -1.0, 1.0)
        close(q, ql * s[None, :], 1e-11); close(t, tl * s[:, None], 1e-11)
        assert np.all(np.diag(t) > 0)
        close(q @ t, a, 1e-12)
    # ill-conditioned but full rank: still orthonormal to machine precision
    a = rng.standard_normal((60, 8)) @ np.diag(10.0 ** -np.arange(8))
    q, t = thin_qr_positive(a)
    close(q.T @ q, np.eye(8), 1e-13)
    qg, tg = gram_schmidt_loops(rng.standard_normal((9, 4)).tolist())
    close(np.array(qg).T @ np.array(qg), np.eye(4), 1e-12)


def test_col_norm_definition():
    r = np.array([[3.0, 0.0, 1.0], [4.0, 0.0, -1.0]])
    q = col_norm(r)
    close(q[:, 0], [0.6, 0.8]); close(q[:, 1], [0.0, 0.0]); close(q[:, 2], [1 / math.sqrt(2), -1 / math.sqrt(2)])


def test_bf16_rounding_known_patterns():
    # exact values, ties to even, and the step above a tie
    vals = np.array([1.0, -2.0, 1.0 + 2.0 ** -8, 1.0 + 3.0 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -30,
                     0.0, 3.140625, 2.0 ** -126, 65280.0])
    bits = f64_to_bf16_bits(vals)
    assert bits.tolist() == [0x3F80, 0xC000, 0x3F80, 0x3F82, 0x3F81, 0x0000, 0x4049, 0x0080, 0x477F]
    close(bf16_bits_to_f64(bits)[[0, 1, 6]], [1.0, -2.0, 3.140625])


def test_bf16_rounding_matches_torch_on_fp32_values():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(12)
    v = (rng.standard_normal(20000) * 10.0 ** rng.uniform(-6, 4, 20000)).astype(np.float32)
    ours = f64_to_bf16_bits(v.astype(np.float64))
    theirs = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, theirs)
    back = bf16_bits_to_f64(ours)
    assert np.array_equal(back, torch.from_numpy(v).to(torch.bfloat16).to(torch.float64).numpy())


def test_double_rounding_is_avoided():
    # 1 + 2^-8 + 2^-40 lies just above a bf16 tie; rounding through fp32 first would
    # land exactly on the tie and round down to even.
    v = np.array([1.0 + 2.0 ** -8 + 2.0 ** -40])
    assert f64_to_bf16_bits(v)[0] == 0x3F81


# ----------------------------------------------------------------- planted mistakes

class _DropGradient(OrthDionOracle):
    def buffer(self, m_prev, g):
        return g.copy()


class _BufferSign(OrthDionOracle):
    def buffer(self, m_prev, g):
        return g - m_prev


class _ProjectTransposed(OrthDionOracle):
    def project(self, b, q_prev):
        return b.T @ q_prev if b.shape[0] == b.shape[1] else b @ q_prev


class _NoSignFix(OrthDionOracle):
    def orth(self, a):
        q, t = np.linalg.qr(a)
        return q, t


class _OrthIsColNorm(OrthDionOracle):
    def orth(self, a):
        return col_norm(a), np.diag(np.sqrt(np.sum(a * a, axis=0)))


class _PolarOrth(OrthDionOracle):
    def orth(self, a):
        u, s, vt = np.linalg.svd(a, full_matrices=False)
        return u @ vt, vt.T @ np.diag(s) @ vt


class _BackProjectRaw(OrthDionOracle):
    def step(self, x, g, m_prev, q_prev):
        out = super().step(x, g, m_prev, q_prev)
        return out

    def back_project(self, b, p):
        return b.T @ (p * 1.0001)


class _UpdateSign(OrthDionOracle):
    def update(self, x, p, q):
        return x + self.lr * (p @ q.T)


class _UpdateTransposed(OrthDionOracle):
    def update(self, x, p, q):
        d = p @ q.T
        return x - self.lr * (d.T if d.shape[0] == d.shape[1] else d)


class _EfDropsFactor(OrthDionOracle):
    def error_feedback(self, b, p, r):
        return b - p @ r.T if self.ef == "dion" else super().error_feedback(b, p, r)


class _EfUsesMu(OrthDionOracle):
    def error_feedback(self, b, p, r):
        return b - self.mu * (p @ r.T) if self.ef == "dion" else super().error_feedback(b, p, r)


class _EfPaperScalesOnlyProjection(OrthDionOracle):
    def error_feedback(self, b, p, r):
        return b - self.mu * (p @ r.T) if self.ef == "paper" else super().error_feedback(b, p, r)


class _ColNormByMax(OrthDionOracle):
    def right_factor(self, r):
        if self.variant == "colnorm":
            return r / np.max(np.abs(r), axis=0)[None, :], None
        return super().right_factor(r)


class _ColNormRows(OrthDionOracle):
    def right_factor(self, r):
        if self.variant == "colnorm":
            return r / np.sqrt(np.sum(r * r, axis=1))[:, None], None
        return super().right_factor(r)


class _NoWarmStart(OrthDionOracle):
    def run(self, x, grads, m0, q0):
        outs = []
        x_cur, m_cur = x, m0
        for g in grads:
            o = self.step(x_cur, g, m_cur, q0)
            outs.append(o)
            x_cur = o["X_bits"] if self.x_bf16 else o["X"]
            m_cur = o["M"]
        return outs


class _QrOfRawRightFactor(OrthDionOracle):
    """orthogonalises B^T P_raw instead of B^T P (a different basis of the same span)."""

    def step(self, x, g, m_prev, q_prev):
        out = super().step(x, g, m_prev, q_prev)
        if self.variant == "qr":
            q, t = thin_qr_positive(out["B"].T @ out["P_raw"])
            out["Q"], out["T_Q"] = q, t
            out["D"] = out["P"] @ q.T
            out["X"] = (bf16_bits_to_f64(x) if np.asarray(x).dtype == np.uint16 else np.asarray(x, float)) \
                - self.lr * out["D"]
        return out


MUTANTS = [_DropGradient, _BufferSign, _ProjectTransposed, _NoSignFix, _OrthIsColNorm, _PolarOrth,
           _BackProjectRaw, _UpdateSign, _UpdateTransposed, _EfDropsFactor, _EfUsesMu,
           _EfPaperScalesOnlyProjection, _ColNormByMax, _ColNormRows, _NoWarmStart,
           _QrOfRawRightFactor]


@pytest.mark.parametrize("mutant", MUTANTS, ids=lambda c: c.__name__)
def test_pins_catch_planted_mistake(mutant):
    failures = []
    for pin in PINS:
        try:
            pin(lambda **kw: mutant(**kw))
        except AssertionError:
            failures.append(pin.__name__)
        except Exception as exc:            # a mutant may also break shapes
            failures.append(pin.__name__ + ":" + type(exc).__name__)
    assert failures, f"no pin notices {mutant.__name__}"
