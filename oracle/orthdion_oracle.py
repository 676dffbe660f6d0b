"""fp64 CPU oracle of one Orth-Dion / stripped-Dion optimizer step.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the HIP path
is judged against.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import it; the product path never does, and it shares no
code with the HIP sources.

What it computes (paper Alg. 1, "Orth-Dion / Stripped Dion (one step)", and the
two listings of App. B.1), in the notation of the library interface
(paper name -> name here):  buffer M_t -> B,  residual R_t -> M,  U_t -> P,
W_t -> R,  right factor V -> Q,  eta -> lr.

    B      = M + G                     Alg. 1 line 1  (buffer = gradient + residual)
    P_raw  = B Q_prev                  Alg. 1 line 2  (one subspace-iteration step)
    P      = orth(P_raw)               Alg. 1 line 2  (left factor via QR)
    R      = B^T P                     Alg. 1 line 3
    Q      = orth(R)  |  ColNorm(R)    Alg. 1 line 4  (Orth-Dion | Dion, Sec. 2 table)
    X_new  = X - lr P Q^T              Alg. 1 lines 5-6
    M_new  = a B - b P R^T             Alg. 1 line 7 and the reading below
    Q_prev = Q                         Alg. 1 line 8  (warm start)

Readings of points the paper leaves open:
  * orth(A) is the Q factor of the thin QR factorisation A = Q T whose triangular
    factor has a positive diagonal.  The paper only says "QR"; for full column
    rank this factor is unique, which is what makes P Q^T well defined (a
    different orthonormal basis of the same span gives a different update).
  * error feedback: the library's default is M_new = B - (1 - mu) P R^T
    ("dion" form: a = 1, b = 1 - mu).  Alg. 1 line 7 prints
    beta (B - P (P^T B)) ("paper" form: a = b = beta, with beta passed as mu).
    Both are a B - b P R^T and coincide at mu = 0 / beta = 1.
  * ColNorm divides each column of R by its Euclidean length (abstract and
    Sec. 3: unit-length columns, Gram diagonal 1); no epsilon is added.
  * bf16 parameters: the new parameter is the fp64 result rounded to bfloat16
    with round-to-nearest-even; the paper does not discuss rounding.

Every product is a plain numpy matmul in float64; the QR is Householder
reflections written out below.  Nothing is blocked, fused or reordered.

``OrthDionOracle(qr="library")`` takes the same thin QR factor (Alg. 1 lines 2 and 4; the
positive-diagonal factor is unique for full column rank) from numpy's QR routine with the
signs fixed afterwards, instead of the reflections written out here.  It exists for the
parity tests at the largest benchmark shapes (rank >= 1024), where the written-out
reflections take minutes per matrix; the two routes are pinned against each other and
against the same closed forms in the CPU tests.  The default stays the written-out one.
"""
from __future__ import annotations

from typing import Dict, Optional, Tuple

import numpy as np

__all__ = ["thin_qr_positive", "thin_qr_library", "col_norm", "ef_coefficients", "OrthDionOracle",
           "bf16_bits_to_f64", "f64_to_bf16_bits", "rel_fro", "effective_rank", "diagnostics", "gradient_persistence", "rank_policy",
           "resize_right_factor"]


# ---------------------------------------------------------------- storage helpers

def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of bfloat16 bit patterns (uint16) as float64."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64 to bfloat16, round-to-nearest-even, directly from the fp64 value
    (no intermediate fp32 rounding).  Finite inputs in bf16's normal range only."""
    x = np.asarray(x, dtype=np.float64)
    mant, expo = np.frexp(x)                     # x = mant * 2^expo, 0.5 <= |mant| < 1
    # bf16 keeps 8 significant bits: quantum is 2^(expo - 8); subnormals: 2^-133
    q = np.ldexp(1.0, np.maximum(expo - 8, -133))
    y = np.rint(x / q) * q                       # rint = round half to even
    y32 = y.astype(np.float32)                   # exact: y has <= 8 significant bits
    return (y32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def rel_fro(a: np.ndarray, b: np.ndarray) -> float:
    """||a - b||_F / ||b||_F in float64 (b is the reference)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = float(np.linalg.norm(b))
    num = float(np.linalg.norm(a - b))
    return num / den if den > 0.0 else num


# ---------------------------------------------------------------- orth / ColNorm

def thin_qr_positive(a: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Thin QR of ``a`` (rows >= cols) by Householder reflections: ``a = q @ t`` with
    ``q`` having orthonormal columns and ``t`` upper triangular with ``diag(t) > 0``.

    This is the ``orth`` of Alg. 1 lines 2 and 4 under the positive-diagonal reading.
    """
    a = np.array(a, dtype=np.float64, copy=True)
    rows, cols = a.shape
    if rows < cols:
        raise ValueError("thin QR needs rows >= cols")
    vs = []
    for j in range(cols):
        x = a[j:, j]
        normx = np.sqrt(np.dot(x, x))
        v = x.copy()
        if normx > 0.0:
            alpha = -normx if x[0] >= 0.0 else normx     # reflect x onto alpha * e_1
            v[0] -= alpha
            vnorm = np.sqrt(np.dot(v, v))
            if vnorm > 0.0:
                v /= vnorm
                a[j:, j:] -= 2.0 * np.outer(v, v @ a[j:, j:])
        else:
            v[:] = 0.0
        vs.append(v)
    t = np.triu(a[:cols, :cols])
    q = np.zeros((rows, cols), dtype=np.float64)
    q[:cols, :cols] = np.eye(cols)
    for j in range(cols - 1, -1, -1):                    # q = H_0 H_1 ... H_{c-1} [I; 0]
        v = vs[j]
        q[j:, :] -= 2.0 * np.outer(v, v @ q[j:, :])
    sign = np.where(np.diag(t) < 0.0, -1.0, 1.0)
    return q * sign[None, :], t * sign[:, None]


def thin_qr_library(a: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """The same factorisation as ``thin_qr_positive`` (``a = q @ t``, orthonormal ``q``, upper
    triangular ``t`` with ``diag(t) > 0``; Alg. 1 lines 2 and 4) with numpy's thin QR as the
    library step: column j of ``q`` and row j of ``t`` change sign wherever ``t[j, j] < 0``."""
    a = np.asarray(a, dtype=np.float64)
    if a.shape[0] < a.shape[1]:
        raise ValueError("thin QR needs rows >= cols")
    q, t = np.linalg.qr(a, mode="reduced")
    sign = np.where(np.diag(t) < 0.0, -1.0, 1.0)
    return q * sign[None, :], np.triu(t) * sign[:, None]


def col_norm(r: np.ndarray) -> np.ndarray:
    """ColNorm of the Dion variant: every column rescaled to unit Euclidean length.
    A zero column is left as zeros."""
    r = np.asarray(r, dtype=np.float64)
    lengths = np.sqrt(np.sum(r * r, axis=0))
    safe = np.where(lengths > 0.0, lengths, 1.0)
    return r / safe[None, :]


def ef_coefficients(mu: float, ef: str) -> Tuple[float, float]:
    """(a, b) of ``M_new = a B - b P R^T``: "dion" -> (1, 1 - mu); "polyak" -> (mu, 0); "paper" -> (mu, mu)
    (Alg. 1 line 7 with beta = mu)."""
    if ef == "dion":
        return 1.0, 1.0 - float(mu)
    if ef == "paper":
        return float(mu), float(mu)
    if ef == "polyak":
        # "PolyakDion" of Sec. 6.3 / App. H: residual identically zero, explicit momentum mu.
        # Reading: the momentum is heavy-ball on the buffer, B_t = mu B_{t-1} + G_t.
        return float(mu), 0.0
    raise ValueError("ef must be 'dion', 'paper' or 'polyak'")


# ---------------------------------------------------------------- the step

class OrthDionOracle:
    """One matrix, stepped in float64.  Each sub-step is its own method so that a
    test can plant a mistake in exactly one of them and check that the pins notice."""

    def __init__(self, mu: float = 0.95, lr: float = 0.01, variant: str = "qr",
                 ef: str = "dion", x_bf16: bool = False, qr: str = "householder"):
        if variant not in ("qr", "colnorm"):
            raise ValueError("variant must be 'qr' or 'colnorm'")
        if qr not in ("householder", "library"):
            raise ValueError("qr must be 'householder' or 'library'")
        self.mu, self.lr, self.variant, self.ef, self.x_bf16 = float(mu), float(lr), variant, ef, bool(x_bf16)
        self.qr = qr
        ef_coefficients(mu, ef)

    # Alg. 1 line 1
    def buffer(self, m_prev: np.ndarray, g: np.ndarray) -> np.ndarray:
        return m_prev + g

    # Alg. 1 line 2 (product)
    def project(self, b: np.ndarray, q_prev: np.ndarray) -> np.ndarray:
        return b @ q_prev

    # Alg. 1 lines 2 and 4 (orth)
    def orth(self, a: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
        return thin_qr_library(a) if self.qr == "library" else thin_qr_positive(a)

    # Alg. 1 line 3
    def back_project(self, b: np.ndarray, p: np.ndarray) -> np.ndarray:
        return b.T @ p

    # Alg. 1 line 4
    def right_factor(self, r: np.ndarray) -> Tuple[np.ndarray, Optional[np.ndarray]]:
        if self.variant == "qr":
            return self.orth(r)
        return col_norm(r), None

    # Alg. 1 lines 5-6
    def update(self, x: np.ndarray, p: np.ndarray, q: np.ndarray) -> np.ndarray:
        return x - self.lr * (p @ q.T)

    # Alg. 1 line 7 / default form
    def error_feedback(self, b: np.ndarray, p: np.ndarray, r: np.ndarray) -> np.ndarray:
        a_coef, b_coef = ef_coefficients(self.mu, self.ef)
        return a_coef * b - b_coef * (p @ r.T)

    def step(self, x, g, m_prev, q_prev) -> Dict[str, np.ndarray]:
        """Inputs: X and G as float arrays or uint16 bf16 bit patterns; M, Q float.
        Returns every intermediate; ``X`` is the fp64 result, ``X_bits`` its bf16
        rounding when the parameter is stored in bf16."""
        x = bf16_bits_to_f64(x) if np.asarray(x).dtype == np.uint16 else np.asarray(x, dtype=np.float64)
        g = bf16_bits_to_f64(g) if np.asarray(g).dtype == np.uint16 else np.asarray(g, dtype=np.float64)
        m_prev = np.asarray(m_prev, dtype=np.float64)
        q_prev = np.asarray(q_prev, dtype=np.float64)
        b = self.buffer(m_prev, g)
        p_raw = self.project(b, q_prev)
        p, t_p = self.orth(p_raw)
        r = self.back_project(b, p)
        q, t_q = self.right_factor(r)
        x_new = self.update(x, p, q)
        m_new = self.error_feedback(b, p, r)
        out = {"B": b, "P_raw": p_raw, "P": p, "T_P": t_p, "R": r, "Q": q, "T_Q": t_q,
               "X": x_new, "M": m_new, "D": p @ q.T}
        if self.x_bf16:
            out["X_bits"] = f64_to_bf16_bits(x_new)
        return out

    def run(self, x, grads, m0, q0):
        """Free-running trajectory: ``grads`` is an iterable of gradients.  With bf16
        parameters the stored (rounded) X is what the next step reads; M and Q stay in
        float64.  Returns the list of per-step outputs."""
        outs = []
        x_cur, m_cur, q_cur = x, m0, q0
        for g in grads:
            o = self.step(x_cur, g, m_cur, q_cur)
            outs.append(o)
            x_cur = o["X_bits"] if self.x_bf16 else o["X"]
            m_cur, q_cur = o["M"], o["Q"]
        return outs


# ---------------------------------------------------------------- diagnostics and rank policy

def effective_rank(r: np.ndarray) -> float:
    """Estimated effective rank of App. B.2 / Sec. 6: exp(-sum p log p) with
    p_i = ||R[:, i]||_2 / sum_j ||R[:, j]||_2 (terms with p_i = 0 contribute 0)."""
    r = np.asarray(r, dtype=np.float64)
    lengths = np.sqrt(np.sum(r * r, axis=0))
    total = float(np.sum(lengths))
    if total <= 0.0:
        return 0.0
    p = lengths / total
    nz = p > 0.0
    return float(np.exp(-np.sum(p[nz] * np.log(p[nz]))))


def diagnostics(step_out: Dict[str, np.ndarray], m_prev, g) -> Dict[str, float]:
    """Per-step scalars the paper logs, from one step's intermediates:
      b_norm, r_norm       ||B||_F and ||R||_F = ||P^T B||_F
      tracking_error       ||(I - P P^T) B||_F / ||B||_F            (Sec. 6', App. J key quantities)
      residual_ratio       ||M_prev||_F / ||G||_F  (R-norm ratio)   (Sec. 6', App. J)
      inner                <B, P Q^T>                               (Lemma 4.2; = trace(T_Q) for QR)
      nu                   sigma_1(Q), the dual-norm factor         (Prop. 3.1, Lemma 4.1)
      erank                estimated effective rank of R            (Sec. 6, App. B.2)
    """
    g = bf16_bits_to_f64(g) if np.asarray(g).dtype == np.uint16 else np.asarray(g, dtype=np.float64)
    m_prev = np.asarray(m_prev, dtype=np.float64)
    b, p, r, q = step_out["B"], step_out["P"], step_out["R"], step_out["Q"]
    b_norm = float(np.linalg.norm(b))
    resid = b - p @ (p.T @ b)
    gn = float(np.linalg.norm(g))
    return {
        "b_norm": b_norm,
        "r_norm": float(np.linalg.norm(r)),
        "tracking_error": float(np.linalg.norm(resid)) / b_norm if b_norm > 0 else 0.0,
        "residual_ratio": float(np.linalg.norm(m_prev)) / gn if gn > 0 else 0.0,
        "inner": float(np.sum(b * (p @ q.T))),
        "nu": float(np.linalg.norm(q, 2)),
        "erank": effective_rank(r),
    }


def gradient_persistence(p_t, g_t, p_prev, g_prev) -> float:
    """phi_t = cos of the angle between the out-of-subspace parts of two consecutive gradients,
    (I - P_t P_t^T) G_t and (I - P_{t-1} P_{t-1}^T) G_{t-1}, as matrices under the Frobenius
    inner product (Sec. 6.3, App. J key quantities).  Its sign names the error-feedback regime:
    coherent (> 0), stochastic (about 0), anti-correlated (< 0)."""
    def outside(p, g):
        g = bf16_bits_to_f64(g) if np.asarray(g).dtype == np.uint16 else np.asarray(g, dtype=np.float64)
        p = np.asarray(p, dtype=np.float64)
        return g - p @ (p.T @ g)
    a, b = outside(p_t, g_t), outside(p_prev, g_prev)
    na, nb = float(np.linalg.norm(a)), float(np.linalg.norm(b))
    return float(np.sum(a * b)) / (na * nb) if na > 0 and nb > 0 else 0.0


def rank_policy(e_t: float, r_t: int, ema_prev: float, r_min: int, r_max: int, alpha: float,
                gamma: float) -> Tuple[float, int]:
    """Ada-Orth-Dion rank selection (App. B.2, Alg. 2): EMA of the effective-rank estimate,
    buffer multiplier, ceiling, clip to [r_min, r_max], multiple of 8.  Reading: "rounded to
    multiple of 8" rounds up (the multiplier is a safety margin) and the result is clipped
    again so that it never leaves [r_min, r_max] (both taken to be multiples of 8).
    Returns (new EMA, next rank)."""
    ema = alpha * float(e_t) + (1.0 - alpha) * float(ema_prev)
    target = int(np.ceil(gamma * ema))
    nxt = min(max(target, int(r_min)), int(r_max))
    nxt = ((nxt + 7) // 8) * 8
    nxt = min(max(nxt, int(r_min)), int(r_max))
    return ema, nxt


def resize_right_factor(q: np.ndarray, r_new: int, pad: Optional[np.ndarray] = None) -> np.ndarray:
    """Rank change of the warm-start factor (App. B.2, Alg. 2, "truncate or pad").  Reading:
    truncation keeps the leading r_new columns; growth appends the columns of ``pad``
    (n x (r_new - r_old)), which the caller draws -- the paper does not say with what the
    factor is padded, and zero columns would make the next projection rank deficient."""
    q = np.asarray(q)
    n, r_old = q.shape
    if r_new <= r_old:
        return q[:, :r_new].copy()
    if pad is None or pad.shape != (n, r_new - r_old):
        raise ValueError("growing the rank needs pad of shape (n, r_new - r_old)")
    return np.concatenate([q, np.asarray(pad, dtype=q.dtype)], axis=1)
