/*
 * orthdion.h - C ABI of the MI355X-native Orth-Dion optimizer step.
 *
 * One call of orthdion_step performs, for every matrix of the set, one step of the
 * paper's Alg. 1 ("Orth-Dion / Stripped Dion (one step)"; the two variants are also
 * listed in App. B.1).  In this interface's letters (paper's letters in brackets):
 *
 *   B      = M + G                   [M_t = G_t + R_t]            Alg. 1 line 1
 *   P      = orth(B Q)               [U_t = orth(M_t V_{t-1})]    Alg. 1 line 2
 *   R      = B^T P                   [W_t = M_t^T U_t]            Alg. 1 line 3
 *   Q      = orth(R) | ColNorm(R)    [V_t]   Orth-Dion | Dion     Alg. 1 line 4, Sec. 2 table
 *   X      = X - lr P Q^T            [X_{t+1} = X_t - eta D_t]    Alg. 1 lines 5-6
 *   M      = a B - b P R^T           [R_{t+1}]                    Alg. 1 line 7 (see orthdion_ef)
 *   Q is kept for the next step      [warm start]                 Alg. 1 line 8
 *
 * orth(A) is the Q factor of the thin QR factorisation of A whose triangular factor has a
 * positive diagonal.  ColNorm rescales every column to unit Euclidean length.
 *
 * Memory: every matrix is row-major.  X, G, M are m x n with leading dimensions ldx, ldg,
 * ldm (in elements); Q is n x r, densely packed (leading dimension r).  X and G are fp32 or
 * bf16 as configured; M and Q are always fp32.  All buffers named "device" are device
 * (HBM) pointers owned by the caller; pointer *arrays* are host arrays.  The library never
 * allocates or frees device memory and never synchronises the device or a stream, except
 * orthdion_get_info / orthdion_get_warnings / orthdion_get_diagnostics, which wait for the
 * stream they are given.  orthdion_step creates, at its first call that is not under stream
 * capture and only when it has a use for them, two more streams and four events (runtime
 * objects of the handle, released by orthdion_destroy).  Ranks above 256 in fast precision
 * fork the guard of the second CholeskyQR pass onto one of them; a handle with two groups
 * (orthdion_config.groups) runs the second group's step on the other.  Every fork is joined
 * to the caller's stream again before the kernels that need it, at the latest before the call
 * returns, so the caller sees a single stream; under capture all branches are part of the
 * graph.
 *
 * Errors: every function returns ORTHDION_OK (0) or a negative orthdion_status; nothing
 * throws or aborts.  Numerical breakdown found on the device (a rank-deficient or
 * non-finite factor, outside the method's domain: Lemma 4.3 assumes full rank) does not
 * fail the call; it is reported per matrix by orthdion_get_info and leaves that matrix's
 * outputs unspecified.
 */
#ifndef ORTHDION_H
#define ORTHDION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct orthdion_ctx* orthdion_handle;   /* opaque; host memory only */

typedef enum {
  ORTHDION_OK = 0,
  ORTHDION_E_INVALID_ARG = -1,        /* enum out of range, nmat < 1, non-finite mu / lr ...   */
  ORTHDION_E_NULL_PTR = -2,
  ORTHDION_E_BAD_SHAPE = -3,          /* see orthdion_matdesc                                   */
  ORTHDION_E_WORKSPACE_TOO_SMALL = -4,
  ORTHDION_E_MISALIGNED = -5,         /* a device pointer is not 16-byte aligned                */
  ORTHDION_E_HIP = -6,                /* a HIP call failed; hipGetLastError has the cause       */
  ORTHDION_E_NO_STEP = -7,            /* orthdion_get_info before any orthdion_step             */
  ORTHDION_E_NO_MEMORY = -8           /* a host allocation failed                               */
} orthdion_status;

typedef enum { ORTHDION_F32 = 0, ORTHDION_BF16 = 1 } orthdion_dtype;

/* Alg. 1 line 4: QR orthogonalisation (Orth-Dion, the paper's method) or Dion's column
 * normalisation. */
typedef enum { ORTHDION_QR = 0, ORTHDION_COLNORM = 1 } orthdion_variant;

/* Error-feedback form, both M = a B - b P R^T:
 *   ORTHDION_EF_DION   a = 1,  b = 1 - mu   (momentum form; the default)
 *   ORTHDION_EF_PAPER  a = mu, b = mu       (Alg. 1 line 7 with beta = mu)
 *   ORTHDION_EF_POLYAK a = mu, b = 0        (no error feedback: the buffer is plain heavy-ball
 *                                            momentum of the gradients, the "PolyakDion"
 *                                            comparison of Sec. 6.3 / App. H)
 * The first two coincide at mu = 0 / beta = 1. */
typedef enum { ORTHDION_EF_DION = 0, ORTHDION_EF_PAPER = 1, ORTHDION_EF_POLYAK = 2 } orthdion_ef;

/* Arithmetic of the large contractions (B Q, B^T P, P R^T, P Q^T).  Accumulation is always
 * fp32; the orthogonalisations always use split-bf16 operands (>= 16 significant bits).
 *   ORTHDION_PREC_AUTO   FAST when X and G are both bf16, otherwise EXACT
 *   ORTHDION_PREC_FAST   fp16 matrix-core operands under a power-of-two scale (11 bits)
 *   ORTHDION_PREC_EXACT  three-way split bf16 operands, six products (24 bits) */
typedef enum { ORTHDION_PREC_AUTO = 0, ORTHDION_PREC_FAST = 1, ORTHDION_PREC_EXACT = 2 } orthdion_precision;

/* One parameter matrix.  Requirements (else ORTHDION_E_BAD_SHAPE):
 *   m, n, r multiples of 8 (the paper's adaptive-rank policy, App. B.2, rounds ranks to
 *   multiples of 8);  8 <= r <= min(m, n);  ldx, ldg, ldm >= n and multiples of 8;
 *   m, n < 2^24. */
typedef struct {
  int64_t m, n;
  int32_t r;
  int64_t ldx, ldg, ldm;
} orthdion_matdesc;

typedef struct {
  orthdion_dtype x_dtype, g_dtype;
  orthdion_variant variant;
  orthdion_ef ef;
  orthdion_precision precision;
  float mu;     /* momentum / error-feedback coefficient, 0 <= mu <= 1                  */
  float lr;     /* step size eta; any scale factor or schedule is folded in by the caller */
  int32_t groups; /* 0 = chosen by the library (two for a set of several matrices with 2^26 to
                   * 2^29 elements in all, else one), 1, or 2.  With two groups the launch
                   * batches are dealt to two sets of about equal work whose steps run side
                   * by side, one on the caller's stream and one on a stream of the handle:
                   * what one set leaves idle (its Cholesky chains, short launches) the other
                   * one uses.  No result depends on it, bit for bit.                        */
} orthdion_config;

/* Builds a handle for a fixed set of nmat matrices (host-side planning only; the handle
 * holds shapes and hyper-parameters, no numerical state: the optimizer state is the
 * caller's X, M, Q buffers).  `mats` and `cfg` are copied. */
int orthdion_create(orthdion_handle* out, const orthdion_matdesc* mats, int32_t nmat,
                    const orthdion_config* cfg);

/* Bytes of device scratch orthdion_step needs; the caller allocates it (256-byte aligned).
 * Its contents are meaningless between steps except for the debug layout below. */
size_t orthdion_workspace_bytes(orthdion_handle h);

/* 1 or 2: the number of groups the handle's matrices were dealt into (orthdion_config.groups;
 * 2 only when the set has at least two launch batches); 0 for a NULL handle. */
int32_t orthdion_get_groups(orthdion_handle h);

int orthdion_set_lr(orthdion_handle h, float lr);
int orthdion_set_mu(orthdion_handle h, float mu);
int orthdion_set_variant(orthdion_handle h, orthdion_variant v);

/* One optimizer step over the whole matrix set, enqueued on `stream` (a hipStream_t passed
 * as void*, 0 = the null stream); returns without waiting.
 *   X  host array of nmat device pointers, x_dtype, updated in place
 *   G  host array of nmat device pointers, g_dtype, read only
 *   M  host array of nmat device pointers, fp32, updated in place
 *   Q  host array of nmat device pointers, fp32 n x r; on entry the previous right factor
 *      (any full-column-rank n x r matrix for the first step), on exit the new one
 * Buffers must not overlap each other or the workspace.  Steps of one handle must be
 * enqueued on one stream at a time (they share the workspace). */
int orthdion_step(orthdion_handle h, void* const* X, const void* const* G, float* const* M,
                  float* const* Q, void* workspace, size_t workspace_bytes, void* stream);

/* Waits for `stream`, then copies the per-matrix breakdown words of the last step to
 * info_host[nmat]: 0 = fine; k > 0 = the left factor B Q lost rank (or went non-finite) at
 * column k (k = r when the loss only shows as a failed orthogonality check after the first
 * CholeskyQR pass); k < 0 = the same for the right factor (QR) or a zero column (ColNorm)
 * at column -k. */
int orthdion_get_info(orthdion_handle h, int32_t* info_host, void* stream);

/* Waits for `stream`, then copies the per-matrix warning bits of the last step to
 * warn_host[nmat] (host array).  A warning does not invalidate the step: the results are
 * delivered, but with less accuracy than the precision mode promises.  The fast precision
 * reads B = M + G (Alg. 1 line 1) and R (line 3) as fp16 under power-of-two scales that are
 * derived from 32 sampled rows of B; the pass that sees every entry anyway checks the sample.
 *   ORTHDION_WARN_B_CLIPPED     an entry of B exceeded the fp16 range under its scale and was
 *                               clipped in the projection and back-projection
 *   ORTHDION_WARN_R_CLIPPED     the same for an entry of R in the error-feedback product
 *   ORTHDION_WARN_B_SCALE_BLIND every sampled row of B was zero although B is not: no scale
 *                               was applied, small entries may have been flushed
 *   ORTHDION_WARN_WAIT_EXPIRED  a bounded wait inside the Cholesky kernel ran out (a defect,
 *                               not a property of the data); orthdion_get_info reports the
 *                               matrix as broken down as well
 * Exact precision never clips (no scale is involved); its words stay zero. */
#define ORTHDION_WARN_B_CLIPPED 1u
#define ORTHDION_WARN_R_CLIPPED 2u
#define ORTHDION_WARN_B_SCALE_BLIND 4u
#define ORTHDION_WARN_WAIT_EXPIRED 8u
int orthdion_get_warnings(orthdion_handle h, uint32_t* warn_host, void* stream);

/* Debug / test hook: byte offsets inside the workspace of what the last step left for
 * matrix `index`: P (m x r fp32), R (n x r fp32), and the two triangular factors of each
 * CholeskyQR2 orthogonalisation (r x r fp32 each; orth(.)'s triangular factor is
 * t2 * t1).  Any output pointer may be NULL. */
int orthdion_workspace_layout(orthdion_handle h, int32_t index, size_t* off_p, size_t* off_r,
                              size_t* off_tp1, size_t* off_tp2, size_t* off_tq1, size_t* off_tq2);

/* Optional timing of the phases of orthdion_step with HIP events recorded on the step's
 * own stream (host-side resources only; do not use while the stream is being captured into
 * a graph).  A phase with one kernel (PROJ, BACK, EFX) is timed by that dispatch's own start
 * and stop time stamps (the figure a kernel trace reports), the others between two recorded
 * events.
 *   orthdion_profile_begin  brackets every phase whose bit (1u << phase) is set in
 *                           phase_mask, for the next max_steps calls of orthdion_step.
 *   orthdion_profile_end    waits for the recorded events, then writes, per phase, the summed
 *                           elapsed milliseconds and the number of intervals summed (steps x
 *                           shape-class batches) into two arrays of ORTHDION_NPHASE entries.
 * The CHOL and GUARD phases do not depend on m and n and run once for all matrices of one rank
 * r, whatever their shape class: they contribute one interval per step and distinct rank
 * (the GUARD interval is empty for r <= 256, where the guard is part of the FINISH phase).  For
 * r <= 32 the factorisation is part of the first kernel of the ORTH phase that follows (one
 * launch does it together with the triangular product), and the CHOL interval is empty. */
typedef enum {
  ORTHDION_PHASE_STATS = 0,        /* sampled scale of B for the fp16 operand format      */
  ORTHDION_PHASE_PROJ = 1,         /* kernel: P_raw partials = (M + G) Q      (line 2)    */
  ORTHDION_PHASE_PROJ_REDUCE = 2,  /* second stage of the split contraction               */
  ORTHDION_PHASE_GRAM_LEFT = 3,    /* Gram matrix of P_raw                    (line 2)    */
  ORTHDION_PHASE_CHOL_LEFT = 4,    /* its Cholesky factor and inverse; see below          */
  ORTHDION_PHASE_ORTH_LEFT = 5,    /* second CholeskyQR pass of P up to its deviation     */
  ORTHDION_PHASE_GUARD_LEFT = 6,   /* re-factorisation of ill-conditioned matrices, r > 256 */
  ORTHDION_PHASE_FINISH_LEFT = 7,  /* P = orth(P_raw) written out             (line 2)    */
  ORTHDION_PHASE_BACK = 8,         /* kernel: R partials = (M + G)^T P        (line 3)    */
  ORTHDION_PHASE_BACK_REDUCE = 9,
  ORTHDION_PHASE_GRAM_RIGHT = 10,  /* Gram matrix of R (QR variant only)      (line 4)    */
  ORTHDION_PHASE_CHOL_RIGHT = 11,  /* its Cholesky factor and inverse (QR variant only)   */
  ORTHDION_PHASE_ORTH_RIGHT = 12,  /* second pass of Q up to its deviation (QR variant)   */
  ORTHDION_PHASE_GUARD_RIGHT = 13, /* as GUARD_LEFT (QR variant only)                     */
  ORTHDION_PHASE_FINISH_RIGHT = 14,/* Q = orth(R) written out, or ColNorm(R)  (line 4)    */
  ORTHDION_PHASE_EFX = 15,         /* kernel: error feedback + update         (lines 5-7) */
  ORTHDION_NPHASE = 16
} orthdion_phase;
int orthdion_profile_begin(orthdion_handle h, uint32_t phase_mask, int32_t max_steps);
int orthdion_profile_end(orthdion_handle h, float* ms_per_phase, int32_t* count_per_phase);

/* ---- Optional per-step diagnostics (quantities the paper logs: Sec. 4.3 tracking error,
 * Sec. 6.3 R-norm ratio, Prop. 3.1 / Lemma 4.1 dual-norm factor nu, Lemma 4.2 inner product,
 * App. B.2 estimated effective rank).  Off by default; when on, every orthdion_step also
 * enqueues a few extra kernels (one more pass over M and G, one over R, a Gram matrix of
 * the new Q and 128 power iterations on it) that fill a table in the workspace.
 *   orthdion_set_diagnostics  enable != 0 switches them on for the following steps.
 *   orthdion_get_diagnostics  copies the table of the most recent step to the host array
 *                             out_host[nmat][ORTHDION_NDIAG] (matrix order of
 *                             orthdion_create) and synchronises `stream` (the step's stream).
 *                             ORTHDION_E_NO_STEP when the last step ran without diagnostics.
 * Columns of the table (fp32; sums of squares are accumulated in fp64):
 *   B_NORM          ||M_prev + G||_F
 *   R_NORM          ||R||_F = ||P^T B||_F
 *   TRACKING_ERROR  ||(I - P P^T) B||_F / ||B||_F, evaluated as sqrt(||B||^2 - ||R||^2) / ||B||
 *                   (P has orthonormal columns); absolute accuracy about 1e-3 in FAST precision
 *   RESIDUAL_RATIO  ||M_prev||_F / ||G||_F (0 when G = 0)
 *   INNER           <B, P Q^T>: trace of orth(R)'s triangular factor (QR), sum of the column
 *                   lengths of R (ColNorm)
 *   NU              sigma_1(Q_new), from power iteration on Q^T Q (a lower estimate, relative
 *                   error (lambda_2 / lambda_1)^256)
 *   ERANK           exp(-sum p_i log p_i), p_i = ||R[:, i]|| / sum_j ||R[:, j]||
 *   G_NORM          ||G||_F                                                              */
typedef enum {
  ORTHDION_DIAG_B_NORM = 0,
  ORTHDION_DIAG_R_NORM = 1,
  ORTHDION_DIAG_TRACKING_ERROR = 2,
  ORTHDION_DIAG_RESIDUAL_RATIO = 3,
  ORTHDION_DIAG_INNER = 4,
  ORTHDION_DIAG_NU = 5,
  ORTHDION_DIAG_ERANK = 6,
  ORTHDION_DIAG_G_NORM = 7,
  ORTHDION_NDIAG = 8
} orthdion_diag;
int orthdion_set_diagnostics(orthdion_handle h, int32_t enable);
int orthdion_get_diagnostics(orthdion_handle h, float* out_host, void* stream);

/* ---- Adaptive rank (App. B.2, Alg. 2).  Host-only arithmetic:
 *   ema_out = alpha * e_t + (1 - alpha) * ema_prev
 *   r_next  = clip(ceil(gamma * ema_out), r_min, r_max), rounded up to a multiple of 8 and
 *             clipped again (the paper leaves the rounding direction open).
 * e_t is the ERANK diagnostic of the step just taken.  r_min and r_max must be multiples of
 * 8 with 8 <= r_min <= r_max; alpha in [0, 1]; gamma > 0; else ORTHDION_E_INVALID_ARG. */
int orthdion_rank_policy(float e_t, float ema_prev, int32_t r_min, int32_t r_max, float alpha, float gamma,
                         float* ema_out, int32_t* r_next);

/* Rank change of the warm-start factor (Alg. 2: "truncate or pad"): q_new (n x r_new,
 * ld r_new, device) receives the leading min(r_old, r_new) columns of q_old (n x r_old,
 * ld r_old, device); when r_new > r_old the remaining columns are copied from `pad`
 * (n x (r_new - r_old), row-major, device; the caller draws them, e.g. N(0, 1/n); NULL is
 * an error then, since zero columns would make the next projection rank deficient).  The
 * buffers must not overlap.  Only enqueues work on `stream`.  A handle has fixed ranks: after
 * a rank change create a new handle for the new shapes (host-side work only). */
int orthdion_resize_q(const float* q_old, int64_t n, int32_t r_old, float* q_new, int32_t r_new,
                      const float* pad, void* stream);

/* ---- The step without a workspace argument, for callers that cannot allocate device memory
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
 * Identical to orthdion_step, kernels included, except that the workspace is a device array
 * inside the library, ORTHDION_STATIC_SCRATCH_BYTES long (128 MiB; every GPU the library runs
 * on holds it until the process ends).  X, G, M, Q and `stream` as for orthdion_step; the
 * current device must be the one the buffers and the stream belong to.  Calls no allocating
 * routine.  A handle whose orthdion_workspace_bytes exceeds the array (one 4096 x 4096 matrix at
 * r = 256 needs 92 MiB) is refused with ORTHDION_E_WORKSPACE_TOO_SMALL.  All calls on one GPU -
 * from any handle or stream - share the one array: calls that overlap in time on a GPU race;
 * enqueue them on one stream, or order the streams with events.  orthdion_get_info,
 * orthdion_get_diagnostics and orthdion_workspace_layout refer to the array after such a
 * step (offsets then count from its start, which the library does not expose). */
#define ORTHDION_STATIC_SCRATCH_BYTES ((size_t)128 << 20)
size_t orthdion_static_scratch_bytes(void);
int orthdion_step_static(orthdion_handle h, void* const* X, const void* const* G, float* const* M,
                         float* const* Q, void* stream);

const char* orthdion_strerror(int status);

int orthdion_destroy(orthdion_handle h);

#ifdef __cplusplus
}
#endif

#endif /* ORTHDION_H */
