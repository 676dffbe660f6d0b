// Host-callable launchers of the HIP kernels of the Orth-Dion step (defined in
// od_kernels.hip).  Every launcher only enqueues work on `stream`; none synchronises
// or allocates.  A launch covers the matrices of one shape class (same m, n, r),
// `nb` of them, at most od::kMaxBatch.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace od {

constexpr int kMaxBatchHost = 32;

// Caller-owned buffers of the matrices of one shape class.
struct MatPtrs {
  void* X[kMaxBatchHost];
  const void* G[kMaxBatchHost];
  float* M[kMaxBatchHost];
  float* Q[kMaxBatchHost];
};

enum Prec : int { PREC_F16 = 0, PREC_BF3 = 1 };   // operand format of the big contractions

struct ClassDims {
  int m, n, r, nb;
  int64_t ldx, ldg, ldm;
  int x_bf16, g_bf16;
  int col_fast;        // error-feedback pass: consecutive workgroups walk along a row of tiles (set by its launcher)
};

// A workspace array with one slice per matrix of the class.
struct WsArr {
  float* base;
  int64_t stride;      // elements between consecutive matrices
};

// A workspace array of pre-scaled fp16 operand words, one slice per matrix.
struct HalfArr {
  uint16_t* base;
  int64_t stride;      // elements between consecutive matrices
};

// A launch made conditional, matrix by matrix, on a scale-table word written by an earlier
// kernel of the same stream: matrix z is processed only if
// (scal[z * kScalPerMat + slot] > thr) == (want != 0).  scal == nullptr: unconditional.
struct Pred {
  const float* scal;
  int slot;
  float thr;
  int want;
};

// scal layout per matrix (floats): [1] scale of R, [2] / [3] largest deviation of the
// first-pass Gram matrix of the left / right factor from identity, [8..39] sampled row sums
// of squares of B
constexpr int kScalPerMat = 40;
constexpr int kScalSample = 8;
// info layout per matrix (ints): [0] left-factor breakdown column, [1] right-factor
// breakdown column (1-based, 0 = none), [2] zero-column flag of ColNorm, [3] warning bits
// (results are delivered, but with less accuracy than the precision mode promises)
constexpr int kInfoPerMat = 4;
constexpr int kWarnSlot = 3;
constexpr int kWarnBClipped = 1;       // an entry of B = M + G exceeded the fp16 range under its sampled scale
constexpr int kWarnRClipped = 2;       // the same for R = B^T P
constexpr int kWarnBScaleBlind = 4;    // the sampled rows of B were all zero although B is not
constexpr int kWarnWaitExpired = 8;    // a bounded wait inside the Cholesky kernel ran out
// Second CholeskyQR pass: up to kFirstOrderDeviation (largest entry of the first pass's
// G - I) the pass is the first-order correction I - Phi(E), whose O(E^2) remainder then stays
// near the rounding of the measurement itself; above it, up to kMaxGramDeviation, a second
// factorisation of I + E is run for that matrix; beyond that the matrix is flagged.
constexpr float kFirstOrderDeviation = 1.0e-3f;
constexpr float kMaxGramDeviation = 0.5f;
// smallest ratio of diagonal entries of the first pass's triangular factor (about the
// reciprocal condition number of the factor) that still counts as full rank
constexpr float kMinPivotRatio = 1.0e-3f;

// first kernel of a step in fast precision: clears the matrices' scale words [0..7] and flag
// words, samples sums of squares of B (for its fp16 scale) and writes Q as pre-scaled fp16,
// transposed [r][n]
hipError_t launch_stats(const ClassDims& d, const MatPtrs& ptrs, float* scal, int* info, HalfArr qht, hipStream_t st);

// whether launch_proj (fast precision) works on 64-row tiles for this shape class: the
// caller sizes the number of splits accordingly
bool proj_uses_flat_tiles(int m, int r, int nb);
// whether launch_proj / launch_back (fast precision) take the direct-to-LDS kernel for this shape
// class (128-row tiles, stream_tile_cols(r) columns, one workgroup per CU): the caller sizes
// the number of splits accordingly
bool stream_kernel_eligible(const ClassDims& d);
int stream_tile_cols(int r);
// P_raw partials: part[split][m][r] = (M+G)[:, k-range] * Q[k-range, :]
hipError_t launch_proj(const ClassDims& d, const MatPtrs& ptrs, Prec prec, const float* scal,
                       WsArr part, int splits, HalfArr qht, hipStream_t st);
// R partials: part[split][n][r] = (M+G)[k-range, :]^T * P[k-range, :]
// Where back_writes_fp16_copy holds (fast precision, one split, the direct-to-LDS kernel) and
// `rh`, `info` are given, the launch also writes R as pre-scaled fp16 and checks its range, and
// launch_reduce_r is not needed.
bool back_writes_fp16_copy(const ClassDims& d, Prec prec, int splits);
hipError_t launch_back(const ClassDims& d, const MatPtrs& ptrs, Prec prec, const float* scal,
                       WsArr p, WsArr part, int splits, HalfArr pht, hipStream_t st, HalfArr rh = HalfArr{nullptr, 0},
                       int* info = nullptr);
// out[i] = sum_s part[s * count + i], i < count, per matrix
hipError_t launch_reduce(int nb, WsArr part, int splits, int64_t count, WsArr out, hipStream_t st, Pred pred = Pred{nullptr, 0, 0.f, 0});
// the same for R (n x r), also written as pre-scaled fp16 [n][r]; with one split `part` may be
// `out` itself (the back-projection wrote R in place): then only the fp16 copy is written
hipError_t launch_reduce_r(const ClassDims& d, WsArr part, int splits, WsArr out, HalfArr rh, const float* scal, int* info, hipStream_t st);

// Gram partials: part[split][r][r] = A[k-range, :]^T A[k-range, :], A is rows x r (ld r)
// Operand format (`mode`): kGramBF2 / kGramBF3 two- / three-way split bf16 (3 / 6 products,
// 16 / 24 bits), kGramH2 two-term scaled fp16 (3 products, 22 bits).  kGramH2 needs the
// operand's scale: `side` 0 = P_raw, 1 = R (scale derived from the sampled scale of B in
// `scal`, shape in `d`), 2 = a nearly orthonormal factor (fixed scale, d and scal unused).
enum : int { kGramBF2 = 0, kGramBF3 = 1, kGramH2 = 2 };
hipError_t launch_gram(int nb, int rows, int r, WsArr a, WsArr part, int splits, int mode, hipStream_t st,
                       const ClassDims* d = nullptr, const float* scal = nullptr, int side = -1);
// out = A * W, A rows x r, W r x r upper triangular (both ld r); the result goes to the
// callers' Q buffers when q_ptrs is given, else to the workspace array `out`.
// With hn.base / ht.base non-null the result is also stored as fp16 scaled by 2^10, in
// natural [rows][r] and transposed [r][rows] layout.
hipError_t launch_apply(int nb, int rows, int r, WsArr a, WsArr w, WsArr out, const MatPtrs* q_ptrs, HalfArr hn,
                        HalfArr ht, int exact, hipStream_t st, Pred pred = Pred{nullptr, 0, 0.f, 0});
// out = A - A * Phi with Phi upper triangular and small (the first-order second pass of
// CholeskyQR2): A enters in fp32, the correction is a single fp16 product.  `phit` is Phi^T as
// fp16 scaled by 2^13, [r][r] per matrix (written by launch_corr).  Outputs as above.
hipError_t launch_apply_correction(int nb, int rows, int r, WsArr a, HalfArr phit, WsArr out, const MatPtrs* q_ptrs,
                                   HalfArr hn, HalfArr ht, hipStream_t st, Pred pred = Pred{nullptr, 0, 0.f, 0});

// Cholesky factor and its inverse of the SPD r x r matrices `gram` (ld r): gram = T^T T,
// W = T^-1, both upper triangular with zeros below the diagonal.  The matrices need not belong
// to one shape class: the work depends on r only, so one call serves every matrix of that
// rank.  For r <= 256 one workgroup per matrix does everything; above, the factorisation is
// blocked, `gram` is destroyed and `tmp` is r x r scratch.  A non-positive or non-finite pivot
// writes its 1-based column to info[mat * kInfoPerMat + info_slot] (first failure wins); the
// factors of such a matrix are unspecified (they may hold NaN).
// With `splits` > 1 (r <= 256 only) `gram` holds that many partial sums per matrix, `split_stride`
// elements apart, which the factorisation adds up itself.
hipError_t launch_cholinv(int nb, int r, WsArr gram, WsArr t, WsArr w, WsArr tmp, int* info, int info_slot,
                          hipStream_t st, Pred pred = Pred{nullptr, 0, 0.f, 0}, int splits = 1, int64_t split_stride = 0);

// r <= 32: Cholesky factor and inverse of `gram`, A1 = A0 W1 and the Gram partials of A1
// (`splits` of them, r x r each, in `part`) in one launch; T1 and W1 are written as by
// launch_cholinv, a bad pivot is reported the same way.
// `gram` holds `gram_splits` partial sums per matrix, r * r elements apart (launch_small_gram).
hipError_t launch_small_first_pass(int nb, int rows, int r, WsArr a0, WsArr gram, int gram_splits, WsArr t1, WsArr w1, WsArr a1,
                                   WsArr part, int splits, int* info, int info_slot, hipStream_t st);
// r <= 32: Gram partials of A0 in plain fp32, part[split][r][r]
hipError_t launch_small_gram(int nb, int rows, int r, WsArr a0, WsArr part, int splits, hipStream_t st);

// First-order second pass: from the Gram partials of a nearly orthonormal matrix writes
// T2 = I + Phi(E), and either W2 = I - Phi(E) (fp32) or, with phit.base non-null, Phi(E)^T as
// fp16 scaled by 2^13 ([r][r], stride phit.stride) instead; max |E| into scal[mat][scal_slot]
// (must be zeroed); a deviation above kMaxGramDeviation (or NaN) is a breakdown:
// info[mat][info_slot] = r unless already set.
// Also reads the diagonal of the first pass's factor `t1`: a ratio of its smallest to its
// largest entry below kMinPivotRatio reports the matrix as numerically rank deficient.
hipError_t launch_corr(int nb, int r, WsArr part, int splits, WsArr t1, WsArr t2, WsArr w2, HalfArr phit, float* scal,
                       int scal_slot, int* info, int info_slot, hipStream_t st);

// scal[mat][1] = power-of-two scale for R from trace(gram) = ||R||_F^2 (rows n, cols r)
hipError_t launch_scale_from_trace(int nb, int n, int r, WsArr gram, float* scal, hipStream_t st);

// ColNorm: Q[:, c] = R[:, c] / ||R[:, c]||; also writes the scale of R.  `part` holds
// slabs x r partial sums per matrix, `colsq` r reciprocal lengths per matrix.
hipError_t launch_colnorm(int nb, int n, int r, WsArr rr, const MatPtrs& ptrs, WsArr part, int slabs, WsArr colsq,
                          float* scal, int* info, HalfArr qh, hipStream_t st);

// M_new = a (M+G) - b P R^T ;  X_new = X - lr P Q^T   (one pass over M, G, X)
// A matrix whose info words report a breakdown keeps its X and gets M_new = a (M + G): its
// factors are unspecified and must not reach the caller's state.
hipError_t launch_efx(const ClassDims& d, const MatPtrs& ptrs, Prec prec, const float* scal, const int* info, WsArr p,
                      WsArr rr, float a_coef, float b_coef, float lr, hipStream_t st);

// the same pass from the pre-scaled fp16 factors (fast precision); also checks every entry of
// B against its sampled fp16 scale and sets the warning bits of `info`
hipError_t launch_efx_h(const ClassDims& d, const MatPtrs& ptrs, const float* scal, int* info, HalfArr ph, HalfArr rh,
                        HalfArr qh, float a_coef, float b_coef, float lr, hipStream_t st);

// ---- optional diagnostics (od_diag.hip) ----
constexpr int kDiagPerMat = 8;     // floats reported per matrix
constexpr int kDaccPerMat = 8;     // fp64 accumulators per matrix: [3] ||R||^2, [4] sum of column lengths of R,
                                   // [5] sum of len * log(len), [6] trace of the right triangular factor, [7] lambda_max
constexpr int kDiagBlocks = 128;   // workgroups (partial triples of 4 doubles) per matrix of the norm pass

// dpart[mat][kDiagBlocks][4] = partial sums of squares of M, G, M + G
hipError_t launch_diag_norms(const ClassDims& d, const MatPtrs& ptrs, double* dpart, hipStream_t st);
// column lengths of R (n x r, ld r) -> dacc[mat][3..5]; `part` needs slabs * r floats per matrix
hipError_t launch_diag_cols(int nb, int n, int r, WsArr rr, WsArr part, int slabs, double* dacc, hipStream_t st);
// dacc[mat][6] = sum_i t1[i][i] * t2[i][i]
hipError_t launch_diag_trace(int nb, int r, WsArr t1, WsArr t2, double* dacc, hipStream_t st);
// out[mat] = callers' Q (n x r)
hipError_t launch_gather_q(int nb, int n, int r, const MatPtrs& ptrs, WsArr out, hipStream_t st);
// dacc[mat][7] = largest eigenvalue of the symmetric PSD r x r matrix `gram` after `iters` power
// iterations; xbuf needs 2 r floats per matrix (used for r > 512)
hipError_t launch_power(int nb, int r, WsArr gram, WsArr xbuf, int iters, double* dacc, hipStream_t st);
// diag[mat][0..7] = ||B||, ||R||, tracking error, ||M_prev|| / ||G||, <B, P Q^T>, nu, effective rank, ||G||
hipError_t launch_diag_final(int nb, const double* dpart, const double* dacc, int colnorm, float* diag, hipStream_t st);
// q_new (n x r_new) = leading min(r_old, r_new) columns of q_old, then columns of pad (n x (r_new - r_old))
hipError_t launch_resize_q(const float* q_old, int64_t n, int r_old, float* q_new, int r_new, const float* pad, hipStream_t st);

// The next launch_proj / launch_back / launch_efx / launch_efx_h of this thread records the
// start and stop time stamps of its kernel in the two events (one shot).
void time_next_launch(hipEvent_t start, hipEvent_t stop);

hipError_t launch_fill_int(int* p, int64_t count, int value, hipStream_t st);
hipError_t launch_fill_f32(float* p, int64_t count, float value, hipStream_t st);

}  // namespace od
