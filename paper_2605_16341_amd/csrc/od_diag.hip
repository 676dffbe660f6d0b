// Optional per-step diagnostics of the Orth-Dion step and the rank-change helper, as HIP
// kernels for gfx950.  All of them are bandwidth-trivial next to the step itself; they favour
// accuracy (fp64 accumulation of sums of squares) and determinism (fixed reduction trees).
//
// Quantities (paper notation in brackets):
//   ||B||_F, ||G||_F, ||M_prev||_F      buffer, gradient, residual norms     (App. J)
//   ||R||_F = ||P^T B||_F               captured energy                      (Alg. 1 line 3)
//   tracking error                      sqrt(||B||^2 - ||R||^2) / ||B||      (Sec. 4.3; P orthonormal)
//   residual ratio                      ||M_prev|| / ||G||   [R-norm ratio]  (Sec. 6.3)
//   inner product <B, P Q^T>            trace of the triangular factor of R (QR, Lemma 4.2),
//                                       sum of column lengths of R (ColNorm)
//   nu = sigma_1(Q)                     dual-norm factor                     (Prop. 3.1, Lemma 4.1)
//   estimated effective rank            exp(entropy of normalised column lengths of R)  (App. B.2)
#include "od_kernels.h"

#include "od_common.h"

namespace od {

#define OD_CHECK_LAUNCH()                       \
  do {                                          \
    hipError_t e_ = hipGetLastError();          \
    if (e_ != hipSuccess) return e_;            \
  } while (0)

// Sum over the workgroup (256 threads) of one double per thread; result valid in thread 0.
OD_DEV double block_sum_256(double v, double* red) {
  const int tid = threadIdx.x;
  __syncthreads();
  red[tid] = v;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (tid < w) red[tid] += red[tid + w];
    __syncthreads();
  }
  return red[0];
}

// ------------------------------------------------------------------------------------
// sums of squares of M_prev, G and B = M_prev + G, one partial triple per workgroup
// ------------------------------------------------------------------------------------
template <bool GBF>
__global__ __launch_bounds__(256) void k_diag_norms(ClassDims d, MatPtrs ptrs, double* dpart) {
  const int z = blockIdx.y, tid = threadIdx.x;
  const float* mp = ptrs.M[z];
  const int n4 = d.n / 4;
  const int64_t groups = (int64_t)d.m * n4;
  double sm = 0.0, sg = 0.0, sb = 0.0;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + tid; idx < groups; idx += (int64_t)gridDim.x * 256) {
    const int64_t i = idx / n4;
    const int j = (int)(idx - i * n4) * 4;
    f32x4 mv = *reinterpret_cast<const f32x4*>(mp + i * d.ldm + j);
    float g[4];
    if constexpr (GBF) {
      u32x2 raw = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint16_t*>(ptrs.G[z]) + i * d.ldg + j);
      g[0] = bf16_lo(raw[0]); g[1] = bf16_hi(raw[0]); g[2] = bf16_lo(raw[1]); g[3] = bf16_hi(raw[1]);
    } else {
      f32x4 raw = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(ptrs.G[z]) + i * d.ldg + j);
      g[0] = raw[0]; g[1] = raw[1]; g[2] = raw[2]; g[3] = raw[3];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const double a = (double)mv[e], b = (double)g[e], c = a + b;
      sm += a * a;
      sg += b * b;
      sb += c * c;
    }
  }
  __shared__ double red[256];
  const double tm = block_sum_256(sm, red);
  const double tg = block_sum_256(sg, red);
  const double tb = block_sum_256(sb, red);
  if (tid == 0) {
    double* o = dpart + ((int64_t)z * kDiagBlocks + blockIdx.x) * 4;
    o[0] = tm; o[1] = tg; o[2] = tb; o[3] = 0.0;
  }
}

// ------------------------------------------------------------------------------------
// column sums of squares of R: partials over slabs of rows, then lengths and their sums
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_diag_colsq(int n, int r, WsArr rr, WsArr part, int slabs) {
  const int z = blockIdx.z, slab = blockIdx.y;
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int per = (n + slabs - 1) / slabs;
  const int r0 = slab * per, r1 = (r0 + per) < n ? (r0 + per) : n;
  if (c >= r) return;
  const float* src = rr.base + (int64_t)z * rr.stride;
  double acc = 0.0;
  for (int i = r0; i < r1; ++i) {
    const double v = (double)src[(int64_t)i * r + c];
    acc += v * v;
  }
  part.base[(int64_t)z * part.stride + (int64_t)slab * r + c] = (float)acc;
}

__global__ __launch_bounds__(256) void k_diag_cols_final(int r, WsArr part, int slabs, double* dacc) {
  const int z = blockIdx.x, tid = threadIdx.x;
  double s2 = 0.0, sl = 0.0, sll = 0.0;
  for (int c = tid; c < r; c += 256) {
    double s = 0.0;
#pragma unroll 8
    for (int k = 0; k < slabs; ++k) s += (double)part.base[(int64_t)z * part.stride + (int64_t)k * r + c];
    s2 += s;
    const double len = sqrt(s);
    sl += len;
    if (len > 0.0) sll += len * log(len);
  }
  __shared__ double red[256];
  const double t2 = block_sum_256(s2, red);
  const double tl = block_sum_256(sl, red);
  const double tll = block_sum_256(sll, red);
  if (tid == 0) {
    double* o = dacc + (int64_t)z * kDaccPerMat;
    o[3] = t2; o[4] = tl; o[5] = tll;
  }
}

// trace of T2 * T1 (both upper triangular): sum of products of the diagonals
__global__ __launch_bounds__(256) void k_diag_trace(int r, WsArr t1, WsArr t2, double* dacc) {
  const int z = blockIdx.x, tid = threadIdx.x;
  const float* a = t1.base + (int64_t)z * t1.stride;
  const float* b = t2.base + (int64_t)z * t2.stride;
  double s = 0.0;
  for (int i = tid; i < r; i += 256) s += (double)a[(int64_t)i * r + i] * (double)b[(int64_t)i * r + i];
  __shared__ double red[256];
  const double t = block_sum_256(s, red);
  if (tid == 0) dacc[(int64_t)z * kDaccPerMat + 6] = t;
}

// copy of the callers' Q (n x r, ld r) into a workspace array
__global__ __launch_bounds__(256) void k_gather_q(int n, int r, MatPtrs ptrs, WsArr out) {
  const int z = blockIdx.y;
  const f32x4* src = reinterpret_cast<const f32x4*>(ptrs.Q[z]);
  f32x4* dst = reinterpret_cast<f32x4*>(out.base + (int64_t)z * out.stride);
  const int64_t n4 = (int64_t)n * r / 4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

// ------------------------------------------------------------------------------------
// largest eigenvalue of the r x r Gram matrix of Q by power iteration; nu = sqrt of it.
// x <- G x / ||x||; after the last product ||G x^|| estimates the eigenvalue from below with
// relative error O((lambda_2 / lambda_1)^(2 k)).
// ------------------------------------------------------------------------------------
constexpr int kPowerThreads = 1024;
constexpr int kPowerMaxR = 2048;          // x kept in LDS

OD_DEV float power_start(int i) { return 1.f + 0.5f * __sinf(0.7f * (float)i); }

// y[i] = scale * sum_j g[i][j] x[j] for rows i = row0 + wave, row0 + wave + nwaves, ... < row1
OD_DEV void power_rows(const float* g, const float* x_lds, int r, int row0, int row1, float scale, float* y) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  for (int i = row0 + wave; i < row1; i += nw) {
    const float* row = g + (int64_t)i * r;
    float acc = 0.f;
    for (int j = lane * 4; j < r; j += 256) {
      f32x4 a = *reinterpret_cast<const f32x4*>(row + j);
      f32x4 b = *reinterpret_cast<const f32x4*>(x_lds + j);
      acc += a[0] * b[0] + a[1] * b[1] + a[2] * b[2] + a[3] * b[3];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) y[i] = acc * scale;
  }
}

OD_DEV float block_sumsq(const float* v, int r, float* red) {
  const int tid = threadIdx.x;
  float s = 0.f;
  for (int i = tid; i < r; i += blockDim.x) s += v[i] * v[i];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  __syncthreads();
  if ((tid & 63) == 0) red[tid >> 6] = s;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += red[w];
  return t;
}

// one workgroup per matrix, all iterations inside (small r: the matrix stays in L2)
__global__ __launch_bounds__(kPowerThreads) void k_power(int r, WsArr gram, int iters, double* dacc) {
  __shared__ __align__(16) float x[kPowerMaxR];
  __shared__ __align__(16) float y[kPowerMaxR];
  __shared__ float red[kPowerThreads / 64];
  const int z = blockIdx.x, tid = threadIdx.x;
  const float* g = gram.base + (int64_t)z * gram.stride;
  for (int i = tid; i < r; i += kPowerThreads) x[i] = power_start(i);
  float lam = 0.f;
  for (int it = 0; it < iters; ++it) {
    const float s = block_sumsq(x, r, red);          // barriers inside: x complete
    const float inv = s > 0.f ? rsqrtf(s) : 0.f;
    power_rows(g, x, r, 0, r, inv, y);
    __syncthreads();
    for (int i = tid; i < r; i += kPowerThreads) x[i] = y[i];
    __syncthreads();
  }
  lam = sqrtf(block_sumsq(x, r, red));
  if (tid == 0) dacc[(int64_t)z * kDaccPerMat + 7] = (double)lam;
}

// large r: one launch per iteration, rows spread over workgroups; xin / xout ping-pong
__global__ __launch_bounds__(256) void k_power_init(int r, WsArr xbuf) {
  const int z = blockIdx.y;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < r) xbuf.base[(int64_t)z * xbuf.stride + i] = power_start(i);
}
__global__ __launch_bounds__(256) void k_power_step(int r, WsArr gram, WsArr xbuf, int src_half, int rows_per_wg) {
  __shared__ __align__(16) float x[kPowerMaxR];
  __shared__ float red[4];
  const int z = blockIdx.y, tid = threadIdx.x;
  const float* g = gram.base + (int64_t)z * gram.stride;
  const float* xin = xbuf.base + (int64_t)z * xbuf.stride + (int64_t)src_half * r;
  float* xout = xbuf.base + (int64_t)z * xbuf.stride + (int64_t)(src_half ^ 1) * r;
  for (int i = tid; i < r; i += 256) x[i] = xin[i];
  const float s = block_sumsq(x, r, red);
  const float inv = s > 0.f ? rsqrtf(s) : 0.f;
  const int row0 = blockIdx.x * rows_per_wg;
  const int row1 = (row0 + rows_per_wg) < r ? (row0 + rows_per_wg) : r;
  power_rows(g, x, r, row0, row1, inv, xout);
}
__global__ __launch_bounds__(256) void k_power_final(int r, WsArr xbuf, int src_half, double* dacc) {
  __shared__ float red[4];
  const int z = blockIdx.x;
  const float* x = xbuf.base + (int64_t)z * xbuf.stride + (int64_t)src_half * r;
  const float s = block_sumsq(x, r, red);
  if (threadIdx.x == 0) dacc[(int64_t)z * kDaccPerMat + 7] = (double)sqrtf(s);
}

// ------------------------------------------------------------------------------------
// the reported scalars, one thread per matrix
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_diag_final(int nb, const double* dpart, const double* dacc, int colnorm, float* diag) {
  const int z = blockIdx.x * 64 + threadIdx.x;
  if (z >= nb) return;
  double sm = 0.0, sg = 0.0, sb = 0.0;
  for (int k = 0; k < kDiagBlocks; ++k) {
    const double* p = dpart + ((int64_t)z * kDiagBlocks + k) * 4;
    sm += p[0]; sg += p[1]; sb += p[2];
  }
  const double* a = dacc + (int64_t)z * kDaccPerMat;
  const double r2 = a[3], sl = a[4], sll = a[5];
  float* o = diag + (int64_t)z * kDiagPerMat;
  const double gap = sb - r2;
  o[0] = (float)sqrt(sb);
  o[1] = (float)sqrt(r2);
  o[2] = sb > 0.0 ? (float)sqrt((gap > 0.0 ? gap : 0.0) / sb) : 0.f;
  o[3] = sg > 0.0 ? (float)sqrt(sm / sg) : 0.f;
  o[4] = (float)(colnorm ? sl : a[6]);
  o[5] = (float)sqrt(a[7]);
  o[6] = sl > 0.0 ? (float)exp(log(sl) - sll / sl) : 0.f;
  o[7] = (float)sqrt(sg);
}

// ------------------------------------------------------------------------------------
// rank change of the warm-start factor: keep the leading columns, append caller-supplied ones
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_resize_q(const float* q_old, int64_t n, int r_old, float* q_new, int r_new,
                                                  const float* pad) {
  const int64_t total = n * r_new;
  const int keep = r_old < r_new ? r_old : r_new;
  const int extra = r_new - keep;
  for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
    const int64_t i = idx / r_new;
    const int c = (int)(idx - i * r_new);
    q_new[idx] = c < keep ? q_old[i * r_old + c] : pad[i * extra + (c - keep)];
  }
}

// ------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------
hipError_t launch_diag_norms(const ClassDims& d, const MatPtrs& ptrs, double* dpart, hipStream_t st) {
  if (d.g_bf16) hipLaunchKernelGGL(k_diag_norms<true>, dim3(kDiagBlocks, d.nb), dim3(256), 0, st, d, ptrs, dpart);
  else hipLaunchKernelGGL(k_diag_norms<false>, dim3(kDiagBlocks, d.nb), dim3(256), 0, st, d, ptrs, dpart);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_diag_cols(int nb, int n, int r, WsArr rr, WsArr part, int slabs, double* dacc, hipStream_t st) {
  hipLaunchKernelGGL(k_diag_colsq, dim3((r + 255) / 256, slabs, nb), dim3(256), 0, st, n, r, rr, part, slabs);
  OD_CHECK_LAUNCH();
  hipLaunchKernelGGL(k_diag_cols_final, dim3(nb), dim3(256), 0, st, r, part, slabs, dacc);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_diag_trace(int nb, int r, WsArr t1, WsArr t2, double* dacc, hipStream_t st) {
  hipLaunchKernelGGL(k_diag_trace, dim3(nb), dim3(256), 0, st, r, t1, t2, dacc);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_gather_q(int nb, int n, int r, const MatPtrs& ptrs, WsArr out, hipStream_t st) {
  int64_t n4 = (int64_t)n * r / 4;
  int blocks = (int)((n4 + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(k_gather_q, dim3(blocks, nb), dim3(256), 0, st, n, r, ptrs, out);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_power(int nb, int r, WsArr gram, WsArr xbuf, int iters, double* dacc, hipStream_t st) {
  if (r > kPowerMaxR || xbuf.stride < 2 * (int64_t)r) return hipErrorInvalidValue;
  if (r <= 512) {
    hipLaunchKernelGGL(k_power, dim3(nb), dim3(kPowerThreads), 0, st, r, gram, iters, dacc);
    OD_CHECK_LAUNCH();
    return hipSuccess;
  }
  hipLaunchKernelGGL(k_power_init, dim3((r + 255) / 256, nb), dim3(256), 0, st, r, xbuf);
  OD_CHECK_LAUNCH();
  const int rows_per_wg = 8;
  int half = 0;
  for (int it = 0; it < iters; ++it) {
    hipLaunchKernelGGL(k_power_step, dim3((r + rows_per_wg - 1) / rows_per_wg, nb), dim3(256), 0, st, r, gram, xbuf, half, rows_per_wg);
    OD_CHECK_LAUNCH();
    half ^= 1;
  }
  hipLaunchKernelGGL(k_power_final, dim3(nb), dim3(256), 0, st, r, xbuf, half, dacc);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_diag_final(int nb, const double* dpart, const double* dacc, int colnorm, float* diag, hipStream_t st) {
  hipLaunchKernelGGL(k_diag_final, dim3((nb + 63) / 64), dim3(64), 0, st, nb, dpart, dacc, colnorm, diag);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_resize_q(const float* q_old, int64_t n, int r_old, float* q_new, int r_new, const float* pad, hipStream_t st) {
  int64_t total = n * r_new;
  int blocks = (int)((total + 255) / 256);
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(k_resize_q, dim3(blocks), dim3(256), 0, st, q_old, n, r_old, q_new, r_new, pad);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

}  // namespace od
