// HIP kernels of the Orth-Dion optimizer step for gfx950 (CDNA4) and their launchers.
//
// Notation follows the library interface: B = M + G (paper Alg. 1 line 1, never stored),
// P_raw = B Q (line 2), P = orth(P_raw) (line 2), R = B^T P (line 3), Q = orth(R) or
// ColNorm(R) (line 4), X -= lr P Q^T (lines 5-6), M = a B - b P R^T (line 7).
#include "od_kernels.h"

#include <hip/hip_ext.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "od_chol.h"
#include "od_dma.h"
#include "od_gemm.h"

namespace od {

static_assert(kMaxBatchHost == kMaxBatch, "batch limit");

// ------------------------------------------------------------------------------------
// tile shapes
// ------------------------------------------------------------------------------------
typedef Tile<128, 256, 32, 2, 2> TileWide;     // r > 128: wave tile 64 x 128
typedef Tile<128, 128, 32, 2, 2> TileSquare;   // wave tile 64 x 64
typedef Tile<128, 64, 32, 4, 1> TileNarrow;    // r <= 64: wave tile 32 x 64
typedef Tile<64, 256, 32, 2, 2> TileFlat;      // projection, r > 128: twice the row panels, half the splits (wave tile 32 x 128)
typedef Tile<256, 256, 32, 2, 2> TileHuge;    // back-projection, r > 256: wave tile 128 x 128, one workgroup per CU
typedef Tile<128, 128, 64, 2, 2> TileSquareDeepK;   // single-part operands: half the k steps at the same LDS footprint
typedef Tile<64, 64, 64, 2, 2> TileSmall;      // wave tile 32 x 32: small problems that need many workgroups

typedef short s16x4 __attribute__((ext_vector_type(4)));    // result of the LDS transpose read
constexpr float kUnitScale = 1024.f;           // scale of orthonormal / unit-column factors in fp16

OD_DEV bool pred_on(const Pred& p, int z) {
  if (p.scal == nullptr) return true;
  return (p.scal[z * kScalPerMat + p.slot] > p.thr) == (p.want != 0);
}

OD_DEV int split_begin(int K, int splits, int KT, int s, int* kend) {
  int per = ((K + splits - 1) / splits + KT - 1) / KT * KT;
  int kb = s * per;
  int ke = kb + per;
  *kend = ke < K ? ke : K;
  return kb;
}

template <class GSrc>
OD_DEV SrcSum<GSrc> make_b_source(const ClassDims& d, const MatPtrs& ptrs, int z) {
  SrcSum<GSrc> s;
  s.m = SrcF32{ptrs.M[z], d.m, d.n, d.ldm};
  s.g = GSrc{reinterpret_cast<decltype(GSrc::p)>(ptrs.G[z]), d.m, d.n, d.ldg};
  return s;
}

// ------------------------------------------------------------------------------------
// sampled power-of-two scale of B for the fp16 operand format
// ------------------------------------------------------------------------------------
OD_DEV float pow2_scale_for_rms(float ms) {
  if (ms > 0.f && ms < 3.0e38f) return ldexpf(1.f, -ilogbf(sqrtf(ms)));
  return 1.f;
}

constexpr int kStatRows = 32;      // sampled rows per matrix, one workgroup each

template <class GSrc>
OD_DEV void stats_block(const ClassDims& d, const MatPtrs& ptrs, float* scal, int z) {
  const int tid = threadIdx.x;
  SrcSum<GSrc> b = make_b_source<GSrc>(d, ptrs, z);
  const int nrows = d.m < kStatRows ? d.m : kStatRows;
  float acc = 0.f;
  const int groups = d.n / 8;
  if ((int)blockIdx.x < nrows)
  for (int idx = tid; idx < groups; idx += 256) {
    int s = blockIdx.x, c = idx * 8;
    int row = (int)(((int64_t)s * d.m) / nrows);
    float x[8];
    SrcSum<GSrc>::unpack8(b.load8(row, c), x);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc += x[i] * x[i];
  }
  __shared__ float red[256];
  red[tid] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (tid < w) red[tid] += red[tid + w];
    __syncthreads();
  }
  if (tid == 0) scal[z * kScalPerMat + kScalSample + blockIdx.x] = red[0];
}

// Q (n x r fp32, the caller's state) -> pre-scaled fp16, transposed to [r][n]
OD_DEV void prep_q_block(const ClassDims& d, const MatPtrs& ptrs, HalfArr qht, int z, int bx, int by) {
  __shared__ uint16_t tile[64][66];
  const int tid = threadIdx.x;
  const int k0 = bx * 64, c0 = by * 64;       // k over n, c over r
  const float* q = ptrs.Q[z];
  uint16_t* out = qht.base + (int64_t)z * qht.stride;
  for (int idx = tid; idx < 64 * 16; idx += 256) {            // 64 rows (k) x 16 groups of 4 columns
    const int kk = idx / 16, cg = (idx % 16) * 4;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (k0 + kk < d.n && c0 + cg < d.r) v = *reinterpret_cast<const f32x4*>(q + (int64_t)(k0 + kk) * d.r + c0 + cg);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      _Float16 x = (_Float16)__builtin_amdgcn_fmed3f(v[e] * kUnitScale, -65504.f, 65504.f);
      tile[cg + e][kk] = __builtin_bit_cast(uint16_t, x);
    }
  }
  __syncthreads();
  for (int idx = tid; idx < 64 * 16; idx += 256) {            // 64 rows (c) x 16 groups of 4 k
    const int cc = idx / 16, kg = (idx % 16) * 4;
    if (c0 + cc < d.r && k0 + kg < d.n) {
      u32x2 h = {(uint32_t)tile[cc][kg] | ((uint32_t)tile[cc][kg + 1] << 16),
                 (uint32_t)tile[cc][kg + 2] | ((uint32_t)tile[cc][kg + 3] << 16)};
      *reinterpret_cast<u32x2*>(out + (int64_t)(c0 + cc) * d.n + k0 + kg) = h;
    }
  }
}

// First kernel of a step in fast precision, one launch for three small jobs: workgroups
// 0 .. kStatRows-1 of a matrix sample the scale of B (the first of them also clears the
// matrix's flag and scale words), the others convert Q.
template <class GSrc>
__global__ __launch_bounds__(256) void k_prologue(ClassDims d, MatPtrs ptrs, float* scal, int* info, HalfArr qht) {
  const int z = blockIdx.y, bx = blockIdx.x;
  if (bx < kStatRows) {
    if (bx == 0) {
      if (threadIdx.x < kScalSample) scal[z * kScalPerMat + threadIdx.x] = 0.f;
      if (threadIdx.x < kInfoPerMat) info[z * kInfoPerMat + threadIdx.x] = 0;
    }
    stats_block<GSrc>(d, ptrs, scal, z);
  } else {
    const int t = bx - kStatRows, tiles_k = (d.n + 63) / 64;
    prep_q_block(d, ptrs, qht, z, t % tiles_k, t / tiles_k);
  }
}

// scale of B from the sampled row sums of squares (same value in every consumer)
OD_DEV float b_scale(const ClassDims& d, const float* scal, int z) {
  const int nrows = d.m < kStatRows ? d.m : kStatRows;
  // all kStatRows slots are written (zero beyond nrows): fixed-size vector loads, no loop-carried latency
  const f32x4* p = reinterpret_cast<const f32x4*>(scal + z * kScalPerMat + kScalSample);
  f32x4 acc4 = p[0];
#pragma unroll
  for (int i = 1; i < kStatRows / 4; ++i) acc4 += p[i];
  const float tot = (acc4[0] + acc4[1]) + (acc4[2] + acc4[3]);
  return pow2_scale_for_rms(tot / ((float)nrows * (float)d.n));
}

// ------------------------------------------------------------------------------------
// P_raw = B Q  (split over n)                                       Alg. 1 line 2
// ------------------------------------------------------------------------------------
// scale of R = B^T P in fp16: P is orthonormal, so rms(R) <= rms(B) sqrt(m / r); a power of
// two derived from the scale of B alone, known before R exists
OD_DEV float r_scale(const ClassDims& d, const float* scal, int z) {
  return ldexpf(b_scale(d, scal, z), -(ilogbf((float)d.m / (float)d.r) / 2));
}

// Second argument of __launch_bounds__ (waves per SIMD the register allocation must allow;
// with 4-wave workgroups that is workgroups per CU).  Register stages of a deep prefetch on
// top of 8 accumulator tiles, or 16 accumulator tiles alone, need more than 256 registers.
template <class T, int PF>
constexpr int min_waves_per_simd() { return ((PF > 1 && T::FM * T::FN >= 8) || T::FM * T::FN >= 16) ? 1 : 2; }

template <class T, class Num, class GSrc, int PF>
__global__ __launch_bounds__(T::THREADS, (min_waves_per_simd<T, PF>())) void k_proj(ClassDims d, MatPtrs ptrs, const float* scal, WsArr part, int splits, HalfArr qht, int rotate) {
  extern __shared__ __align__(16) char lds[];
  const int tiles_n = (d.r + T::NT - 1) / T::NT;
  // the column tiles of one row panel read the same part of B: keep them on one XCD
  const int bid = tiles_n > 1 ? xcd_contiguous(blockIdx.x, gridDim.x) : blockIdx.x;
  const int tn = bid % tiles_n, tm = bid / tiles_n;
  const int split = blockIdx.y, z = blockIdx.z;
  SrcSum<GSrc> a = make_b_source<GSrc>(d, ptrs, z);
  SrcF32 b{ptrs.Q[z], d.n, d.r, d.r};
  int kend;
  const int kbeg = split_begin(d.n, splits, T::KT, split, &kend);
  const float sa = Num::F16 ? b_scale(d, scal, z) : 1.f;
  const float sb = Num::F16 ? kUnitScale : 1.f;
  f32x16 acc[T::FM][T::FN];
  zero_acc<T>(acc);
  if constexpr (Num::F16) {
    // Q as pre-scaled fp16, transposed to [r][n] so that k is contiguous
    SrcH16 bh{qht.base + (int64_t)z * qht.stride, d.r, d.n, d.n};
    // Row panels of one matrix read the same columns of B at the same time, and with a row
    // stride that is a multiple of the memory-channel interleave they all land on the same
    // channels: start every panel at a different k step then.
    if constexpr (PF > 1)
      gemm_mainloop_deep<T, Num, KC, SrcSum<GSrc>, KC, SrcH16, PF>(a, bh, tm * T::MT, tn * T::NT, kbeg, kend, sa, sb, lds, acc, rotate ? tm : 0);
    else
      gemm_mainloop<T, Num, KC, SrcSum<GSrc>, KC, SrcH16>(a, bh, tm * T::MT, tn * T::NT, kbeg, kend, sa, sb, lds, acc, rotate ? tm : 0);
  } else {
    gemm_mainloop<T, Num, KC, SrcSum<GSrc>, KS, SrcF32>(a, b, tm * T::MT, tn * T::NT, kbeg, kend, sa, sb, lds, acc);
  }
  const float inv = 1.f / (sa * sb);
  float* out = part.base + (int64_t)z * part.stride + (int64_t)split * d.m * d.r;
  for_each_acc<T>(acc, tm * T::MT, tn * T::NT, [&](int row, int col, float v) {
    if (row < d.m && col < d.r) out[(int64_t)row * d.r + col] = v * inv;
  });
}

// ------------------------------------------------------------------------------------
// R = B^T P  (split over m)                                         Alg. 1 line 3
// ------------------------------------------------------------------------------------
template <class T, class Num, class GSrc, int PF>
__global__ __launch_bounds__(T::THREADS, (min_waves_per_simd<T, PF>())) void k_back(ClassDims d, MatPtrs ptrs, const float* scal, WsArr p, WsArr part, int splits, HalfArr pht) {
  extern __shared__ __align__(16) char lds[];
  const int tiles_n = (d.r + T::NT - 1) / T::NT;
  // as in the projection: the column tiles of one panel of B share an XCD's L2
  const int bid = tiles_n > 1 ? xcd_contiguous(blockIdx.x, gridDim.x) : blockIdx.x;
  const int tn = bid % tiles_n, tm = bid / tiles_n;
  const int split = blockIdx.y, z = blockIdx.z;
  SrcSum<GSrc> a = make_b_source<GSrc>(d, ptrs, z);      // read as [k = row i][operand row = column j]
  SrcF32 b{p.base + (int64_t)z * p.stride, d.m, d.r, d.r};
  int kend;
  const int kbeg = split_begin(d.m, splits, T::KT, split, &kend);
  const float sa = Num::F16 ? b_scale(d, scal, z) : 1.f;
  const float sb = Num::F16 ? kUnitScale : 1.f;
  f32x16 acc[T::FM][T::FN];
  zero_acc<T>(acc);
  if constexpr (Num::F16) {
    SrcH16 bh{pht.base + (int64_t)z * pht.stride, d.r, d.m, d.m};      // P^T as fp16, [r][m]
    if constexpr (PF > 1)
      gemm_mainloop_deep<T, Num, KS, SrcSum<GSrc>, KC, SrcH16, PF>(a, bh, tm * T::MT, tn * T::NT, kbeg, kend, sa, sb, lds, acc);
    else
      gemm_mainloop<T, Num, KS, SrcSum<GSrc>, KC, SrcH16>(a, bh, tm * T::MT, tn * T::NT, kbeg, kend, sa, sb, lds, acc);
  } else {
    gemm_mainloop<T, Num, KS, SrcSum<GSrc>, KS, SrcF32>(a, b, tm * T::MT, tn * T::NT, kbeg, kend, sa, sb, lds, acc);
  }
  const float inv = 1.f / (sa * sb);
  float* out = part.base + (int64_t)z * part.stride + (int64_t)split * d.n * d.r;
  for_each_acc<T>(acc, tm * T::MT, tn * T::NT, [&](int row, int col, float v) {
    if (row < d.n && col < d.r) out[(int64_t)row * d.r + col] = v * inv;
  });
}

// ------------------------------------------------------------------------------------
// deterministic second stage of the split contractions
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_reduce(WsArr part, int splits, int64_t count, WsArr out, Pred pred) {
  const int z = blockIdx.y;
  if (!pred_on(pred, z)) return;
  const float* src = part.base + (int64_t)z * part.stride;
  float* dst = out.base + (int64_t)z * out.stride;
  const int64_t n4 = count / 4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
    f32x4 s = reinterpret_cast<const f32x4*>(src)[i];
#pragma unroll 8
    for (int k = 1; k < splits; ++k) {       // unrolled: the loads of eight partials are in flight together
      f32x4 v = reinterpret_cast<const f32x4*>(src + (int64_t)k * count)[i];
      s += v;
    }
    reinterpret_cast<f32x4*>(dst)[i] = s;
  }
}

// the same for R, which is also stored as pre-scaled fp16 for the error-feedback kernel
__global__ __launch_bounds__(256) void k_reduce_r(ClassDims d, WsArr part, int splits, WsArr out, HalfArr rh, const float* scal, int* info) {
  const int z = blockIdx.y;
  const float* src = part.base + (int64_t)z * part.stride;
  float* dst = out.base + (int64_t)z * out.stride;
  uint16_t* dh = rh.base + (int64_t)z * rh.stride;
  const int64_t count = (int64_t)d.n * d.r, n4 = count / 4;
  const float sr = r_scale(d, scal, z);
  float rmax = 0.f;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
    f32x4 s = reinterpret_cast<const f32x4*>(src)[i];
#pragma unroll 8
    for (int k = 1; k < splits; ++k) s += reinterpret_cast<const f32x4*>(src + (int64_t)k * count)[i];
    if (dst != src) reinterpret_cast<f32x4*>(dst)[i] = s;     // in place (one split): only the fp16 copy is new
    u32x2 h = {pack_f16_sat(s[0] * sr, s[1] * sr), pack_f16_sat(s[2] * sr, s[3] * sr)};
    reinterpret_cast<u32x2*>(dh)[i] = h;
    rmax = fmaxf(rmax, fmaxf(fmaxf(fabsf(s[0]), fabsf(s[1])), fmaxf(fabsf(s[2]), fabsf(s[3]))));
  }
  // a clipped entry (or a NaN) is reported, not hidden
  if (!(rmax * sr <= 65504.f)) atomicOr(&info[z * kInfoPerMat + kWarnSlot], kWarnRClipped);
}

// ------------------------------------------------------------------------------------
// Gram matrix A^T A (split over rows)                 CholeskyQR for orth(), Alg. 1 l. 2, 4
// ------------------------------------------------------------------------------------
// Power-of-two scale of a Gram operand in the two-term fp16 format.  side 0: P_raw = B Q, whose
// rms is at most rms(B) sqrt(n / r) for an orthonormal Q; side 1: R = B^T P, at most
// rms(B) sqrt(m / r); both brought to about 2^6 .. 2^7, which leaves 2^9 of headroom for
// entries above the rms and saturates beyond.  side 2: a nearly orthonormal factor (entries
// at most about one): 2^12.
constexpr float kGramUnitScale = 4096.f;
OD_DEV float gram_operand_scale(const ClassDims& d, const float* scal, int side, int z) {
  if (side == 2) return kGramUnitScale;
  const float sb = b_scale(d, scal, z);
  const float ratio = side == 0 ? (float)d.n / (float)d.r : (float)d.m / (float)d.r;
  return ldexpf(sb, 6 - ilogbf(ratio) / 2);
}

template <class T, class Num>
__global__ __launch_bounds__(T::THREADS) void k_gram(int rows, int r, WsArr a, WsArr part, int splits, ClassDims d, const float* scal, int side) {
  static_assert(T::MT == T::NT, "the tile grid of a symmetric result must be symmetric");
  extern __shared__ __align__(16) char lds[];
  const int tiles = (r + T::NT - 1) / T::NT;
  // The result is symmetric: only the tiles (tm, tn) with tm <= tn are computed, row by row
  // of the tile grid, and an off-diagonal tile is stored a second time, transposed.
  // All tiles of one row split read the same rows of A.  Workgroups go to the 8 XCDs round robin
  // by their flattened index; each XCD gets one contiguous range of the order (matrix, split,
  // tile), so those tiles run under one L2 and A comes from HBM once.  (Taken per matrix, 20
  // workgroups spread over all XCDs: the counters showed three times the input fetched.)
  const int per_z = (int)gridDim.x * (int)gridDim.y;
  const int flat = xcd_contiguous((int)blockIdx.x + (int)gridDim.x * ((int)blockIdx.y + (int)gridDim.y * (int)blockIdx.z),
                                  per_z * (int)gridDim.z);
  const int z = flat / per_z, logical = flat - z * per_z;
  int tm = 0, tn = logical % (int)gridDim.x;
  while (tn >= tiles - tm) { tn -= tiles - tm; ++tm; }
  tn += tm;
  const int split = logical / (int)gridDim.x;
  SrcF32 s{a.base + (int64_t)z * a.stride, rows, r, r};
  int kend;
  const int kbeg = split_begin(rows, splits, T::KT, split, &kend);
  f32x16 acc[T::FM][T::FN];
  zero_acc<T>(acc);
  const float sc = Num::F16 ? gram_operand_scale(d, scal, side, z) : 1.f;
  gemm_mainloop_deep<T, Num, KSF, SrcF32, KSF, SrcF32, 3>(s, s, tm * T::MT, tn * T::NT, kbeg, kend, sc, sc, lds, acc);
  if constexpr (Num::F16) {
    const float inv = 1.f / (sc * sc);
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
      for (int fn = 0; fn < T::FN; ++fn)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[fm][fn][v] *= inv;
  }
  float* out = part.base + (int64_t)z * part.stride + (int64_t)split * r * r;
  for_each_acc<T>(acc, tm * T::MT, tn * T::NT, [&](int row, int col, float v) {
    if (row < r && col < r) out[(int64_t)row * r + col] = v;
  });
  if (tm != tn) {
    // lane (c, h) holds rows 8q + 4h .. 8q + 4h + 3 of column c: four consecutive entries of
    // row c of the transposed tile (r is a multiple of 8, so they are inside or outside together)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / T::WN, wn = wave % T::WN;
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
      for (int fn = 0; fn < T::FN; ++fn) {
        const int col = tn * T::NT + wn * T::WTN + fn * 32 + (lane & 31);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row0 = tm * T::MT + wm * T::WTM + fm * 32 + 8 * q + 4 * (lane >> 5);
          if (col < r && row0 < r) {
            const f32x4 v4 = {acc[fm][fn][4 * q], acc[fm][fn][4 * q + 1], acc[fm][fn][4 * q + 2], acc[fm][fn][4 * q + 3]};
            *reinterpret_cast<f32x4*>(out + (int64_t)col * r + row0) = v4;
          }
        }
      }
  }
}

// ------------------------------------------------------------------------------------
// out = A W with W upper triangular (the triangular solve of CholeskyQR as a product
// with the explicit inverse factor)
//
// CORR: the second pass of CholeskyQR2 in correction form.  `w` holds Phi(E) (entries far
// below one) and the result is A - A Phi: the product is a small correction of A, so one fp16
// product (A scaled by 2^10, Phi by 2^13: relative error 2^-11 of a term of size |E|) is
// enough, and A itself enters in full fp32 precision.
// ------------------------------------------------------------------------------------
constexpr float kPhiScale = 8192.f;
template <class T, class Num, bool DEEP, bool CORR>
__global__ __launch_bounds__(T::THREADS) void k_apply(int rows, int r, WsArr a, WsArr w, HalfArr wh, WsArr out, MatPtrs ptrs,
                                                      int to_q, HalfArr hn, HalfArr ht, Pred pred) {
  extern __shared__ __align__(16) char lds[];
  if (!pred_on(pred, blockIdx.z)) return;
  const int tiles_n = (r + T::NT - 1) / T::NT;
  // the column tiles of one row panel of A share an XCD's L2
  const int bid = tiles_n > 1 ? xcd_contiguous(blockIdx.x, gridDim.x) : blockIdx.x;
  const int tn = bid % tiles_n, tm = bid / tiles_n;
  const int z = blockIdx.z;
  SrcF32 sa{a.base + (int64_t)z * a.stride, rows, r, r};
  SrcF32 sw{w.base + (int64_t)z * w.stride, r, r, r};
  int kend = (tn + 1) * T::NT;          // W[k][j] = 0 for k > j
  if (kend > r) kend = r;
  f32x16 acc[T::FM][T::FN];
  zero_acc<T>(acc);
  if constexpr (CORR) {
    // Phi arrives as ready operand words (fp16, scaled, transposed to [column][k]): its tiles go
    // to LDS as they are, without the transposition and conversion a fp32 source needs
    SrcH16 swh{wh.base + (int64_t)z * wh.stride, r, r, r};
    if constexpr (DEEP) gemm_mainloop_deep<T, Num, KC, SrcF32, KC, SrcH16, 3>(sa, swh, tm * T::MT, tn * T::NT, 0, kend, kUnitScale, 1.f, lds, acc);
    else gemm_mainloop<T, Num, KC, SrcF32, KC, SrcH16>(sa, swh, tm * T::MT, tn * T::NT, 0, kend, kUnitScale, 1.f, lds, acc);
  } else {
    if constexpr (DEEP) gemm_mainloop_deep<T, Num, KC, SrcF32, KS, SrcF32, 3>(sa, sw, tm * T::MT, tn * T::NT, 0, kend, 1.f, 1.f, lds, acc);
    else gemm_mainloop<T, Num, KC, SrcF32, KS, SrcF32>(sa, sw, tm * T::MT, tn * T::NT, 0, kend, 1.f, 1.f, lds, acc);
  }
  if constexpr (CORR) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave / T::WN, wn = wave % T::WN;
    constexpr float inv = 1.f / (kUnitScale * kPhiScale);
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
      for (int fn = 0; fn < T::FN; ++fn)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = tm * T::MT + wm * T::WTM + fm * 32 + acc_row(v, lane);
          const int col = tn * T::NT + wn * T::WTN + fn * 32 + acc_col(lane);
          const float a1 = (row < rows && col < r) ? sa.p[(int64_t)row * r + col] : 0.f;
          acc[fm][fn][v] = a1 - inv * acc[fm][fn][v];
        }
  }
  float* dst = to_q ? ptrs.Q[z] : out.base + (int64_t)z * out.stride;
  for_each_acc<T>(acc, tm * T::MT, tn * T::NT, [&](int row, int col, float v) {
    if (row < rows && col < r) dst[(int64_t)row * r + col] = v;
  });
  // pre-scaled fp16 copies of the (orthonormal) result for the large contractions
  if (hn.base != nullptr) {
    uint16_t* h = hn.base + (int64_t)z * hn.stride;
    for_each_acc<T>(acc, tm * T::MT, tn * T::NT, [&](int row, int col, float v) {
      if (row < rows && col < r) {
        _Float16 x = (_Float16)__builtin_amdgcn_fmed3f(v * kUnitScale, -65504.f, 65504.f);
        h[(int64_t)row * r + col] = __builtin_bit_cast(uint16_t, x);
      }
    });
  }
  if (ht.base != nullptr) {     // transposed [r][rows]: 4 consecutive rows of one column per store
    uint16_t* h = ht.base + (int64_t)z * ht.stride;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / T::WN, wn = wave % T::WN;
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
      for (int fn = 0; fn < T::FN; ++fn) {
        const int col = tn * T::NT + wn * T::WTN + fn * 32 + (lane & 31);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row = tm * T::MT + wm * T::WTM + fm * 32 + 8 * q + 4 * (lane >> 5);
          if (col < r && row < rows) {
            u32x2 hv = {pack_f16_sat(acc[fm][fn][4 * q] * kUnitScale, acc[fm][fn][4 * q + 1] * kUnitScale),
                        pack_f16_sat(acc[fm][fn][4 * q + 2] * kUnitScale, acc[fm][fn][4 * q + 3] * kUnitScale)};
            *reinterpret_cast<u32x2*>(h + (int64_t)col * rows + row) = hv;
          }
        }
      }
  }
}

// ------------------------------------------------------------------------------------
// r <= 32: the first CholeskyQR pass in one launch.  At this size every kernel of the pass is
// a few microseconds of latency, so three of them become one: every workgroup factors the
// (reduced) Gram matrix for itself in its first wave (one 32 x 32 tile, padded with the
// identity), applies W = T^-1 to its share of the rows in plain fp32 and leaves the Gram
// partial of the rows it has just produced for the second pass.  Workgroup 0 of a matrix also
// writes T1 and W1.  One thread per row; `part` receives `splits` partial sums of r x r.
// ------------------------------------------------------------------------------------
constexpr int kSmallRows = 256, kSmallPitch = 36;

// Sum of a^T a over the 64 rows a wave owns of the tile S ([rows][kSmallPitch], 32 columns) on
// the matrix cores: fp32 32x32x2 products with both operands the same register (lane (c, h)
// feeds row 2i + h, column c).
OD_DEV f32x16 small_gram_rows(const float* S, int wave, int lane, f32x16 acc) {
  const float* sw = S + (wave * 64 + (lane >> 5)) * kSmallPitch + (lane & 31);
#pragma unroll 8
  for (int i = 0; i < 32; ++i) {
    const float a = sw[2 * i * kSmallPitch];
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, a, acc, 0, 0, 0);
  }
  return acc;
}
// The four waves' tiles summed through S (then [wave][32][kSmallPitch]) and stored as r x r.
OD_DEV void small_gram_store(float* S, const f32x16& acc, int r, float* out, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int v = 0; v < 16; ++v) S[(wave * 32 + acc_row(v, lane)) * kSmallPitch + (lane & 31)] = acc[v];
  __syncthreads();
  const int gi = tid >> 3, gj = 4 * (tid & 7);
  f32x4 g = *reinterpret_cast<const f32x4*>(S + gi * kSmallPitch + gj);
#pragma unroll
  for (int w = 1; w < 4; ++w) g += *reinterpret_cast<const f32x4*>(S + (w * 32 + gi) * kSmallPitch + gj);
  if (gi < r && gj < r) *reinterpret_cast<f32x4*>(out + (int64_t)gi * r + gj) = g;
}

// r <= 32: Gram partials A^T A of `splits` row ranges, one thread per row, in plain fp32.
__global__ __launch_bounds__(kSmallRows) void k_small_gram(int rows, int r, WsArr a0, WsArr part, int splits) {
  __shared__ __align__(16) float S[kSmallRows * kSmallPitch];
  const int z = blockIdx.y, split = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int kend;
  const int kbeg = split_begin(rows, splits, 8, split, &kend);
  const float* A = a0.base + (int64_t)z * a0.stride;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  for (int base = kbeg; base < kend; base += kSmallRows) {
    const int row = base + tid;
#pragma unroll
    for (int j4 = 0; j4 < 8; ++j4) {
      f32x4 v4 = {0.f, 0.f, 0.f, 0.f};
      if (row < kend && 4 * j4 < r) v4 = *reinterpret_cast<const f32x4*>(A + (int64_t)row * r + 4 * j4);
      *reinterpret_cast<f32x4*>(S + tid * kSmallPitch + 4 * j4) = v4;
    }
    __syncthreads();
    acc = small_gram_rows(S, wave, lane, acc);
    __syncthreads();
  }
  small_gram_store(S, acc, r, part.base + (int64_t)z * part.stride + (int64_t)split * r * r, tid);
}

__global__ __launch_bounds__(kSmallRows) void k_small_first_pass(int rows, int r, WsArr a0, WsArr gram, int gram_splits, WsArr t1,
                                                                WsArr w1, WsArr a1, WsArr part, int splits, int* info,
                                                                int info_slot) {
  __shared__ __align__(16) float Wl[32 * kSmallPitch];           // W[k][j]
  __shared__ __align__(16) float S[kSmallRows * kSmallPitch];    // the rows of a1 of one pass
  const int z = blockIdx.y, split = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (wave == 0) {
    const float* G = gram.base + (int64_t)z * gram.stride;
    const int c = lane & 31, h = lane >> 5;
    // accumulator layout (lane = column c, registers = rows) read through the mirrored element
    // of the symmetric matrix: four consecutive entries of row c
    f32x16 d, zt;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int gi = 8 * q + 4 * h;
      f32x4 v4 = {0.f, 0.f, 0.f, 0.f};
      if (c < r && gi < r) {
        // `gram_splits` partial sums, r * r apart, added in order
#pragma unroll 8
        for (int sp = 0; sp < gram_splits; ++sp) v4 += *reinterpret_cast<const f32x4*>(G + (int64_t)sp * r * r + (int64_t)c * r + gi);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) d[4 * q + e] = (c < r && gi < r) ? v4[e] : ((gi + e == c) ? 1.f : 0.f);
    }
    const int bad = diag_tile_factor(d, zt, lane);
    if (bad != 0 && lane == 0) atomicCAS(&info[z * kInfoPerMat + info_slot], 0, bad);
    // zt = M with W = M^T: lane c holds row c of W
#pragma unroll
    for (int v = 0; v < 16; ++v) Wl[c * kSmallPitch + acc_row(v, lane)] = zt[v];
    if (split == 0 && c < r) {
      float* tp = t1.base + (int64_t)z * t1.stride;
      float* wp = w1.base + (int64_t)z * w1.stride;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int gi = 8 * q + 4 * h;
        if (gi < r) {
#pragma unroll
          for (int e = 0; e < 4; ++e) tp[(int64_t)(gi + e) * r + c] = d[4 * q + e];
          const f32x4 v4 = {zt[4 * q], zt[4 * q + 1], zt[4 * q + 2], zt[4 * q + 3]};
          *reinterpret_cast<f32x4*>(wp + (int64_t)c * r + gi) = v4;
        }
      }
    }
  }
  int kend;
  const int kbeg = split_begin(rows, splits, 8, split, &kend);
  const float* A = a0.base + (int64_t)z * a0.stride;
  float* O = a1.base + (int64_t)z * a1.stride;
  // Gram of the produced rows, 64 per wave and pass; the four tiles are summed at the end
  f32x16 gacc;
#pragma unroll
  for (int v = 0; v < 16; ++v) gacc[v] = 0.f;
  bool first = true;
  for (int base = kbeg; base < kend; base += kSmallRows) {
    const int row = base + tid;
    const bool valid = row < kend;
    // this thread's row of A waits in its own row of S (which takes the row of a1 further down)
    float* xs = S + tid * kSmallPitch;
#pragma unroll
    for (int j4 = 0; j4 < 8; ++j4) {
      f32x4 v4 = {0.f, 0.f, 0.f, 0.f};
      if (valid && 4 * j4 < r) v4 = *reinterpret_cast<const f32x4*>(A + (int64_t)row * r + 4 * j4);
      *reinterpret_cast<f32x4*>(xs + 4 * j4) = v4;
    }
    // the first rows are requested before the wait for the factorisation
    if (first) { __syncthreads(); first = false; }
    // o = x W, W upper triangular: column block jb takes k <= 4 jb + 3.  Four k per turn of a
    // loop that stays rolled: unrolled, all 144 reads of W were issued ahead of the arithmetic
    // and a quarter of them spilled to scratch memory.
    f32x4 o[8];
#pragma unroll
    for (int jb = 0; jb < 8; ++jb) o[jb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int kb = 0; kb < 8; ++kb) {
      const f32x4 x4 = *reinterpret_cast<const f32x4*>(xs + 4 * kb);
#pragma unroll
      for (int jb = 0; jb < 8; ++jb) {
        if (jb >= kb) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const f32x4 w4 = *reinterpret_cast<const f32x4*>(Wl + (4 * kb + i) * kSmallPitch + 4 * jb);
#pragma unroll
            for (int e = 0; e < 4; ++e) o[jb][e] = fmaf(x4[i], w4[e], o[jb][e]);
          }
        }
      }
    }
#pragma unroll
    for (int jb = 0; jb < 8; ++jb) {
      if (valid && 4 * jb < r) *reinterpret_cast<f32x4*>(O + (int64_t)row * r + 4 * jb) = o[jb];
      *reinterpret_cast<f32x4*>(S + tid * kSmallPitch + 4 * jb) = valid ? o[jb] : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    __syncthreads();
    gacc = small_gram_rows(S, wave, lane, gacc);
    __syncthreads();
  }
  if (first) __syncthreads();          // a workgroup without rows still meets the others' barrier count
  small_gram_store(S, gacc, r, part.base + (int64_t)z * part.stride + (int64_t)split * r * r, tid);
}

// ------------------------------------------------------------------------------------
// small general product on r x r workspace matrices, used by the blocked Cholesky and
// triangular inverse:  C[cr.., cc..] = alpha * A * B + beta * C over Mc x Nc x Kc with
// block origins that advance affinely with the inner batch index q.
// ------------------------------------------------------------------------------------
struct SgemmArgs {
  WsArr a, b, c;
  int r;                 // all three are r x r, ld r
  int a_r0, a_k0, b_k0, b_c0, c_r0, c_c0;
  int q_step;            // every origin advances by q * q_step
  int nq;
  int Mc, Nc, Kc;
  float alpha, beta;
  Pred pred;
};

template <class D> OD_DEV constexpr bool DirA_is_kc() { return false; }
template <> OD_DEV constexpr bool DirA_is_kc<KC>() { return true; }

OD_DEV SrcF32 sub_view(const float* base, int r, int row0, int col0, int rows, int cols) {
  int R = r - row0, C = r - col0;
  if (R > rows) R = rows;
  if (C > cols) C = cols;
  if (R < 0) R = 0;
  if (C < 0) C = 0;
  return SrcF32{base + (int64_t)row0 * r + col0, R, C, r};
}

template <class T, class Num, class DirA>
OD_DEV void sgemm_tile(const SgemmArgs& g, int bx, int bz, char* lds) {
  const int tiles_n = (g.Nc + T::NT - 1) / T::NT;
  const int tn = bx % tiles_n, tm = bx / tiles_n;
  const int q = bz % g.nq, z = bz / g.nq;
  if (!pred_on(g.pred, z)) return;      // uniform over the workgroup: nobody reaches a barrier
  const int o = q * g.q_step;
  const float* ap = g.a.base + (int64_t)z * g.a.stride;
  const float* bp = g.b.base + (int64_t)z * g.b.stride;
  float* cp = g.c.base + (int64_t)z * g.c.stride;
  SrcF32 sa = DirA_is_kc<DirA>() ? sub_view(ap, g.r, g.a_r0 + o, g.a_k0 + o, g.Mc, g.Kc)
                                 : sub_view(ap, g.r, g.a_k0 + o, g.a_r0 + o, g.Kc, g.Mc);
  SrcF32 sb = sub_view(bp, g.r, g.b_k0 + o, g.b_c0 + o, g.Kc, g.Nc);
  f32x16 acc[T::FM][T::FN];
  zero_acc<T>(acc);
  gemm_mainloop_deep<T, Num, DirA, SrcF32, KSF, SrcF32, 3>(sa, sb, tm * T::MT, tn * T::NT, 0, g.Kc, 1.f, 1.f, lds, acc);
  const int cr = g.c_r0 + o, cc = g.c_c0 + o;
  for_each_acc<T>(acc, tm * T::MT, tn * T::NT, [&](int row, int col, float v) {
    if (row < g.Mc && col < g.Nc && cr + row < g.r && cc + col < g.r) {
      float* dst = cp + (int64_t)(cr + row) * g.r + (cc + col);
      float old = g.beta != 0.f ? *dst : 0.f;
      *dst = g.alpha * v + g.beta * old;
    }
  });
}

template <class T, class Num, class DirA>
__global__ __launch_bounds__(T::THREADS) void k_sgemm(SgemmArgs g) {
  extern __shared__ __align__(16) char lds[];
  sgemm_tile<T, Num, DirA>(g, blockIdx.x, blockIdx.z, lds);
}

// Two independent products in one launch (the first `tiles1` workgroups of a matrix work on
// g1, the rest on g2): the blocked factorisation is a chain of short launches, and pairing
// the products that do not depend on each other shortens it.
template <class T, class Num, class DirA1, class DirA2>
__global__ __launch_bounds__(T::THREADS) void k_sgemm_pair(SgemmArgs g1, SgemmArgs g2, int tiles1) {
  extern __shared__ __align__(16) char lds[];
  if ((int)blockIdx.x < tiles1) sgemm_tile<T, Num, DirA1>(g1, blockIdx.x, blockIdx.z, lds);
  else sgemm_tile<T, Num, DirA2>(g2, blockIdx.x - tiles1, blockIdx.z, lds);
}

// Look-ahead of the blocked factorisation: workgroup 0 of a matrix factors the next diagonal
// block (whose own update has already been applied) while the others apply the rest of the
// current block's trailing update (g1, g2) and finish block column p of the inverse (g3).
// The products run on the first T::THREADS threads of their workgroups; the surplus waves end
// at once (a barrier counts only the waves that are still alive).
template <class T>
__global__ __launch_bounds__(kCholThreads) void k_chol_ahead(CholArgs ca, SgemmArgs g1, SgemmArgs g2, SgemmArgs g3, int tiles1, int tiles2) {
  extern __shared__ __align__(16) char lds[];
  typedef NumBF<3> Num;
  if (blockIdx.x == 0) {
    chol256_block(ca, blockIdx.z, lds);
    return;
  }
  if ((int)threadIdx.x >= T::THREADS) return;
  const int bx = (int)blockIdx.x - 1;
  if (bx < tiles1) sgemm_tile<T, Num, KSF>(g1, bx, blockIdx.z, lds);
  else if (bx < tiles1 + tiles2) sgemm_tile<T, Num, KSF>(g2, bx - tiles1, blockIdx.z, lds);
  else sgemm_tile<T, Num, KC>(g3, bx - tiles1 - tiles2, blockIdx.z, lds);
}

constexpr int kLeaf = kCholMax;   // diagonal block of the blocked factorisation

// ------------------------------------------------------------------------------------
// Second CholeskyQR pass as a first-order correction.  After the first pass the Gram matrix
// is I + E with small E; its Cholesky factor is I + Phi(E) + O(E^2), Phi = strict upper
// triangle + half the diagonal, and the inverse factor I - Phi(E) + O(E^2).  Writes
// T2 = I + Phi(E), W2 = I - Phi(E) and the largest |E| entry (scal[mat][scal_slot]).
// ------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_corr(int r, WsArr part, int splits, WsArr t1, WsArr t2, WsArr w2, HalfArr phit, float* scal,
                                              int scal_slot, int* info, int info_slot) {
  const int z = blockIdx.y;
  const float* src = part.base + (int64_t)z * part.stride;
  float* tp = t2.base + (int64_t)z * t2.stride;
  float* wp = w2.base + (int64_t)z * w2.stride;
  const int64_t count = (int64_t)r * r;
  float emax = 0.f;
  // four consecutive entries of one row per thread (r is a multiple of 8)
  for (int64_t i4 = (int64_t)blockIdx.x * 256 + threadIdx.x; i4 < count / 4; i4 += (int64_t)gridDim.x * 256) {
    const int64_t idx = i4 * 4;
    const int i = (int)(idx / r), j0 = (int)(idx % r);
    f32x4 g = reinterpret_cast<const f32x4*>(src)[i4];
#pragma unroll 8
    for (int sp = 1; sp < splits; ++sp) g += reinterpret_cast<const f32x4*>(src + (int64_t)sp * count)[i4];
    f32x4 to, wo, pt;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int j = j0 + c;
      const float e = (i == j) ? g[c] - 1.f : g[c];
      emax = fmaxf(emax, fabsf(e));
      float phi = 0.f;
      if (j > i) phi = e;
      else if (j == i) phi = 0.5f * e;
      const float id = (i == j) ? 1.f : 0.f;
      to[c] = id + phi;
      wo[c] = id - phi;
      // E is symmetric, so row i of Phi^T (the operand layout [column][k]) is made of the same
      // entries of row i of E, taken below the diagonal instead of above
      float lower = 0.f;
      if (j < i) lower = e;
      else if (j == i) lower = 0.5f * e;
      pt[c] = lower * kPhiScale;
    }
    reinterpret_cast<f32x4*>(tp)[i4] = to;
    if (phit.base == nullptr) {
      reinterpret_cast<f32x4*>(wp)[i4] = wo;
    } else {
      const u32x2 h = {pack_f16_sat(pt[0], pt[1]), pack_f16_sat(pt[2], pt[3])};
      reinterpret_cast<u32x2*>(phit.base + (int64_t)z * phit.stride)[i4] = h;
    }
  }
  __shared__ float red[256];
  red[threadIdx.x] = emax;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + w]);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    float v = red[0];
    if (!(v == v)) v = 3.0e38f;       // NaN -> huge
    atomicMax(reinterpret_cast<int*>(scal + z * kScalPerMat + scal_slot), __float_as_int(v));
    // The first pass left the factor far from orthonormal: the input had (numerically) less
    // than full column rank, which the Cholesky pivots alone do not always show.
    if (v > kMaxGramDeviation) atomicCAS(&info[z * kInfoPerMat + info_slot], 0, r);
  }
  // Numerical rank: the diagonal of the first pass's triangular factor spans the factor's
  // condition number from below.  Beyond about 1 / sqrt(rounding of the Gram matrix) the small
  // pivots are rounding noise - CholeskyQR would return an orthonormal basis of that noise -
  // so such a matrix is reported as rank deficient whatever deviation the noise happened to leave.
  if (blockIdx.x == 0) {
    const float* t = t1.base + (int64_t)z * t1.stride;
    float lo = 3.0e38f, hi = 0.f;
    for (int i = threadIdx.x; i < r; i += 256) {
      const float d = t[(int64_t)i * r + i];
      lo = fminf(lo, d == d ? d : 0.f);
      hi = fmaxf(hi, d);
    }
    __shared__ float rlo[256], rhi[256];
    rlo[threadIdx.x] = lo;
    rhi[threadIdx.x] = hi;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
      if ((int)threadIdx.x < w) {
        rlo[threadIdx.x] = fminf(rlo[threadIdx.x], rlo[threadIdx.x + w]);
        rhi[threadIdx.x] = fmaxf(rhi[threadIdx.x], rhi[threadIdx.x + w]);
      }
      __syncthreads();
    }
    if (threadIdx.x == 0 && !(rlo[0] > kMinPivotRatio * rhi[0])) atomicCAS(&info[z * kInfoPerMat + info_slot], 0, r);
  }
}

// ------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------
// zero the r x r matrices of two per-matrix workspace arrays, all matrices in one launch
__global__ __launch_bounds__(256) void k_zero_pair(WsArr a, WsArr b, int64_t count, Pred pred) {
  const int z = blockIdx.y;
  if (!pred_on(pred, z)) return;
  f32x4* pa = reinterpret_cast<f32x4*>(a.base + (int64_t)z * a.stride);
  f32x4* pb = reinterpret_cast<f32x4*>(b.base + (int64_t)z * b.stride);
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count / 4; i += (int64_t)gridDim.x * 256) {
    pa[i] = zero;
    pb[i] = zero;
  }
}
__global__ __launch_bounds__(256) void k_fill_f32(float* p, int64_t count, float v) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) p[i] = v;
}
__global__ __launch_bounds__(256) void k_fill_i32(int* p, int64_t count, int v) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) p[i] = v;
}


__global__ __launch_bounds__(256) void k_scale_from_trace(int n, int r, WsArr gram, float* scal) {
  const int z = blockIdx.x, tid = threadIdx.x;
  const float* g = gram.base + (int64_t)z * gram.stride;
  float acc = 0.f;
  for (int i = tid; i < r; i += 256) acc += g[(int64_t)i * r + i];
  __shared__ float red[256];
  red[tid] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (tid < w) red[tid] += red[tid + w];
    __syncthreads();
  }
  if (tid == 0) scal[z * kScalPerMat + 1] = pow2_scale_for_rms(red[0] / ((float)n * (float)r));
}

// ColNorm stage 1: partial column sums of squares over a slab of rows (deterministic)
__global__ __launch_bounds__(256) void k_colsq_partial(int n, int r, WsArr rr, WsArr part, int slabs) {
  const int z = blockIdx.z, slab = blockIdx.y;
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int per = (n + slabs - 1) / slabs;
  const int r0 = slab * per, r1 = (r0 + per) < n ? (r0 + per) : n;
  if (c >= r) return;
  const float* src = rr.base + (int64_t)z * rr.stride;
  float acc = 0.f;
  for (int i = r0; i < r1; ++i) {
    float v = src[(int64_t)i * r + c];
    acc += v * v;
  }
  part.base[(int64_t)z * part.stride + (int64_t)slab * r + c] = acc;
}
// stage 2: column lengths, the scale of R, and the zero-column flag
__global__ __launch_bounds__(256) void k_colsq_final(int n, int r, WsArr part, int slabs, WsArr colsq, float* scal, int* info) {
  const int z = blockIdx.x, tid = threadIdx.x;
  float tot = 0.f;
  for (int c = tid; c < r; c += 256) {
    float s = 0.f;
#pragma unroll 8
    for (int k = 0; k < slabs; ++k) s += part.base[(int64_t)z * part.stride + (int64_t)k * r + c];
    tot += s;
    float len = sqrtf(s);
    float inv = 0.f;
    if (len > 1e-30f && len < 3.0e38f) inv = 1.f / len;
    else atomicCAS(&info[z * kInfoPerMat + 2], 0, c + 1);
    colsq.base[(int64_t)z * colsq.stride + c] = inv;
  }
  __shared__ float red[256];
  red[tid] = tot;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (tid < w) red[tid] += red[tid + w];
    __syncthreads();
  }
  if (tid == 0) scal[z * kScalPerMat + 1] = pow2_scale_for_rms(red[0] / ((float)n * (float)r));
}
// stage 3: Q = R * diag(1/len)
__global__ __launch_bounds__(256) void k_colnorm_apply(int n, int r, WsArr rr, WsArr colsq, MatPtrs ptrs, HalfArr qh) {
  const int z = blockIdx.y;
  const float* src = rr.base + (int64_t)z * rr.stride;
  const float* inv = colsq.base + (int64_t)z * colsq.stride;
  float* q = ptrs.Q[z];
  const int64_t n4 = (int64_t)n * r / 4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256) {
    int c = (int)((i * 4) % r);
    f32x4 v = reinterpret_cast<const f32x4*>(src)[i];
    f32x4 s = *reinterpret_cast<const f32x4*>(inv + c);
    f32x4 o = v * s;
    reinterpret_cast<f32x4*>(q)[i] = o;
    if (qh.base != nullptr) {
      u32x2 h = {pack_f16_sat(o[0] * kUnitScale, o[1] * kUnitScale), pack_f16_sat(o[2] * kUnitScale, o[3] * kUnitScale)};
      reinterpret_cast<u32x2*>(qh.base + (int64_t)z * qh.stride)[i] = h;
    }
  }
}

// ------------------------------------------------------------------------------------
// Error feedback and parameter update in one pass over M, G and X:
//   M_new = a (M + G) - b P R^T     (Alg. 1 line 7 / default form)
//   X_new = X - lr P Q^T            (Alg. 1 lines 5-6)
// The products are computed transposed (tile rows = columns j of the matrix) so that each
// lane owns 4 consecutive j of one row i and moves M, G, X with vector accesses.
// ------------------------------------------------------------------------------------
OD_DEV bool matrix_flagged(const int* info, int z) {
  const int* w = info + z * kInfoPerMat;
  return (w[0] | w[1] | w[2]) != 0;
}

// The fast-precision contractions read B = M + G as fp16 under a scale sampled from 32 rows.
// The pass that sees every entry of B anyway (error feedback) checks the sample: `bmax` is the
// largest |B| this lane has met.
OD_DEV void report_b_range(const ClassDims& d, const float* scal, int* info, int z, float bmax) {
  const float sb = b_scale(d, scal, z);
  int warn = 0;
  if (!(bmax * sb <= 65504.f)) warn |= kWarnBClipped;
  if (bmax > 0.f) {
    const f32x4* p = reinterpret_cast<const f32x4*>(scal + z * kScalPerMat + kScalSample);
    f32x4 acc4 = p[0];
#pragma unroll
    for (int i = 1; i < kStatRows / 4; ++i) acc4 += p[i];
    if ((acc4[0] + acc4[1]) + (acc4[2] + acc4[3]) == 0.f) warn |= kWarnBScaleBlind;
  }
  if (warn != 0) atomicOr(&info[z * kInfoPerMat + kWarnSlot], warn);
}

template <class T, class Num, bool XBF, bool GBF>
__global__ __launch_bounds__(T::THREADS) void k_efx(ClassDims d, MatPtrs ptrs, const float* scal, const int* info, WsArr p, WsArr rr,
                                                    float a_coef, float b_coef, float lr) {
  extern __shared__ __align__(16) char lds[];
  const int tiles_i = (d.m + T::NT - 1) / T::NT;
  const int ti = blockIdx.x % tiles_i, tj = blockIdx.x / tiles_i;
  const int z = blockIdx.z;
  SrcF32 sp{p.base + (int64_t)z * p.stride, d.m, d.r, d.r};
  SrcF32 sr{rr.base + (int64_t)z * rr.stride, d.n, d.r, d.r};
  SrcF32 sq{ptrs.Q[z], d.n, d.r, d.r};
  const float s_r = Num::F16 ? scal[z * kScalPerMat + 1] : 1.f;
  const float s_u = Num::F16 ? kUnitScale : 1.f;
  f32x16 acc_r[T::FM][T::FN], acc_q[T::FM][T::FN];
  zero_acc<T>(acc_r);
  zero_acc<T>(acc_q);
  gemm_mainloop<T, Num, KC, SrcF32, KC, SrcF32>(sr, sp, tj * T::MT, ti * T::NT, 0, d.r, s_r, s_u, lds, acc_r);
  gemm_mainloop<T, Num, KC, SrcF32, KC, SrcF32>(sq, sp, tj * T::MT, ti * T::NT, 0, d.r, s_u, s_u, lds, acc_q);
  const float cr = b_coef / (s_r * s_u), cq = lr / (s_u * s_u);
  if (matrix_flagged(info, z)) {        // unspecified factors (possibly NaN) never reach X and M
    zero_acc<T>(acc_r);
    zero_acc<T>(acc_q);
  }

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / T::WN, wn = wave % T::WN;
  float* Mz = ptrs.M[z];
#pragma unroll
  for (int fn = 0; fn < T::FN; ++fn) {
    const int i = ti * T::NT + wn * T::WTN + fn * 32 + (lane & 31);
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm) {
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const int j = tj * T::MT + wm * T::WTM + fm * 32 + 8 * vq + 4 * (lane >> 5);
        if (i < d.m && j < d.n) {
          float g[4], x[4];
          if constexpr (GBF) {
            u32x2 gv = *reinterpret_cast<const u32x2*>(reinterpret_cast<const uint16_t*>(ptrs.G[z]) + (int64_t)i * d.ldg + j);
            g[0] = bf16_lo(gv[0]); g[1] = bf16_hi(gv[0]); g[2] = bf16_lo(gv[1]); g[3] = bf16_hi(gv[1]);
          } else {
            f32x4 gv = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(ptrs.G[z]) + (int64_t)i * d.ldg + j);
            g[0] = gv[0]; g[1] = gv[1]; g[2] = gv[2]; g[3] = gv[3];
          }
          f32x4* mp = reinterpret_cast<f32x4*>(Mz + (int64_t)i * d.ldm + j);
          f32x4 mv = *mp, mo;
#pragma unroll
          for (int e = 0; e < 4; ++e) mo[e] = a_coef * (mv[e] + g[e]) - cr * acc_r[fm][fn][4 * vq + e];
          *mp = mo;
          if constexpr (XBF) {
            u32x2* xp = reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(ptrs.X[z]) + (int64_t)i * d.ldx + j);
            u32x2 xv = *xp;
            x[0] = bf16_lo(xv[0]); x[1] = bf16_hi(xv[0]); x[2] = bf16_lo(xv[1]); x[3] = bf16_hi(xv[1]);
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] -= cq * acc_q[fm][fn][4 * vq + e];
            u32x2 xo;
            xo[0] = pack_bf16_rne(x[0], x[1]);
            xo[1] = pack_bf16_rne(x[2], x[3]);
            *xp = xo;
          } else {
            f32x4* xp = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(ptrs.X[z]) + (int64_t)i * d.ldx + j);
            f32x4 xv = *xp;
#pragma unroll
            for (int e = 0; e < 4; ++e) xv[e] -= cq * acc_q[fm][fn][4 * vq + e];
            *xp = xv;
          }
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------
// The same pass with every factor already in matrix-core format (fp16, pre-scaled by its
// producer): P [m][r], R [n][r], Q [n][r].  Tile: 128 rows i x 128 columns j, 8 waves.
//   * one K loop feeds both products from one P tile;
//   * wave w owns rows 32 (w % 4) .. +31 and the column half 64 (w / 4) .. +63; the R and Q
//     tiles are laid out in LDS so that lane c of the wave's two accumulator blocks holds
//     columns 2c and 2c + 1: every lane moves pairs, every wave instruction moves whole
//     256-byte (M) or 128-byte (G, X) row segments;
//   * all M, G, X values of the lane are requested together after the K loop; two workgroups
//     per CU (16 waves) overlap one's HBM traffic with the other's products.  (Requests
//     issued before the K loop would not overlap it: the loop's waits for its own operand
//     loads complete in issue order, behind the older requests.)
// ------------------------------------------------------------------------------------
// (second bound: four waves per SIMD, i.e. at most 128 registers, so that two of these 8-wave
// workgroups share a CU as the last point above needs)
// streamed once and not needed again before they are evicted anyway: keep them from pushing the
// factor panels out of L2 (used for long K loops, where the panels are re-read by many tiles)
template <bool STREAM, class V>
OD_DEV V ld_stream(const V* p) {
  if constexpr (STREAM) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool STREAM, class V>
OD_DEV void st_stream(V* p, V v) {
  if constexpr (STREAM) __builtin_nontemporal_store(v, p);
  else *p = v;
}

template <bool XBF, bool GBF, bool STREAM>
__global__ __launch_bounds__(512, 4) void k_efx_h(ClassDims d, MatPtrs ptrs, const float* scal, int* info, HalfArr ph, HalfArr rh,
                                               HalfArr qh, float a_coef, float b_coef, float lr) {
  constexpr int TJ = 128, TI = 128, KT = 32, PITCH = KT * 2 + 16, PLANE = 128 * PITCH, BUF = 3 * PLANE;
  extern __shared__ __align__(16) char lds[];
  const int tiles_i = (d.m + TI - 1) / TI;
  int ti = blockIdx.x % tiles_i, tj = blockIdx.x / tiles_i;
  if (d.col_fast) {
    const int tiles_jj = (d.n + TJ - 1) / TJ;
    tj = blockIdx.x % tiles_jj;
    ti = blockIdx.x / tiles_jj;
  }
  if (d.r > 256) {
    // Long K loops re-read the panels of P, R and Q often enough to matter: bands of eight tile
    // columns, row-major inside a band, one contiguous range of that order per XCD, so that the
    // 64 workgroups an XCD holds at a time form an 8 x 8 block of tiles and every panel fetched
    // into its L2 serves eight of them (measured -4 to -5 %; at r = 256 the plain order is 2 us
    // faster).
    const int tiles_j = (d.n + TJ - 1) / TJ;
    const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
    const int band = logical / (tiles_i * 8);
    const int in_band = logical - band * tiles_i * 8;
    const int bw = min(8, tiles_j - band * 8);
    ti = in_band / bw;
    tj = band * 8 + in_band % bw;
  }
  const int z = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wi = wave & 3, wj = wave >> 2, c = lane & 31;
  SrcH16 sp{ph.base + (int64_t)z * ph.stride, d.m, d.r, d.r};
  SrcH16 sr{rh.base + (int64_t)z * rh.stride, d.n, d.r, d.r};
  SrcH16 sq{qh.base + (int64_t)z * qh.stride, d.n, d.r, d.r};
  // loader: thread t brings 16 bytes (8 k) of row t / 4 of each tile
  const int lrow = tid >> 2, lkg = tid & 3;
  const int jj = lrow & 63;
  const int prow = (lrow & 64) + (jj & 1) * 32 + (jj >> 1);     // LDS position of column lrow of the R / Q tiles
  const int off_p = lrow * PITCH + lkg * 16, off_rq = prow * PITCH + lkg * 16;

  f32x16 acc_r[2], acc_q[2];
#pragma unroll
  for (int f = 0; f < 2; ++f)
#pragma unroll
    for (int v = 0; v < 16; ++v) { acc_r[f][v] = 0.f; acc_q[f][v] = 0.f; }

  u32x4 nr = sr.load8(tj * TJ + lrow, lkg * 8), nq = sq.load8(tj * TJ + lrow, lkg * 8), np = sp.load8(ti * TI + lrow, lkg * 8);
  *reinterpret_cast<u32x4*>(lds + off_rq) = nr;
  *reinterpret_cast<u32x4*>(lds + PLANE + off_rq) = nq;
  *reinterpret_cast<u32x4*>(lds + 2 * PLANE + off_p) = np;
  __syncthreads();
  int buf = 0;
  for (int k = 0; k < d.r; k += KT) {
    const bool more = (k + KT) < d.r;
    if (more) {
      nr = sr.load8(tj * TJ + lrow, k + KT + lkg * 8);
      nq = sq.load8(tj * TJ + lrow, k + KT + lkg * 8);
      np = sp.load8(ti * TI + lrow, k + KT + lkg * 8);
    }
    const char* base = lds + buf * BUF;
#pragma unroll
    for (int kk = 0; kk < KT / 16; ++kk) {
      const int off = c * PITCH + (2 * kk + (lane >> 5)) * 16;
      const u32x4 fp = *reinterpret_cast<const u32x4*>(base + 2 * PLANE + (wi * 32) * PITCH + off);
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        const u32x4 fr = *reinterpret_cast<const u32x4*>(base + (wj * 64 + f * 32) * PITCH + off);
        const u32x4 fq = *reinterpret_cast<const u32x4*>(base + PLANE + (wj * 64 + f * 32) * PITCH + off);
        acc_r[f] = mfma_32x32x16<true>(fp, fr, acc_r[f]);
        acc_q[f] = mfma_32x32x16<true>(fp, fq, acc_q[f]);
      }
    }
    if (more) {
      char* nb = lds + (buf ^ 1) * BUF;
      *reinterpret_cast<u32x4*>(nb + off_rq) = nr;
      *reinterpret_cast<u32x4*>(nb + PLANE + off_rq) = nq;
      *reinterpret_cast<u32x4*>(nb + 2 * PLANE + off_p) = np;
    }
    __syncthreads();
    buf ^= 1;
  }

  // ---- epilogue: this lane's 16 rows x 2 adjacent columns, in two halves of 8 rows; within a
  // half every load is issued before the first store
  const int j0 = tj * TJ + 64 * wj + 2 * c;
  float* __restrict__ Mz = ptrs.M[z];
  const char* __restrict__ Gz = reinterpret_cast<const char*>(ptrs.G[z]);
  char* __restrict__ Xz = reinterpret_cast<char*>(ptrs.X[z]);
  constexpr int GE = GBF ? 2 : 4, XE = XBF ? 2 : 4;
  const float s_r = r_scale(d, scal, z);
  const float cr = b_coef / (s_r * kUnitScale), cq = lr / (kUnitScale * kUnitScale);
  if (matrix_flagged(info, z)) {        // unspecified factors (possibly NaN) never reach X and M
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int v = 0; v < 16; ++v) { acc_r[f][v] = 0.f; acc_q[f][v] = 0.f; }
  }
  float bmax = 0.f;
#pragma unroll
  for (int hv = 0; hv < 2; ++hv) {
    f32x2 mv[8], gv[8], xv[8];
    uint32_t gp[8], xp[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int v = 8 * hv + u;
      const int i = ti * TI + 32 * wi + acc_row(v, lane);
      mv[u] = f32x2{0.f, 0.f};
      gp[u] = 0u; xp[u] = 0u; gv[u] = f32x2{0.f, 0.f}; xv[u] = f32x2{0.f, 0.f};
      if (i < d.m && j0 < d.n) {
        mv[u] = ld_stream<STREAM>(reinterpret_cast<const f32x2*>(Mz + (int64_t)i * d.ldm + j0));
        if constexpr (GBF) gp[u] = ld_stream<STREAM>(reinterpret_cast<const uint32_t*>(Gz + ((int64_t)i * d.ldg + j0) * GE));
        else gv[u] = ld_stream<STREAM>(reinterpret_cast<const f32x2*>(Gz + ((int64_t)i * d.ldg + j0) * GE));
        if constexpr (XBF) xp[u] = ld_stream<STREAM>(reinterpret_cast<const uint32_t*>(Xz + ((int64_t)i * d.ldx + j0) * XE));
        else xv[u] = ld_stream<STREAM>(reinterpret_cast<const f32x2*>(Xz + ((int64_t)i * d.ldx + j0) * XE));
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int v = 8 * hv + u;
      const int i = ti * TI + 32 * wi + acc_row(v, lane);
      if (i < d.m && j0 < d.n) {
        f32x2 g = gv[u], x = xv[u];
        if constexpr (GBF) g = f32x2{bf16_lo(gp[u]), bf16_hi(gp[u])};
        if constexpr (XBF) x = f32x2{bf16_lo(xp[u]), bf16_hi(xp[u])};
        f32x2 mo, xo;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const float bval = mv[u][e] + g[e];
          bmax = fmaxf(bmax, fabsf(bval));
          mo[e] = a_coef * bval - cr * acc_r[e][v];
          xo[e] = x[e] - cq * acc_q[e][v];
        }
        st_stream<STREAM>(reinterpret_cast<f32x2*>(Mz + (int64_t)i * d.ldm + j0), mo);
        if constexpr (XBF) st_stream<STREAM>(reinterpret_cast<uint32_t*>(Xz + ((int64_t)i * d.ldx + j0) * XE), pack_bf16_rne(xo[0], xo[1]));
        else st_stream<STREAM>(reinterpret_cast<f32x2*>(Xz + ((int64_t)i * d.ldx + j0) * XE), xo);
      }
    }
  }
  report_b_range(d, scal, info, z, bmax);
}

// ------------------------------------------------------------------------------------
// The same pass with direct-to-LDS operand loads (r a multiple of 32).  Tile: 128 rows i x
// 128 columns j, 4 waves; wave (wi, wj) owns rows 64 wi .. +63 and columns 64 wj .. +63 of BOTH
// products: eight 32 x 32 accumulators (two row blocks x even / odd columns x {P R^T, P Q^T}),
// six LDS operand reads for eight matrix-core products per 16-deep step (0.75 per product,
// against 1.25 with 32 x 64 wave tiles).  Three LDS stages of 32-deep P, R, Q tiles are kept
// in flight by `dma16` (od_dma.h), one barrier per step.  The R / Q rows arrive permuted so
// that operand row rho of parity f is column 2 rho + f: lane c then owns the adjacent columns
// 2c, 2c + 1 and every wave instruction of the epilogue moves whole 256-byte (M) or 128-byte
// (G, X) row segments, as in k_efx_h.  Two workgroups per CU (72 KB of LDS each): one streams
// M, G, X while the other multiplies.
// ------------------------------------------------------------------------------------
template <bool XBF, bool GBF, bool STREAM, int WI>
__global__ __launch_bounds__(128 * WI, (WI == 2 ? 2 : 1)) void k_efx_d(ClassDims d, MatPtrs ptrs, const float* scal, int* info, HalfArr ph,
                                                                     HalfArr rh, HalfArr qh, float a_coef, float b_coef, float lr) {
  constexpr int TI = 64 * WI, TJ = 128, KT = 32, ROWB = KT * 2, ST = 3, NW = 2 * WI;
  constexpr int PLANE = 128 * ROWB, STAGE = 2 * PLANE + TI * ROWB;       // R | Q | P
  constexpr int CPW = (16 + TI / 16) / NW;                    // 1 KB chunks per wave and stage
  extern __shared__ __align__(16) char lds[];
  const int tiles_i = (d.m + TI - 1) / TI;
  int ti = blockIdx.x % tiles_i, tj = blockIdx.x / tiles_i;
  if (d.col_fast) {
    const int tiles_jj = (d.n + TJ - 1) / TJ;
    tj = blockIdx.x % tiles_jj;
    ti = blockIdx.x / tiles_jj;
  }
  if (d.r > 256) {
    // bands of eight tile columns, one contiguous range of that order per XCD (see k_efx_h)
    const int tiles_j = (d.n + TJ - 1) / TJ;
    const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
    const int band = logical / (tiles_i * 8);
    const int in_band = logical - band * tiles_i * 8;
    const int bw = min(8, tiles_j - band * 8);
    ti = in_band / bw;
    tj = band * 8 + in_band % bw;
  }
  const int z = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, c = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = wave % WI, wj = wave / WI;

  // ---- this lane's share of every stage: chunk = 16 LDS rows of one of the three tiles
  const uint16_t* gp[CPW];
  uint32_t loff[CPW];
  const uint32_t lds0 = lds_offset_of(lds);
#pragma unroll
  for (int q = 0; q < CPW; ++q) {
    const int chunk = wave + NW * q;                // 0..7 R, 8..15 Q, 16.. P
    const int which = chunk < 16 ? chunk >> 3 : 2, rel = chunk < 16 ? chunk & 7 : chunk - 16;
    const int row = rel * 16 + (lane >> 2), slot = lane & 3;
    const int kg = slot ^ swz32(row);
    int grow;
    const uint16_t* base;
    if (which == 2) {
      grow = min(ti * TI + row, d.m - 1);
      base = ph.base + (int64_t)z * ph.stride;
    } else {
      const int col = (row & 64) + 2 * (row & 31) + ((row >> 5) & 1);     // LDS row -> tile column
      grow = min(tj * TJ + col, d.n - 1);
      base = (which == 0 ? rh.base + (int64_t)z * rh.stride : qh.base + (int64_t)z * qh.stride);
    }
    gp[q] = base + (int64_t)grow * d.r + kg * 8;
    loff[q] = lds0 + which * PLANE + rel * 1024;
  }
  const int nsteps = d.r / KT;
  auto issue = [&](int step) {
    const uint32_t boff = (uint32_t)(step % ST) * STAGE;
#pragma unroll
    for (int q = 0; q < CPW; ++q) dma16(gp[q] + step * KT, loff[q] + boff);
  };

  f32x16 acc_r[2][2], acc_q[2][2];
#pragma unroll
  for (int fm = 0; fm < 2; ++fm)
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int v = 0; v < 16; ++v) { acc_r[fm][f][v] = 0.f; acc_q[fm][f][v] = 0.f; }

#pragma unroll
  for (int s = 0; s < ST - 1; ++s)
    if (s < nsteps) issue(s);

  const int prow = wi * 64 + c, jrow = wj * 64 + c;
  for (int i = 0; i < nsteps; ++i) {
    // stage i has landed when at most the loads of the one younger stage are outstanding
    if (i + ST - 2 < nsteps) __builtin_amdgcn_s_waitcnt(vmcnt_only((ST - 2) * CPW));
    else __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (i + ST - 1 < nsteps) issue(i + ST - 1);       // into the buffer every wave has finished reading
    const char* base = lds + (i % ST) * STAGE;
#pragma unroll
    for (int kk = 0; kk < KT / 16; ++kk) {
      const int kg = 2 * kk + (lane >> 5);
      u32x4 fp[2], fr[2], fq[2];
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        const int rp = prow + 32 * f, rj = jrow + 32 * f;
        fp[f] = *reinterpret_cast<const u32x4*>(base + 2 * PLANE + rp * ROWB + ((kg ^ swz32(rp)) * 16));
        fr[f] = *reinterpret_cast<const u32x4*>(base + rj * ROWB + ((kg ^ swz32(rj)) * 16));
        fq[f] = *reinterpret_cast<const u32x4*>(base + PLANE + rj * ROWB + ((kg ^ swz32(rj)) * 16));
      }
#pragma unroll
      for (int fm = 0; fm < 2; ++fm)
#pragma unroll
        for (int f = 0; f < 2; ++f) {
          acc_r[fm][f] = mfma_32x32x16<true>(fp[fm], fr[f], acc_r[fm][f]);
          acc_q[fm][f] = mfma_32x32x16<true>(fp[fm], fq[f], acc_q[fm][f]);
        }
    }
  }

  // ---- epilogue: 2 row blocks x 16 rows x 2 adjacent columns per lane, in four parts of 8
  // rows; within a part every load is issued before the first store
  const int j0 = tj * TJ + 64 * wj + 2 * c;
  float* __restrict__ Mz = ptrs.M[z];
  const char* __restrict__ Gz = reinterpret_cast<const char*>(ptrs.G[z]);
  char* __restrict__ Xz = reinterpret_cast<char*>(ptrs.X[z]);
  constexpr int GE = GBF ? 2 : 4, XE = XBF ? 2 : 4;
  const float s_r = r_scale(d, scal, z);
  const float cr = b_coef / (s_r * kUnitScale), cq = lr / (kUnitScale * kUnitScale);
  if (matrix_flagged(info, z)) {        // unspecified factors (possibly NaN) never reach X and M
#pragma unroll
    for (int fm = 0; fm < 2; ++fm)
#pragma unroll
      for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int v = 0; v < 16; ++v) { acc_r[fm][f][v] = 0.f; acc_q[fm][f][v] = 0.f; }
  }
  float bmax = 0.f;
#pragma unroll
  for (int part = 0; part < 4; ++part) {
    const int fm = part >> 1, hv = part & 1;
    f32x2 mv[8], gv[8], xv[8];
    uint32_t gpk[8], xpk[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int v = 8 * hv + u;
      const int i = ti * TI + 64 * wi + 32 * fm + acc_row(v, lane);
      mv[u] = f32x2{0.f, 0.f};
      gpk[u] = 0u; xpk[u] = 0u; gv[u] = f32x2{0.f, 0.f}; xv[u] = f32x2{0.f, 0.f};
      if (i < d.m && j0 < d.n) {
        mv[u] = ld_stream<STREAM>(reinterpret_cast<const f32x2*>(Mz + (int64_t)i * d.ldm + j0));
        if constexpr (GBF) gpk[u] = ld_stream<STREAM>(reinterpret_cast<const uint32_t*>(Gz + ((int64_t)i * d.ldg + j0) * GE));
        else gv[u] = ld_stream<STREAM>(reinterpret_cast<const f32x2*>(Gz + ((int64_t)i * d.ldg + j0) * GE));
        if constexpr (XBF) xpk[u] = ld_stream<STREAM>(reinterpret_cast<const uint32_t*>(Xz + ((int64_t)i * d.ldx + j0) * XE));
        else xv[u] = ld_stream<STREAM>(reinterpret_cast<const f32x2*>(Xz + ((int64_t)i * d.ldx + j0) * XE));
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int v = 8 * hv + u;
      const int i = ti * TI + 64 * wi + 32 * fm + acc_row(v, lane);
      if (i < d.m && j0 < d.n) {
        f32x2 g = gv[u], x = xv[u];
        if constexpr (GBF) g = f32x2{bf16_lo(gpk[u]), bf16_hi(gpk[u])};
        if constexpr (XBF) x = f32x2{bf16_lo(xpk[u]), bf16_hi(xpk[u])};
        f32x2 mo, xo;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const float bval = mv[u][e] + g[e];
          bmax = fmaxf(bmax, fabsf(bval));
          mo[e] = a_coef * bval - cr * acc_r[fm][e][v];
          xo[e] = x[e] - cq * acc_q[fm][e][v];
        }
        st_stream<STREAM>(reinterpret_cast<f32x2*>(Mz + (int64_t)i * d.ldm + j0), mo);
        if constexpr (XBF) st_stream<STREAM>(reinterpret_cast<uint32_t*>(Xz + ((int64_t)i * d.ldx + j0) * XE), pack_bf16_rne(xo[0], xo[1]));
        else st_stream<STREAM>(reinterpret_cast<f32x2*>(Xz + ((int64_t)i * d.ldx + j0) * XE), xo);
      }
    }
  }
  report_b_range(d, scal, info, z, bmax);
}

// ------------------------------------------------------------------------------------
// Projection and back-projection with every global load direct to LDS (fast precision, bf16
// gradients, r >= 128):
//   TRANS = false   out[i][c] = sum_j (M + G)[i][j] Qt[c][j]     P_raw = B Q      (Alg. 1 line 2)
//   TRANS = true    out[j][c] = sum_i (M + G)[i][j] Pt[c][i]     R = B^T P        (Alg. 1 line 3)
// One workgroup (8 waves, 2 x 4) computes 128 output rows x NT columns over a K range; wave
// tile 64 x NT / 4.  Per 32-deep step:
//   * the factor operand (Qt / Pt: fp16 words, k contiguous) arrives by `dma16` in the swizzled
//     layout of od_dma.h, two stages;
//   * the streamed operand arrives raw - the fp32 tile of M and the bf16 tile of G, exactly as
//     they lie in memory - by `dma16` into three staging stages, so two steps of HBM traffic
//     (48 KB per CU) are in flight with no staging registers and no compiler-scheduled waits;
//     all threads then turn one raw stage into fp16 operand words of (M + G) * scale in a
//     double-buffered operand tile while the matrix cores work on the previous one;
//   * TRANS: the operand tile keeps memory's [k = i][j] order and the wave reads its
//     [row = j][8 consecutive k] fragments with the LDS transpose read (`ds_read_b64_tr_b16`:
//     within 16 lanes, lane c receives element c % 4 of the 8 bytes addressed by lanes
//     4 e + c / 4, e = 0..3; so lanes 4 e + q address row k0 + e, columns j0 + 4 q .. + 3, and
//     lane c receives k0 .. k0 + 3 of column j0 + c); rows are 320 bytes apart so that the four
//     rows a half-wave touches fall into different banks.
// One barrier per step.  Waits count loads: per step and wave kCB factor loads, then kNR raw loads.
// ------------------------------------------------------------------------------------
template <bool TRANS, int NT, int SB>
__global__ __launch_bounds__(512, 1) void k_stream_d(ClassDims d, MatPtrs ptrs, const float* scal, WsArr part, int splits, HalfArr fh, HalfArr rh,
                                                  int* info, int rotate) {
  constexpr int MT = 128, KT = 32, ROWB = 64, SR = 3;
  constexpr int FN = NT / 128;                                // 32-column accumulator blocks per wave
  constexpr int B_STAGE = NT * ROWB, RAW_M = MT * KT * 4, RAW_G = MT * KT * 2, RAW_STAGE = RAW_M + RAW_G;
  constexpr int A_PITCH = TRANS ? 320 : ROWB, A_ROWS = TRANS ? KT : MT, A_BYTES = A_ROWS * A_PITCH;
  constexpr int OFF_RAW = SB * B_STAGE, OFF_A = OFF_RAW + SR * RAW_STAGE;
  constexpr int kCB = NT / 16 / 8, kNR = 3;                   // 1 KB chunks per wave: factor stage, raw stage (2 of M, 1 of G)
  extern __shared__ __align__(16) char lds[];
  const int Mdim = TRANS ? d.n : d.m, Kdim = TRANS ? d.m : d.n;
  const int tiles_n = (d.r + NT - 1) / NT;
  // Workgroups go to the 8 XCDs round robin by their flattened index.  Each XCD gets one
  // contiguous range of the order (matrix, split, row panel, column tile): the workgroups that
  // run side by side under one L2 then read the same k range of the same factor operand (and
  // the column tiles of a row panel the same raw tile), instead of 16 different ones.
  const int per_z = (int)gridDim.x * (int)gridDim.y;
  const int logical = xcd_contiguous((int)blockIdx.x + (int)gridDim.x * ((int)blockIdx.y + (int)gridDim.y * (int)blockIdx.z),
                                     per_z * (int)gridDim.z);
  const int z = logical / per_z, in_z = logical - z * per_z;
  const int split = in_z / (int)gridDim.x, bid = in_z - split * (int)gridDim.x;
  const int tn = bid % tiles_n, tm = bid / tiles_n;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  int kend;
  const int kbeg = split_begin(Kdim, splits, KT, split, &kend);
  const int nsteps = kend > kbeg ? (kend - kbeg + KT - 1) / KT : 0;
  // rotated k order (the projection of one matrix whose rows lie a multiple of 32 KB apart):
  // every row panel starts its k range `rotate` steps after the panel before it, otherwise all
  // panels would read the same columns - the same memory channels - in lockstep
  const int rot = (rotate > 0 && nsteps > 0) ? (int)(((int64_t)tm * rotate) % nsteps) : 0;
  auto k_of = [&](int step) {
    int s2 = step + rot;
    if (s2 >= nsteps) s2 -= nsteps;
    return kbeg + s2 * KT;
  };
  const float sa = b_scale(d, scal, z);
  const uint32_t lds0 = lds_offset_of(lds);
  const float* Mz = ptrs.M[z];
  const uint16_t* Gz = reinterpret_cast<const uint16_t*>(ptrs.G[z]);
  const uint16_t* Fz = fh.base + (int64_t)z * fh.stride;      // [r][Kdim]

  // ---- factor operand: chunk = 16 rows (output columns) x 64 bytes
  const uint16_t* fp[kCB];
  uint32_t foff[kCB];
#pragma unroll
  for (int q = 0; q < kCB; ++q) {
    const int chunk = wave + 8 * q;
    const int row = chunk * 16 + (lane >> 2), kg = (lane & 3) ^ swz32(row);
    fp[q] = Fz + (int64_t)min(tn * NT + row, d.r - 1) * Kdim + kg * 8;
    foff[q] = lds0 + chunk * 1024;
  }
  // ---- raw operand: M chunks of 1 KB (not TRANS: 8 rows x 128 B; TRANS: 2 rows x 512 B), G
  // chunks of 1 KB (16 rows x 64 B; 4 rows x 256 B).  Wave w moves M chunks w and w + 8 and G chunk w.
  // Addresses are clamped into the matrix; what lies outside is zeroed at conversion.
  int64_t raw_off[kNR];          // element offset of this lane's 16 bytes at k step 0
  uint32_t roff[kNR];
#pragma unroll
  for (int q = 0; q < kNR; ++q) {
    const bool isg = q == 2;
    const int chunk = isg ? wave : wave + 8 * q;
    int row, col;                // within the tile: row along the matrix's rows, col along its columns
    if (!TRANS) {
      row = isg ? chunk * 16 + (lane >> 2) : chunk * 8 + (lane >> 3);
      col = isg ? (lane & 3) * 8 : (lane & 7) * 4;
    } else {
      row = isg ? chunk * 4 + (lane >> 4) : chunk * 2 + (lane >> 5);
      col = isg ? (lane & 15) * 8 : (lane & 31) * 4;
    }
    // not TRANS: rows are output rows (fixed), columns advance with k; TRANS: the other way round
    const int grow = TRANS ? row : min(tm * MT + row, d.m - 1);
    const int gcol = TRANS ? min(tm * MT + col, d.n - (isg ? 8 : 4)) : col;
    raw_off[q] = (int64_t)grow * (isg ? d.ldg : d.ldm) + gcol;
    roff[q] = lds0 + OFF_RAW + (isg ? RAW_M : 0) + chunk * 1024;
  }
  auto issue_f = [&](int step) {
    const uint32_t boff = (uint32_t)(step % SB) * B_STAGE;
    const int k0 = min(k_of(step), Kdim - KT);                // a clamped step only meets zeros of the other operand
#pragma unroll
    for (int q = 0; q < kCB; ++q) dma16(fp[q] + k0, foff[q] + boff);
  };
  auto issue_raw = [&](int step) {
    const uint32_t boff = (uint32_t)(step % SR) * RAW_STAGE;
    const int k0 = k_of(step);
#pragma unroll
    for (int q = 0; q < kNR; ++q) {
      const bool isg = q == 2;
      int64_t off;
      if (!TRANS) off = raw_off[q] + min(k0, d.n - KT);        // clamped like the factor operand
      else off = raw_off[q] + (int64_t)min(k0, d.m - KT) * (isg ? d.ldg : d.ldm);
      if (isg) dma16(Gz + off, roff[q] + boff);
      else dma16(Mz + off, roff[q] + boff);
    }
  };
  // A step whose k range was clamped re-reads earlier k positions: conversion zeroes every k
  // outside [k0, kend) of the step, and every row / column outside the matrix.
  auto convert = [&](int step) {
    const char* raw = lds + OFF_RAW + (step % SR) * RAW_STAGE;
    char* abuf = lds + OFF_A + (step & 1) * A_BYTES;
    const int k0 = k_of(step);
    const int kld = TRANS ? min(k0, d.m - KT) : min(k0, d.n - KT);       // where the loaded tile really starts
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int e = tid + 512 * h;                             // 16 bytes of M = 4 elements each
      const f32x4 mv = *reinterpret_cast<const f32x4*>(raw + e * 16);
      const u32x2 gv = *reinterpret_cast<const u32x2*>(raw + RAW_M + e * 8);
      int row, col;                                            // tile row along the matrix's rows, column along its columns
      if (!TRANS) { row = e >> 3; col = (e & 7) * 4; }
      else { row = e >> 5; col = (e & 31) * 4; }
      const int kk = (TRANS ? row : col) + kld;                // global k of the first element
      float x[4] = {mv[0] + bf16_lo(gv[0]), mv[1] + bf16_hi(gv[0]), mv[2] + bf16_lo(gv[1]), mv[3] + bf16_hi(gv[1])};
      bool ok;
      if (!TRANS) ok = tm * MT + row < d.m && kk >= k0 && kk < kend;       // k advances in groups of 4 inside multiples of 8
      else ok = kk >= k0 && kk < kend && tm * MT + col < d.n;
      if (!TRANS && tm * MT + row >= d.m) ok = false;
      u32x2 w = {0u, 0u};
      if (ok) { w[0] = pack_f16_sat(x[0] * sa, x[1] * sa); w[1] = pack_f16_sat(x[2] * sa, x[3] * sa); }
      if (!TRANS) {
        const int kg = col >> 3;
        *reinterpret_cast<u32x2*>(abuf + row * ROWB + ((kg ^ swz32(row)) * 16) + (col & 4) * 2) = w;
      } else {
        *reinterpret_cast<u32x2*>(abuf + row * A_PITCH + col * 2) = w;
      }
    }
  };

  f32x16 acc[2][FN];
#pragma unroll
  for (int fm = 0; fm < 2; ++fm)
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[fm][fn][v] = 0.f;

  if (nsteps > 0) {
    issue_raw(0);
    issue_f(0);
    if (nsteps > 1) issue_raw(1);
    if (SB == 3 && nsteps > 1) issue_f(1);
    if (nsteps > 2) issue_raw(2);
    if (nsteps > 2) __builtin_amdgcn_s_waitcnt(vmcnt_only(2 * kNR + (SB == 3 ? kCB : 0)));
    else __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    convert(0);
  }
  const int arow = wm * 64 + (lane & 31), brow = wn * (NT / 4) + (lane & 31);
  for (int i = 0; i < nsteps; ++i) {
    // factor stage i and raw stage i + 1 have landed when only raw stage i + 2 (and, with three
    // factor stages, factor stage i + 1 issued before it) is outstanding
    if (i + 2 < nsteps) __builtin_amdgcn_s_waitcnt(vmcnt_only(kNR + (SB == 3 ? kCB : 0)));
    else __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (i + SB - 1 < nsteps) issue_f(i + SB - 1);
    if (i + 3 < nsteps) issue_raw(i + 3);
    if (i + 1 < nsteps) convert(i + 1);
    const char* ab = lds + OFF_A + (i & 1) * A_BYTES;
    const char* bb = lds + (i % SB) * B_STAGE;
#pragma unroll
    for (int kk = 0; kk < KT / 16; ++kk) {
      const int kg = 2 * kk + (lane >> 5);
      u32x4 af[2], bf[FN];
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        if constexpr (!TRANS) {
          const int r0 = arow + 32 * f;
          af[f] = *reinterpret_cast<const u32x4*>(ab + r0 * ROWB + ((kg ^ swz32(r0)) * 16));
        } else {
          // lane l = 16 b + i: addresses row k = 16 kk + 8 (b >> 1) + i / 4 (+ 4), columns j0 + 16 (b & 1) + 4 (i % 4)
          const int b = lane >> 4, ii = lane & 15;
          const int k = 16 * kk + 8 * (b >> 1) + (ii >> 2);
          const int j = wm * 64 + 32 * f + 16 * (b & 1) + 4 * (ii & 3);
          const char* p0 = ab + k * A_PITCH + j * 2;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p0));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p0 + 4 * A_PITCH));
          const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
          af[f] = u32x4{l2[0], l2[1], h2[0], h2[1]};
        }
      }
#pragma unroll
      for (int f = 0; f < FN; ++f) {
        const int r0 = brow + 32 * f;
        bf[f] = *reinterpret_cast<const u32x4*>(bb + r0 * ROWB + ((kg ^ swz32(r0)) * 16));
      }
#pragma unroll
      for (int fm = 0; fm < 2; ++fm)
#pragma unroll
        for (int fn = 0; fn < FN; ++fn) acc[fm][fn] = mfma_32x32x16<true>(af[fm], bf[fn], acc[fm][fn]);
    }
  }
  const float inv = 1.f / (sa * kUnitScale);
  float* out = part.base + (int64_t)z * part.stride + (int64_t)split * Mdim * d.r;
#pragma unroll
  for (int fm = 0; fm < 2; ++fm)
#pragma unroll
    for (int fn = 0; fn < FN; ++fn)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = tm * MT + wm * 64 + fm * 32 + acc_row(v, lane);
        const int col = tn * NT + wn * (NT / 4) + fn * 32 + acc_col(lane);
        if (row < Mdim && col < d.r) out[(int64_t)row * d.r + col] = acc[fm][fn][v] * inv;
      }
  // A single split of the back-projection is R itself: its pre-scaled fp16 copy (what
  // k_reduce_r would make in a pass of its own) is written here, with the same range check.
  if (TRANS && rh.base != nullptr) {
    const float sr = r_scale(d, scal, z) * inv;
    uint16_t* dh = rh.base + (int64_t)z * rh.stride;
    float rmax = 0.f;
#pragma unroll
    for (int fm = 0; fm < 2; ++fm)
#pragma unroll
      for (int fn = 0; fn < FN; ++fn)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = tm * MT + wm * 64 + fm * 32 + acc_row(v, lane);
          const int col = tn * NT + wn * (NT / 4) + fn * 32 + acc_col(lane);
          if (row < Mdim && col < d.r) {
            const float x = acc[fm][fn][v] * sr;
            rmax = fmaxf(rmax, fabsf(x));
            dh[(int64_t)row * d.r + col] = __builtin_bit_cast(uint16_t, (_Float16)__builtin_amdgcn_fmed3f(x, -65504.f, 65504.f));
          }
        }
    if (!(rmax <= 65504.f)) atomicOr(&info[z * kInfoPerMat + kWarnSlot], kWarnRClipped);
  }
}

// ====================================================================================
// launchers
// ====================================================================================
#define OD_CHECK_LAUNCH()                       \
  do {                                          \
    hipError_t e_ = hipGetLastError();          \
    if (e_ != hipSuccess) return e_;            \
  } while (0)

// One-shot timing of the next streaming kernel (projection, back-projection, error feedback):
// the events receive the start and stop time stamps of the dispatch itself, without the
// gaps around separately recorded events.
static thread_local hipEvent_t g_time_start = nullptr, g_time_stop = nullptr;
void time_next_launch(hipEvent_t start, hipEvent_t stop) { g_time_start = start; g_time_stop = stop; }

template <class K, class... Args>
static void launch_timed(K kernel, dim3 grid, dim3 block, int lds, hipStream_t st, Args... args) {
  if (g_time_start != nullptr) {
    hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, st, g_time_start, g_time_stop, 0u, args...);
    g_time_start = nullptr;
    g_time_stop = nullptr;
  } else {
    hipLaunchKernelGGL(kernel, grid, block, lds, st, args...);
  }
}

// Development switch: ORTHDION_KERNELS="efx=old,..." selects the previous kernel of a phase,
// so that two generations can be timed in one process.  Unset in normal use.
static bool kernel_choice(const char* phase, const char* value) {
  const char* env = std::getenv("ORTHDION_KERNELS");
  if (env == nullptr) return false;
  char key[64];
  std::snprintf(key, sizeof(key), "%s=%s", phase, value);
  return std::strstr(env, key) != nullptr;
}

template <class K>
static hipError_t allow_lds(K kernel, int bytes) {
  if (bytes > 64 * 1024) return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  return hipSuccess;
}

hipError_t launch_fill_int(int* p, int64_t count, int value, hipStream_t st) {
  if (count <= 0) return hipSuccess;
  int blocks = (int)((count + 255) / 256);
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(k_fill_i32, dim3(blocks), dim3(256), 0, st, p, count, value);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_fill_f32(float* p, int64_t count, float v, hipStream_t st) {
  if (count <= 0) return hipSuccess;
  int blocks = (int)((count + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(k_fill_f32, dim3(blocks), dim3(256), 0, st, p, count, v);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_stats(const ClassDims& d, const MatPtrs& ptrs, float* scal, int* info, HalfArr qht, hipStream_t st) {
  const dim3 grid(kStatRows + ((d.n + 63) / 64) * ((d.r + 63) / 64), d.nb);
  if (d.g_bf16) hipLaunchKernelGGL(k_prologue<SrcBF16>, grid, dim3(256), 0, st, d, ptrs, scal, info, qht);
  else hipLaunchKernelGGL(k_prologue<SrcF32>, grid, dim3(256), 0, st, d, ptrs, scal, info, qht);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

template <class T, class Num, class GSrc, int PF = 1>
static hipError_t proj_t(const ClassDims& d, const MatPtrs& ptrs, const float* scal, WsArr part, int splits, HalfArr qht, hipStream_t st) {
  constexpr int lds = T::template lds_bytes<Num>();
  hipError_t e = allow_lds(k_proj<T, Num, GSrc, PF>, lds);
  if (e != hipSuccess) return e;
  dim3 grid(((d.m + T::MT - 1) / T::MT) * ((d.r + T::NT - 1) / T::NT), splits, d.nb);
  // one matrix whose rows are a multiple of 32 KB apart (in M): measured 10-20 % faster with
  // rotated k order at 8192 columns; with several matrices in flight the order does not matter
  const int rotate = (d.nb == 1 && (d.ldm * (int64_t)sizeof(float)) % 32768 == 0) ? 1 : 0;
  launch_timed(k_proj<T, Num, GSrc, PF>, grid, dim3(T::THREADS), lds, st, d, ptrs, scal, part, splits, qht, rotate);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}
// Few wide tiles need many splits to fill the chip; 64-row tiles get there with half of them,
// i.e. half the partial sums to write and to add up.  With enough tiles the wide one wins.
bool proj_uses_flat_tiles(int m, int r, int nb) {
  return r > 128 && (int64_t)((m + 127) / 128) * ((r + 255) / 256) * nb < 256;
}
template <class GSrc>
static hipError_t proj_g(const ClassDims& d, const MatPtrs& ptrs, Prec prec, const float* scal, WsArr part, int splits, HalfArr qht, hipStream_t st) {
  if (prec == PREC_BF3) {
    // small problems: 64-deep steps halve the number of round trips of a loop that is all latency
    if ((int64_t)((d.m + 127) / 128) * ((d.r + 127) / 128) * splits * d.nb < 256)
      return proj_t<TileSmall, NumBF<3>, GSrc>(d, ptrs, scal, part, splits, qht, st);
    return proj_t<TileSquare, NumBF<3>, GSrc>(d, ptrs, scal, part, splits, qht, st);
  }
  if (d.r <= 64) return proj_t<TileNarrow, NumF16, GSrc>(d, ptrs, scal, part, splits, qht, st);
  if (d.r <= 128) return proj_t<TileSquare, NumF16, GSrc>(d, ptrs, scal, part, splits, qht, st);
  if (proj_uses_flat_tiles(d.m, d.r, d.nb)) {
    // long enough K loops per column tile pay for a second register stage
    if (d.r > 256) return proj_t<TileFlat, NumF16, GSrc, 2>(d, ptrs, scal, part, splits, qht, st);
    return proj_t<TileFlat, NumF16, GSrc>(d, ptrs, scal, part, splits, qht, st);
  }
  return proj_t<TileWide, NumF16, GSrc>(d, ptrs, scal, part, splits, qht, st);
}
template <bool TRANS, int NT>
static hipError_t stream_d_t(const ClassDims& d, const MatPtrs& ptrs, const float* scal, WsArr part, int splits, HalfArr fh, hipStream_t st,
                             HalfArr rh = HalfArr{nullptr, 0}, int* info = nullptr) {
  constexpr int SB = NT == 512 ? 2 : 3;
  constexpr int lds = SB * NT * 64 + 3 * (128 * 32 * 6) + 2 * (TRANS ? 32 * 320 : 128 * 64);
  hipError_t e = allow_lds(k_stream_d<TRANS, NT, SB>, lds);
  if (e != hipSuccess) return e;
  const int Mdim = TRANS ? d.n : d.m;
  dim3 grid(((Mdim + 127) / 128) * ((d.r + NT - 1) / NT), splits, d.nb);
  // rotated k order for the projection of a single matrix at 8192 columns (see the kernel): 120 ->
  // 102 us at r = 256.  With several matrices in flight the order does not matter, and the
  // 512-column tiles of the larger ranks are not waiting for memory (no gain measured there).
  const int rotate = (!TRANS && NT == 256 && d.nb == 1 && (d.ldm * (int64_t)sizeof(float)) % 32768 == 0) ? 1 : 0;
  launch_timed(k_stream_d<TRANS, NT, SB>, grid, dim3(512), lds, st, d, ptrs, scal, part, splits, fh, rh, info, rotate);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}
// shapes the direct-to-LDS contraction takes (fast precision only): bf16 gradients, a rank
// that fills its 256- or 512-column tiles reasonably, at least one whole 32-deep step
bool stream_kernel_eligible(const ClassDims& d) {
  return d.g_bf16 && d.r >= 192 && d.m >= 32 && d.n >= 32 && !kernel_choice("stream", "old");
}
int stream_tile_cols(int r) { return r <= 256 ? 256 : 512; }

hipError_t launch_proj(const ClassDims& d, const MatPtrs& ptrs, Prec prec, const float* scal, WsArr part, int splits, HalfArr qht, hipStream_t st) {
  if (prec == PREC_F16 && stream_kernel_eligible(d))
    return stream_tile_cols(d.r) == 256 ? stream_d_t<false, 256>(d, ptrs, scal, part, splits, qht, st)
                                        : stream_d_t<false, 512>(d, ptrs, scal, part, splits, qht, st);
  return d.g_bf16 ? proj_g<SrcBF16>(d, ptrs, prec, scal, part, splits, qht, st) : proj_g<SrcF32>(d, ptrs, prec, scal, part, splits, qht, st);
}

template <class T, class Num, class GSrc, int PF = 1>
static hipError_t back_t(const ClassDims& d, const MatPtrs& ptrs, const float* scal, WsArr p, WsArr part, int splits, HalfArr pht, hipStream_t st) {
  constexpr int lds = T::template lds_bytes<Num>();
  hipError_t e = allow_lds(k_back<T, Num, GSrc, PF>, lds);
  if (e != hipSuccess) return e;
  dim3 grid(((d.n + T::MT - 1) / T::MT) * ((d.r + T::NT - 1) / T::NT), splits, d.nb);
  launch_timed(k_back<T, Num, GSrc, PF>, grid, dim3(T::THREADS), lds, st, d, ptrs, scal, p, part, splits, pht);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}
template <class GSrc>
static hipError_t back_g(const ClassDims& d, const MatPtrs& ptrs, Prec prec, const float* scal, WsArr p, WsArr part, int splits, HalfArr pht, hipStream_t st) {
  if (prec == PREC_BF3) {
    if ((int64_t)((d.n + 127) / 128) * ((d.r + 127) / 128) * splits * d.nb < 256)
      return back_t<TileSmall, NumBF<3>, GSrc>(d, ptrs, scal, p, part, splits, pht, st);
    return back_t<TileSquare, NumBF<3>, GSrc>(d, ptrs, scal, p, part, splits, pht, st);
  }
  if (d.r <= 64) return back_t<TileNarrow, NumF16, GSrc>(d, ptrs, scal, p, part, splits, pht, st);
  if (d.r <= 128) return back_t<TileSquare, NumF16, GSrc>(d, ptrs, scal, p, part, splits, pht, st);
  // several column tiles per row panel: 256 x 256 tiles halve the operand traffic per product
  // and run one workgroup per CU with two register stages of loads in flight
  if (d.r > 256) return back_t<TileHuge, NumF16, GSrc, 2>(d, ptrs, scal, p, part, splits, pht, st);
  return back_t<TileWide, NumF16, GSrc>(d, ptrs, scal, p, part, splits, pht, st);
}
bool back_writes_fp16_copy(const ClassDims& d, Prec prec, int splits) { return prec == PREC_F16 && splits == 1 && stream_kernel_eligible(d); }

hipError_t launch_back(const ClassDims& d, const MatPtrs& ptrs, Prec prec, const float* scal, WsArr p, WsArr part, int splits, HalfArr pht, hipStream_t st,
                       HalfArr rh, int* info) {
  if (prec == PREC_F16 && stream_kernel_eligible(d)) {
    const HalfArr none{nullptr, 0};
    const bool copy = back_writes_fp16_copy(d, prec, splits) && rh.base != nullptr && info != nullptr;
    return stream_tile_cols(d.r) == 256 ? stream_d_t<true, 256>(d, ptrs, scal, part, splits, pht, st, copy ? rh : none, info)
                                        : stream_d_t<true, 512>(d, ptrs, scal, part, splits, pht, st, copy ? rh : none, info);
  }
  return d.g_bf16 ? back_g<SrcBF16>(d, ptrs, prec, scal, p, part, splits, pht, st) : back_g<SrcF32>(d, ptrs, prec, scal, p, part, splits, pht, st);
}

hipError_t launch_reduce(int nb, WsArr part, int splits, int64_t count, WsArr out, hipStream_t st, Pred pred) {
  int64_t n4 = count / 4;
  int blocks = (int)((n4 + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(k_reduce, dim3(blocks, nb), dim3(256), 0, st, part, splits, count, out, pred);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_reduce_r(const ClassDims& d, WsArr part, int splits, WsArr out, HalfArr rh, const float* scal, int* info, hipStream_t st) {
  int64_t n4 = (int64_t)d.n * d.r / 4;
  int blocks = (int)((n4 + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(k_reduce_r, dim3(blocks, d.nb), dim3(256), 0, st, d, part, splits, out, rh, scal, info);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

template <class T, class Num>
static hipError_t gram_tt(int nb, int rows, int r, WsArr a, WsArr part, int splits, hipStream_t st, const ClassDims& d, const float* scal, int side) {
  constexpr int lds = T::template lds_bytes<Num>();
  hipError_t e = allow_lds(k_gram<T, Num>, lds);
  if (e != hipSuccess) return e;
  int tiles = (r + T::NT - 1) / T::NT;
  hipLaunchKernelGGL((k_gram<T, Num>), dim3(tiles * (tiles + 1) / 2, splits, nb), dim3(T::THREADS), lds, st, rows, r, a, part, splits, d, scal, side);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}
template <class Num>
static hipError_t gram_t(int nb, int rows, int r, WsArr a, WsArr part, int splits, hipStream_t st, const ClassDims& d, const float* scal, int side) {
  // few large tiles leave most of the chip idle: use small ones until the grid fills it
  const int big = ((r + 127) / 128) * ((r + 127) / 128) * splits * nb;
  if (big < 512) return gram_tt<TileSmall, Num>(nb, rows, r, a, part, splits, st, d, scal, side);
  return gram_tt<TileSquare, Num>(nb, rows, r, a, part, splits, st, d, scal, side);
}
hipError_t launch_gram(int nb, int rows, int r, WsArr a, WsArr part, int splits, int mode, hipStream_t st, const ClassDims* d,
                       const float* scal, int side) {
  const ClassDims none = {};
  if (mode == kGramH2) {
    if (side != 2 && (d == nullptr || scal == nullptr)) return hipErrorInvalidValue;
    return gram_t<NumH2>(nb, rows, r, a, part, splits, st, d ? *d : none, scal, side);
  }
  return mode == kGramBF3 ? gram_t<NumBF<3>>(nb, rows, r, a, part, splits, st, none, nullptr, -1)
                          : gram_t<NumBF<2>>(nb, rows, r, a, part, splits, st, none, nullptr, -1);
}

template <class T, class Num, bool DEEP, bool CORR>
static hipError_t apply_tt(int nb, int rows, int r, WsArr a, WsArr w, HalfArr wh, WsArr out, const MatPtrs* ptrs, HalfArr hn, HalfArr ht, hipStream_t st, Pred pred) {
  constexpr int lds = T::template lds_bytes<Num>();
  hipError_t e = allow_lds(k_apply<T, Num, DEEP, CORR>, lds);
  if (e != hipSuccess) return e;
  MatPtrs none = {};
  dim3 grid(((rows + T::MT - 1) / T::MT) * ((r + T::NT - 1) / T::NT), 1, nb);
  hipLaunchKernelGGL((k_apply<T, Num, DEEP, CORR>), grid, dim3(T::THREADS), lds, st, rows, r, a, w, wh, out, ptrs ? *ptrs : none, ptrs ? 1 : 0, hn, ht, pred);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}
template <class Num, bool CORR>
static hipError_t apply_t(int nb, int rows, int r, WsArr a, WsArr w, HalfArr wh, WsArr out, const MatPtrs* ptrs, HalfArr hn, HalfArr ht, hipStream_t st, Pred pred) {
  const int big = ((rows + 127) / 128) * ((r + 127) / 128) * nb;
  if (big < 512) return apply_tt<TileSmall, Num, true, CORR>(nb, rows, r, a, w, wh, out, ptrs, hn, ht, st, pred);
  // 128 columns per tile: the loop of a column tile ends at its last row of W (upper triangular),
  // so narrower tiles skip more of the zero half than 256-column ones would (measured -10 %)
  // one operand part leaves LDS room for 64-deep steps at two workgroups per CU (measured -13 to
  // -23 %); with two parts the deeper tile halves the occupancy and loses
  if constexpr (Num::PARTS == 1) return apply_tt<TileSquareDeepK, Num, false, CORR>(nb, rows, r, a, w, wh, out, ptrs, hn, ht, st, pred);
  else return apply_tt<TileSquare, Num, false, CORR>(nb, rows, r, a, w, wh, out, ptrs, hn, ht, st, pred);
}
hipError_t launch_apply(int nb, int rows, int r, WsArr a, WsArr w, WsArr out, const MatPtrs* q_ptrs, HalfArr hn, HalfArr ht, int exact, hipStream_t st, Pred pred) {
  const HalfArr none{nullptr, 0};
  return exact ? apply_t<NumBF<3>, false>(nb, rows, r, a, w, none, out, q_ptrs, hn, ht, st, pred) : apply_t<NumBF<2>, false>(nb, rows, r, a, w, none, out, q_ptrs, hn, ht, st, pred);
}
hipError_t launch_apply_correction(int nb, int rows, int r, WsArr a, HalfArr phit, WsArr out, const MatPtrs* q_ptrs, HalfArr hn, HalfArr ht, hipStream_t st, Pred pred) {
  const WsArr unused{nullptr, 0};
  return apply_t<NumF16, true>(nb, rows, r, a, unused, phit, out, q_ptrs, hn, ht, st, pred);
}

template <class T, class Num, class DirA>
static hipError_t sgemm_tt(int nb, const SgemmArgs& g, hipStream_t st) {
  constexpr int lds = T::template lds_bytes<Num>();
  hipError_t e = allow_lds(k_sgemm<T, Num, DirA>, lds);
  if (e != hipSuccess) return e;
  dim3 grid(((g.Mc + T::MT - 1) / T::MT) * ((g.Nc + T::NT - 1) / T::NT), 1, nb * g.nq);
  hipLaunchKernelGGL((k_sgemm<T, Num, DirA>), grid, dim3(T::THREADS), lds, st, g);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}
template <class Num, class DirA>
static hipError_t sgemm_t(int nb, const SgemmArgs& g, hipStream_t st) {
  const int big = ((g.Mc + 127) / 128) * ((g.Nc + 127) / 128) * nb * g.nq;
  if (big < 256) return sgemm_tt<TileSmall, Num, DirA>(nb, g, st);      // one 128 x 128 tile per CU fills the chip
  return sgemm_tt<TileSquare, Num, DirA>(nb, g, st);
}
static hipError_t sgemm(int nb, const SgemmArgs& g, bool a_kc, int exact, hipStream_t st) {
  if (g.Mc <= 0 || g.Nc <= 0 || g.Kc <= 0 || g.nq <= 0) return hipSuccess;
  if (exact) return a_kc ? sgemm_t<NumBF<3>, KC>(nb, g, st) : sgemm_t<NumBF<3>, KSF>(nb, g, st);
  return a_kc ? sgemm_t<NumBF<2>, KC>(nb, g, st) : sgemm_t<NumBF<2>, KSF>(nb, g, st);
}

// g1 with A read as [k][row] (KSF) and g2 with A read as [row][k] (KC), six-product operands,
// in one launch; either may be empty.  Both have nq = 1.
template <class T>
static hipError_t sgemm_pair_tt(int nb, const SgemmArgs& g1, const SgemmArgs& g2, hipStream_t st) {
  typedef NumBF<3> Num;
  constexpr int lds = T::template lds_bytes<Num>();
  hipError_t e = allow_lds(k_sgemm_pair<T, Num, KSF, KC>, lds);
  if (e != hipSuccess) return e;
  const int tiles1 = ((g1.Mc + T::MT - 1) / T::MT) * ((g1.Nc + T::NT - 1) / T::NT);
  const int tiles2 = ((g2.Mc + T::MT - 1) / T::MT) * ((g2.Nc + T::NT - 1) / T::NT);
  hipLaunchKernelGGL((k_sgemm_pair<T, Num, KSF, KC>), dim3(tiles1 + tiles2, 1, nb), dim3(T::THREADS), lds, st, g1, g2, tiles1);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}
static hipError_t sgemm_pair(int nb, const SgemmArgs& g1, const SgemmArgs& g2, hipStream_t st) {
  const bool has1 = g1.Mc > 0 && g1.Nc > 0 && g1.Kc > 0, has2 = g2.Mc > 0 && g2.Nc > 0 && g2.Kc > 0;
  if (!has1 && !has2) return hipSuccess;
  if (!has2) return sgemm(nb, g1, false, 1, st);
  if (!has1) return sgemm(nb, g2, true, 1, st);
  const int big = (((g1.Mc + 127) / 128) * ((g1.Nc + 127) / 128) + ((g2.Mc + 127) / 128) * ((g2.Nc + 127) / 128)) * nb;
  if (big < 256) return sgemm_pair_tt<TileSmall>(nb, g1, g2, st);
  return sgemm_pair_tt<TileSquare>(nb, g1, g2, st);
}

hipError_t launch_cholinv(int nb, int r, WsArr gram, WsArr t, WsArr w, WsArr tmp, int* info, int info_slot,
                          hipStream_t st, Pred pred, int splits, int64_t split_stride) {
  hipError_t e = allow_lds(k_chol256, kCholLds);
  if (e != hipSuccess) return e;
  const int nblk = (r + kLeaf - 1) / kLeaf;
  CholArgs ca = {};
  ca.t = t; ca.w = w; ca.r = r; ca.info = info; ca.info_slot = info_slot;
  ca.src = gram; ca.splits = 1; ca.split_stride = 0;
  ca.pred = pred;
  if (nblk == 1) {
    ca.splits = splits; ca.split_stride = split_stride;
    ca.blk = 0;
    hipLaunchKernelGGL(k_chol256, dim3(nb), dim3(kCholThreads), kCholLds, st, ca);
    OD_CHECK_LAUNCH();
    return hipSuccess;
  }
  // lower block triangles of T and W are never written below; clear them once
  {
    const int64_t count = (int64_t)r * r;          // a multiple of 64
    int blocks = (int)((count / 4 + 255) / 256);
    if (blocks > 256) blocks = 256;
    hipLaunchKernelGGL(k_zero_pair, dim3(blocks, nb), dim3(256), 0, st, t, w, count, pred);
    OD_CHECK_LAUNCH();
  }
  // Step p: the diagonal block (T_pp, W_pp) is factored; then
  //   (1) the panel of the factor      T(p, rest) = W_pp^T G(p, rest)
  //       and, for the inverse,        tmp(0:p, p) = T(0:p, p) W_pp              (one launch)
  //   (2) the update of the next diagonal block alone
  //                                    G(p+1, p+1) -= T(p, p+1)^T T(p, p+1)      (one short launch)
  //   (3) one launch: the factorisation of block p + 1, beside the rest of the trailing update
  //       G(rest, rest) -= T(p, rest)^T T(p, rest) and block column p of the inverse,
  //       W(0:p, p) = -W(0:p, 0:p) tmp(0:p, p)
  // (the inverse of [[A, b], [0, c]] is [[A^-1, -A^-1 b c^-1], [0, c^-1]]).  The serial chain is
  // the factorisations and launches (1), (2); the bulk of the update hides behind a factorisation.
  auto tiles_of = [](const SgemmArgs& g, int mt) { return g.Mc > 0 && g.Nc > 0 && g.Kc > 0 ? ((g.Mc + mt - 1) / mt) * ((g.Nc + mt - 1) / mt) : 0; };
  for (int p = 0; p < nblk; ++p) {
    if (p == 0) {
      ca.blk = 0;
      hipLaunchKernelGGL(k_chol256, dim3(nb), dim3(kCholThreads), kCholLds, st, ca);
      OD_CHECK_LAUNCH();
    }
    const int o = p * kLeaf, o1 = (p + 1) * kLeaf, rest = r > o1 ? r - o1 : 0;
    const int bw = r - o < kLeaf ? r - o : kLeaf;       // width of block column p
    SgemmArgs panel = {}, prod = {}, trail = {}, wcol = {};
    panel.pred = prod.pred = trail.pred = wcol.pred = pred;
    panel.r = prod.r = trail.r = wcol.r = r;
    panel.nq = prod.nq = trail.nq = wcol.nq = 1;
    if (rest > 0) {
      panel.a = w; panel.b = gram; panel.c = t;
      panel.a_r0 = o; panel.a_k0 = o; panel.b_k0 = o; panel.b_c0 = o1; panel.c_r0 = o; panel.c_c0 = o1;
      panel.Mc = kLeaf; panel.Nc = rest; panel.Kc = kLeaf; panel.alpha = 1.f; panel.beta = 0.f;
      trail.a = t; trail.b = t; trail.c = gram;
      trail.a_r0 = o1; trail.a_k0 = o; trail.b_k0 = o; trail.b_c0 = o1; trail.c_r0 = o1; trail.c_c0 = o1;
      trail.Mc = rest; trail.Nc = rest; trail.Kc = kLeaf; trail.alpha = -1.f; trail.beta = 1.f;
    }
    if (p > 0) {
      prod.a = t; prod.b = w; prod.c = tmp;
      prod.a_r0 = 0; prod.a_k0 = o; prod.b_k0 = o; prod.b_c0 = o; prod.c_r0 = 0; prod.c_c0 = o;
      prod.Mc = o; prod.Nc = bw; prod.Kc = bw; prod.alpha = 1.f; prod.beta = 0.f;
      wcol.a = w; wcol.b = tmp; wcol.c = w;
      wcol.a_r0 = 0; wcol.a_k0 = 0; wcol.b_k0 = 0; wcol.b_c0 = o; wcol.c_r0 = 0; wcol.c_c0 = o;
      wcol.Mc = o; wcol.Nc = bw; wcol.Kc = o; wcol.alpha = -1.f; wcol.beta = 0.f;
    }
    if ((e = sgemm_pair(nb, panel, prod, st)) != hipSuccess) return e;
    if (rest == 0) {
      if ((e = sgemm_pair(nb, trail, wcol, st)) != hipSuccess) return e;
      continue;
    }
    // the trailing update in three pieces: the next diagonal block, the columns right of it
    // (all rows), and the rows below it (its own columns)
    const int nb1 = rest < kLeaf ? rest : kLeaf, o2 = o1 + nb1;
    SgemmArgs diag = trail, right = trail, below = trail;
    diag.Mc = nb1; diag.Nc = nb1;
    right.b_c0 = o2; right.c_c0 = o2; right.Nc = rest - nb1;
    below.a_r0 = o2; below.c_r0 = o2; below.Mc = rest - nb1; below.Nc = nb1;
    if ((e = sgemm(nb, diag, false, 1, st)) != hipSuccess) return e;
    ca.blk = p + 1;
    const int big = (tiles_of(right, 128) + tiles_of(below, 128) + tiles_of(wcol, 128)) * nb;
    if (big < 256) {
      typedef TileSmall T;
      constexpr int lds = T::lds_bytes<NumBF<3>>() > kCholLds ? T::lds_bytes<NumBF<3>>() : kCholLds;
      if ((e = allow_lds(k_chol_ahead<T>, lds)) != hipSuccess) return e;
      const int t1 = tiles_of(right, T::MT), t2 = tiles_of(below, T::MT), t3 = tiles_of(wcol, T::MT);
      hipLaunchKernelGGL(k_chol_ahead<T>, dim3(1 + t1 + t2 + t3, 1, nb), dim3(kCholThreads), lds, st, ca, right, below, wcol, t1, t2);
    } else {
      typedef TileSquare T;
      constexpr int lds = T::lds_bytes<NumBF<3>>() > kCholLds ? T::lds_bytes<NumBF<3>>() : kCholLds;
      if ((e = allow_lds(k_chol_ahead<T>, lds)) != hipSuccess) return e;
      const int t1 = tiles_of(right, T::MT), t2 = tiles_of(below, T::MT), t3 = tiles_of(wcol, T::MT);
      hipLaunchKernelGGL(k_chol_ahead<T>, dim3(1 + t1 + t2 + t3, 1, nb), dim3(kCholThreads), lds, st, ca, right, below, wcol, t1, t2);
    }
    OD_CHECK_LAUNCH();
  }
  return hipSuccess;
}

hipError_t launch_small_gram(int nb, int rows, int r, WsArr a0, WsArr part, int splits, hipStream_t st) {
  if (r > 32) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_small_gram, dim3(splits, nb), dim3(kSmallRows), 0, st, rows, r, a0, part, splits);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_small_first_pass(int nb, int rows, int r, WsArr a0, WsArr gram, int gram_splits, WsArr t1, WsArr w1, WsArr a1,
                                   WsArr part, int splits, int* info, int info_slot, hipStream_t st) {
  if (r > 32) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_small_first_pass, dim3(splits, nb), dim3(kSmallRows), 0, st, rows, r, a0, gram, gram_splits, t1, w1, a1,
                     part, splits, info, info_slot);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_corr(int nb, int r, WsArr part, int splits, WsArr t1, WsArr t2, WsArr w2, HalfArr phit, float* scal, int scal_slot,
                       int* info, int info_slot, hipStream_t st) {
  int64_t count = (int64_t)r * r;
  int blocks = (int)((count / 4 + 255) / 256);
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(k_corr, dim3(blocks, nb), dim3(256), 0, st, r, part, splits, t1, t2, w2, phit, scal, scal_slot, info, info_slot);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_scale_from_trace(int nb, int n, int r, WsArr gram, float* scal, hipStream_t st) {
  hipLaunchKernelGGL(k_scale_from_trace, dim3(nb), dim3(256), 0, st, n, r, gram, scal);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t launch_colnorm(int nb, int n, int r, WsArr rr, const MatPtrs& ptrs, WsArr part, int slabs, WsArr colsq,
                          float* scal, int* info, HalfArr qh, hipStream_t st) {
  hipLaunchKernelGGL(k_colsq_partial, dim3((r + 255) / 256, slabs, nb), dim3(256), 0, st, n, r, rr, part, slabs);
  OD_CHECK_LAUNCH();
  hipLaunchKernelGGL(k_colsq_final, dim3(nb), dim3(256), 0, st, n, r, part, slabs, colsq, scal, info);
  OD_CHECK_LAUNCH();
  int64_t n4 = (int64_t)n * r / 4;
  int blocks = (int)((n4 + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(k_colnorm_apply, dim3(blocks, nb), dim3(256), 0, st, n, r, rr, colsq, ptrs, qh);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}

template <class T, class Num, bool XBF, bool GBF>
static hipError_t efx_tt(const ClassDims& d, const MatPtrs& ptrs, const float* scal, const int* info, WsArr p, WsArr rr, float a_coef,
                         float b_coef, float lr, hipStream_t st) {
  constexpr int lds = T::template lds_bytes<Num>();
  hipError_t e = allow_lds(k_efx<T, Num, XBF, GBF>, lds);
  if (e != hipSuccess) return e;
  dim3 grid(((d.m + T::NT - 1) / T::NT) * ((d.n + T::MT - 1) / T::MT), 1, d.nb);
  launch_timed(k_efx<T, Num, XBF, GBF>, grid, dim3(T::THREADS), lds, st, d, ptrs, scal, info, p, rr, a_coef, b_coef, lr);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}
template <class Num, bool XBF, bool GBF>
static hipError_t efx_t(const ClassDims& d, const MatPtrs& ptrs, const float* scal, const int* info, WsArr p, WsArr rr, float a_coef,
                        float b_coef, float lr, hipStream_t st) {
  // small problems: more, smaller tiles (the kernel is a few microseconds of latency per tile)
  if ((int64_t)((d.m + 127) / 128) * ((d.n + 127) / 128) * d.nb < 256)
    return efx_tt<TileSmall, Num, XBF, GBF>(d, ptrs, scal, info, p, rr, a_coef, b_coef, lr, st);
  return efx_tt<TileSquare, Num, XBF, GBF>(d, ptrs, scal, info, p, rr, a_coef, b_coef, lr, st);
}
template <class Num>
static hipError_t efx_n(const ClassDims& d, const MatPtrs& ptrs, const float* scal, const int* info, WsArr p, WsArr rr, float a_coef,
                        float b_coef, float lr, hipStream_t st) {
  if (d.x_bf16) return d.g_bf16 ? efx_t<Num, true, true>(d, ptrs, scal, info, p, rr, a_coef, b_coef, lr, st)
                                : efx_t<Num, true, false>(d, ptrs, scal, info, p, rr, a_coef, b_coef, lr, st);
  return d.g_bf16 ? efx_t<Num, false, true>(d, ptrs, scal, info, p, rr, a_coef, b_coef, lr, st)
                  : efx_t<Num, false, false>(d, ptrs, scal, info, p, rr, a_coef, b_coef, lr, st);
}
template <bool XBF, bool GBF>
static hipError_t efx_h_t(const ClassDims& d_in, const MatPtrs& ptrs, const float* scal, int* info, HalfArr ph, HalfArr rh, HalfArr qh,
                          float a_coef, float b_coef, float lr, hipStream_t st) {
  ClassDims d = d_in;
  // up to r = 256 (above, the XCD-aware band order takes over) consecutive workgroups walk along a
  // row of tiles, i.e. through consecutive addresses of M, G, X, instead of down a column of tiles
  // whose rows lie a whole leading dimension apart: 8192 x 8192: 172 -> 156 us at r = 16, 233 ->
  // 224 us at r = 256; no difference at 4096 x 4096
  d.col_fast = d.r <= 256 ? 1 : 0;
  dim3 grid(((d.m + 127) / 128) * ((d.n + 127) / 128), 1, d.nb);
  const bool stream = d.r > 256 || (int64_t)d.m * d.n * d.nb >= ((int64_t)48 << 20);
  // ranks that are whole 32-deep steps take the direct-to-LDS kernel
  if (d.r % 32 == 0 && d.r >= 64 && !kernel_choice("efx", "old")) {
    // r > 256: 256-row tiles (one 8-wave workgroup per CU) while they still fill the chip twice:
    // a third less operand traffic into LDS per product than 128-row tiles
    const int64_t tall = (int64_t)((d.m + 255) / 256) * ((d.n + 127) / 128) * d.nb;
    if (d.r > 256 && tall >= 512 && !kernel_choice("efx", "dma128")) {
      constexpr int lds_t = 3 * (2 * 128 + 256) * 64;
      hipError_t e = stream ? allow_lds(k_efx_d<XBF, GBF, true, 4>, lds_t) : allow_lds(k_efx_d<XBF, GBF, false, 4>, lds_t);
      if (e != hipSuccess) return e;
      const dim3 tgrid(((d.m + 255) / 256) * ((d.n + 127) / 128), 1, d.nb);
      if (stream) launch_timed(k_efx_d<XBF, GBF, true, 4>, tgrid, dim3(512), lds_t, st, d, ptrs, scal, info, ph, rh, qh, a_coef, b_coef, lr);
      else launch_timed(k_efx_d<XBF, GBF, false, 4>, tgrid, dim3(512), lds_t, st, d, ptrs, scal, info, ph, rh, qh, a_coef, b_coef, lr);
      OD_CHECK_LAUNCH();
      return hipSuccess;
    }
    constexpr int lds_d = 3 * 3 * 128 * 64;
    hipError_t e = stream ? allow_lds(k_efx_d<XBF, GBF, true, 2>, lds_d) : allow_lds(k_efx_d<XBF, GBF, false, 2>, lds_d);
    if (e != hipSuccess) return e;
    if (stream) launch_timed(k_efx_d<XBF, GBF, true, 2>, grid, dim3(256), lds_d, st, d, ptrs, scal, info, ph, rh, qh, a_coef, b_coef, lr);
    else launch_timed(k_efx_d<XBF, GBF, false, 2>, grid, dim3(256), lds_d, st, d, ptrs, scal, info, ph, rh, qh, a_coef, b_coef, lr);
    OD_CHECK_LAUNCH();
    return hipSuccess;
  }
  constexpr int lds = 2 * 3 * 128 * 80;
  // also for sets far beyond the Infinity Cache at any rank: nontemporal stores leave no dirty
  // lines behind for the next kernel to wait on (measured on 8192 x 8192: the step is 2-7 % faster)
  if (d.r > 256 || (int64_t)d.m * d.n * d.nb >= ((int64_t)48 << 20)) launch_timed(k_efx_h<XBF, GBF, true>, grid, dim3(512), lds, st, d, ptrs, scal, info, ph, rh, qh, a_coef, b_coef, lr);
  else launch_timed(k_efx_h<XBF, GBF, false>, grid, dim3(512), lds, st, d, ptrs, scal, info, ph, rh, qh, a_coef, b_coef, lr);
  OD_CHECK_LAUNCH();
  return hipSuccess;
}
hipError_t launch_efx_h(const ClassDims& d, const MatPtrs& ptrs, const float* scal, int* info, HalfArr ph, HalfArr rh,
                        HalfArr qh, float a_coef, float b_coef, float lr, hipStream_t st) {
  if (d.x_bf16) return d.g_bf16 ? efx_h_t<true, true>(d, ptrs, scal, info, ph, rh, qh, a_coef, b_coef, lr, st)
                                : efx_h_t<true, false>(d, ptrs, scal, info, ph, rh, qh, a_coef, b_coef, lr, st);
  return d.g_bf16 ? efx_h_t<false, true>(d, ptrs, scal, info, ph, rh, qh, a_coef, b_coef, lr, st)
                  : efx_h_t<false, false>(d, ptrs, scal, info, ph, rh, qh, a_coef, b_coef, lr, st);
}

hipError_t launch_efx(const ClassDims& d, const MatPtrs& ptrs, Prec prec, const float* scal, const int* info, WsArr p, WsArr rr,
                      float a_coef, float b_coef, float lr, hipStream_t st) {
  return prec == PREC_BF3 ? efx_n<NumBF<3>>(d, ptrs, scal, info, p, rr, a_coef, b_coef, lr, st)
                          : efx_n<NumF16>(d, ptrs, scal, info, p, rr, a_coef, b_coef, lr, st);
}

}  // namespace od
