// Cholesky factorisation and triangular inverse of one SPD block of up to 256 x 256 in a
// single workgroup (8 waves):  G = T^T T with T upper triangular, W = T^-1.
//
// Used by the CholeskyQR orthogonalisation (orth() of Alg. 1 lines 2 and 4): T is the
// triangular factor of the thin QR, W turns the triangular solve into a product.
//
// Layout of the computation (8 waves: wave 3 runs the serial chain of diagonal tiles, the
// other seven are workers)
//   * The block is cut into 32 x 32 tiles; the tiles (I, K) with I < K are kept as
//     matrix-core accumulators (16 registers per lane: register v of lane l is row
//     8 (v / 4) + 4 (l / 32) + v % 4, column l % 32), spread over the workers so that every
//     row and column of tiles is shared out evenly.  The diagonal tiles wait in LDS.
//   * Step J, (a): the diagonal wave factors tile (J, J) in place, four rows at a time.
//     The 4 x 4 diagonal block is gathered with readlane, factored and inverted in scalar
//     (wave-uniform) arithmetic; the new rows are a 4 x 4 product inside each lane; the
//     rank-4 trailing update of the tile is two fp32 matrix-core products (32x32x2).  The
//     same operations applied to an identity tile give the inverse of the tile's factor.
//     (b): the owner of tile (J, K) forms T(J, K) = W_JJ^T S(J, K) on the matrix cores (the
//     accumulator tile serves directly as the k-side operand), writes it out, publishes it
//     to LDS already split into three bf16 terms in the operand's register order, and
//     subtracts T(J, K)^T T(J, K) from the waiting diagonal tile (K, K).  Tile (J, J+1) goes
//     first: as soon as it is done the diagonal wave starts on (J+1, J+1) while the workers
//     finish (b) and do (c).
//     (c): every remaining tile gets S(I, K) -= T(J, I)^T T(J, K) from those LDS operands.
//   * The inverse is built alongside, right-looking, as V = W^T (lower triangular): once
//     T(I, K) has left its accumulator the same registers collect
//     S'(K, I) = sum_{I <= L < K} T(L, K)^T V(L, I) in the (c) phases, and in (b) of step K
//     V(K, I) = -W_KK^T S'(K, I) is written out and published to LDS for the rows below.
//   * Waves hand tiles over through LDS words (signal / bounded wait); the one barrier per
//     step waits for LDS traffic only, so the global stores of finished tiles never stall
//     the loop.  Panel and inverse products use three-way split bf16 operands (six
//     products, 24 significant bits).
#pragma once

#include <type_traits>

#include "od_common.h"
#include "od_kernels.h"

namespace od {

constexpr int kCholMax = 256;          // largest block one workgroup factors
constexpr int kCT = 32;                // tile size
constexpr int kCNT = kCholMax / kCT;   // 8 tiles per side
constexpr int kCTiles = kCNT * (kCNT + 1) / 2;   // 36
constexpr int kCholThreads = 512;      // 8 waves: two per SIMD
constexpr int kCholDiagWave = 3;       // the serial chain; the other seven are workers
constexpr int kCWorkers = 7;
constexpr int kCSlots = 4;             // off-diagonal tiles per worker: 28 over 7 workers, four each
constexpr int kCPitch = 36;            // floats per row of an fp32 LDS tile (16-byte aligned, conflict free)
constexpr int kCTileF = kCT * kCPitch; // floats per fp32 LDS tile
constexpr int kPPitch = 80;            // bytes per row of a pre-split operand tile (32 bf16 + pad)
constexpr int kPPlane = kCT * kPPitch; // bytes per part of a pre-split tile
constexpr int kPTile = 3 * kPPlane;    // bytes per pre-split tile
// LDS: Wt[2] fp32 (W_JJ^T of even / odd steps) | panel[8] pre-split T(J, K)^T | vpanel[8] pre-split V(J, I)
constexpr int kCholOffPanel = 2 * kCTileF * 4;
constexpr int kCholOffVPanel = kCholOffPanel + kCNT * kPTile;
constexpr int kCholOffSync = kCholOffVPanel + kCNT * kPTile;   // published[8] | s_ready[8] (ints)
constexpr int kCholOffStash = kCholOffSync + 2 * kCNT * 4;      // two fp32 tile images: S(J, J+1) for the diagonal wave
constexpr int kCholLds = kCholOffStash + 2 * 4096;
constexpr int kCholSpinLimit = 1 << 22;  // bound of every wait below (never reached: the producers do not wait)

struct CholArgs {
  WsArr src;           // Gram block source: `splits` partial sums, `split_stride` elements apart
  int splits;
  int64_t split_stride;
  WsArr t, w;          // outputs, r x r each (ld r)
  int r;               // matrix order (ld of everything)
  int blk;             // which diagonal block of kCholMax
  int* info;
  int info_slot;
  Pred pred;           // the matrix is skipped unless its predicate holds
};

// tile (I, K), I < K, of slot s of worker u, four bits per slot, 15 = no tile (kept in scalar
// registers: a table in memory would cost a dependent load per use).  Tile (I, K) belongs
// to worker (I + K) mod 7: four tiles each, and in every step the panel tiles (one row and one
// column of tiles, sums I + K that span eight consecutive values) go to seven different
// workers but for one pair.
OD_DEV uint64_t own_rows(int u) {
  return u == 0 ? 0x3210ull : u == 1 ? 0x3210ull : u == 2 ? 0x4320ull : u == 3 ? 0x4310ull : u == 4 ? 0x5410ull : u == 5 ? 0x5210ull
       : u == 6 ? 0x6210ull : 0xffffull;
}
OD_DEV uint64_t own_cols(int u) {
  return u == 0 ? 0x4567ull : u == 1 ? 0x5671ull : u == 2 ? 0x5672ull : u == 3 ? 0x6723ull : u == 4 ? 0x6734ull : u == 5 ? 0x7345ull
       : u == 6 ? 0x7456ull : 0xffffull;
}

// A diagonal tile waiting in LDS in accumulator layout: plane q holds registers 4q .. 4q+3
// of every lane (16 bytes per lane, conflict free).
OD_DEV f32x16 load_dtile(const char* p, int lane) {
  f32x16 t;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(p + q * 1024 + lane * 16);
#pragma unroll
    for (int e = 0; e < 4; ++e) t[4 * q + e] = v[e];
  }
  return t;
}
OD_DEV void store_dtile(char* p, const f32x16& t, int lane) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const f32x4 v = {t[4 * q], t[4 * q + 1], t[4 * q + 2], t[4 * q + 3]};
    *reinterpret_cast<f32x4*>(p + q * 1024 + lane * 16) = v;
  }
}

// workgroup barrier that orders LDS traffic only (outstanding global stores keep flying)
OD_DEV void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

OD_DEV float lane_bcast(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// 1/sqrt(d) to fp32 accuracy: hardware estimate (1 ulp) plus one Newton step.
OD_DEV float fast_rsqrt(float d) {
  float y = __builtin_amdgcn_rsqf(d);
  return y * fmaf(-0.5f * d * y, y, 1.5f);
}

// Three-way split bf16 operand words of 8 floats.
OD_DEV void split3(const float* x, u32x4* parts) { NumBF<3>::pack(x, 1.f, parts); }

OD_DEV void negate3(u32x4* parts) {
#pragma unroll
  for (int s = 0; s < 3; ++s)
#pragma unroll
    for (int i = 0; i < 4; ++i) parts[s][i] ^= 0x80008000u;
}

OD_DEV f32x16 mma6(const u32x4* a, const u32x4* b, f32x16 c) {
#pragma unroll
  for (int i = 2; i >= 0; --i)
#pragma unroll
    for (int j = 2 - i; j >= 0; --j) c = mfma_32x32x16<false>(a[i], b[j], c);
  return c;
}

// Operand of k-step kk from an fp32 LDS tile stored [row][k] with pitch kCPitch: this lane's
// row is l % 32 and its 8 k-slots are 16 kk + 4 g + {0..3} and 16 kk + 8 + 4 g + {0..3}
// (the rows an accumulator lane holds in registers 8 kk .. 8 kk + 7).
OD_DEV void lds_operand(const float* tile, int lane, int kk, u32x4* parts) {
  const float* p = tile + (lane & 31) * kCPitch + 16 * kk + 4 * (lane >> 5);
  f32x4 lo = *reinterpret_cast<const f32x4*>(p);
  f32x4 hi = *reinterpret_cast<const f32x4*>(p + 8);
  float x[8] = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  split3(x, parts);
}
// k-side operand of k-step kk straight from an accumulator tile.
OD_DEV void acc_operand(const f32x16& acc, int kk, u32x4* parts) {
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = acc[8 * kk + e];
  split3(x, parts);
}

// Pre-split operand tile in LDS: the transpose of an accumulator tile (element (row, col) is
// operand row col, k = row), three bf16 planes, each row holding its 32 k in register order
// so that the operand words of k-step kk are one 16-byte read per plane.
OD_DEV void store_presplit(char* tile, const f32x16& acc, int lane) {
  char* p = tile + (lane & 31) * kPPitch + (lane >> 5) * 16;
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    u32x4 parts[3];
    acc_operand(acc, kk, parts);
#pragma unroll
    for (int s = 0; s < 3; ++s) *reinterpret_cast<u32x4*>(p + s * kPPlane + kk * 32) = parts[s];
  }
}
OD_DEV void load_presplit(const char* tile, int lane, int kk, u32x4* parts) {
  const char* p = tile + (lane & 31) * kPPitch + (lane >> 5) * 16 + kk * 32;
#pragma unroll
  for (int s = 0; s < 3; ++s) parts[s] = *reinterpret_cast<const u32x4*>(p + s * kPPlane);
}

// Producer / consumer hand-off between the waves of the workgroup through LDS words.  The
// producer's earlier LDS writes are complete before the word changes; a consumer that has
// seen the value may read them.  Producers never wait on consumers, so every wait ends; it
// is bounded anyway so that a wave can always run to the end of the kernel.
OD_DEV void lds_signal_add(int* word, int lane) {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  if (lane == 0) __hip_atomic_fetch_add(word, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
// Returns false when the bound ran out (the caller reports it; the kernel still ends).
OD_DEV bool lds_wait_ge(int* word, int target) {
  bool seen = false;
  for (int spins = 0; spins < kCholSpinLimit; ++spins) {
    if (__hip_atomic_load(word, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= target) { seen = true; break; }
    __builtin_amdgcn_s_sleep(1);
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
  return seen;
}

// ---------------------------------------------------------------------------------------
// Diagonal tile: in-place upper Cholesky factor of the symmetric tile `d` and, in `zt`, the
// inverse of its transpose (M = L^-1, lower triangular), both in accumulator layout.
// Returns the 1-based index of the first bad pivot within the tile, or 0.
// ---------------------------------------------------------------------------------------
// value of `x` held by the lanes of half `hh`, in both halves
OD_DEV float half_bcast(float x, int hh) {
  const uint32_t u = __float_as_uint(x);
  // swaps lanes 32..63 of the first operand with lanes 0..31 of the second:
  // [0] = the lower half's values in both halves, [1] = the upper half's
  auto pr = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(hh ? pr[1] : pr[0]);
}

OD_DEV f32x16 mfma_f32_k2(float a, float b, f32x16 c) {
  // D(32x32) += A(32x2) B(2x32) in fp32: lane l holds A[l % 32][l / 32] and B[l / 32][l % 32]
  return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

OD_DEV int diag_tile_factor(f32x16& d_io, f32x16& zt_out, int lane) {
  const int c = lane & 31, h = lane >> 5;
  int bad = 0;
  // `d` and `zt` are only ever changed by the matrix-core updates; the finished rows are
  // collected on the side (a finished row of `d` / `zt` itself is never read again)
  f32x16 d = d_io, zt;
  float tfin[16], zfin[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) zt[v] = (acc_row(v, lane) == c) ? 1.f : 0.f;
#pragma unroll
  for (int g = 0; g < 8; ++g) {
    const int q = g >> 1, hh = g & 1, src_lane = 32 * hh + 4 * g;
    // 4 x 4 diagonal block (upper part), wave-uniform
    const float d00 = lane_bcast(d[4 * q + 0], src_lane + 0), d01 = lane_bcast(d[4 * q + 0], src_lane + 1);
    const float d02 = lane_bcast(d[4 * q + 0], src_lane + 2), d03 = lane_bcast(d[4 * q + 0], src_lane + 3);
    const float d11 = lane_bcast(d[4 * q + 1], src_lane + 1), d12 = lane_bcast(d[4 * q + 1], src_lane + 2);
    const float d13 = lane_bcast(d[4 * q + 1], src_lane + 3), d22 = lane_bcast(d[4 * q + 2], src_lane + 2);
    const float d23 = lane_bcast(d[4 * q + 2], src_lane + 3), d33 = lane_bcast(d[4 * q + 3], src_lane + 3);
    // rows 4g .. 4g+3 of both tiles, made available to both lane halves
    float s[4], zz[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      s[e] = half_bcast(d[4 * q + e], hh);
      zz[e] = half_bcast(zt[4 * q + e], hh);
    }
    // pivots: a non-positive or non-finite one is only recorded (the outputs of such a matrix
    // are unspecified); the hardware reciprocal square root (1 ulp) is accurate enough here,
    // since the inverse below is built from the same rounded values
    const float p0 = d00;
    const float i00 = __builtin_amdgcn_rsqf(p0);
    const float t01 = d01 * i00, t02 = d02 * i00, t03 = d03 * i00;
    const float p1 = d11 - t01 * t01;
    const float i11 = __builtin_amdgcn_rsqf(p1);
    const float t12 = (d12 - t01 * t02) * i11, t13 = (d13 - t01 * t03) * i11;
    const float p2 = d22 - t02 * t02 - t12 * t12;
    const float i22 = __builtin_amdgcn_rsqf(p2);
    const float t23 = (d23 - t02 * t03 - t12 * t13) * i22;
    const float p3 = d33 - t03 * t03 - t13 * t13 - t23 * t23;
    const float i33 = __builtin_amdgcn_rsqf(p3);
    // one test per group on the critical path (a NaN or an infinite pivot makes the sum fail
    // the upper bound; fminf alone would skip a NaN); which of the four it was is worked out
    // only when the test fails
    const float pmin = fminf(fminf(p0, p1), fminf(p2, p3)), psum = (p0 + p1) + (p2 + p3);
    if (bad == 0 && !(pmin > 0.f && psum < 3.0e38f)) {
      if (!(p0 > 0.f) || !(p0 < 3.0e38f)) bad = 4 * g + 1;
      else if (!(p1 > 0.f) || !(p1 < 3.0e38f)) bad = 4 * g + 2;
      else if (!(p2 > 0.f) || !(p2 < 3.0e38f)) bad = 4 * g + 3;
      else bad = 4 * g + 4;
    }
    // inverse of the 4 x 4 upper factor
    const float w01 = -(t01 * i11) * i00, w12 = -(t12 * i22) * i11, w23 = -(t23 * i33) * i22;
    const float w02 = -(t01 * w12 + t02 * i22) * i00, w13 = -(t12 * w23 + t13 * i33) * i11;
    const float w03 = -(t01 * w13 + t02 * w23 + t03 * i33) * i00;
    // new rows of the factor and of the inverse: (W4^T s)_a = sum_{b <= a} W4[b][a] s_b
    float tn[4], zn[4];
    tn[0] = i00 * s[0];
    tn[1] = w01 * s[0] + i11 * s[1];
    tn[2] = w02 * s[0] + w12 * s[1] + i22 * s[2];
    tn[3] = w03 * s[0] + w13 * s[1] + w23 * s[2] + i33 * s[3];
    zn[0] = i00 * zz[0];
    zn[1] = w01 * zz[0] + i11 * zz[1];
    zn[2] = w02 * zz[0] + w12 * zz[1] + i22 * zz[2];
    zn[3] = w03 * zz[0] + w13 * zz[1] + w23 * zz[2] + i33 * zz[3];
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (c < 4 * g + e) tn[e] = 0.f;                // row 4g+e of an upper factor starts at its diagonal
    if (g < 7) {
      // rank-4 update of both tiles, -T_g^T T_g and -T_g^T Z_g, as two k = 2 products each:
      // the lower lane half carries rows 4g, 4g+2 and the upper half rows 4g+1, 4g+3
      const float t01v = h ? tn[1] : tn[0], t23v = h ? tn[3] : tn[2];
      const float z01v = h ? zn[1] : zn[0], z23v = h ? zn[3] : zn[2];
      d = mfma_f32_k2(-t01v, t01v, d);
      zt = mfma_f32_k2(-t01v, z01v, zt);
      d = mfma_f32_k2(-t23v, t23v, d);
      zt = mfma_f32_k2(-t23v, z23v, zt);
    }
    // the rows of this group are final (register 4q + e of lane half hh; the other half's
    // turn for these registers comes with the next group)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (hh == 0) { tfin[4 * q + e] = tn[e]; zfin[4 * q + e] = zn[e]; }
      else if (h == 1) { tfin[4 * q + e] = tn[e]; zfin[4 * q + e] = zn[e]; }
    }
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) { d_io[v] = tfin[v]; zt_out[v] = zfin[v]; }
  return bad;
}

// The factorisation of block `a.blk` of matrix `z` by one workgroup of kCholThreads threads;
// `lds_raw`: kCholLds bytes.
OD_DEV void chol256_block(const CholArgs& a, int z, char* lds_raw) {
  float* Wt = reinterpret_cast<float*>(lds_raw);                         // W_JJ^T, [i][k], buffer J & 1
  char* panel = lds_raw + kCholOffPanel;                                 // T(J, K)^T pre-split, one tile per K
  char* vpanel = lds_raw + kCholOffVPanel;                               // V(J, I) pre-split, one tile per I; before
                                                                         // step I-1 ends: the waiting tile (I, I)
  int* published = reinterpret_cast<int*>(lds_raw + kCholOffSync);       // tiles of step J published so far
  int* s_ready = published + kCNT;                                       // S(J, J+1) has its last update and is in the stash
  char* stash = lds_raw + kCholOffStash;                                 // buffer J & 1

  const int tid = threadIdx.x, lane = tid & 63;
  // uniform over the workgroup, before any barrier or LDS hand-off
  if (a.pred.scal != nullptr && (a.pred.scal[z * kScalPerMat + a.pred.slot] > a.pred.thr) != (a.pred.want != 0)) return;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool diag_wave = wave == kCholDiagWave;
  const int worker = diag_wave ? kCWorkers : (wave < kCholDiagWave ? wave : wave - 1);
  const uint64_t ownI = own_rows(worker), ownK = own_cols(worker);
  const int r = a.r;
  const int o = a.blk * kCholMax;
  const int nb = (r - o) < kCholMax ? (r - o) : kCholMax;     // order of this block
  const int nt = (nb + kCT - 1) / kCT;                        // active tiles per side
  const int64_t off = (int64_t)o * r + o;
  const float* src = a.src.base + (int64_t)z * a.src.stride + off;
  float* tg = a.t.base + (int64_t)z * a.t.stride + off;
  float* wg = a.w.base + (int64_t)z * a.w.stride + off;
  const int col = lane & 31, half = lane >> 5;
  if (tid < 2 * kCNT) published[tid] = 0;

  // ---- tiles strictly below the diagonal of T and W are zero and written by nobody else:
  // one tile per iteration (256 threads x 16 bytes = one 32 x 32 tile)
  if (tid < 256) {
    for (int I = 1; I < nt; ++I)
      for (int K = 0; K < I; ++K) {
        const int gi = I * kCT + (tid >> 3), gj = K * kCT + (tid & 7) * 4;
        if (gi < nb && gj < nb) {
          const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
          *reinterpret_cast<f32x4*>(tg + (int64_t)gi * r + gj) = zero;
          *reinterpret_cast<f32x4*>(wg + (int64_t)gi * r + gj) = zero;
        }
      }
  }

  // ---- load: every tile is read straight into accumulator layout through the transposed
  // element (the matrix is symmetric): lane column c needs rows 8q + 4h + {0..3} of its
  // column, which are four consecutive entries of row c of the mirrored tile.  Addresses are
  // clamped into the block, so all loads are unconditional and in flight together; identity
  // outside the block.
  auto load_tile = [&](int I, int K) {
    f32x16 t;
    const int gj = K * kCT + col, gjc = gj < nb ? gj : nb - 1;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int gi = I * kCT + 8 * q + 4 * half, gic = gi < nb ? gi : nb - 4;
      const float* p = src + (int64_t)gjc * r + gic;
      f32x4 v4 = *reinterpret_cast<const f32x4*>(p);
      for (int sp = 1; sp < a.splits; ++sp) v4 += *reinterpret_cast<const f32x4*>(p + (int64_t)sp * a.split_stride);
#pragma unroll
      for (int e = 0; e < 4; ++e) t[4 * q + e] = v4[e];
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int gi = I * kCT + acc_row(v, lane);
      if (gi >= nb || gj >= nb) t[v] = (gi == gj) ? 1.f : 0.f;
    }
    return t;
  };
  f32x16 acc[kCSlots];
#pragma unroll
  for (int s = 0; s < kCSlots; ++s) {
    const int I = (int)(ownI >> (4 * s)) & 15, K = (int)(ownK >> (4 * s)) & 15;
    if (K < nt) acc[s] = load_tile(I, K);
    else {
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[s][v] = 0.f;
    }
  }

  // ================================ factorisation ================================
  // (a) tile (J, J): factor, invert, write T_JJ and W_JJ, publish W_JJ^T
  auto do_diag = [&](int J, f32x16 d) {
    f32x16 zt;
    const int bad = diag_tile_factor(d, zt, lane);
    if (bad != 0 && lane == 0) atomicCAS(&a.info[z * kInfoPerMat + a.info_slot], 0, o + J * kCT + bad);
    const int nv = (nb - J * kCT) < kCT ? (nb - J * kCT) : kCT;   // valid rows / cols of this tile
    // zt = M = V(J, J) with W_JJ = M^T:  Wt[i][k] = M[i][k]
    float* wt = Wt + (J & 1) * kCTileF;
#pragma unroll
    for (int v = 0; v < 16; ++v) wt[acc_row(v, lane) * kCPitch + col] = zt[v];
    store_presplit(vpanel + J * kPTile, zt, lane);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      // global W_JJ[c][rows] (row c of W = column c of M), 4 consecutive entries
      if (col < nv && 8 * q < nv) {
        const f32x4 v4 = {zt[4 * q], zt[4 * q + 1], zt[4 * q + 2], zt[4 * q + 3]};
        *reinterpret_cast<f32x4*>(wg + (int64_t)(J * kCT + col) * r + J * kCT + 8 * q + 4 * half) = v4;
      }
    }
    if (col < nv) {
      float* tp = tg + (int64_t)(J * kCT + 4 * half) * r + J * kCT + col;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (8 * q < nv) {
#pragma unroll
          for (int e = 0; e < 4; ++e) tp[(int64_t)(8 * q + e) * r] = d[4 * q + e];
        }
      }
    }
  };
  // tile += sign * A^T B with both operands pre-split in LDS
  auto lds_product = [&](f32x16& tile, const char* pa, const char* pb, bool negate) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      u32x4 ap[3], bp[3];
      load_presplit(pa, lane, kk, ap);
      load_presplit(pb, lane, kk, bp);
      if (negate) negate3(ap);
      tile = mma6(ap, bp, tile);
    }
  };
  // (b) for one owned tile of step J: T(J, K) = W_JJ^T S(J, K) (row tile) or V(J, I) = -W_JJ^T S'(J, I)
  // (column tile), written out and published.  fp32 products (32x32x2): step (q, e) contracts
  // over k = 8q + e (lower lane half) and 8q + 4 + e (upper half), which is exactly the row an
  // accumulator lane keeps in register 4q + e, so the k-side operand needs no data movement
  // and nothing is split.
  auto panel_tile = [&](f32x16& tile, const f32x4 (&mrow)[4], int J, int I, int K, bool row_tile) {
    const int nvr = (nb - J * kCT) < kCT ? (nb - J * kCT) : kCT;
    // two independent accumulation chains keep the matrix core busy back to back
    f32x16 res, res2;
#pragma unroll
    for (int v = 0; v < 16; ++v) { res[v] = 0.f; res2[v] = 0.f; }
#pragma unroll
    for (int q = 0; q < 4; q += 2)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        res = mfma_f32_k2(mrow[q][e], tile[4 * q + e], res);
        res2 = mfma_f32_k2(mrow[q + 1][e], tile[4 * q + 4 + e], res2);
      }
#pragma unroll
    for (int v = 0; v < 16; ++v) res[v] = row_tile ? (res[v] + res2[v]) : -(res[v] + res2[v]);
    if (row_tile) {
      // block orders are multiples of 8, so rows 8q .. 8q+7 are valid or not together
      if (K * kCT + col < nb) {
        float* tp = tg + (int64_t)(J * kCT + 4 * half) * r + K * kCT + col;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (8 * q < nvr) {
#pragma unroll
            for (int e = 0; e < 4; ++e) tp[(int64_t)(8 * q + e) * r] = res[4 * q + e];
          }
        }
      }
      store_presplit(panel + K * kPTile, res, lane);
#pragma unroll
      for (int v = 0; v < 16; ++v) tile[v] = 0.f;       // from now on the sum S'(K, J)
      // the waiting diagonal tile (K, K) -= T(J, K)^T T(J, K), operands read back from the panel
      // (tile (J+1, J+1) gets this update from the diagonal wave itself, which is about to factor it)
      if (K != J + 1) {
        char* dk = vpanel + K * kPTile;
        f32x16 dt = load_dtile(dk, lane);
        lds_product(dt, panel + K * kPTile, panel + K * kPTile, true);
        store_dtile(dk, dt, lane);
      }
      lds_signal_add(published + J, lane);
    } else {
      store_presplit(vpanel + I * kPTile, res, lane);
      lds_signal_add(published + J, lane);
      // W(I*32 + c, J*32 + i) = V(J, I)(i, c): four consecutive columns per store
      if (I * kCT + col < nb) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (8 * q < nvr) {
            const f32x4 v4 = {res[4 * q], res[4 * q + 1], res[4 * q + 2], res[4 * q + 3]};
            *reinterpret_cast<f32x4*>(wg + (int64_t)(I * kCT + col) * r + J * kCT + 8 * q + 4 * half) = v4;
          }
        }
      }
    }
  };

  if (diag_wave) {
    // the diagonal tiles: (0, 0) is factored at once, the others wait in LDS for their updates
    for (int I = 1; I < nt; ++I) store_dtile(vpanel + I * kPTile, load_tile(I, I), lane);
    do_diag(0, load_tile(0, 0));
  } else {
    // tile (0, 1) as loaded is what the diagonal wave needs first
#pragma unroll
    for (int s = 0; s < kCSlots; ++s) {
      const int I = (int)(ownI >> (4 * s)) & 15, K = (int)(ownK >> (4 * s)) & 15;
      if (I == 0 && K == 1 && K < nt) store_dtile(stash, acc[s], lane);     // made visible by the barrier below
    }
  }
  lds_barrier();
  bool expired = false;
  // One loop per role (the branch is wave-uniform and both loops pass the same nt barriers): in
  // the diagonal wave's loop the workers' accumulators are dead, so its serial chain keeps its
  // operands in registers.
  if (diag_wave) {
    for (int J = 0; J < nt; ++J) {
      // ---- the serial chain stays in this wave: T(J, J+1) = W_JJ^T S(J, J+1) from the stash,
      // tile (J+1, J+1) -= T^T T (both fp32 products with the accumulator as k-side operand,
      // see panel_tile), then its factorisation.  The workers form T(J, J+1) again for the panel.
      if (J + 1 < nt) {
        if (J > 0 && !lds_wait_ge(s_ready + J, 1)) expired = true;
        const f32x16 sj = load_dtile(stash + (J & 1) * 4096, lane);
        f32x16 dn = load_dtile(vpanel + (J + 1) * kPTile, lane);
        const float* wt = Wt + (J & 1) * kCTileF;
        f32x4 mrow[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) mrow[q] = *reinterpret_cast<const f32x4*>(wt + col * kCPitch + 8 * q + 4 * half);
        f32x16 t1, t2;
#pragma unroll
        for (int v = 0; v < 16; ++v) { t1[v] = 0.f; t2[v] = 0.f; }
#pragma unroll
        for (int q = 0; q < 4; q += 2)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            t1 = mfma_f32_k2(mrow[q][e], sj[4 * q + e], t1);
            t2 = mfma_f32_k2(mrow[q + 1][e], sj[4 * q + 4 + e], t2);
          }
#pragma unroll
        for (int v = 0; v < 16; ++v) t1[v] += t2[v];
#pragma unroll
        for (int v = 0; v < 16; ++v) dn = mfma_f32_k2(-t1[v], t1[v], dn);
        do_diag(J + 1, dn);
      }
      // the next step rewrites the panels and the other Wt buffer
      lds_barrier();
    }
  } else {
    for (int J = 0; J < nt; ++J) {
      // ---- (b) row J of T and row J of V; the tile the diagonal wave waits for goes first
      const float* wt = Wt + (J & 1) * kCTileF;
      f32x4 mrow[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) mrow[q] = *reinterpret_cast<const f32x4*>(wt + col * kCPitch + 8 * q + 4 * half);
#pragma unroll
      for (int s = 0; s < kCSlots; ++s) {
        const int I = (int)(ownI >> (4 * s)) & 15, K = (int)(ownK >> (4 * s)) & 15;
        if (I == J && K == J + 1 && K < nt) panel_tile(acc[s], mrow, J, I, K, true);
      }
#pragma unroll
      for (int s = 0; s < kCSlots; ++s) {
        const int I = (int)(ownI >> (4 * s)) & 15, K = (int)(ownK >> (4 * s)) & 15;
        const bool row_tile = I == J && K > J + 1 && K < nt, col_tile = K == J && I < J;
        if (row_tile || col_tile) panel_tile(acc[s], mrow, J, I, K, row_tile);
      }
      // ---- (c) once all nt - 1 tiles of the step are published:
      // S(I, K) -= T(J, I)^T T(J, K) for J < I < K;  S'(K, I) += T(J, K)^T V(J, I) for I <= J < K
      if (!lds_wait_ge(published + J, nt - 1)) expired = true;
#pragma unroll
      for (int s = 0; s < kCSlots; ++s) {
        const int I = (int)(ownI >> (4 * s)) & 15, K = (int)(ownK >> (4 * s)) & 15;
        if (K > J && K < nt) {
          if (I > J) lds_product(acc[s], panel + I * kPTile, panel + K * kPTile, true);
          else lds_product(acc[s], panel + K * kPTile, vpanel + I * kPTile, false);
          // S(J+1, J+2) is final now: hand it to the diagonal wave
          if (I == J + 1 && K == J + 2) {
            store_dtile(stash + ((J + 1) & 1) * 4096, acc[s], lane);
            lds_signal_add(s_ready + J + 1, lane);
          }
        }
      }
      lds_barrier();
    }
  }
  // a wait that ran out means a tile was used before its producer finished: the factors of this
  // matrix are wrong, which the breakdown word says (the warning bit says why)
  if (expired && lane == 0) {
    atomicOr(&a.info[z * kInfoPerMat + kWarnSlot], kWarnWaitExpired);
    atomicCAS(&a.info[z * kInfoPerMat + a.info_slot], 0, o + 1);
  }
}

__global__ __launch_bounds__(kCholThreads) void k_chol256(CholArgs a) {
  extern __shared__ __align__(16) char lds_raw[];
  chol256_block(a, blockIdx.x, lds_raw);
}

}  // namespace od
