// Cholesky factorisation and triangular inverse of one SPD block of up to 256 x 256 in a
// single workgroup (4 waves):  G = T^T T with T upper triangular, W = T^-1.
//
// Used by the CholeskyQR orthogonalisation (orth() of Alg. 1 lines 2 and 4): T is the
// triangular factor of the thin QR, W turns the triangular solve into a product.
//
// Layout of the computation
//   * The block is cut into 32 x 32 tiles; only tiles (I, K) with I <= K are kept, each as a
//     matrix-core accumulator (16 registers per lane: register v of lane l is row
//     8 (v / 4) + 4 (l / 32) + v % 4, column l % 32) owned by one wave, so the trailing
//     matrix never leaves the register file.
//   * Step J, (a): the owner of the diagonal tile factors it in place, four rows at a time.
//     The 4 x 4 diagonal block is gathered with readlane, factored and inverted in scalar
//     (wave-uniform) arithmetic; the new rows are a 4 x 4 product inside each lane; the
//     rank-4 trailing update of the tile is one matrix-core product whose operands are the
//     four registers just written.  The same operations applied to an identity tile give
//     the inverse of the tile's factor at no extra data movement.
//     (b): owners of the tiles (J, K) form T(J, K) = W_JJ^T S(J, K) on the matrix cores, the
//     accumulator tile serving directly as the k-side operand, and publish it to LDS
//     already split into three bf16 terms in the operand's register order.
//     (c): every remaining tile gets S(I, K) -= T(J, I)^T T(J, K) from those LDS operands.
//   * All products use three-way split bf16 operands (six products, 24 significant bits).
//   * The inverse is then built one block column per wave by back substitution with the
//     same tile products; T is read back from global memory (written earlier by this same
//     workgroup), the diagonal inverses from LDS.
#pragma once

#include "od_common.h"
#include "od_kernels.h"

namespace od {

constexpr int kCholMax = 256;          // largest block one workgroup factors
constexpr int kCT = 32;                // tile size
constexpr int kCNT = kCholMax / kCT;   // 8 tiles per side
constexpr int kCTiles = kCNT * (kCNT + 1) / 2;   // 36
constexpr int kCSlots = kCTiles / 4;   // 9 tiles per wave
constexpr int kCPitch = 36;            // floats per row of an fp32 LDS tile (16-byte aligned, conflict free)
constexpr int kCTileF = kCT * kCPitch; // floats per fp32 LDS tile
constexpr int kPPitch = 80;            // bytes per row of a pre-split operand tile (32 bf16 + pad)
constexpr int kPPlane = kCT * kPPitch; // bytes per part of a pre-split tile
constexpr int kPTile = 3 * kPPlane;    // bytes per pre-split tile
constexpr int kStagePitch = kCholMax + 4;        // floats per staged input row
// LDS: Wrow[8] fp32 | Wt fp32 | panel[8] pre-split | (input staging aliases the panel)
constexpr int kCholOffWt = kCNT * kCTileF * 4;
constexpr int kCholOffPanel = kCholOffWt + kCTileF * 4;
constexpr int kCholPanelBytes = kCNT * kPTile;
constexpr int kCholStageBytes = kCT * kStagePitch * 4;
constexpr int kCholLds = kCholOffPanel + (kCholPanelBytes > kCholStageBytes ? kCholPanelBytes : kCholStageBytes);

#ifdef OD_CHOL_TIMING
#define OD_TICK(slot) do { if (lane == 0) a.dbg[(z * 4 + wave) * 64 + (slot)] = wall_clock64(); } while (0)
#else
#define OD_TICK(slot) do { } while (0)
#endif

struct CholArgs {
  WsArr src;           // Gram block source: `splits` partial sums, `split_stride` elements apart
  int splits;
  int64_t split_stride;
  WsArr t, w;          // outputs, r x r each (ld r)
  int r;               // matrix order (ld of everything)
  int blk;             // which diagonal block of kCholMax
  int* info;
  int info_slot;
#ifdef OD_CHOL_TIMING
  long long* dbg;
#endif
};

// tile enumeration: I descending, K ascending; tile t belongs to wave t % 4, slot t / 4
__device__ __constant__ const unsigned char kTileI[kCTiles] = {7, 6, 6, 5, 5, 5, 4, 4, 4, 4, 3, 3, 3, 3, 3, 2, 2, 2,
                                                               2, 2, 2, 1, 1, 1, 1, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0, 0};
__device__ __constant__ const unsigned char kTileK[kCTiles] = {7, 6, 7, 5, 6, 7, 4, 5, 6, 7, 3, 4, 5, 6, 7, 2, 3, 4,
                                                               5, 6, 7, 1, 2, 3, 4, 5, 6, 7, 0, 1, 2, 3, 4, 5, 6, 7};

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

// the same for 4 values in the first four k-slots, the other four being zero
OD_DEV void split3_four(const float* x, u32x4* parts) {
  float rem[4] = {x[0], x[1], x[2], x[3]};
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    const uint32_t p0 = pack_bf16_rne(rem[0], rem[1]), p1 = pack_bf16_rne(rem[2], rem[3]);
    parts[s] = u32x4{p0, p1, 0u, 0u};
    if (s < 2) {
      rem[0] -= bf16_lo(p0); rem[1] -= bf16_hi(p0); rem[2] -= bf16_lo(p1); rem[3] -= bf16_hi(p1);
    }
  }
}

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
// The same from a row-major global matrix (ld elements); rows >= rows_valid or k >= k_valid read 0.
OD_DEV void global_operand(const float* base, int64_t ld, int rows_valid, int k_valid, int lane, int kk, u32x4* parts) {
  const int row = lane & 31, k0 = 16 * kk + 4 * (lane >> 5);
  float x[8];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int k = k0 + 8 * h;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (row < rows_valid && k < k_valid) v = *reinterpret_cast<const f32x4*>(base + (int64_t)row * ld + k);
#pragma unroll
    for (int e = 0; e < 4; ++e) x[4 * h + e] = v[e];
  }
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

// ---------------------------------------------------------------------------------------
// Diagonal tile: in-place upper Cholesky factor of the symmetric tile `d` and, in `zt`, the
// inverse of its transpose (M = L^-1, lower triangular), both in accumulator layout.
// Returns the 1-based index of the first bad pivot within the tile, or 0.
// ---------------------------------------------------------------------------------------
OD_DEV int diag_tile_factor(f32x16& d, f32x16& zt, int lane) {
  const int c = lane & 31, h = lane >> 5;
  int bad = 0;
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
    float p0 = d00;
    if (!(p0 > 0.f) || p0 > 3.0e38f) { if (bad == 0) bad = 4 * g + 1; p0 = 1.f; }
    const float i00 = fast_rsqrt(p0);
    const float t01 = d01 * i00, t02 = d02 * i00, t03 = d03 * i00;
    float p1 = d11 - t01 * t01;
    if (!(p1 > 0.f) || p1 > 3.0e38f) { if (bad == 0) bad = 4 * g + 2; p1 = 1.f; }
    const float i11 = fast_rsqrt(p1);
    const float t12 = (d12 - t01 * t02) * i11, t13 = (d13 - t01 * t03) * i11;
    float p2 = d22 - t02 * t02 - t12 * t12;
    if (!(p2 > 0.f) || p2 > 3.0e38f) { if (bad == 0) bad = 4 * g + 3; p2 = 1.f; }
    const float i22 = fast_rsqrt(p2);
    const float t23 = (d23 - t02 * t03 - t12 * t13) * i22;
    float p3 = d33 - t03 * t03 - t13 * t13 - t23 * t23;
    if (!(p3 > 0.f) || p3 > 3.0e38f) { if (bad == 0) bad = 4 * g + 4; p3 = 1.f; }
    const float i33 = fast_rsqrt(p3);
    // inverse of the 4 x 4 upper factor
    const float w01 = -(t01 * i11) * i00, w12 = -(t12 * i22) * i11, w23 = -(t23 * i33) * i22;
    const float w02 = -(t01 * w12 + t02 * i22) * i00, w13 = -(t12 * w23 + t13 * i33) * i11;
    const float w03 = -(t01 * w13 + t02 * w23 + t03 * i33) * i00;
    // new rows of the factor and of the inverse: (W4^T s)_a = sum_{b <= a} W4[b][a] s_b
    const float s0 = d[4 * q + 0], s1 = d[4 * q + 1], s2 = d[4 * q + 2], s3 = d[4 * q + 3];
    const float z0 = zt[4 * q + 0], z1 = zt[4 * q + 1], z2 = zt[4 * q + 2], z3 = zt[4 * q + 3];
    float tn[4], zn[4];
    tn[0] = i00 * s0;
    tn[1] = w01 * s0 + i11 * s1;
    tn[2] = w02 * s0 + w12 * s1 + i22 * s2;
    tn[3] = w03 * s0 + w13 * s1 + w23 * s2 + i33 * s3;
    zn[0] = i00 * z0;
    zn[1] = w01 * z0 + i11 * z1;
    zn[2] = w02 * z0 + w12 * z1 + i22 * z2;
    zn[3] = w03 * z0 + w13 * z1 + w23 * z2 + i33 * z3;
    const bool mine = h == hh;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (!mine || c < 4 * g + e) tn[e] = 0.f;       // row 4g+e of an upper factor starts at its diagonal
      if (!mine) zn[e] = 0.f;
    }
    if (g < 7) {
      // rank-4 update of both tiles: -T_g^T T_g and -T_g^T Z_g; the four values sit in the
      // first k-slots of this lane half, every other slot is zero
      u32x4 ta[3], tb[3], zb[3];
      split3_four(tn, tb);
      split3_four(zn, zb);
#pragma unroll
      for (int s = 0; s < 3; ++s) ta[s] = tb[s];
      negate3(ta);
      d = mma6(ta, tb, d);
      zt = mma6(ta, zb, zt);
    }
    // the rows of this group are final: put them (back) in place
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (mine) { d[4 * q + e] = tn[e]; zt[4 * q + e] = zn[e]; }
    }
  }
  return bad;
}

__global__ __launch_bounds__(256) void k_chol256(CholArgs a) {
  extern __shared__ __align__(16) char lds_raw[];
  float* Wrow = reinterpret_cast<float*>(lds_raw);                       // W_JJ, [i][k], one tile per J
  float* Wt = reinterpret_cast<float*>(lds_raw + kCholOffWt);            // W_JJ^T of the current step
  char* panel = lds_raw + kCholOffPanel;                                 // T(J, K)^T pre-split, one tile per K
  float* stage = reinterpret_cast<float*>(lds_raw + kCholOffPanel);      // input rows (before the loop only)

  const int z = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = a.r;
  const int o = a.blk * kCholMax;
  const int nb = (r - o) < kCholMax ? (r - o) : kCholMax;     // order of this block
  const int nt = (nb + kCT - 1) / kCT;                        // active tiles per side
  const int64_t off = (int64_t)o * r + o;
  const float* src = a.src.base + (int64_t)z * a.src.stride + off;
  float* tg = a.t.base + (int64_t)z * a.t.stride + off;
  float* wg = a.w.base + (int64_t)z * a.w.stride + off;
  const int col = lane & 31, half = lane >> 5;
  OD_TICK(0);

  // ---- tiles strictly below the diagonal of T and W are zero and written by nobody else
  {
    const int lower = nt * (nt - 1) / 2;
    for (int idx = tid; idx < lower * kCT * (kCT / 4); idx += 256) {
      const int tile = idx / (kCT * (kCT / 4)), e = idx % (kCT * (kCT / 4));
      // tile -> (I, K) with I > K: row-wise enumeration of the strict lower triangle
      int I = 1, base = 0;
      while (base + I <= tile) { base += I; ++I; }
      const int K = tile - base;
      const int gi = I * kCT + e / (kCT / 4), gj = K * kCT + (e % (kCT / 4)) * 4;
      if (gi < nb && gj < nb) {
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
        *reinterpret_cast<f32x4*>(tg + (int64_t)gi * r + gj) = zero;
        *reinterpret_cast<f32x4*>(wg + (int64_t)gi * r + gj) = zero;
      }
    }
  }

  // ---- load: 32 rows at a time through LDS (coalesced reads), then each owner picks its
  // tiles up in accumulator layout; identity outside the block
  f32x16 acc[kCSlots];
#pragma unroll
  for (int s = 0; s < kCSlots; ++s)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[s][v] = 0.f;
  constexpr int kPer = kCT * (kCholMax / 4) / 256;      // float4 per thread per 32 rows
  f32x4 pre[kPer];
  auto fetch = [&](int I) {
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const int idx = tid + u * 256;
      const int rr = idx / (kCholMax / 4), c4 = (idx % (kCholMax / 4)) * 4;
      f32x4 v4 = {0.f, 0.f, 0.f, 0.f};
      if (I * kCT + rr < nb && c4 < nb) {
        const float* p = src + (int64_t)(I * kCT + rr) * r + c4;
        v4 = *reinterpret_cast<const f32x4*>(p);
        for (int sp = 1; sp < a.splits; ++sp) v4 += *reinterpret_cast<const f32x4*>(p + (int64_t)sp * a.split_stride);
      }
      pre[u] = v4;
    }
  };
  fetch(0);
  for (int I = 0; I < nt; ++I) {
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const int idx = tid + u * 256;
      *reinterpret_cast<f32x4*>(stage + (idx / (kCholMax / 4)) * kStagePitch + (idx % (kCholMax / 4)) * 4) = pre[u];
    }
    __syncthreads();
    if (I + 1 < nt) fetch(I + 1);      // in flight while this block is picked up
#pragma unroll
    for (int s = 0; s < kCSlots; ++s) {
      const int t = s * 4 + wave;
      if (kTileI[t] == I && kTileK[t] < nt) {
        const int K = kTileK[t];
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[s][v] = stage[acc_row(v, lane) * kStagePitch + K * kCT + col];
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int s = 0; s < kCSlots; ++s) {
    const int t = s * 4 + wave, I = kTileI[t], K = kTileK[t];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int gi = I * kCT + acc_row(v, lane), gj = K * kCT + col;
      const bool inside = I < nt && K < nt && gi < nb && gj < nb;
      if (!inside) acc[s][v] = (gi == gj) ? 1.f : 0.f;
    }
  }
  OD_TICK(1);

  // ================================ factorisation ================================
  // (a) for tile (J, J): factor, invert, publish W_JJ (LDS and global) and T_JJ (global)
  auto do_diag = [&](int J) {
    const int t = (7 - J) * (8 - J) / 2;      // position of (J, J) in the enumeration
    const int slot = t >> 2;
    f32x16 d, zt;
#pragma unroll
    for (int s = 0; s < kCSlots; ++s)
      if (s == slot) d = acc[s];
    const int bad = diag_tile_factor(d, zt, lane);
    if (bad != 0 && lane == 0) atomicCAS(&a.info[z * kInfoPerMat + a.info_slot], 0, o + J * kCT + bad);
    const int nv = (nb - J * kCT) < kCT ? (nb - J * kCT) : kCT;   // valid rows / cols of this tile
    // zt = M with W_JJ = M^T.  LDS: Wt[i][k] = W_JJ[k][i] = M[i][k];  Wrow[i][k] = W_JJ[i][k] = M[k][i]
    float* wr = Wrow + J * kCTileF;
#pragma unroll
    for (int v = 0; v < 16; ++v) Wt[acc_row(v, lane) * kCPitch + col] = zt[v];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      f32x4 v4 = {zt[4 * q], zt[4 * q + 1], zt[4 * q + 2], zt[4 * q + 3]};
      *reinterpret_cast<f32x4*>(wr + col * kCPitch + 8 * q + 4 * half) = v4;
      // global W_JJ[c][rows] (row c of W = column c of M), 4 consecutive entries
      if (col < nv && 8 * q + 4 * half < nv)
        *reinterpret_cast<f32x4*>(wg + (int64_t)(J * kCT + col) * r + J * kCT + 8 * q + 4 * half) = v4;
    }
    if (col < nv) {
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (acc_row(v, lane) < nv) tg[(int64_t)(J * kCT + acc_row(v, lane)) * r + J * kCT + col] = d[v];
    }
  };
  // (c) for one owned tile: S(I, K) -= T(J, I)^T T(J, K)
  auto update_tile = [&](f32x16& tile, int I, int K) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
      u32x4 ap[3], bp[3];
      load_presplit(panel + I * kPTile, lane, kk, ap);
      load_presplit(panel + K * kPTile, lane, kk, bp);
      negate3(ap);
      tile = mma6(ap, bp, tile);
    }
  };

  if (((7 * 8 / 2) & 3) == wave) do_diag(0);
  __syncthreads();
  for (int J = 0; J < nt; ++J) {
    OD_TICK(4 + 4 * J);
    // ---- (b) row panel: T(J, K) = W_JJ^T S(J, K), K > J
#pragma unroll
    for (int s = 0; s < kCSlots; ++s) {
      const int t = s * 4 + wave, I = kTileI[t], K = kTileK[t];
      if (I == J && K > J && K < nt) {
        f32x16 res;
#pragma unroll
        for (int v = 0; v < 16; ++v) res[v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          u32x4 ap[3], bp[3];
          lds_operand(Wt, lane, kk, ap);
          acc_operand(acc[s], kk, bp);
          res = mma6(ap, bp, res);
        }
        acc[s] = res;
        store_presplit(panel + K * kPTile, res, lane);
        const int nvr = (nb - J * kCT) < kCT ? (nb - J * kCT) : kCT;
        if (K * kCT + col < nb) {
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (acc_row(v, lane) < nvr) tg[(int64_t)(J * kCT + acc_row(v, lane)) * r + K * kCT + col] = res[v];
        }
      }
    }
    __syncthreads();
    OD_TICK(5 + 4 * J);
    // ---- (c) trailing update, J < I <= K.  The owner of the next diagonal tile updates it
    // first and factors it at once, while the other waves finish their updates.
    const int tn = (6 - J) * (7 - J) / 2;           // position of (J + 1, J + 1)
    const bool next_mine = (J + 1 < nt) && ((tn & 3) == wave);
    if (next_mine) {
#pragma unroll
      for (int s = 0; s < kCSlots; ++s)
        if (s == (tn >> 2)) update_tile(acc[s], J + 1, J + 1);
      do_diag(J + 1);
    }
    OD_TICK(6 + 4 * J);
#pragma unroll
    for (int s = 0; s < kCSlots; ++s) {
      const int t = s * 4 + wave, I = kTileI[t], K = kTileK[t];
      if (I > J && K < nt && !(next_mine && t == tn)) update_tile(acc[s], I, K);
    }
    OD_TICK(7 + 4 * J);
    // next (b) reads Wt (written above) and rewrites `panel` (read above)
    __syncthreads();
  }
  OD_TICK(40);     // the loop's last barrier also makes all of T (global) visible to this workgroup
  OD_TICK(41);

  // ================================ inverse ================================
  // Wave w builds block columns K = 7 - w and w (the long and the short one pair up).
  for (int pass = 0; pass < 2; ++pass) {
    const int K = pass == 0 ? (kCNT - 1 - wave) : wave;
    if (K >= nt) continue;
    f32x16 wcol[kCNT];        // W(I, K), I <= K
#pragma unroll
    for (int Ii = kCNT - 1; Ii >= 0; --Ii) {
      if (Ii > K) continue;
      if (Ii == K) {
#pragma unroll
        for (int v = 0; v < 16; ++v) wcol[Ii][v] = Wrow[K * kCTileF + acc_row(v, lane) * kCPitch + col];
        continue;
      }
      // S = sum_{L = Ii+1..K} T(Ii, L) W(L, K)
      f32x16 sacc;
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
      for (int L = kCNT - 1; L >= 1; --L) {
        if (L <= Ii || L > K) continue;
        const float* tb = tg + (int64_t)(Ii * kCT) * r + L * kCT;
        const int kvalid = nb - L * kCT;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          u32x4 ap[3], bp[3];
          global_operand(tb, r, kCT, kvalid, lane, kk, ap);
          acc_operand(wcol[L], kk, bp);
          sacc = mma6(ap, bp, sacc);
        }
      }
      // W(Ii, K) = -W_II S
      f32x16 res;
#pragma unroll
      for (int v = 0; v < 16; ++v) res[v] = 0.f;
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        u32x4 ap[3], bp[3];
        lds_operand(Wrow + Ii * kCTileF, lane, kk, ap);
        negate3(ap);
        acc_operand(sacc, kk, bp);
        res = mma6(ap, bp, res);
      }
      wcol[Ii] = res;
      if (K * kCT + col < nb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) wg[(int64_t)(Ii * kCT + acc_row(v, lane)) * r + K * kCT + col] = res[v];
      }
    }
  }
  OD_TICK(42);
}

}  // namespace od
