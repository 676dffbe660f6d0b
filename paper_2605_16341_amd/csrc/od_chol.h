// Cholesky factorisation and triangular inverse of one SPD block of up to 256 x 256 in a
// single workgroup (4 waves):  G = T^T T with T upper triangular, W = T^-1.
//
// Used by the CholeskyQR orthogonalisation (orth() of Alg. 1 lines 2 and 4): T is the
// triangular factor of the thin QR, W turns the triangular solve into a product.
//
// Layout of the computation
//   * The block is cut into 32 x 32 tiles; only tiles (I, K) with I <= K are kept, each as a
//     matrix-core accumulator (16 registers per lane) owned by one wave, so the trailing
//     matrix never leaves the register file.
//   * Step J: (a) the owner of the diagonal tile factors it and inverts its factor inside
//     the wave, rows in lanes, columns in registers, broadcasting with readlane;
//     (b) the owners of the tiles (J, K) form T(J, K) = W_JJ^T S(J, K) on the matrix cores;
//     (c) every remaining tile gets S(I, K) -= T(J, I)^T T(J, K).
//     An accumulator tile serves directly as the k-side operand of the next product: register
//     v of lane l is row 8 (v / 4) + 4 (l / 32) + v % 4, and the other operand is read from
//     LDS in that same row order, so no data moves between lanes.
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
constexpr int kCPitch = 36;            // floats per LDS tile row (16-byte aligned, conflict free)
constexpr int kCTileF = kCT * kCPitch; // floats per LDS tile
// LDS: Wrow[8] | Wt | Dtmp | panel[8]
constexpr int kCholLds = (kCNT + 1 + 1 + kCNT) * kCTileF * 4;

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
  float* scal;         // if non-null: scal[z * kScalPerMat + 1] = power-of-two scale from the trace
  int trace_rows;      // rows of the tall matrix whose Gram this is (for the scale)
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

// 1/sqrt(d) and 1/d to fp32 accuracy: hardware estimate (1 ulp) plus one Newton step.
OD_DEV float fast_rsqrt(float d) {
  float y = __builtin_amdgcn_rsqf(d);
  return y * fmaf(-0.5f * d * y, y, 1.5f);
}
OD_DEV float fast_rcp(float d) {
  float y = __builtin_amdgcn_rcpf(d);
  return y * fmaf(-d, y, 2.f);
}

OD_DEV void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  __builtin_amdgcn_wave_barrier();
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

// A-side operand of k-step kk from an LDS tile stored [row][k] with pitch kCPitch:
// this lane's row is l % 32 and its 8 k-slots are 16 kk + 4 g + {0..3} and 16 kk + 8 + 4 g + {0..3}.
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

// Transposed store of an accumulator tile into an LDS tile: element (row, col) -> [col][row].
OD_DEV void store_tile_transposed(float* tile, const f32x16& acc, int lane) {
  float* p = tile + (lane & 31) * kCPitch + 4 * (lane >> 5);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    f32x4 v = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
    *reinterpret_cast<f32x4*>(p + 8 * q) = v;
  }
}

__global__ __launch_bounds__(256) void k_chol256(CholArgs a) {
  extern __shared__ __align__(16) char lds_raw[];
  float* Wrow = reinterpret_cast<float*>(lds_raw);            // W_JJ, [i][k], one tile per J
  float* Wt = Wrow + kCNT * kCTileF;                         // W_JJ^T of the current step
  float* Dtmp = Wt + kCTileF;                                // staging of the diagonal tile
  float* panel = Dtmp + kCTileF;                             // T(J, K)^T, one tile per K

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
  // ---- load the owned tiles (sum of the split partials); identity outside the block
  f32x16 acc[kCSlots];
  float tr = 0.f;
#pragma unroll
  for (int s = 0; s < kCSlots; ++s)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[s][v] = 0.f;
  // split by split, so that the loads of one split are all in flight together.  The Gram
  // matrix is symmetric: the 4 consecutive rows a lane needs of column gj are read as 4
  // consecutive columns of row gj (one 16-byte load).
  for (int sp = 0; sp < a.splits; ++sp) {
    const float* sp_src = src + (int64_t)sp * a.split_stride;
#pragma unroll
    for (int s = 0; s < kCSlots; ++s) {
      const int t = s * 4 + wave, I = kTileI[t], K = kTileK[t];
      if (I < nt && K < nt) {
        const int gj = K * kCT + col;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int gi = I * kCT + 8 * q + 4 * half;
          if (gi < nb && gj < nb) {
            f32x4 v4 = *reinterpret_cast<const f32x4*>(sp_src + (int64_t)gj * r + gi);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[s][4 * q + e] += v4[e];
          }
        }
      }
    }
  }
#pragma unroll
  for (int s = 0; s < kCSlots; ++s) {
    const int t = s * 4 + wave, I = kTileI[t], K = kTileK[t];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int gi = I * kCT + acc_row(v, lane), gj = K * kCT + col;
      const bool inside = I < nt && K < nt && gi < nb && gj < nb;
      if (!inside) acc[s][v] = (gi == gj) ? 1.f : 0.f;
      else if (gi == gj) tr += acc[s][v];
    }
  }
  if (a.scal != nullptr) {       // trace -> power-of-two scale of the tall matrix (uniform branch)
    __shared__ float s_tr[256];
    s_tr[tid] = tr;
    __syncthreads();
    for (int w2 = 128; w2 > 0; w2 >>= 1) {
      if (tid < w2) s_tr[tid] += s_tr[tid + w2];
      __syncthreads();
    }
    if (tid == 0) {
      float ms = s_tr[0] / ((float)a.trace_rows * (float)r);
      float sc = 1.f;
      if (ms > 0.f && ms < 3.0e38f) sc = ldexpf(1.f, -ilogbf(sqrtf(ms)));
      a.scal[z * kScalPerMat + 1] = sc;
    }
  }
  __syncthreads();

  OD_TICK(1);
  // ================================ factorisation ================================
  for (int J = 0; J < nt; ++J) {
    OD_TICK(2 + 4 * J);
    // ---- (a) diagonal tile: Cholesky and inverse inside the owning wave
    {
      // tile (J, J) is entry t = sum_{i=J+1..7} (8 - i) = (7 - J)(8 - J) / 2 of the enumeration
      const int t = (7 - J) * (8 - J) / 2;
      if ((t & 3) == wave) {
        const int slot = t >> 2;
        f32x16 d;
#pragma unroll
        for (int s = 0; s < kCSlots; ++s)
          if (s == slot) d = acc[s];
        // stage [row][col] so that lane i can pick up row i
#pragma unroll
        for (int v = 0; v < 16; ++v) Dtmp[acc_row(v, lane) * kCPitch + col] = d[v];
        wave_lds_fence();
        float rowv[32];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          f32x4 v4 = *reinterpret_cast<const f32x4*>(Dtmp + col * kCPitch + 4 * q);
          rowv[4 * q] = v4[0]; rowv[4 * q + 1] = v4[1]; rowv[4 * q + 2] = v4[2]; rowv[4 * q + 3] = v4[3];
        }
        // right-looking Cholesky, lane i = row i (both lane halves compute the same)
        int bad = 0;
#pragma unroll
        for (int k = 0; k < 32; ++k) {
          float dk = lane_bcast(rowv[k], k);
          if (!(dk > 0.f) || dk > 3.0e38f) {
            if (bad == 0) bad = J * kCT + k + 1;
            dk = 1.f;
          }
          const float rs = fast_rsqrt(dk);
          const float sq = dk * rs;
          const float tk = rowv[k] * (rs * rs);
          rowv[k] = (col == k) ? sq : rowv[k] * rs;
#pragma unroll
          for (int j = k + 1; j < 32; ++j) rowv[j] = fmaf(-tk, lane_bcast(rowv[j], k), rowv[j]);
          __builtin_amdgcn_sched_barrier(0);     // keep the broadcasts of one column together
        }
#pragma unroll
        for (int j = 0; j < 32; ++j)
          if (j > col) rowv[j] = 0.f;            // rowv[j] = L[col][j]
        if (bad != 0 && lane == 0) {
          atomicCAS(&a.info[z * kInfoPerMat + a.info_slot], 0, o + bad);
        }
        // inverse of L: lane c = column c, m[i] = M[i][c]
        float m[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) {
          float s = 0.f;
#pragma unroll
          for (int k = 0; k < i; ++k) s = fmaf(lane_bcast(rowv[k], i), m[k], s);
          const float dinv = fast_rcp(lane_bcast(rowv[i], i));
          m[i] = ((col == i) ? 1.f : -s) * dinv;
          __builtin_amdgcn_sched_barrier(0);
        }
        const int nv = (nb - J * kCT) < kCT ? (nb - J * kCT) : kCT;   // valid rows / cols of this tile
        if (half == 0) {
          // W_JJ^T = M, [i][k] = M[i][k]: lane k holds column k
#pragma unroll
          for (int i = 0; i < 32; ++i) Wt[i * kCPitch + col] = m[i];
          // W_JJ, [c][i] = M[i][c]: lane c writes its 32 values contiguously
          float* wr = Wrow + J * kCTileF + col * kCPitch;
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            f32x4 v4 = {m[4 * q], m[4 * q + 1], m[4 * q + 2], m[4 * q + 3]};
            *reinterpret_cast<f32x4*>(wr + 4 * q) = v4;
          }
          // global: T_JJ[j][i] = L[i][j];  W_JJ[c][i] = M[i][c]
          if (col < nv) {
            float* tcol = tg + (int64_t)(J * kCT) * r + J * kCT + col;
#pragma unroll
            for (int j = 0; j < 32; ++j)
              if (j < nv) tcol[(int64_t)j * r] = rowv[j];
            float* wrow = wg + (int64_t)(J * kCT + col) * r + J * kCT;
#pragma unroll
            for (int q = 0; q < 8; ++q)
              if (4 * q < nv) {
                f32x4 v4 = {m[4 * q], m[4 * q + 1], m[4 * q + 2], m[4 * q + 3]};
                *reinterpret_cast<f32x4*>(wrow + 4 * q) = v4;
              }
          }
        }
      }
    }
    OD_TICK(3 + 4 * J);
    __syncthreads();
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
        store_tile_transposed(panel + K * kCTileF, res, lane);
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
    // ---- (c) trailing update: S(I, K) -= T(J, I)^T T(J, K), J < I <= K
#pragma unroll
    for (int s = 0; s < kCSlots; ++s) {
      const int t = s * 4 + wave, I = kTileI[t], K = kTileK[t];
      if (I > J && K < nt) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          u32x4 ap[3], bp[3];
          lds_operand(panel + I * kCTileF, lane, kk, ap);
          lds_operand(panel + K * kCTileF, lane, kk, bp);
          negate3(ap);
          acc[s] = mma6(ap, bp, acc[s]);
        }
      }
    }
    // the next (a) writes Wt / Dtmp only after every wave is done with this step's (b);
    // the next (b) writes `panel` only after the barrier that follows (a).
  }
  OD_TICK(40);
  __syncthreads();     // all of T is in global memory and visible to this workgroup
  OD_TICK(41);

  // ================================ inverse ================================
  // Wave w builds block columns K = w, 7 - w (in that order the long and the short one pair up).
  for (int pass = 0; pass < 2; ++pass) {
    const int K = pass == 0 ? (kCNT - 1 - wave) : wave;
    if (K >= nt) continue;
    f32x16 wcol[kCNT];        // W(I, K), I <= K
    // W(K, K) from LDS in accumulator layout
#pragma unroll
    for (int v = 0; v < 16; ++v) wcol[kCNT - 1][v] = 0.f;
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
  // lower block triangle of T and W inside this block: zero (tiles strictly below the diagonal)
  for (int idx = tid; idx < nb * nb; idx += 256) {
    const int i = idx / nb, j = idx % nb;
    if ((i / kCT) > (j / kCT)) {
      tg[(int64_t)i * r + j] = 0.f;
      wg[(int64_t)i * r + j] = 0.f;
    }
  }
}

}  // namespace od
