// LDS-tiled matrix-core contraction for gfx950: one workgroup computes an MT x NT tile of
// C = A * B^T-like products over a K range, with both operands staged through LDS as
// [row][k] tiles of 16-byte k-groups (8 half-precision values), double buffered.
//
// Operand tiles come from "loaders" that read global memory in whichever direction is
// contiguous and always write the same LDS layout:
//   LoadKC  memory is [operand row][k]  (k contiguous): one 8-element vector load per item.
//   LoadKS  memory is [k][operand row]  (operand row contiguous): eight 4-element loads
//           (8 consecutive k, 4 consecutive operand rows) transposed in registers.
// The loads of step i+1 are issued before the matrix-core work of step i and converted
// and written to the other LDS buffer after it, so one barrier per step suffices.
#pragma once

#include <type_traits>

#include "od_common.h"

namespace od {

template <int MT_, int NT_, int KT_, int WM_, int WN_>
struct Tile {
  static constexpr int MT = MT_, NT = NT_, KT = KT_, WM = WM_, WN = WN_;
  static constexpr int THREADS = kWave * WM * WN;
  static constexpr int WTM = MT / WM, WTN = NT / WN;      // per-wave tile
  static constexpr int FM = WTM / 32, FN = WTN / 32;      // 32x32 accumulator tiles per wave
  static constexpr int KG = KT / 8;                       // 16-byte k-groups per row
  static constexpr int PITCH = KT * 2 + 16;               // bytes per LDS row (padded)
  static constexpr int PLANE_A = MT * PITCH, PLANE_B = NT * PITCH;
  static_assert(MT % (32 * WM) == 0 && NT % (32 * WN) == 0 && KT % 16 == 0, "tile shape");
  template <class Num>
  static constexpr int lds_bytes() { return 2 * Num::PARTS * (PLANE_A + PLANE_B); }
};

template <class Src, int ROWS, int KT, int PITCH, int THREADS>
struct LoadKC {
  static constexpr int KG = KT / 8, ITEMS = ROWS * KG, PER = (ITEMS + THREADS - 1) / THREADS;
  typename Src::Raw8 raw[PER];
  OD_DEV void load(const Src& s, int row0, int k0, int tid) {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int item = tid + p * THREADS;
      if (ITEMS % THREADS == 0 || item < ITEMS) raw[p] = s.load8(row0 + item / KG, k0 + (item % KG) * 8);
    }
  }
  // the tile rows and every k below kpad lie inside the source
  OD_DEV static bool interior(const Src& s, int row0, int kpad) { return row0 + ROWS <= s.rows() && kpad <= s.cols(); }
  // load() for an interior tile: no bounds checks, hence no branches
  OD_DEV void loadu(const Src& s, int row0, int k0, int tid) {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int item = tid + p * THREADS;
      if (ITEMS % THREADS != 0) item %= ITEMS;         // surplus threads repeat a valid item; store() skips them
      raw[p] = s.load8u(row0 + item / KG, k0 + (item % KG) * 8);
    }
  }
  template <class Num>
  OD_DEV void store(char* lds, int plane, float scale, int tid) const {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int item = tid + p * THREADS;
      if (ITEMS % THREADS == 0 || item < ITEMS) {
        char* dst = lds + (item / KG) * PITCH + (item % KG) * 16;
        if constexpr (Src::PACKED) {
          static_assert(Num::PARTS == 1, "packed operands have one part");
          *reinterpret_cast<u32x4*>(dst) = raw[p];
        } else {
          float x[8];
          Src::unpack8(raw[p], x);
          u32x4 w[Num::PARTS];
          Num::pack(x, scale, w);
#pragma unroll
          for (int s = 0; s < Num::PARTS; ++s) *reinterpret_cast<u32x4*>(dst + s * plane) = w[s];
        }
      }
    }
  }
};

template <class Src, int ROWS, int KT, int PITCH, int THREADS>
struct LoadKS {
  static constexpr int RQ = ROWS / 4, KG = KT / 8, ITEMS = RQ * KG, PER = (ITEMS + THREADS - 1) / THREADS;
  typename Src::Raw4 raw[PER][8];
  OD_DEV void load(const Src& s, int row0, int k0, int tid) {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int item = tid + p * THREADS;
      if (ITEMS % THREADS == 0 || item < ITEMS) {
        int rq = item % RQ, kg = item / RQ;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) raw[p][kk] = s.load4(k0 + kg * 8 + kk, row0 + rq * 4);
      }
    }
  }
  OD_DEV static bool interior(const Src& s, int row0, int kpad) { return kpad <= s.rows() && row0 + ROWS <= s.cols(); }
  OD_DEV void loadu(const Src& s, int row0, int k0, int tid) {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int item = tid + p * THREADS;
      if (ITEMS % THREADS != 0) item %= ITEMS;
      int rq = item % RQ, kg = item / RQ;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) raw[p][kk] = s.load4u(k0 + kg * 8 + kk, row0 + rq * 4);
    }
  }
  template <class Num>
  OD_DEV void store(char* lds, int plane, float scale, int tid) const {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int item = tid + p * THREADS;
      if (ITEMS % THREADS == 0 || item < ITEMS) {
        int rq = item % RQ, kg = item / RQ;
        float x[8][4];
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) Src::unpack4(raw[p][kk], x[kk]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float col[8];
#pragma unroll
          for (int kk = 0; kk < 8; ++kk) col[kk] = x[kk][j];
          u32x4 w[Num::PARTS];
          Num::pack(col, scale, w);
          char* dst = lds + (rq * 4 + j) * PITCH + kg * 16;
#pragma unroll
          for (int s = 0; s < Num::PARTS; ++s) *reinterpret_cast<u32x4*>(dst + s * plane) = w[s];
        }
      }
    }
  }
};

// LoadKS for tiles so small that four-row items would leave most threads without work:
// one operand row and 8 consecutive k per item, eight scalar loads (adjacent lanes read
// adjacent rows, so a wave instruction still covers whole 256-byte segments).
template <class Src, int ROWS, int KT, int PITCH, int THREADS>
struct LoadKS1 {
  static constexpr int KG = KT / 8, ITEMS = ROWS * KG, PER = (ITEMS + THREADS - 1) / THREADS;
  float raw[PER][8];
  OD_DEV void load(const Src& s, int row0, int k0, int tid) {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int item = tid + p * THREADS;
      if (ITEMS % THREADS == 0 || item < ITEMS) {
        int row = item % ROWS, kg = item / ROWS;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) raw[p][kk] = s.load1(k0 + kg * 8 + kk, row0 + row);
      }
    }
  }
  OD_DEV static bool interior(const Src& s, int row0, int kpad) { return kpad <= s.rows() && row0 + ROWS <= s.cols(); }
  OD_DEV void loadu(const Src& s, int row0, int k0, int tid) {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int item = tid + p * THREADS;
      if (ITEMS % THREADS != 0) item %= ITEMS;
      int row = item % ROWS, kg = item / ROWS;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) raw[p][kk] = s.load1u(k0 + kg * 8 + kk, row0 + row);
    }
  }
  template <class Num>
  OD_DEV void store(char* lds, int plane, float scale, int tid) const {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int item = tid + p * THREADS;
      if (ITEMS % THREADS == 0 || item < ITEMS) {
        int row = item % ROWS, kg = item / ROWS;
        u32x4 w[Num::PARTS];
        Num::pack(raw[p], scale, w);
        char* dst = lds + row * PITCH + kg * 16;
#pragma unroll
        for (int s = 0; s < Num::PARTS; ++s) *reinterpret_cast<u32x4*>(dst + s * plane) = w[s];
      }
    }
  }
};

// Loader selection by direction tag.
struct KC {};
struct KS {};
struct KSF {};
template <class Dir, class Src, int ROWS, int KT, int PITCH, int THREADS>
struct LoaderFor;
template <class Src, int ROWS, int KT, int PITCH, int THREADS>
struct LoaderFor<KC, Src, ROWS, KT, PITCH, THREADS> { typedef LoadKC<Src, ROWS, KT, PITCH, THREADS> type; };
template <class Src, int ROWS, int KT, int PITCH, int THREADS>
struct LoaderFor<KS, Src, ROWS, KT, PITCH, THREADS> { typedef LoadKS<Src, ROWS, KT, PITCH, THREADS> type; };
// KSF: like KS, but the one-row loader wherever four-row items would not occupy every thread
template <class Src, int ROWS, int KT, int PITCH, int THREADS>
struct LoaderFor<KSF, Src, ROWS, KT, PITCH, THREADS> {
  static constexpr bool kFine = Src::HAS_LOAD1 && (ROWS / 4) * (KT / 8) < THREADS;
  typedef typename std::conditional<kFine, LoadKS1<Src, ROWS, KT, PITCH, THREADS>, LoadKS<Src, ROWS, KT, PITCH, THREADS>>::type type;
};

// One KT-deep step of matrix-core work from the LDS tiles.
template <class T, class Num>
OD_DEV void mma_step(const char* ldsA, const char* ldsB, f32x16 (&acc)[T::FM][T::FN], int wm, int wn, int lane) {
#pragma unroll
  for (int kk = 0; kk < T::KT / 16; ++kk) {
    const int kg = 2 * kk + (lane >> 5);
    u32x4 af[Num::PARTS][T::FM], bf[Num::PARTS][T::FN];
#pragma unroll
    for (int s = 0; s < Num::PARTS; ++s) {
#pragma unroll
      for (int fm = 0; fm < T::FM; ++fm)
        af[s][fm] = *reinterpret_cast<const u32x4*>(ldsA + s * T::PLANE_A + (wm * T::WTM + fm * 32 + (lane & 31)) * T::PITCH + kg * 16);
#pragma unroll
      for (int fn = 0; fn < T::FN; ++fn)
        bf[s][fn] = *reinterpret_cast<const u32x4*>(ldsB + s * T::PLANE_B + (wn * T::WTN + fn * 32 + (lane & 31)) * T::PITCH + kg * 16);
    }
#pragma unroll
    for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
      for (int fn = 0; fn < T::FN; ++fn)
#pragma unroll
        for (int i = Num::PARTS - 1; i >= 0; --i)
#pragma unroll
          for (int j = Num::PARTS - 1 - i; j >= 0; --j)
            acc[fm][fn] = mfma_32x32x16<Num::F16>(af[i][fm], bf[j][fn], acc[fm][fn]);
  }
}

// The main loop: acc += sum over k in [kbeg, kend) of A(m0.., k) * B(n0.., k).
// `lds` must hold T::lds_bytes<Num>() bytes.  Ends with all waves past their last LDS read.
template <class T, class Num, class DirA, class SrcA, class DirB, class SrcB>
OD_DEV void gemm_mainloop(const SrcA& a, const SrcB& b, int m0, int n0, int kbeg, int kend,
                          float scaleA, float scaleB, char* lds, f32x16 (&acc)[T::FM][T::FN], int rot = 0) {
  typedef typename LoaderFor<DirA, SrcA, T::MT, T::KT, T::PITCH, T::THREADS>::type LA;
  typedef typename LoaderFor<DirB, SrcB, T::NT, T::KT, T::PITCH, T::THREADS>::type LB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / T::WN, wn = wave % T::WN;
  constexpr int BUF = Num::PARTS * (T::PLANE_A + T::PLANE_B);
  constexpr int OFF_B = Num::PARTS * T::PLANE_A;
  LA la;
  LB lb;
  if (kbeg >= kend) return;
  // The KT-deep steps are taken in rotated order, starting at step `rot` (mod the step
  // count).  Workgroups that run side by side and would otherwise walk the same k positions
  // in lockstep get different rotations from their caller (see k_proj).
  const int nsteps = (kend - kbeg + T::KT - 1) / T::KT;
  int cur = rot % nsteps;
  la.load(a, m0, kbeg + cur * T::KT, tid);
  lb.load(b, n0, kbeg + cur * T::KT, tid);
  la.template store<Num>(lds, T::PLANE_A, scaleA, tid);
  lb.template store<Num>(lds + OFF_B, T::PLANE_B, scaleB, tid);
  __syncthreads();
  int buf = 0;
  for (int i = 0; i < nsteps; ++i) {
    const bool more = (i + 1) < nsteps;
    cur = (cur + 1 == nsteps) ? 0 : cur + 1;
    if (more) {
      la.load(a, m0, kbeg + cur * T::KT, tid);
      lb.load(b, n0, kbeg + cur * T::KT, tid);
    }
    mma_step<T, Num>(lds + buf * BUF, lds + buf * BUF + OFF_B, acc, wm, wn, lane);
    if (more) {
      la.template store<Num>(lds + (buf ^ 1) * BUF, T::PLANE_A, scaleA, tid);
      lb.template store<Num>(lds + (buf ^ 1) * BUF + OFF_B, T::PLANE_B, scaleB, tid);
    }
    __syncthreads();
    buf ^= 1;
  }
}

// The same loop with the global loads of PF steps in flight (PF register stages per
// operand).  For short K loops on small grids, where a workgroup cannot hide the load
// latency behind other workgroups: the loads of step i + PF are issued before the
// matrix-core work of step i.
template <class T, class Num, class DirA, class SrcA, class DirB, class SrcB, int PF>
OD_DEV void gemm_mainloop_deep(const SrcA& a, const SrcB& b, int m0, int n0, int kbeg, int kend,
                               float scaleA, float scaleB, char* lds, f32x16 (&acc)[T::FM][T::FN], int rot = 0) {
  typedef typename LoaderFor<DirA, SrcA, T::MT, T::KT, T::PITCH, T::THREADS>::type LA;
  typedef typename LoaderFor<DirB, SrcB, T::NT, T::KT, T::PITCH, T::THREADS>::type LB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / T::WN, wn = wave % T::WN;
  constexpr int BUF = Num::PARTS * (T::PLANE_A + T::PLANE_B);
  constexpr int OFF_B = Num::PARTS * T::PLANE_A;
  if (kbeg >= kend) return;
  const int nsteps = (kend - kbeg + T::KT - 1) / T::KT;
  rot %= nsteps;
  // step i works on the k range of step (i + rot) mod nsteps (see gemm_mainloop)
  auto k_of = [&](int i) { const int c = i + rot; return kbeg + (c >= nsteps ? c - nsteps : c) * T::KT; };
  LA la[PF];
  LB lb[PF];
  // (small tiles are chosen for short K loops on small grids: they keep the simple loop only)
  if (T::MT * T::NT >= 128 * 128 && nsteps >= 2 * PF && LA::interior(a, m0, kbeg + nsteps * T::KT) &&
      LB::interior(b, n0, kbeg + nsteps * T::KT)) {
    // Both tiles lie inside their sources for every step: loads without bounds checks, and a
    // main loop of straight-line code, so that the wait before a store to LDS is for the
    // oldest register stage only (the younger PF - 1 stay in flight across the barrier).
#pragma unroll
    for (int p = 0; p < PF; ++p) {
      la[p].loadu(a, m0, k_of(p), tid);
      lb[p].loadu(b, n0, k_of(p), tid);
    }
    la[0].template store<Num>(lds, T::PLANE_A, scaleA, tid);
    lb[0].template store<Num>(lds + OFF_B, T::PLANE_B, scaleB, tid);
    __syncthreads();
    int i = 0;
    for (; i + 2 * PF <= nsteps; i += PF) {        // every refill below is a step that exists
#pragma unroll
      for (int j = 0; j < PF; ++j) {
        const int step = i + j, buf = step & 1;    // step lives in register stage j
        la[j].loadu(a, m0, k_of(step + PF), tid);
        lb[j].loadu(b, n0, k_of(step + PF), tid);
        __builtin_amdgcn_sched_barrier(0);         // the loads stay ahead of the matrix-core work
        mma_step<T, Num>(lds + buf * BUF, lds + buf * BUF + OFF_B, acc, wm, wn, lane);
        la[(j + 1) % PF].template store<Num>(lds + (buf ^ 1) * BUF, T::PLANE_A, scaleA, tid);
        lb[(j + 1) % PF].template store<Num>(lds + (buf ^ 1) * BUF + OFF_B, T::PLANE_B, scaleB, tid);
        __syncthreads();
      }
    }
    // the last PF .. 2 PF - 1 steps: stage t % PF holds step i + t, the tile of step i is in LDS
#pragma unroll
    for (int t = 0; t < 2 * PF - 1; ++t) {
      const int step = i + t, buf = step & 1;
      if (step < nsteps) {
        if (step + PF < nsteps) {
          la[t % PF].loadu(a, m0, k_of(step + PF), tid);
          lb[t % PF].loadu(b, n0, k_of(step + PF), tid);
        }
        mma_step<T, Num>(lds + buf * BUF, lds + buf * BUF + OFF_B, acc, wm, wn, lane);
        if (step + 1 < nsteps) {
          la[(t + 1) % PF].template store<Num>(lds + (buf ^ 1) * BUF, T::PLANE_A, scaleA, tid);
          lb[(t + 1) % PF].template store<Num>(lds + (buf ^ 1) * BUF + OFF_B, T::PLANE_B, scaleB, tid);
        }
        __syncthreads();
      }
    }
    return;
  }
#pragma unroll
  for (int p = 0; p < PF; ++p) {
    if (p < nsteps) {
      la[p].load(a, m0, k_of(p), tid);
      lb[p].load(b, n0, k_of(p), tid);
    }
  }
  la[0].template store<Num>(lds, T::PLANE_A, scaleA, tid);
  lb[0].template store<Num>(lds + OFF_B, T::PLANE_B, scaleB, tid);
  __syncthreads();
  for (int i0 = 0; i0 < nsteps; i0 += PF) {
#pragma unroll
    for (int j = 0; j < PF; ++j) {
      const int i = i0 + j;                    // step i lives in register stage j
      if (i < nsteps) {
        const int buf = i & 1;
        if (i + PF < nsteps) {                 // stage j went to LDS one step ago: refill it
          la[j].load(a, m0, k_of(i + PF), tid);
          lb[j].load(b, n0, k_of(i + PF), tid);
        }
        mma_step<T, Num>(lds + buf * BUF, lds + buf * BUF + OFF_B, acc, wm, wn, lane);
        if (i + 1 < nsteps) {
          la[(j + 1) % PF].template store<Num>(lds + (buf ^ 1) * BUF, T::PLANE_A, scaleA, tid);
          lb[(j + 1) % PF].template store<Num>(lds + (buf ^ 1) * BUF + OFF_B, T::PLANE_B, scaleB, tid);
        }
        __syncthreads();
      }
    }
  }
}

template <class T>
OD_DEV void zero_acc(f32x16 (&acc)[T::FM][T::FN]) {
#pragma unroll
  for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
    for (int fn = 0; fn < T::FN; ++fn)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[fm][fn][v] = 0.f;
}

// Visit every accumulator element of this lane: f(row, col, value) in tile coordinates
// offset by (m0, n0).
template <class T, class F>
OD_DEV void for_each_acc(const f32x16 (&acc)[T::FM][T::FN], int m0, int n0, F&& f) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / T::WN, wn = wave % T::WN;
#pragma unroll
  for (int fm = 0; fm < T::FM; ++fm)
#pragma unroll
    for (int fn = 0; fn < T::FN; ++fn)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        f(m0 + wm * T::WTM + fm * 32 + acc_row(v, lane), n0 + wn * T::WTN + fn * 32 + acc_col(lane), acc[fm][fn][v]);
}

}  // namespace od
