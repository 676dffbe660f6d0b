// Shared device-side building blocks of the Orth-Dion HIP path for gfx950 (CDNA4):
// register/LDS vector types, matrix-core (MFMA) wrappers with their lane layouts,
// number formats for the matrix-core operands, and global-memory tile sources.
//
// Nothing here is shared with the CPU oracle.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace od {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kMaxBatch = 32;       // matrices of one shape class per launch
constexpr int kWave = 64;

#define OD_DEV __device__ __forceinline__

// ---------------------------------------------------------------------------------
// Matrix-core wrapper: D(32x32) += A(32x16) * B(16x32), fp32 accumulate.
// Operand fragment of lane l: row (A) or column (B) index l % 32, and the 8 consecutive
// k values 8*(l/32) .. 8*(l/32)+7, packed two per dword.  Accumulator register v of lane
// l is element (row 8*(v/4) + 4*(l/32) + v%4, column l%32).
// ---------------------------------------------------------------------------------
template <bool F16>
OD_DEV f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c) {
  if constexpr (F16) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
}

// Workgroups are handed to the 8 XCDs (each with its own L2) round robin by their flattened
// index.  This maps the hardware index to a logical one such that every XCD works on one
// contiguous range of logical indices, so neighbours in tile order share an L2.
OD_DEV int xcd_contiguous(int bid, int n) {
  constexpr int kXcd = 8;
  const int xcd = bid % kXcd, slot = bid / kXcd;
  const int q = n / kXcd, rem = n % kXcd;
  return xcd * q + (xcd < rem ? xcd : rem) + slot;
}

OD_DEV int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }
OD_DEV int acc_col(int lane) { return lane & 31; }

// ---------------------------------------------------------------------------------
// bf16 helpers (storage format of X and G in the bf16 configurations)
// ---------------------------------------------------------------------------------
OD_DEV float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
OD_DEV float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
OD_DEV float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

OD_DEV uint32_t pack_bf16_rne(float lo, float hi) {
  bf16x2 p;
  p[0] = (__bf16)lo;        // v_cvt_pk_bf16_f32: round to nearest even
  p[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, p);
}

// ---------------------------------------------------------------------------------
// Number formats of the matrix-core operands.  `pack(x, scale, out)` turns 8 fp32 values
// into PARTS operand words; the products (i, j) with i + j < PARTS are accumulated.
//   NumF16      one fp16 value per element after multiplying by a power-of-two scale
//               (11 significant bits; the scale keeps the data inside fp16's range and the
//               conversion saturates instead of overflowing).
//   NumBF<S>    the value split into S bf16 terms (8, 16, 24 significant bits); 1, 3 or 6
//               products.  No scale: bf16 has fp32's exponent range.
// ---------------------------------------------------------------------------------
struct NumF16 {
  static constexpr int PARTS = 1;
  static constexpr bool F16 = true;
  OD_DEV static void pack(const float* x, float scale, u32x4* out) {
    u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float a = __builtin_amdgcn_fmed3f(x[2 * i] * scale, -65504.f, 65504.f);
      float b = __builtin_amdgcn_fmed3f(x[2 * i + 1] * scale, -65504.f, 65504.f);
      f16x2 p;
      p[0] = (_Float16)a;
      p[1] = (_Float16)b;
      w[i] = __builtin_bit_cast(uint32_t, p);
    }
    out[0] = w;
  }
};

// The value times a power-of-two scale split into two fp16 terms, hi + lo (22 significant
// bits), three products (hi hi, hi lo, lo hi): close to the three-way bf16 split at half
// its matrix-core work.  The scale must bring the data near the top of fp16's range: a term
// below 2^-14 (hi) or 2^-24 (lo) loses bits, which only matters for entries far below the rest.
struct NumH2 {
  static constexpr int PARTS = 2;
  static constexpr bool F16 = true;
  OD_DEV static void pack(const float* x, float scale, u32x4* out) {
    u32x4 hi, lo;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float a = __builtin_amdgcn_fmed3f(x[2 * i] * scale, -65504.f, 65504.f);
      const float b = __builtin_amdgcn_fmed3f(x[2 * i + 1] * scale, -65504.f, 65504.f);
      f16x2 h;
      h[0] = (_Float16)a;
      h[1] = (_Float16)b;
      f16x2 l;
      l[0] = (_Float16)(a - (float)h[0]);
      l[1] = (_Float16)(b - (float)h[1]);
      hi[i] = __builtin_bit_cast(uint32_t, h);
      lo[i] = __builtin_bit_cast(uint32_t, l);
    }
    out[0] = hi;
    out[1] = lo;
  }
};

template <int S>
struct NumBF {
  static constexpr int PARTS = S;
  static constexpr bool F16 = false;
  OD_DEV static void pack(const float* x, float /*scale*/, u32x4* out) {
    float rem[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) rem[i] = x[i];
#pragma unroll
    for (int s = 0; s < S; ++s) {
      u32x4 w;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint32_t p = pack_bf16_rne(rem[2 * i], rem[2 * i + 1]);
        w[i] = p;
        if (s + 1 < S) {
          rem[2 * i] -= bf16_lo(p);
          rem[2 * i + 1] -= bf16_hi(p);
        }
      }
      out[s] = w;
    }
  }
};

// ---------------------------------------------------------------------------------
// Global-memory sources of operand tiles.  A source is a row-major matrix view with
// R rows, C columns and leading dimension ld (elements).  load8(r, c) returns the 8
// consecutive elements (r, c..c+7), load4(r, c) the 4 elements (r, c..c+3); positions
// outside the view read as zero.  C is a multiple of 8, so a group of 8 (or 4) aligned
// columns is either wholly inside or wholly outside.  load8u / load4u / load1u are the same
// reads without the bounds check, for tiles known to lie inside the view: a checked load is
// a branch, and past a branch the compiler waits for every outstanding load, not just the
// oldest, which defeats a multi-stage prefetch.
// ---------------------------------------------------------------------------------
struct SrcF32 {
  static constexpr bool PACKED = false;
  static constexpr bool HAS_LOAD1 = true;
  OD_DEV float load1(int r, int c) const { return (r < R && c < C) ? p[(int64_t)r * ld + c] : 0.f; }
  const float* p;
  int R, C;
  int64_t ld;
  OD_DEV int rows() const { return R; }
  OD_DEV int cols() const { return C; }
  struct Raw8 { f32x4 a, b; };
  typedef f32x4 Raw4;
  OD_DEV Raw8 load8u(int r, int c) const {
    const f32x4* q = reinterpret_cast<const f32x4*>(p + (int64_t)r * ld + c);
    return Raw8{q[0], q[1]};
  }
  OD_DEV Raw4 load4u(int r, int c) const { return *reinterpret_cast<const f32x4*>(p + (int64_t)r * ld + c); }
  OD_DEV float load1u(int r, int c) const { return p[(int64_t)r * ld + c]; }
  OD_DEV Raw8 load8(int r, int c) const {
    Raw8 v;
    if (r < R && c < C) {
      const f32x4* q = reinterpret_cast<const f32x4*>(p + (int64_t)r * ld + c);
      v.a = q[0];
      v.b = q[1];
    } else {
      v.a = f32x4{0.f, 0.f, 0.f, 0.f};
      v.b = v.a;
    }
    return v;
  }
  OD_DEV Raw4 load4(int r, int c) const {
    if (r < R && c < C) return *reinterpret_cast<const f32x4*>(p + (int64_t)r * ld + c);
    return f32x4{0.f, 0.f, 0.f, 0.f};
  }
  OD_DEV static void unpack8(const Raw8& v, float* x) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[i] = v.a[i]; x[4 + i] = v.b[i]; }
  }
  OD_DEV static void unpack4(const Raw4& v, float* x) {
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = v[i];
  }
};

struct SrcBF16 {
  static constexpr bool PACKED = false;
  static constexpr bool HAS_LOAD1 = false;
  const uint16_t* p;
  int R, C;
  int64_t ld;
  OD_DEV int rows() const { return R; }
  OD_DEV int cols() const { return C; }
  typedef u32x4 Raw8;
  typedef u32x2 Raw4;
  OD_DEV Raw8 load8u(int r, int c) const { return *reinterpret_cast<const u32x4*>(p + (int64_t)r * ld + c); }
  OD_DEV Raw4 load4u(int r, int c) const { return *reinterpret_cast<const u32x2*>(p + (int64_t)r * ld + c); }
  OD_DEV Raw8 load8(int r, int c) const {
    if (r < R && c < C) return *reinterpret_cast<const u32x4*>(p + (int64_t)r * ld + c);
    return u32x4{0u, 0u, 0u, 0u};
  }
  OD_DEV Raw4 load4(int r, int c) const {
    if (r < R && c < C) return *reinterpret_cast<const u32x2*>(p + (int64_t)r * ld + c);
    return u32x2{0u, 0u};
  }
  OD_DEV static void unpack8(const Raw8& v, float* x) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[2 * i] = bf16_lo(v[i]); x[2 * i + 1] = bf16_hi(v[i]); }
  }
  OD_DEV static void unpack4(const Raw4& v, float* x) {
#pragma unroll
    for (int i = 0; i < 2; ++i) { x[2 * i] = bf16_lo(v[i]); x[2 * i + 1] = bf16_hi(v[i]); }
  }
};

// Operand words already in matrix-core format (fp16, scaled by their producer): a loader
// copies them to LDS untouched.  Only read along k (load8).
struct SrcH16 {
  static constexpr bool PACKED = true;
  static constexpr bool HAS_LOAD1 = false;
  const uint16_t* p;
  int R, C;
  int64_t ld;
  OD_DEV int rows() const { return R; }
  OD_DEV int cols() const { return C; }
  typedef u32x4 Raw8;
  typedef u32x2 Raw4;
  OD_DEV Raw8 load8u(int r, int c) const { return *reinterpret_cast<const u32x4*>(p + (int64_t)r * ld + c); }
  OD_DEV Raw4 load4u(int r, int c) const { return *reinterpret_cast<const u32x2*>(p + (int64_t)r * ld + c); }
  OD_DEV Raw8 load8(int r, int c) const {
    if (r < R && c < C) return *reinterpret_cast<const u32x4*>(p + (int64_t)r * ld + c);
    return u32x4{0u, 0u, 0u, 0u};
  }
  OD_DEV Raw4 load4(int, int) const { return u32x2{0u, 0u}; }
  OD_DEV static void unpack8(const Raw8&, float* x) {
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = 0.f;
  }
  OD_DEV static void unpack4(const Raw4&, float* x) {
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = 0.f;
  }
};

OD_DEV uint32_t pack_f16_sat(float lo, float hi) {
  f16x2 p;
  p[0] = (_Float16)__builtin_amdgcn_fmed3f(lo, -65504.f, 65504.f);
  p[1] = (_Float16)__builtin_amdgcn_fmed3f(hi, -65504.f, 65504.f);
  return __builtin_bit_cast(uint32_t, p);
}

// The buffer B = M + G of the method, formed on the fly from the fp32 momentum and the
// gradient in its storage type; never written to memory.
template <class GSrc>
struct SrcSum {
  static constexpr bool PACKED = false;
  static constexpr bool HAS_LOAD1 = false;
  SrcF32 m;
  GSrc g;
  OD_DEV int rows() const { return m.R; }
  OD_DEV int cols() const { return m.C; }
  struct Raw8 { SrcF32::Raw8 a; typename GSrc::Raw8 b; };
  struct Raw4 { SrcF32::Raw4 a; typename GSrc::Raw4 b; };
  OD_DEV Raw8 load8u(int r, int c) const { return Raw8{m.load8u(r, c), g.load8u(r, c)}; }
  OD_DEV Raw4 load4u(int r, int c) const { return Raw4{m.load4u(r, c), g.load4u(r, c)}; }
  OD_DEV Raw8 load8(int r, int c) const { return Raw8{m.load8(r, c), g.load8(r, c)}; }
  OD_DEV Raw4 load4(int r, int c) const { return Raw4{m.load4(r, c), g.load4(r, c)}; }
  OD_DEV static void unpack8(const Raw8& v, float* x) {
    float y[8];
    SrcF32::unpack8(v.a, x);
    GSrc::unpack8(v.b, y);
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] += y[i];
  }
  OD_DEV static void unpack4(const Raw4& v, float* x) {
    float y[4];
    SrcF32::unpack4(v.a, x);
    GSrc::unpack4(v.b, y);
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] += y[i];
  }
};

}  // namespace od
