// Direct global-to-LDS operand loads for gfx950 and the LDS layout they fill.
//
// `global_load_lds_dwordx4` moves 16 bytes per lane from a per-lane global address straight
// into LDS at (M0 base) + 16 * lane: one wave instruction fills 1 KB of consecutive LDS with
// no staging registers, asynchronously (it counts in vmcnt like any load).  A [row][k] operand
// tile with 64-byte rows (32 half-precision k) therefore arrives as chunks of 16 consecutive
// LDS rows; which *global* row and k-group a lane fetches is free, so
//   * the 16-byte k-groups of a row are stored XOR-swizzled by (row >> 2) & 3: the 16 lanes a
//     `ds_read_b128` serves per clock (16 consecutive rows, one k-group) then hit 16 different
//     bank groups without any padding, and
//   * rows can be permuted on the way in (the error-feedback kernel interleaves even and odd
//     columns that way).
// The compiler knows nothing of these loads: they are issued from inline assembly and waited
// for with explicit `s_waitcnt vmcnt(n)` (loads return in order, so "at most n outstanding"
// means everything older than the youngest n has landed), followed by a workgroup barrier.
#pragma once

#include "od_common.h"

namespace od {

typedef __attribute__((address_space(3))) void* lds_void_ptr;

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and
// 15:14, expcnt 6:4, lgkmcnt 11:8 left at their maxima)
constexpr int vmcnt_only(int n) { return (n & 15) | (((n >> 4) & 3) << 14) | (7 << 4) | (15 << 8); }

OD_DEV uint32_t lds_offset_of(const void* p) { return (uint32_t)(uintptr_t)(lds_void_ptr)(p); }

// one wave: 16 bytes per lane from `gptr` (per lane) to LDS offset `lds_base` (wave uniform) + 16 * lane
OD_DEV void dma16(const void* gptr, uint32_t lds_base) {
  const uint32_t l = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n" ::"v"(gptr), "s"(l) : "memory");
}

// 64-byte rows (KT = 32): k-group kg of row `row` lives in 16-byte slot kg ^ swz32(row)
OD_DEV int swz32(int row) { return (row >> 2) & 3; }

}  // namespace od
