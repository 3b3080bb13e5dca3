// Device-side helpers shared by the PMPD kernels (gfx950, wave64): vector types and the
// bit-plane unpack primitives.
//
// Storage format seen from a wave.  For one (64-row tile, 128-column group, plane k) the store
// holds 1 KiB; lane l = 16 kb + j loads 16 bytes = four 32-bit words, word t holding the plane's
// bit of row 16 t + j of the tile for the 32 columns 32 kb .. 32 kb + 31 of the group.  Inside a
// word, column 8 v + c (v 0..3, c 0..7) uses nibble n = c/2 + 4 (c%2) and, for an even plane
// (0, 2: the upper bit of a 2-bit pair) bit 4n + {1,3,0,2}[v], for an odd plane (1, 3: the lower
// bit) bit (4n + {0,2,31,1}[v]) mod 32.  pair_words() turns a pair of such words into four words
// of eight nibbles 00pp', nibble n of word v belonging to column 8 v + c(n): an fp4 (e2m1) operand
// register set as it is, and two AND/shift steps away from 4-bit codes for the fp16 path.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "pmpd_common.hpp"

namespace pmpd {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
// Pointers into device global memory that were read from a table keep the generic address space;
// naming the global one lets the compiler emit global_load (vmcnt only) instead of flat_load.
typedef const __attribute__((address_space(1))) u32x4* global_u32x4_ptr;
typedef const __attribute__((address_space(1))) uint32_t* global_u32_ptr;

// Masks are made opaque to the optimiser (an empty asm that pins them in SGPRs) so that it
// cannot fold them into distributed ANDs and instead selects one 3-input VALU op each.  No
// instruction is emitted through inline asm, so the compiler's hazard handling sees every op.
__device__ __forceinline__ uint32_t opaque_sgpr(uint32_t v) {
  asm volatile("" : "+s"(v));
  return v;
}

// (a & mask) | (b & ~mask): one v_bitop3_b32 (gfx950's 3-input boolean op).  Truth table index is
// (a << 2) | (b << 1) | mask, so "mask ? a : b" is 0b11100100.
__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) {
  return __builtin_amdgcn_bitop3_b32(a, b, mask, 0xE4);
}

// (a & mask) | c
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t c) { return (a & mask) | c; }

__device__ __forceinline__ uint32_t word_of(const u32x4& v, int d) {
  return d == 0 ? v.x : d == 1 ? v.y : d == 2 ? v.z : v.w;
}

__device__ __forceinline__ float half_bits_to_float(uint32_t bits16) {
  return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(bits16)));
}

// Four words of eight nibbles 00pp' from the plane words of one 2-bit pair: `hi` is the word of
// the even plane (upper bit p), `lo` of the odd plane (lower bit p').  9 VALU ops for 32 weights.
__device__ __forceinline__ void pair_words(uint32_t hi, uint32_t lo, uint32_t (&w)[4]) {
  const uint32_t odd = opaque_sgpr(0xAAAAAAAAu), keep = opaque_sgpr(0x33333333u);
  const uint32_t r1 = bfi(odd, hi, lo);  // odd bits from hi, even bits from lo: columns v = 0, 1
  const uint32_t r2 = bfi(odd, lo, hi);  // even bits from hi, odd bits from lo: columns v = 2, 3
  w[0] = r1 & keep;
  w[1] = (r1 >> 2) & keep;
  w[2] = __builtin_amdgcn_alignbit(r2, r2, 31) & keep;  // rotate left by one
  w[3] = (r2 >> 1) & keep;
}

// The same when the pass stops at the upper bit of the pair (lower plane not read): nibbles 00p0.
__device__ __forceinline__ void single_words(uint32_t hi, uint32_t (&w)[4]) {
  const uint32_t keep = opaque_sgpr(0x22222222u);
  w[0] = hi & keep;
  w[1] = (hi >> 2) & keep;
  w[2] = (hi << 1) & keep;
  w[3] = (hi >> 1) & keep;
}

// Cross-lane moves inside a DPP row of 16 lanes (bound_ctrl: lanes without a source read 0).
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xF, 0xF, true));
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, dpp_u32<CTRL>(__builtin_bit_cast(uint32_t, v)));
}
constexpr int kQuadSwap1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kQuadSwap2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kRowHalfMirror = 0x141;
constexpr int kRowMirror = 0x140;

// Largest value / sum over the 16 lanes of a DPP row (quad swaps, then the two mirrors): every lane gets it.
__device__ __forceinline__ uint32_t row16_max(uint32_t v) {
  uint32_t o = dpp_u32<kQuadSwap1>(v);
  v = v > o ? v : o;
  o = dpp_u32<kQuadSwap2>(v);
  v = v > o ? v : o;
  o = dpp_u32<kRowHalfMirror>(v);
  v = v > o ? v : o;
  o = dpp_u32<kRowMirror>(v);
  return v > o ? v : o;
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_f32<kQuadSwap1>(v);
  v += dpp_f32<kQuadSwap2>(v);
  v += dpp_f32<kRowHalfMirror>(v);
  v += dpp_f32<kRowMirror>(v);
  return v;
}

}  // namespace pmpd
