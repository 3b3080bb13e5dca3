// Device-side helpers shared by the PMPD kernels (gfx950, wave64): vector types, the bit-plane
// unpack primitives and their constants.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "pmpd_common.hpp"

namespace pmpd {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// Pointers into device global memory that were read from a table keep the generic address space;
// naming the global one lets the compiler emit global_load (vmcnt only) instead of flat_load.
typedef const __attribute__((address_space(1))) u32x4* global_u32x4_ptr;
typedef const __attribute__((address_space(1))) uint32_t* global_u32_ptr;
// Wave-uniform reads of x go through the scalar data cache into SGPRs (s_load_dwordx16): the
// constant address space tells the compiler that the memory does not change during the kernel.
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
typedef const __attribute__((address_space(4))) u32x16* const_u32x16_ptr;

__device__ __forceinline__ float dot2(uint32_t w, uint32_t x, float acc) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w), __builtin_bit_cast(half2_t, x), acc, false);
}

// Bit-select and mask-or use compiler-visible operations; the masks are made opaque to the optimiser
// (an empty asm that pins them in SGPRs) so that it cannot fold them into distributed ANDs and
// instead selects one 3-input VALU op each (v_bitop3_b32, v_and_or_b32).  No instruction is
// emitted through inline asm, so the compiler's hazard handling sees every op.
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

// Constants of the unpack, held in registers for the whole kernel.
template <int B>
struct UnpackConsts {
  uint32_t slot[4];   // bit positions congruent to j mod 4
  uint32_t slot2[4];  // slot[j] | slot[j-1]
  uint32_t maskL, maskH, magic;
  __device__ __forceinline__ UnpackConsts() {
#pragma unroll
    for (int j = 0; j < 4; ++j) slot[j] = opaque_sgpr(0x11111111u << j);
#pragma unroll
    for (int j = 0; j < 4; ++j) slot2[j] = opaque_sgpr((0x11111111u << j) | (0x11111111u << ((j + 3) & 3)));
    constexpr uint32_t keep = (0xFu << (4 - B)) & 0xFu;  // top B bits of a 4-bit field
    maskL = opaque_sgpr(keep * 0x00010001u);
    maskH = opaque_sgpr(keep * 0x00100010u);
    magic = 0x64006400u;  // fp16 pair (1024, 1024)
    asm volatile("" : "+v"(magic));
  }
};

__device__ __forceinline__ uint32_t word_of(const u32x4& v, int d) {
  return d == 0 ? v.x : d == 1 ? v.y : d == 2 ? v.z : v.w;
}

__device__ __forceinline__ float half_bits_to_float(uint32_t bits16) {
  return static_cast<float>(__builtin_bit_cast(_Float16, static_cast<uint16_t>(bits16)));
}

// Merge the B plane words of one 32-weight word into the word whose fields (rotated by m)
// are the codes of pairs 4m .. 4m+3.  Plane k sits in sub-slot (3 - k + m) mod 4.
template <int B>
__device__ __forceinline__ uint32_t merge_planes(const UnpackConsts<B>& uc, const uint32_t (&p)[B], int m) {
  if constexpr (B == 4) {
    uint32_t hi = bfi(uc.slot[(3 + m) & 3], p[0], p[1]);
    uint32_t lo = bfi(uc.slot[(1 + m) & 3], p[2], p[3]);
    return bfi(uc.slot2[(3 + m) & 3], hi, lo);
  } else if constexpr (B == 3) {
    uint32_t lo = bfi(uc.slot[(2 + m) & 3], p[1], p[2]);
    return bfi(uc.slot[(3 + m) & 3], p[0], lo);
  } else {
    return bfi(uc.slot[(3 + m) & 3], p[0], p[1]);
  }
}

}  // namespace pmpd
