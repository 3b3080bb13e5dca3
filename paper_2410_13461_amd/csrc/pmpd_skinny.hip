// Skinny batches (3..8 activation vectors) over a list of layers on the int8 matrix cores (gfx950).
// (From 9 vectors, and from 5 at b = 4, the fp16 kernel of pmpd_block16.hip is faster: its cost does not grow with the batch.)
//
// The weights are still read once per step (memory-bound, the paper's decode regime, Section 1 and
// Section 5.2, widened to a few sequences); what changes against the batch-1 kernel is the
// arithmetic.  v_mfma_i32_16x16x64_i8 multiplies 16 weight rows with 16 operand rows exactly, so a
// set of 16 operand rows carries FOUR vectors (three rows each), where the fp8 x fp4 instruction of
// the batch-1 kernel needs a set for two: 2 x 2 small MFMAs per 16 weight rows and group serve up to
// four vectors, and the unpack work per weight does not grow with the batch.
//
// Activations.  Per vector and group of 128 columns the fp16 values are turned into integers
//     X_i = round(x_i 2^(36 - E)),  |X_i| < 2^22,
// E = exponent field of the group's largest magnitude (at least 1).  Every fp16 value within 2^-11 of
// the group's largest is represented exactly; smaller ones are rounded to a multiple of
// 2^-22 of the largest power of two in reach (absolute error below 2^-23 of the group's maximum).
// X_i is written as three balanced base-256 digits, X = p0 + 256 p1 + 65536 p2 with every digit in
// -128..127: byte 0 of X, byte 1 of X + 0x80, byte 2 of X + 0x8080.  The digits of vector 4 s + q
// sit in rows 4 q (p2), 4 q + 1 (p1), 4 q + 2 (p0) of operand set s; row 4 q + 3 is not used.
//
// Weights.  The merged plane words (pair_words) give the 4-bit aligned code q~ as nibbles; two
// AND/shift steps spread them into bytes.  In the storage format lane 16 kb + j of a wave holds 32
// columns of row 16 t + j per word: two MFMAs (h = 0, 1) of K = 64, the lane contributing its columns
// 32 kb + 16 h + {0,4,1,5, 2,6,3,7, 8,12,9,13, 10,14,11,15} in that byte order; the activation image
// is written in the same order.  (Checked on gfx950: operand lane i + 16 kb holds row i, byte e of it
// meets byte e of lane j + 16 kb of the other operand; D[i][j] is in lane j + 16 (i / 4), register i % 4.)
//
// Per group, weight row and vector:  sum_i W_b x = s_g 2^(E-36) (65536 D2 + 256 D1 + D0) + (a_g + s_g 2^(3-b)) X_g
// with Dk = sum q~ p_k exact in int32 and X_g the fp32 sum of the group's x.  Lane l gets the three
// sums of vector 4 s + l / 16 and weight row 16 t + l % 16 in registers 0..2 of D.
//
// Workgroup = 8 waves (4 for up to four vectors), one 64-row tile each over the whole K; the activation
// image of a K-chunk is built once per workgroup in LDS (up to 72 KiB with two workgroups per CU, 36 KiB
// with four) while the first weight loads are in flight.  No atomics, fixed summation order.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "pmpd_common.hpp"
#include "pmpd_device.hpp"

namespace pmpd {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

constexpr int kSkKbStride = 272;                   // bytes between the four 16-lane groups of an operand: 256 + 16, so that
                                                   // the 8-byte writes of a group's 16 staging lanes fall into 16 different bank pairs
constexpr int kSkHalfStride = 4 * kSkKbStride;     // 1088: from MFMA h = 0 to h = 1
constexpr int kSkGroupBytes = 2 * kSkHalfStride;   // 2176 per operand set and group
__host__ __device__ constexpr int sk_budget(int nw) { return nw == 8 ? 72 * 1024 : 36 * 1024; }  // two / four workgroups per CU
constexpr int kSkMaxVectors = 8;

__host__ __device__ inline int sk_sets(int m) { return (m + 3) / 4; }
__host__ __device__ inline int sk_group_bytes(int m) { return sk_sets(m) * kSkGroupBytes + m * 8; }
// Groups per K-chunk: as few chunks as the LDS budget allows, of about equal and even length (a chunk that starts
// at an even group keeps the turns of the two weight register sets, whose loads run on across chunk boundaries).
__host__ __device__ inline int sk_chunk(int n_groups, int m, int nw) {
  const int fit = (sk_budget(nw) / sk_group_bytes(m)) & ~1;
  const int n_chunks = (n_groups + fit - 1) / fit;
  return ((n_groups + n_chunks - 1) / n_chunks + 1) & ~1;
}

// Staging units (one vector x four groups) a wave handles per K-chunk, at most, for SETS operand sets.
constexpr int sk_max_units(int sets, int nw) {
  int worst = 0;
  for (int m = 4 * sets - 3; m <= 4 * sets; ++m) {
    const int fit = sk_budget(nw) / (sets * kSkGroupBytes + m * 8);
    const int units = (m * ((fit + 3) / 4) + nw - 1) / nw;
    worst = units > worst ? units : worst;
  }
  return worst;
}

// Byte k of a, b, c, d as one word (a in the lowest byte).
template <int K>
__device__ __forceinline__ uint32_t gather_bytes(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  constexpr uint32_t sel = 0x0C0C0000u | ((4u + K) << 8) | K;
  const uint32_t ab = __builtin_amdgcn_perm(b, a, sel);
  const uint32_t cd = __builtin_amdgcn_perm(d, c, sel);
  return __builtin_amdgcn_perm(cd, ab, 0x05040100u);
}

struct SkImage {
  char* ops;     // [sets][cg][kSkGroupBytes]
  float* rs;     // [m][cg]: 2^(E - 36) of the vector's group
  float* xsum;   // [m][cg]: fp32 sum of the group's x
  int cg;
  __device__ __forceinline__ SkImage(void* lds, int cg_, int m) : cg(cg_) {
    ops = static_cast<char*>(lds);
    rs = reinterpret_cast<float*>(ops + sk_sets(m) * cg * kSkGroupBytes);
    xsum = rs + m * cg;
  }
};

// Image of four groups (from group gb of a chunk of cn groups) of vector j, by one wave: lane l holds
// columns 8 l .. 8 l + 7 of the four groups in v; a DPP row of 16 lanes is one group.
__device__ __forceinline__ void sk_stage4(const uint4& v, int cn, int gb, const SkImage& im, int j) {
  const int idx = gb * 16 + (threadIdx.x & 63);
  if (idx >= cn * 16) return;  // whole DPP rows drop out together
  char* base = im.ops + (j >> 2) * im.cg * kSkGroupBytes + (4 * (j & 3)) * 16;
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
  us2 mx = __builtin_bit_cast(us2, w[0] & 0x7FFF7FFFu);
  float xs = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    if (q) mx = __builtin_elementwise_max(mx, __builtin_bit_cast(us2, w[q] & 0x7FFF7FFFu));
    xs = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, w[q]), half2_t{1, 1}, xs, false);
  }
  uint32_t E = row16_max(mx.x > mx.y ? mx.x : mx.y) >> 10;
  E = E ? E : 1u;
  const float S = __builtin_bit_cast(float, (163u - E) << 23);  // 2^(36 - E)
  uint32_t b[8];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const half2_t h = __builtin_bit_cast(half2_t, w[q]);
    // 1.5 * 2^23 + X: the integer sits in the low bits of the float (round to nearest even)
    b[2 * q] = __builtin_bit_cast(uint32_t, fmaf(static_cast<float>(h.x), S, 12582912.0f));
    b[2 * q + 1] = __builtin_bit_cast(uint32_t, fmaf(static_cast<float>(h.y), S, 12582912.0f));
  }
  uint32_t b1[8], b2[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    b1[e] = b[e] + 0x80u;
    b2[e] = b[e] - 0x3F7F80u;  // + 0x8080 and the 0x400000 of the float's mantissa taken out
  }
  const int g = idx >> 4, c8 = idx & 15;
  char* dst = base + g * kSkGroupBytes + ((c8 >> 1) & 1) * kSkHalfStride + (c8 >> 2) * kSkKbStride + (c8 & 1) * 8;
  // word order of the weight bytes: columns {0,4,1,5} then {2,6,3,7}
  *reinterpret_cast<uint2*>(dst) = make_uint2(gather_bytes<2>(b2[0], b2[4], b2[1], b2[5]), gather_bytes<2>(b2[2], b2[6], b2[3], b2[7]));
  *reinterpret_cast<uint2*>(dst + 16) = make_uint2(gather_bytes<1>(b1[0], b1[4], b1[1], b1[5]), gather_bytes<1>(b1[2], b1[6], b1[3], b1[7]));
  *reinterpret_cast<uint2*>(dst + 32) = make_uint2(gather_bytes<0>(b[0], b[4], b[1], b[5]), gather_bytes<0>(b[2], b[6], b[3], b[7]));
  xs = row16_sum(xs);
  if (c8 == 0) {
    im.rs[j * im.cg + g] = __builtin_bit_cast(float, (91u + E) << 23);  // 2^(E - 36)
    im.xsum[j * im.cg + g] = xs;
  }
}

// Bytes of the 4-bit aligned codes (B = 2: of q~ / 4) of 16-row block t: two operands of 16 bytes.
// With r1 = odd bits of plane 0 and even bits of plane 1, r2 the other way round (s1, s2 the same from planes 2, 3),
// the upper two bits of the nibbles of the four code words are r1 << 2, r1, rotl(r2, 3), r2 << 1 under the mask
// 0xCCCCCCCC and the lower two s1, s1 >> 2, rotl(s2, 1), s2 >> 1 under its complement, so one 3-input boolean
// operation joins a code word: 14 instructions per 16 rows and group, then 3 per code word to spread the nibbles
// into bytes.  With three planes the lower halves come from plane 2 alone (its odd bits for words 0, 1, its even
// bits for words 2, 3: the bit the complement mask keeps is then the plane's, the other is zero).  With two planes
// the bytes are cut out of r1 and r2 directly.
template <int B>
__device__ __forceinline__ void code_bytes(const u32x4 (&pl)[B], int t, i32x4 (&op)[2]) {
  const uint32_t odd = opaque_sgpr(0xAAAAAAAAu);
  const uint32_t h0 = word_of(pl[0], t), l0 = word_of(pl[1], t);
  const uint32_t r1 = bfi(odd, h0, l0), r2 = bfi(odd, l0, h0);
  if constexpr (B == 2) {
    const uint32_t m2 = opaque_sgpr(0x03030303u);
    op[0] = i32x4{static_cast<int>(r1 & m2), static_cast<int>((r1 >> 4) & m2), static_cast<int>((r1 >> 2) & m2),
                  static_cast<int>((r1 >> 6) & m2)};
    op[1] = i32x4{static_cast<int>(__builtin_amdgcn_alignbit(r2, r2, 31) & m2), static_cast<int>((r2 >> 3) & m2),
                  static_cast<int>((r2 >> 1) & m2), static_cast<int>((r2 >> 5) & m2)};
  } else {
    const uint32_t top = opaque_sgpr(0xCCCCCCCCu), m = opaque_sgpr(0x0F0F0F0Fu);
    uint32_t s1, s2, d;
    if constexpr (B == 4) {
      const uint32_t h1 = word_of(pl[2], t), l1 = word_of(pl[3], t);
      s1 = bfi(odd, h1, l1);
      s2 = bfi(odd, l1, h1);
      d = __builtin_amdgcn_alignbit(s2, s2, 31);
    } else {
      const uint32_t h1 = word_of(pl[2], t);
      s1 = h1 & odd;
      s2 = h1 & opaque_sgpr(0x55555555u);
      d = s2 << 1;
    }
    const uint32_t c0 = bfi(top, r1 << 2, s1), c1 = bfi(top, r1, s1 >> 2);
    const uint32_t c2 = bfi(top, __builtin_amdgcn_alignbit(r2, r2, 29), d), c3 = bfi(top, r2 << 1, s2 >> 1);
    op[0] = i32x4{static_cast<int>(c0 & m), static_cast<int>((c0 >> 4) & m), static_cast<int>(c1 & m), static_cast<int>((c1 >> 4) & m)};
    op[1] = i32x4{static_cast<int>(c2 & m), static_cast<int>((c2 >> 4) & m), static_cast<int>(c3 & m), static_cast<int>((c3 >> 4) & m)};
  }
}

template <int B, int SETS, int NW>
__device__ __forceinline__ void skinny_tiles(const LayerDesc& L, int tile0, const _Float16* __restrict__ x, int m,
                                             float* __restrict__ y, uint4* lds_raw) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int G = L.n_groups;
  const SkImage im(lds_raw, sk_chunk(G, m, NW), m);
  const int tile = tile0 + wave;
  const bool active = tile < L.n_tiles;
  const int64_t tbase = (static_cast<int64_t>(active ? tile : 0) * G) * 64 + lane;
  global_u32x4_ptr pp[B];
#pragma unroll
  for (int k = 0; k < B; ++k) pp[k] = (global_u32x4_ptr)(L.plane[k]) + tbase;
  global_u32x4_ptr sp = (global_u32x4_ptr)(L.sa) + (tbase - lane) / 4 + (lane & 15);

  // operand read address of the lane (16 bytes per MFMA) and the vector whose sums it receives
  const int a_off = (lane >> 4) * kSkKbStride + (lane & 15) * 16;
  int vec[SETS];
#pragma unroll
  for (int s = 0; s < SETS; ++s) {
    const int v = 4 * s + (lane >> 4);
    vec[s] = v < m ? v : m - 1;  // absent vectors repeat the last one; their sums are not stored
  }
  constexpr float kCodeUnit = (B == 2) ? 4.f : 1.f;
  const int inv_m = 65536 / m + 1;  // u / m == (u * inv_m) >> 16 for the few dozen staging units of a chunk
  float yacc[SETS][4];
#pragma unroll
  for (int s = 0; s < SETS; ++s)
#pragma unroll
    for (int t = 0; t < 4; ++t) yacc[s][t] = 0.f;

  // The weight loads run one group ahead through the whole K: the first group of a chunk is requested by the last
  // iteration of the chunk before and is in flight while the image is built.  Past the end the last group is read
  // again (no branch around the loads: the wave keeps counting them).
  u32x4 pa[B], pb[B], sa_a = {0, 0, 0, 0}, sa_b = {0, 0, 0, 0};
  auto load = [&](u32x4 (&dst)[B], u32x4& dsa, int g) {
    const int gl = g < G ? g : G - 1;
#pragma unroll
    for (int k = 0; k < B; ++k) dst[k] = __builtin_nontemporal_load(&pp[k][gl * 64]);
    dsa = sp[gl * 16];
  };
  if (active) load(pa, sa_a, 0);
  for (int c0 = 0; c0 < G; c0 += im.cg) {
    const int cn = (G - c0 < im.cg) ? (G - c0) : im.cg;
    const int g1 = c0 + cn;
    // (vector, block of four groups) units dealt round-robin to the waves: unit u = vector u % m, block u / m.
    // All of a wave's activation loads are issued before the barrier, so that their latency is paid once.
    const int n_units = m * ((cn + 3) >> 2);
    constexpr int kUnits = sk_max_units(SETS, NW);
    uint4 xr[kUnits];
#pragma unroll
    for (int k = 0; k < kUnits; ++k) {
      const int u = wave + k * NW;
      const int blk = (u * inv_m) >> 16, j = u - blk * m, idx = blk * 64 + lane;
      xr[k] = make_uint4(0, 0, 0, 0);
      if (u < n_units && idx < cn * 16) xr[k] = (reinterpret_cast<const uint4*>(x + static_cast<int64_t>(j) * L.in_f) + c0 * 16)[idx];
    }
    if (c0) __syncthreads();  // the previous chunk's image has been consumed
#pragma unroll
    for (int k = 0; k < kUnits; ++k) {
      const int u = wave + k * NW;
      const int blk = (u * inv_m) >> 16;
      if (u < n_units) sk_stage4(xr[k], cn, blk * 4, im, u - blk * m);
    }
    __syncthreads();
    if (active) {
      auto consume = [&](const u32x4 (&pl)[B], const u32x4& csa, int g) {
        const int gr = g - c0;
        i32x4 A[SETS][2];
        float rs[SETS], xg[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
          const char* p = im.ops + (s * im.cg + gr) * kSkGroupBytes + a_off;
          A[s][0] = *reinterpret_cast<const i32x4*>(p);
          A[s][1] = *reinterpret_cast<const i32x4*>(p + kSkHalfStride);
          rs[s] = im.rs[vec[s] * im.cg + gr] * kCodeUnit;
          xg[s] = im.xsum[vec[s] * im.cg + gr];
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          i32x4 op[2];
          code_bytes<B>(pl, t, op);
          const uint32_t w = word_of(csa, t);
          const float sc = half_bits_to_float(w & 0xffffu);
          const float off = fmaf(sc, B == 4 ? 0.5f : B == 3 ? 1.0f : 2.0f, half_bits_to_float(w >> 16));
#pragma unroll
          for (int s = 0; s < SETS; ++s) {
            i32x4 d = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[s][0], op[0], i32x4{0, 0, 0, 0}, 0, 0, 0);
            d = __builtin_amdgcn_mfma_i32_16x16x64_i8(A[s][1], op[1], d, 0, 0, 0);
            // 65536 D2 + 256 D1 + D0: the two low digits are added as integers (below 2^27), one conversion fewer
            const float f = fmaf(static_cast<float>(d[0]), 65536.f, static_cast<float>((d[1] << 8) + d[2]));
            yacc[s][t] = fmaf(sc * rs[s], f, yacc[s][t]);
            yacc[s][t] = fmaf(off, xg[s], yacc[s][t]);
          }
        }
      };
      for (int gc = c0; gc < g1; gc += 2) {
        load(pb, sa_b, gc + 1);
        consume(pa, sa_a, gc);
        load(pa, sa_a, gc + 2);
        if (gc + 1 < g1) consume(pb, sa_b, gc + 1);
      }
    }
  }
  if (active) {
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
      const int v = 4 * s + (lane >> 4);
      if (v < m) {
        float* yo = y + static_cast<int64_t>(v) * L.out_f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int row = tile * 64 + 16 * t + (lane & 15);
          if (row < L.out_f) yo[row] = yacc[s][t];
        }
      }
    }
  }
}

template <int B, int SETS, int NW>
__global__ __launch_bounds__(NW * 64, 4) void pmpd_skinny_stack_kernel(
    const LayerDesc* __restrict__ layers, const WorkItem* __restrict__ items, const _Float16* __restrict__ x_base, int m,
    float* __restrict__ y_base) {
  extern __shared__ uint4 lds[];
  const WorkItem it = items[blockIdx.x];
  const LayerDesc L = layers[it.layer];
  skinny_tiles<B, SETS, NW>(L, it.tile0, x_base + static_cast<int64_t>(m) * L.x_off, m, y_base + static_cast<int64_t>(m) * L.y_off, lds);
}

template <int B, int SETS, int NW>
static hipError_t launch_skinny(const pmpd_stack* st, const _Float16* x, int m, float* y, hipStream_t s) {
  constexpr int list = NW == 8 ? kEightTileList : 0;
  static_assert(kStackTilesPerWg[list] == NW, "one tile per wave");
  // a layer's chunk is at most what the budget holds and at most its own number of groups, both made even
  const int fit = (sk_budget(NW) / sk_group_bytes(m)) & ~1, longest = (st->max_in / kGroup + 1) & ~1;
  const size_t lds = static_cast<size_t>(std::min(fit, longest)) * sk_group_bytes(m);
  auto kernel = pmpd_skinny_stack_kernel<B, SETS, NW>;
  if (lds > 65536) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       sk_budget(NW));
    if (e != hipSuccess) return e;
  }
  const unsigned grid = static_cast<unsigned>(st->items[list].size());
  hipLaunchKernelGGL(kernel, dim3(grid), dim3(NW * 64), lds, s, st->d_layers, st->d_items[list], x, m, y);
  return hipGetLastError();
}

// Up to four vectors: 4-wave workgroups (four per CU); above: 8 waves, so that the image is built half as often.
template <int B>
static hipError_t launch_skinny_b(const pmpd_stack* st, const _Float16* x, int m, float* y, hipStream_t s) {
  return sk_sets(m) == 1 ? launch_skinny<B, 1, 4>(st, x, m, y, s) : launch_skinny<B, 2, 8>(st, x, m, y, s);
}

// Called by the C entry points (pmpd_gemv.hip) for 3 <= m <= 8 vectors over a stack.
hipError_t launch_skinny_stack(const pmpd_stack* st, int b, const void* X, int m, float* Y, hipStream_t s) {
  if (m < 1 || m > kSkMaxVectors) return hipErrorInvalidValue;
  const _Float16* x = static_cast<const _Float16*>(X);
  return b == 4 ? launch_skinny_b<4>(st, x, m, Y, s) : b == 3 ? launch_skinny_b<3>(st, x, m, Y, s) : launch_skinny_b<2>(st, x, m, Y, s);
}

}  // namespace pmpd
