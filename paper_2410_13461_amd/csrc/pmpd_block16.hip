// Batches of 9 to 16 vectors over a list of layers on the fp16 matrix cores (gfx950): one 16-token block per wave
// and 64-row tile, the 4-bit codes fed to the matrix instruction as they are.
//     Y[j][r] = sum_i W_b[r][i] X[j][i],   j < m <= 16
// The decode-phase linear layers of Algorithm 1 (line 16) at a small batch (the paper itself stays at batch 1,
// Section 5.2): the weights are read and unpacked once for all vectors.
//
// Arithmetic.  Per group g of 128 columns (Section 2.1: one scale s_g and minimum a_g per row and group)
//     sum_i W_b x = s_g sum_i q~_i x_i + (a_g + s_g 2^(3-b)) sum_i x_i
// with q~ the 4-bit aligned code.  The integer q~ (0..15) sits in the low four bits of an otherwise zero fp16
// word, which is the subnormal number q~ 2^-24: v_mfma_f32_16x16x32_f16 multiplies subnormal inputs exactly, so
// the code words need no conversion at all, only an AND per pair of columns (after a shift for two of every four
// pairs; the last pair of a word falls out of one packed 16-bit shift).  The products q~ x 2^-24 are exact in
// fp32, the activations are the caller's fp16 values, unscaled and unrounded: the only rounding is that of the
// fp32 accumulation.  The second sum comes from the same instruction, with a second operand of ones.  Scale and
// minimum meet the sums once per group and output: two fused multiply-adds.
//
// Operands.  In the storage format lane 16 kb + j of a wave holds, in word t of a plane, 32 columns of weight row
// 16 t + j.  Merged into four code words (eight codes each, columns 8 v .. 8 v + 7 of the lane's 32), code word v
// is the lane's K slice of matrix instruction v of the group: lane 16 kb + j gives row j for K = 8 kb .. 8 kb + 7,
// meaning columns 32 kb + 8 v + e.  The activations are the first operand: lane 16 kb + i reads token i's same
// eight columns, 16 bytes, from a copy of X in LDS that the four waves of a workgroup share (K is walked in chunks
// of eight groups; read straight from the caches, every load instruction would touch 64 cache lines for 16 bytes
// each).  D[i][j] then sits in lane j + 16 (i / 4), register i % 4: a lane holds row j of the block for four
// tokens, and the row's scale and minimum are in the lane's own scale word.
//
// Against the int8 kernel (pmpd_skinny.hip): no digits, no image to compute, half the matrix instructions at 16
// vectors, and two instead of seven instructions per (16 rows, four vectors) after them; the code words cost 24
// instead of 12 instructions per 16 rows to spread, whatever the batch: 215 / 223 / 198 vector instructions per
// (tile, group) and wave at b = 4 / 3 / 2 against 207 / 210 / 171 at 8 vectors and 294 / 297 / 259 at 16.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "pmpd_common.hpp"
#include "pmpd_device.hpp"

namespace pmpd {

typedef unsigned short us2 __attribute__((ext_vector_type(2)));

constexpr int kB16Waves = 4;  // waves (= 64-row tiles) per workgroup
constexpr int kB16Chunk = 8;  // groups of activations in LDS at a time (even: see the weight loads); 32 KiB at 16 tokens

// The four code words of 16-row block t (eight 4-bit aligned codes q~ each: columns 8 v .. 8 v + 7 of the lane's 32,
// nibbles 0,4 / 1,5 / 2,6 / 3,7 = column pairs (0,1) / (2,3) / (4,5) / (6,7)).  With r1 = odd bits of plane 0 and even
// bits of plane 1, r2 the other way round (s1, s2 the same from planes 2, 3), the upper two bits of the nibbles of
// words 0..3 are r1 << 2, r1, rotl(r2, 3), r2 << 1 under the mask 0xCCCCCCCC and the lower two s1, s1 >> 2,
// rotl(s2, 1), s2 >> 1 under its complement.  With three planes the lower halves come from plane 2 alone (its odd
// bits for words 0, 1, its even bits for words 2, 3); with two planes they are zero.
template <int B>
__device__ __forceinline__ void b16_codes(const u32x4 (&pl)[B], int t, uint32_t (&code)[4]) {
  const uint32_t odd = opaque_sgpr(0xAAAAAAAAu), top = opaque_sgpr(0xCCCCCCCCu);
  const uint32_t h0 = word_of(pl[0], t), l0 = word_of(pl[1], t);
  const uint32_t r1 = bfi(odd, h0, l0), r2 = bfi(odd, l0, h0);
  if constexpr (B == 2) {
    code[0] = (r1 << 2) & top;
    code[1] = r1 & top;
    code[2] = __builtin_amdgcn_alignbit(r2, r2, 29) & top;
    code[3] = (r2 << 1) & top;
  } else {
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
    code[0] = bfi(top, r1 << 2, s1);
    code[1] = bfi(top, r1, s1 >> 2);
    code[2] = bfi(top, __builtin_amdgcn_alignbit(r2, r2, 29), d);
    code[3] = bfi(top, r2 << 1, s2 >> 1);
  }
}

// One code word (eight weights of the lane: the K slice of one matrix instruction) -> the four registers of the
// operand, each a pair of fp16 subnormals q~ 2^-24 for two neighbouring columns.
__device__ __forceinline__ half8_t b16_operand(uint32_t c, uint32_t low4) {
  u32x4 r;
  r.x = c & low4;
  r.y = (c >> 4) & low4;
  r.z = (c >> 8) & low4;
  r.w = __builtin_bit_cast(uint32_t, __builtin_bit_cast(us2, c) >> 12);  // both halves at once: nothing left to mask
  return __builtin_bit_cast(half8_t, r);
}

// Chunk position of 16-byte piece c of token i in the LDS image: pieces are XOR-swizzled so that the operand read
// (lane 16 kb + i fetches piece 4 kb + v of token i) finds the sixteen lanes the hardware serves together in sixteen
// different bank columns (the layout of the prefill kernel's X tile, measured there without bank conflicts).
__device__ __forceinline__ int b16_swz(int r) {
  const int hi = (r >> 2) & 3;
  return (r & 3) | (((0x78 >> (2 * hi)) & 3) << 2);  // hi: 0, 1, 2, 3 -> 0, 2, 3, 1
}

// One workgroup: four row tiles of layer L (one per wave), all m <= 16 tokens, the whole K in chunks of kB16Chunk
// groups whose activations are copied to LDS once for the four waves.
template <int B>
__device__ __forceinline__ void b16_tiles(const LayerDesc& L, int tile0, const _Float16* __restrict__ X, int m, float* __restrict__ Y,
                                          char* lds) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int G = L.n_groups;
  const int tile = tile0 + wave;
  const bool active = tile < L.n_tiles;
  const int64_t tbase = (static_cast<int64_t>(active ? tile : 0) * G) * 64 + lane;
  global_u32x4_ptr pp[B];
#pragma unroll
  for (int k = 0; k < B; ++k) pp[k] = (global_u32x4_ptr)(L.plane[k]) + tbase;
  global_u32x4_ptr sp = (global_u32x4_ptr)(L.sa) + (tbase - lane) / 4 + (lane & 15);

  // Copying: thread 16 j + c moves piece c (8 columns) of token j for every group of the chunk.
  const int pitch = m * 256;  // bytes per group in LDS: m tokens x 128 columns
  const int cj = threadIdx.x >> 4, cc = threadIdx.x & 15;
  const bool copies = cj < m;
  const u32x4* xsrc = reinterpret_cast<const u32x4*>(X + static_cast<int64_t>(copies ? cj : 0) * L.in_f) + cc;
  char* xdst = lds + cj * 256 + ((cc ^ b16_swz(cj)) * 16);
  // First operand of this lane: token lane % 16 (tokens past m repeat the last one; their results are not stored),
  // columns 32 (lane / 16) + 8 v .. + 7 of the group = piece 4 (lane / 16) + v
  const int token = (lane & 15) < m ? (lane & 15) : m - 1;
  const char* xop[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) xop[v] = lds + token * 256 + (((4 * (lane >> 4) + v) ^ b16_swz(token)) * 16);

  float4_t acc_q[4], acc_x[4];  // sum_g s_g sum q~ x 2^-24 and sum_g (a_g + s_g 2^(3-b)) sum x, tokens 4 (lane / 16) + 0..3
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    acc_q[t] = float4_t{0.f, 0.f, 0.f, 0.f};
    acc_x[t] = float4_t{0.f, 0.f, 0.f, 0.f};
  }
  const uint32_t low4 = opaque_sgpr(0x000F000Fu);
  uint32_t one2 = 0x3C003C00u;  // the fp16 pair (1, 1)
  asm volatile("" : "+v"(one2));
  const half8_t ones = __builtin_bit_cast(half8_t, u32x4{one2, one2, one2, one2});
  constexpr float kOff = (B == 4) ? 0.5f : (B == 3) ? 1.0f : 2.0f;  // 2^(3-b)

  u32x4 pa[B], pb[B], sa_a = {0, 0, 0, 0}, sa_b = {0, 0, 0, 0};
  auto load = [&](u32x4 (&dst)[B], u32x4& dsa, int g) {
    const int gl = g < G ? g : G - 1;  // past the end: the last group again (no branch: the wave keeps counting its loads)
#pragma unroll
    for (int k = 0; k < B; ++k) dst[k] = __builtin_nontemporal_load(&pp[k][gl * 64]);
    dsa = sp[gl * 16];
  };
  auto consume = [&](const u32x4 (&pl)[B], const u32x4& csa, int gr) {
    half8_t cx[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) cx[v] = *reinterpret_cast<const half8_t*>(xop[v] + gr * pitch);
    float4_t xs = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int v = 0; v < 4; ++v) xs = __builtin_amdgcn_mfma_f32_16x16x32_f16(cx[v], ones, xs, 0, 0, 0);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      uint32_t code[4];
      b16_codes<B>(pl, t, code);
      float4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int v = 0; v < 4; ++v) d = __builtin_amdgcn_mfma_f32_16x16x32_f16(cx[v], b16_operand(code[v], low4), d, 0, 0, 0);
      const half2_t sm = __builtin_bit_cast(half2_t, word_of(csa, t));
      const float sc = static_cast<float>(sm.x);
      const float off = fmaf(sc, kOff, static_cast<float>(sm.y));
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        acc_q[t][r] = fmaf(sc, d[r], acc_q[t][r]);
        acc_x[t][r] = fmaf(off, xs[r], acc_x[t][r]);
      }
    }
  };

  // The weight loads run one group ahead through the whole K; chunks start at even groups, so the two register sets
  // keep their turns across a chunk boundary and the first group of a chunk is on its way while the chunk is copied.
  // (Two groups ahead, with three register sets, measured slower at b = 4 and the same at b = 2.)
  if (active) load(pa, sa_a, 0);
  for (int c0 = 0; c0 < G; c0 += kB16Chunk) {
    const int g1 = (G - c0 < kB16Chunk) ? G : c0 + kB16Chunk;
    u32x4 xr[kB16Chunk];
#pragma unroll
    for (int k = 0; k < kB16Chunk; ++k) {
      xr[k] = u32x4{0, 0, 0, 0};
      if (copies && c0 + k < g1) xr[k] = xsrc[(c0 + k) * 16];
    }
    if (c0) __syncthreads();  // the previous chunk has been consumed
#pragma unroll
    for (int k = 0; k < kB16Chunk; ++k)
      if (copies && c0 + k < g1) *reinterpret_cast<u32x4*>(xdst + k * pitch) = xr[k];
    __syncthreads();
    if (active) {
      for (int g = c0; g < g1; g += 2) {
        load(pb, sa_b, g + 1);
        consume(pa, sa_a, g - c0);
        load(pa, sa_a, g + 2);
        if (g + 1 < g1) consume(pb, sa_b, g + 1 - c0);
      }
    }
  }
  if (active) {
    const int row0 = tile * 64 + (lane & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int j = 4 * (lane >> 4) + r;
      if (j < m) {
        float* yo = Y + static_cast<int64_t>(j) * L.out_f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int row = row0 + 16 * t;
          if (row < L.out_f) yo[row] = fmaf(acc_q[t][r], 16777216.0f, acc_x[t][r]);
        }
      }
    }
  }
}

template <int B>
__global__ __launch_bounds__(kB16Waves * 64, 3) void pmpd_block16_stack_kernel(const LayerDesc* __restrict__ layers,
                                                                               const WorkItem* __restrict__ items,
                                                                               const _Float16* __restrict__ x_base, int m,
                                                                               float* __restrict__ y_base) {
  extern __shared__ uint4 b16_lds[];
  const WorkItem it = items[blockIdx.x];
  const LayerDesc L = layers[it.layer];
  b16_tiles<B>(L, it.tile0, x_base + static_cast<int64_t>(m) * L.x_off, m, y_base + static_cast<int64_t>(m) * L.y_off,
               reinterpret_cast<char*>(b16_lds));
}

// One layer on its own (pmpd_gemm with 9 to 16 rows of X): workgroup k takes row tiles 4 k .. 4 k + 3.
template <int B>
__global__ __launch_bounds__(kB16Waves * 64, 3) void pmpd_block16_layer_kernel(LayerDesc L, const _Float16* __restrict__ X, int m,
                                                                               float* __restrict__ Y) {
  extern __shared__ uint4 b16_lds[];
  b16_tiles<B>(L, kB16Waves * static_cast<int>(blockIdx.x), X, m, Y, reinterpret_cast<char*>(b16_lds));
}

hipError_t launch_block16_layer(const LayerDesc& d, int b, const void* X, int m, float* Y, hipStream_t s) {
  if (m < 1 || m > 16) return hipErrorInvalidValue;
  const unsigned grid = static_cast<unsigned>((d.n_tiles + kB16Waves - 1) / kB16Waves);
  const size_t lds = static_cast<size_t>(std::min(kB16Chunk, d.n_groups)) * m * 256;
  const _Float16* x = static_cast<const _Float16*>(X);
  if (b == 4) hipLaunchKernelGGL((pmpd_block16_layer_kernel<4>), dim3(grid), dim3(kB16Waves * 64), lds, s, d, x, m, Y);
  else if (b == 3) hipLaunchKernelGGL((pmpd_block16_layer_kernel<3>), dim3(grid), dim3(kB16Waves * 64), lds, s, d, x, m, Y);
  else hipLaunchKernelGGL((pmpd_block16_layer_kernel<2>), dim3(grid), dim3(kB16Waves * 64), lds, s, d, x, m, Y);
  return hipGetLastError();
}

// Called by the C entry points (pmpd_gemv.hip) for batches of one 16-token block over a stack.
hipError_t launch_block16_stack(const pmpd_stack* st, int b, const void* X, int m, float* Y, hipStream_t s) {
  if (m < 1 || m > 16) return hipErrorInvalidValue;
  constexpr int kList = 0;  // 4-tile items: one 64-row tile per wave
  static_assert(kStackTilesPerWg[kList] == kB16Waves, "one tile per wave");
  const unsigned grid = static_cast<unsigned>(st->items[kList].size());
  const _Float16* x = static_cast<const _Float16*>(X);
  const size_t lds = static_cast<size_t>(std::min(kB16Chunk, st->max_in / kGroup)) * m * 256;
  if (b == 4) hipLaunchKernelGGL((pmpd_block16_stack_kernel<4>), dim3(grid), dim3(kB16Waves * 64), lds, s, st->d_layers, st->d_items[kList], x, m, Y);
  else if (b == 3) hipLaunchKernelGGL((pmpd_block16_stack_kernel<3>), dim3(grid), dim3(kB16Waves * 64), lds, s, st->d_layers, st->d_items[kList], x, m, Y);
  else hipLaunchKernelGGL((pmpd_block16_stack_kernel<2>), dim3(grid), dim3(kB16Waves * 64), lds, s, st->d_layers, st->d_items[kList], x, m, Y);
  return hipGetLastError();
}

}  // namespace pmpd
