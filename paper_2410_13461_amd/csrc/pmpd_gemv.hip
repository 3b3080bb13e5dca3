// HIP kernels (gfx950, wave64) and launchers for the PMPD decode linear layers.
//
// Mapping.  Lane l of a wave owns row 64*T + l of a row tile T; the wave walks the
// quantisation groups g of its K-range.  Per (tile, group) the wave issues one coalesced
// 1 KiB nontemporal global_load_dwordx4 per bit-plane (16 bytes = 128 weights of one row per
// lane) and one 256-byte load of the (scale, min) words.  All lanes work on the same columns, so
// the activations are wave-uniform: the batch-1 kernels read them through the scalar cache into
// SGPR operands of v_dot2_f32_f16; the batched kernels read them from LDS as MFMA operands.
// No cross-lane reduction exists; split-K partial sums of different waves meet in LDS in a
// fixed order, so results are run-to-run identical.
//
// Unpack.  The storage format places the bit of plane k for weight u = 2p + half,
// p = 4m + 2v + h, at bit (16 half + 8 v + 4 h + 3 - k + m) mod 32.  For each m one bit-select
// chain (v_bitop3_b32, B-1 ops) merges the B plane words into a word whose 4-bit fields, after a
// rotate by m, are complete codes: byte v, nibble h, 16-bit half `half`.  One v_and_or_b32
// masks the field of both halves and ORs in the fp16 exponent 0x6400, giving the pair
// (1024 + c*q, 1024 + c*q') with c = 1 (low nibble) or 16 (high nibble) without any shift; the
// planes that a b-bit pass does not read are simply absent from the mask, so the field holds
// q~ = q_b * 2^(4-b).  The pair is multiplied with the matching pair of x (products exact, fp32
// accumulation).  The constant 1024 and the factor 16 are removed per group with sums of x
// prepared once per workgroup:
//     sum_i W_b[r][i] x[i] = sum_g { a_g X_g + s_g ( accL + accH/16 + F_g ) }
//     X_g = sum of x over the group, F_g = 2^(3-b) X_g - 1024 (X_g^low + X_g^high / 16)
// where "low"/"high" are the columns whose field is the low/high nibble (i mod 4 < 2 / >= 2).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "pmpd_common.hpp"
#include "pmpd_device.hpp"

#ifndef PMPD_BATCH_WIDE_WAVES
#define PMPD_BATCH_WIDE_WAVES 3  // waves per SIMD the 8-vector, 2-tile kernel is compiled for (168 VGPRs, no spills)
#endif

namespace pmpd {

// =====================================================================================
// Batch 1: VALU dot products, x in SGPRs.

// Masks and fp16 exponents for the merged words that are used without their rotate (m = 1, 2).
template <int B>
struct Batch1Consts {
  uint32_t maskL[2], maskH[2], magic[2];
  __device__ __forceinline__ Batch1Consts() {
    constexpr uint32_t keep = (0xFu << (4 - B)) & 0xFu;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      maskL[i] = opaque_sgpr((keep * 0x00010001u) << (i + 1));
      maskH[i] = opaque_sgpr((keep * 0x00100010u) << (i + 1));
      magic[i] = i == 0 ? 0x60006000u : 0x5C005C00u;  // fp16 pairs (512, 512) and (256, 256)
      asm volatile("" : "+v"(magic[i]));
    }
  }
};

// Offset that the pairs of merged word m carry (see mac_group_sx).
__device__ __forceinline__ float pair_offset(int m) { return m == 1 ? 512.0f : m == 2 ? 256.0f : 1024.0f; }

// Multiply-accumulate one group (128 columns) of the lane's row.
//   pl[k]: the lane's 16 bytes of plane k;
//   xg:    the group's 4 x 16 dwords of x (fp16 pairs in natural column order), read with
//          s_load_dwordx16: they cost neither LDS bandwidth nor vector registers;
//   accL:  comes in holding F_g and leaves holding F_g + sum over low-nibble pairs,
//   accH:  sum over high-nibble pairs (to be divided by 16).
// The merged word of m = 1, 2 is used without the rotate by m: its fields then sit m bits
// higher, which the fp16 exponent absorbs (0x6000 = 512 has ulp 1/2, 0x5C00 = 256 has ulp 1/4),
// so the pair still reads offset + q~ with offset 512 / 256 instead of 1024.  F_g accounts for
// the per-m offsets (stage_group_sums).  m = 3 would put a field across bit 10 and is rotated.
template <int B>
__device__ __forceinline__ void mac_group_sx(const UnpackConsts<B>& uc, const Batch1Consts<B>& bc,
                                             const u32x4 (&pl)[B], const_u32x16_ptr xg, float& accL, float& accH) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const u32x16 xv = xg[d];
    uint32_t p[B];
#pragma unroll
    for (int k = 0; k < B; ++k) p[k] = word_of(pl[k], d);
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const uint32_t u = merge_planes<B>(uc, p, m);
      uint32_t w, w8, mL, mH, mg;
      if (m == 0 || m == 3) {
        w = (m == 0) ? u : __builtin_amdgcn_alignbit(u, u, 3);
        w8 = w >> 8;
        mL = uc.maskL; mH = uc.maskH; mg = uc.magic;
      } else {
        w = u;
        w8 = __builtin_amdgcn_alignbit(u, u, 8);  // rotate: the top field wraps into the low bits
        mL = bc.maskL[m - 1]; mH = bc.maskH[m - 1]; mg = bc.magic[m - 1];
      }
      accL = dot2(and_or(w, mL, mg), xv[4 * m + 0], accL);
      accH = dot2(and_or(w, mH, mg), xv[4 * m + 1], accH);
      accL = dot2(and_or(w8, mL, mg), xv[4 * m + 2], accL);
      accH = dot2(and_or(w8, mH, mg), xv[4 * m + 3], accH);
    }
  }
}

// LDS of a batch-1 workgroup: (X_g, F_g) per group, then NW*64 floats where the split-K partial
// sums meet.
__host__ __device__ inline size_t lds_bytes(int n_groups, int n_waves) {
  return static_cast<size_t>(n_groups) * 8 + static_cast<size_t>(n_waves) * 64 * 4;
}

// Per-group sums of the activation vector, computed by the whole workgroup into LDS.
template <int B, int NW>
__device__ __forceinline__ void stage_group_sums(const _Float16* __restrict__ x, int in_f, float2* cs) {
  const uint4* xg = reinterpret_cast<const uint4*>(x);
  const int n16 = in_f / 8;  // 16 uint4 per group; 16 consecutive threads share a group
  for (int idx = threadIdx.x; idx < n16; idx += NW * 64) {
    const uint4 v = xg[idx];
    // columns 8*idx .. 8*idx+7: (0,1) low, (2,3) high, (4,5) low, (6,7) high
    const half2_t a = __builtin_bit_cast(half2_t, v.x), b = __builtin_bit_cast(half2_t, v.y);
    const half2_t c = __builtin_bit_cast(half2_t, v.z), e = __builtin_bit_cast(half2_t, v.w);
    float lo = (static_cast<float>(a.x) + static_cast<float>(a.y)) + (static_cast<float>(c.x) + static_cast<float>(c.y));
    float hi = (static_cast<float>(b.x) + static_cast<float>(b.y)) + (static_cast<float>(e.x) + static_cast<float>(e.y));
    // these 8 columns belong to merged word m = idx % 4; E collects offset * (low + high/16)
    float X = lo + hi;
    float E = pair_offset(idx & 3) * (lo + hi * 0.0625f);
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {
      X += __shfl_xor(X, off, 16);
      E += __shfl_xor(E, off, 16);
    }
    if ((idx & 15) == 0) cs[idx >> 4] = make_float2(X, X * (B == 4 ? 0.5f : B == 3 ? 1.0f : 2.0f) - E);
  }
}

// One workgroup: TPW = NW / SPLITK consecutive row tiles starting at tile0, each split over
// SPLITK waves along K.  x: in_f fp16, y: out_f fp32.
template <int B, int NW, int SPLITK>
__device__ __forceinline__ void run_tiles(const LayerDesc& L, int tile0, const _Float16* __restrict__ x,
                                          float* __restrict__ y, uint4* lds) {
  static_assert(NW % SPLITK == 0, "waves must divide evenly over the K splits");
  const UnpackConsts<B> uc;
  const Batch1Consts<B> bc;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int G = L.n_groups;
  float2* cs = reinterpret_cast<float2*>(lds);
  float* red = reinterpret_cast<float*>(cs + G);

  const int tile = tile0 + wave / SPLITK;
  const int ks = wave % SPLITK;
  const bool active = tile < L.n_tiles;
  const int64_t base = (static_cast<int64_t>(active ? tile : 0) * G) * 64 + lane;  // + g*64 per group
  global_u32x4_ptr pp[B];
#pragma unroll
  for (int k = 0; k < B; ++k) pp[k] = (global_u32x4_ptr)(L.plane[k]) + base;
  global_u32_ptr sp = (global_u32_ptr)(L.sa) + base;
  const_u32x16_ptr xc = (const_u32x16_ptr)(x);

  float yacc = 0.f;
  const int g0 = G * ks / SPLITK, g1 = G * (ks + 1) / SPLITK;
  const bool work = active && g0 < g1;
  // The next group's plane words are in flight while the current group is consumed.  Weights
  // are read exactly once per pass: nontemporal loads keep them from displacing anything in
  // the caches (measured: the same loop without arithmetic streams 6.7 TB/s with them,
  // 5.8 TB/s without).  Past the end of the range the last group is reloaded (a cache hit)
  // instead of branching around the loads.  Two register sets A and B alternate (the loop is
  // unrolled by two), so nothing is copied.
  u32x4 pa[B], pb[B];
  uint32_t sa_a = 0, sa_b = 0;
  auto load = [&](u32x4 (&dst)[B], uint32_t& dsa, int g) {
    const int gl = g < g1 ? g : g1 - 1;
#pragma unroll
    for (int k = 0; k < B; ++k) dst[k] = __builtin_nontemporal_load(&pp[k][gl * 64]);
    dsa = sp[gl * 64];
  };
  // The first group's loads do not depend on the group sums: issue them before the workgroup
  // computes the sums, so that their latency overlaps the staging and the barrier.
  if (work) load(pa, sa_a, g0);

  stage_group_sums<B, NW>(x, L.in_f, cs);
  __syncthreads();

  if (work) {
    auto consume = [&](const u32x4 (&pl)[B], uint32_t csa, int g) {
      const float2 c = cs[g];
      float accL = c.y, accH = 0.f;
      mac_group_sx<B>(uc, bc, pl, xc + g * 4, accL, accH);
      const float s = half_bits_to_float(csa & 0xffffu);
      const float a = half_bits_to_float(csa >> 16);
      yacc = fmaf(s, fmaf(accH, 0.0625f, accL), yacc);
      yacc = fmaf(a, c.x, yacc);
    };
    for (int gc = g0; gc < g1; gc += 2) {
      load(pb, sa_b, gc + 1);
      consume(pa, sa_a, gc);
      load(pa, sa_a, gc + 2);
      if (gc + 1 < g1) consume(pb, sa_b, gc + 1);
    }
  }
  if constexpr (SPLITK > 1) {
    red[wave * 64 + lane] = yacc;
    __syncthreads();
    if (ks == 0) {
      float sum = yacc;
#pragma unroll
      for (int q = 1; q < SPLITK; ++q) sum += red[(wave + q) * 64 + lane];
      yacc = sum;
    }
  }
  if (ks == 0 && active) {
    const int row = tile * 64 + lane;
    if (row < L.out_f) y[row] = yacc;
  }
}

// =====================================================================================
// MFMA-assisted variant.  Unpack is unchanged; the multiply-accumulate and the sum over K go
// to the matrix pipe, which is otherwise idle, so the VALU only pays for the unpack.
//
// v_mfma_f32_16x16x32_f16 computes D[i][j] += sum_k A[i][k] B[k][j] with lane l holding
// A[l%16][8(l/16) .. 8(l/16)+7] and B[8(l/16) ..][l%16], and D[4(l/16)+t][l%16] in register t.
// A lane's 8 unpacked weights belong to ROW l of the tile, not to row l%16, so the operand is
// read as A[i][8G+t] = w[row 16G+i][t] (G = l/16).  Choosing B[8G+t][j] = x[t] for j == G and 0
// elsewhere gives D[i][j] = sum_t w[16j+i][t] x[t]: column j < 4 of D holds the dot products of
// rows 16j .. 16j+15.  Columns 4*beta + rho carry activation vector beta (up to 4 vectors per
// MFMA, 8 with a second accumulator set), so batches 1..8 read and unpack the weights once.
// The B operand comes straight from LDS with a per-lane address (x for the "diagonal" lanes,
// a block of zeros for the rest): no VALU work.  Low-nibble and high-nibble pairs go to
// separate accumulators DL, DH because they differ by the factor 16 (see the header comment).
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));

// LDS image for the MFMA path: per vector cg groups of x (256 B each, permuted), the (X_g, F_g)
// pairs, 256 zero bytes, then the split-K meeting point (16 B per lane, wave and accumulator set).
// Groups per K-chunk of the batched kernels: the whole row when the m vectors fit in about
// 32 KiB of LDS, else as many groups as fit.
__host__ __device__ inline int chunk_groups(int n_groups, int m) {
  const int fit = (32 * 1024) / (m * 256);
  return n_groups < fit ? n_groups : fit;
}

constexpr int kZeroBlockVec = 20;  // 320 zero bytes: 256 read by the off-diagonal lanes, 64 of phase shift
__host__ __device__ inline size_t lds_bytes_mfma(int cg, int m, int n_waves, int sets_times_tiles) {
  return static_cast<size_t>(m) * cg * 256 + static_cast<size_t>((m * cg + 1) & ~1) * 8 + kZeroBlockVec * 16 +
         static_cast<size_t>(sets_times_tiles) * n_waves * 64 * 16;
}

// Copy groups [c0, c0+cn) of the m vectors into LDS in MFMA operand order.  Within each
// 32-column word the 16 dwords are stored as [L#1][H#1][L#2][H#2], 4 dwords each, where L
// collects the column pairs whose code sits in a low nibble (columns 8q+0,1 and 8q+4,5) and H
// those in a high nibble (8q+2,3 and 8q+6,7); #1 covers columns 0..15 of the word, #2 16..31.
template <int B, int NW>
__device__ __forceinline__ void stage_activations_mfma(const _Float16* __restrict__ x, int in_f, int m, int c0, int cn,
                                                       int cg, uint32_t* xs, float2* cs, uint4* zeros) {
  const int n16 = cn * 16;
  for (int j = 0; j < m; ++j) {
    const uint4* xg = reinterpret_cast<const uint4*>(x + static_cast<int64_t>(j) * in_f) + c0 * 16;
    for (int idx = threadIdx.x; idx < n16; idx += NW * 64) {
      const uint4 v = xg[idx];
      const int q = idx & 3;  // which 8 columns of the 32-column word
      uint32_t* dst = xs + (j * cg * 64) + (idx >> 2) * 16 + (q >> 1) * 8 + (q & 1) * 2;
      *reinterpret_cast<uint2*>(dst) = make_uint2(v.x, v.z);
      *reinterpret_cast<uint2*>(dst + 4) = make_uint2(v.y, v.w);
      const half2_t a = __builtin_bit_cast(half2_t, v.x), b = __builtin_bit_cast(half2_t, v.y);
      const half2_t c = __builtin_bit_cast(half2_t, v.z), e = __builtin_bit_cast(half2_t, v.w);
      float lo = (static_cast<float>(a.x) + static_cast<float>(a.y)) + (static_cast<float>(c.x) + static_cast<float>(c.y));
      float hi = (static_cast<float>(b.x) + static_cast<float>(b.y)) + (static_cast<float>(e.x) + static_cast<float>(e.y));
#pragma unroll
      for (int off = 1; off < 16; off <<= 1) {
        lo += __shfl_xor(lo, off, 16);
        hi += __shfl_xor(hi, off, 16);
      }
      if ((idx & 15) == 0) {
        const float X = lo + hi;
        const float F = X * (B == 4 ? 0.5f : B == 3 ? 1.0f : 2.0f) - 1024.0f * (lo + hi * 0.0625f);
        cs[j * cg + (idx >> 4)] = make_float2(X, F);
      }
    }
  }
  if (threadIdx.x < kZeroBlockVec) zeros[threadIdx.x] = make_uint4(0, 0, 0, 0);
}

__device__ __forceinline__ half8_t as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  u32x4 v = {a, b, c, d};
  return __builtin_bit_cast(half8_t, v);
}

// One workgroup of the MFMA variant.  SETS = 1 serves m <= 4 vectors, SETS = 2 serves m <= 8.
// Each wave owns T consecutive row tiles and reuses every B operand it reads from LDS for all
// of them, which divides the LDS traffic per weight by T.
template <int B, int SETS, int T, int NW, int SPLITK>
__device__ __forceinline__ void run_tiles_mfma(const LayerDesc& L, int tile0, const _Float16* __restrict__ x, int m,
                                               float* __restrict__ y, uint4* lds) {
  static_assert(NW % SPLITK == 0, "waves must divide evenly over the K splits");
  const UnpackConsts<B> uc;
  const uint32_t maskL = uc.maskL, maskH = uc.maskH, magic = uc.magic;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int G = L.n_groups;
  const int cg = chunk_groups(G, m);
  uint32_t* xs = reinterpret_cast<uint32_t*>(lds);
  float2* cs = reinterpret_cast<float2*>(xs + m * cg * 64);
  uint4* zeros = reinterpret_cast<uint4*>(cs + ((m * cg + 1) & ~1));  // keep 16-byte alignment
  float4_t* red = reinterpret_cast<float4_t*>(zeros + kZeroBlockVec);

  const int tile_first = tile0 + (wave / SPLITK) * T;
  const int ks = wave % SPLITK;
  const bool active = tile_first < L.n_tiles;
  // MFMA output geometry of this lane: column j, rows 4*gq .. 4*gq+3 of the 16-row block rho.
  const int j = lane & 15, gq = lane >> 4;
  const int beta = j >> 2, rho = j & 3;
  const int rows0 = 16 * rho + 4 * gq;  // first of the lane's 4 output rows within a tile
  // Tiles past the end of the layer are clamped to the last one (loads stay in bounds, the
  // duplicate result is not stored).
  global_u32x4_ptr pp[T][B];
  global_u32x4_ptr sp[T];
#pragma unroll
  for (int t = 0; t < T; ++t) {
    int tl = tile_first + t;
    tl = tl < L.n_tiles ? tl : L.n_tiles - 1;
    tl = active ? tl : 0;
    const int64_t tbase = (static_cast<int64_t>(tl) * G) * 64;
#pragma unroll
    for (int k = 0; k < B; ++k) pp[t][k] = (global_u32x4_ptr)(L.plane[k]) + tbase + lane;
    sp[t] = (global_u32x4_ptr)((global_u32_ptr)(L.sa) + tbase + rows0);
  }

  // Per-lane LDS addressing of the B operand (bytes from xs): x of vector beta for the
  // "diagonal" lanes; every other lane reads a block of zeros that does not advance with the
  // group and sits 64 bytes out of phase so that the two addresses never share a bank.
  const char* lds_c = reinterpret_cast<const char*>(xs);
  const int zero_off = static_cast<int>(reinterpret_cast<const char*>(zeros) - lds_c) + 64;
  int boff[SETS], bmul[SETS], cidx[SETS];
#pragma unroll
  for (int s = 0; s < SETS; ++s) {
    const int bt = beta + 4 * s;
    const bool diag = (rho == gq) && (bt < m);
    boff[s] = diag ? bt * cg * 256 : zero_off;
    bmul[s] = diag ? 256 : 0;
    cidx[s] = (bt < m ? bt : m - 1) * cg;
  }

  float4_t yacc[T][SETS];
#pragma unroll
  for (int t = 0; t < T; ++t)
#pragma unroll
    for (int s = 0; s < SETS; ++s) yacc[t][s] = float4_t{0.f, 0.f, 0.f, 0.f};

  for (int c0 = 0; c0 < G; c0 += cg) {
    const int cn = (G - c0 < cg) ? (G - c0) : cg;
    if (c0) __syncthreads();
    stage_activations_mfma<B, NW>(x, L.in_f, m, c0, cn, cg, xs, cs, zeros);
    __syncthreads();
    const int g0 = c0 + cn * ks / SPLITK, g1 = c0 + cn * (ks + 1) / SPLITK;
    if (active && g0 < g1) {
      u32x4 nb[T][B];
#pragma unroll
      for (int t = 0; t < T; ++t)
#pragma unroll
        for (int k = 0; k < B; ++k) nb[t][k] = __builtin_nontemporal_load(&pp[t][k][g0 * 64]);
      for (int gc = g0; gc < g1; ++gc) {
        u32x4 cur[T][B];
        u32x4 csa[T];
        const int gl = (gc + 1 < g1) ? (gc + 1) : (g1 - 1);
#pragma unroll
        for (int t = 0; t < T; ++t) {
#pragma unroll
          for (int k = 0; k < B; ++k) cur[t][k] = nb[t][k];
          // scale/min words are needed only after the group's arithmetic: no ring for them
          csa[t] = __builtin_nontemporal_load(&sp[t][gc * 16]);
#pragma unroll
          for (int k = 0; k < B; ++k) nb[t][k] = __builtin_nontemporal_load(&pp[t][k][gl * 64]);
        }

        const char* xb[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) xb[s] = lds_c + boff[s] + (gc - c0) * bmul[s];
        float4_t dl[T][SETS], dh[T][SETS];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          half8_t bL[2][SETS], bH[2][SETS];
#pragma unroll
          for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int s = 0; s < SETS; ++s) {
              bL[q][s] = *reinterpret_cast<const half8_t*>(xb[s] + d * 64 + q * 32);
              bH[q][s] = *reinterpret_cast<const half8_t*>(xb[s] + d * 64 + q * 32 + 16);
            }
#pragma unroll
          for (int t = 0; t < T; ++t) {
            uint32_t p[B];
#pragma unroll
            for (int k = 0; k < B; ++k) p[k] = word_of(cur[t][k], d);
            uint32_t r[4][4];  // r[m][0..3] = (low v0, high v0, low v1, high v1) pairs of word m
#pragma unroll
            for (int mm = 0; mm < 4; ++mm) {
              uint32_t u = merge_planes<B>(uc, p, mm);
              uint32_t w = (mm == 0) ? u : __builtin_amdgcn_alignbit(u, u, mm);
              uint32_t w8 = w >> 8;
              r[mm][0] = and_or(w, maskL, magic);
              r[mm][1] = and_or(w, maskH, magic);
              r[mm][2] = and_or(w8, maskL, magic);
              r[mm][3] = and_or(w8, maskH, magic);
            }
#pragma unroll
            for (int q = 0; q < 2; ++q) {  // columns 16q .. 16q+15 of the word
              const half8_t aL = as_half8(r[2 * q][0], r[2 * q][2], r[2 * q + 1][0], r[2 * q + 1][2]);
              const half8_t aH = as_half8(r[2 * q][1], r[2 * q][3], r[2 * q + 1][1], r[2 * q + 1][3]);
#pragma unroll
              for (int s = 0; s < SETS; ++s) {
                const float4_t zero = {0.f, 0.f, 0.f, 0.f};
                dl[t][s] = __builtin_amdgcn_mfma_f32_16x16x32_f16(aL, bL[q][s], (d == 0 && q == 0) ? zero : dl[t][s], 0, 0, 0);
                dh[t][s] = __builtin_amdgcn_mfma_f32_16x16x32_f16(aH, bH[q][s], (d == 0 && q == 0) ? zero : dh[t][s], 0, 0, 0);
              }
            }
          }
        }
        // scale and minimum of the lane's 4 output rows per tile, once per group
#pragma unroll
        for (int t = 0; t < T; ++t) {
          const uint32_t sa4[4] = {csa[t].x, csa[t].y, csa[t].z, csa[t].w};
#pragma unroll
          for (int s = 0; s < SETS; ++s) {
            const float2 c = cs[cidx[s] + (gc - c0)];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float sc = half_bits_to_float(sa4[e] & 0xffffu);
              const float mn = half_bits_to_float(sa4[e] >> 16);
              const float u = fmaf(dh[t][s][e], 0.0625f, dl[t][s][e]) + c.y;
              yacc[t][s][e] = fmaf(sc, u, yacc[t][s][e]);
              yacc[t][s][e] = fmaf(mn, c.x, yacc[t][s][e]);
            }
          }
        }
      }
    }
  }
  if constexpr (SPLITK > 1) {
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
      for (int s = 0; s < SETS; ++s) red[((t * SETS + s) * NW + wave) * 64 + lane] = yacc[t][s];
    __syncthreads();
    if (ks == 0) {
#pragma unroll
      for (int t = 0; t < T; ++t)
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
          float4_t sum = yacc[t][s];
#pragma unroll
          for (int q = 1; q < SPLITK; ++q) sum += red[((t * SETS + s) * NW + wave + q) * 64 + lane];
          yacc[t][s] = sum;
        }
    }
  }
  if (ks == 0 && active) {
#pragma unroll
    for (int t = 0; t < T; ++t) {
      if (tile_first + t < L.n_tiles) {
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
          const int bt = beta + 4 * s;
          if (bt < m) {
            const int row = (tile_first + t) * 64 + rows0;
            float* yo = y + static_cast<int64_t>(bt) * L.out_f + row;
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (row + e < L.out_f) yo[e] = yacc[t][s][e];
          }
        }
      }
    }
  }
}

template <int B, int T, int NW, int SPLITK>
__global__ __launch_bounds__(NW * 64, 4) void pmpd_gemv_stack_mfma_kernel(const LayerDesc* __restrict__ layers,
                                                                          const WorkItem* __restrict__ items,
                                                                          const _Float16* __restrict__ x_base,
                                                                          float* __restrict__ y_base) {
  extern __shared__ uint4 lds[];
  const WorkItem it = items[blockIdx.x];
  const LayerDesc L = layers[it.layer];
  run_tiles_mfma<B, 1, T, NW, SPLITK>(L, it.tile0, x_base + L.x_off, 1, y_base + L.y_off, lds);
}

template <int B, int SETS, int T, int NW>
__global__ __launch_bounds__(NW * 64, (SETS * T > 2 ? PMPD_BATCH_WIDE_WAVES : 4)) void pmpd_gemm_stack_mfma_kernel(const LayerDesc* __restrict__ layers,
                                                                          const WorkItem* __restrict__ items,
                                                                          const _Float16* __restrict__ x_base, int m,
                                                                          float* __restrict__ y_base) {
  extern __shared__ uint4 lds[];
  const WorkItem it = items[blockIdx.x];
  const LayerDesc L = layers[it.layer];
  run_tiles_mfma<B, SETS, T, NW, 1>(L, it.tile0, x_base + static_cast<int64_t>(m) * L.x_off, m,
                                    y_base + static_cast<int64_t>(m) * L.y_off, lds);
}

template <int B, int SETS, int NW, int SPLITK>
__global__ __launch_bounds__(NW * 64, 4) void pmpd_gemm_layer_mfma_kernel(LayerDesc L, const _Float16* __restrict__ x,
                                                                          int m, float* __restrict__ y) {
  extern __shared__ uint4 lds[];
  run_tiles_mfma<B, SETS, 1, NW, SPLITK>(L, static_cast<int>(blockIdx.x) * (NW / SPLITK), x, m, y, lds);
}

template <int B, int NW, int SPLITK>
__global__ __launch_bounds__(NW * 64, 4) void pmpd_gemv_stack_kernel(const LayerDesc* __restrict__ layers,
                                                                   const WorkItem* __restrict__ items,
                                                                   const _Float16* __restrict__ x_base,
                                                                   float* __restrict__ y_base) {
  extern __shared__ uint4 lds[];
  const WorkItem it = items[blockIdx.x];
  const LayerDesc L = layers[it.layer];
  run_tiles<B, NW, SPLITK>(L, it.tile0, x_base + L.x_off, y_base + L.y_off, lds);
}

template <int B, int NW, int SPLITK>
__global__ __launch_bounds__(NW * 64, 4) void pmpd_gemv_layer_kernel(LayerDesc L, const _Float16* __restrict__ x,
                                                                   float* __restrict__ y) {
  extern __shared__ uint4 lds[];
  run_tiles<B, NW, SPLITK>(L, static_cast<int>(blockIdx.x) * (NW / SPLITK), x, y, lds);
}

// ------------------------------------------------------------------ host side ----
static int32_t hip_fail(hipError_t e, const char* what) {
  return fail(PMPD_EHIP, "%s: %s", what, hipGetErrorString(e));
}

LayerDesc make_desc(const pmpd_layer_t& L, int64_t x_off, int64_t y_off) {
  LayerDesc d;
  for (int k = 0; k < 4; ++k) d.plane[k] = L.planes[k];
  d.sa = L.scale_min;
  d.x_off = x_off;
  d.y_off = y_off;
  d.out_f = L.out_features;
  d.in_f = L.in_features;
  d.n_groups = L.in_features / kGroup;
  d.n_tiles = static_cast<int32_t>(padded_rows(L.out_features) / kTile);
  return d;
}

int32_t check_bits(int32_t b, const char* who) {
  if (b < 2 || b > 4) return fail(PMPD_EINVAL, "%s: bit-width %d outside {2,3,4}", who, b);
  return PMPD_OK;
}

// Launch shapes.  A stack has thousands of row tiles, so whole-K waves (no split) keep x
// staging rare; a single layer has few tiles and splits K to put more waves on the machine.
// Launch shapes.  A stack has thousands of row tiles, so whole-K waves (no split) are enough;
// a single layer has few tiles and splits K to put more waves on the machine.
template <int B, int NW, int SPLITK>
static hipError_t launch_layer(const LayerDesc& d, const void* x, float* y, hipStream_t s) {
  const int tpw = NW / SPLITK;
  const unsigned grid = static_cast<unsigned>((d.n_tiles + tpw - 1) / tpw);
  hipLaunchKernelGGL((pmpd_gemv_layer_kernel<B, NW, SPLITK>), dim3(grid), dim3(NW * 64), lds_bytes(d.n_groups, NW), s, d,
                     static_cast<const _Float16*>(x), y);
  return hipGetLastError();
}

template <int B>
static hipError_t launch_layer_b(const LayerDesc& d, const void* x, float* y, hipStream_t s) {
  // Split K until about 2048 waves exist or a wave would get fewer than 4 groups.
  int splitk = 1;
  while (splitk < 8 && static_cast<int64_t>(d.n_tiles) * splitk < 2048 && d.n_groups / (splitk * 2) >= 4) splitk *= 2;
  switch (splitk) {
    case 1: return launch_layer<B, 4, 1>(d, x, y, s);
    case 2: return launch_layer<B, 4, 2>(d, x, y, s);
    case 4: return launch_layer<B, 4, 4>(d, x, y, s);
    default: return launch_layer<B, 8, 8>(d, x, y, s);
  }
}

template <int B, int SETS, int NW, int SPLITK>
static hipError_t launch_layer_mfma(const LayerDesc& d, const void* x, int m, float* y, hipStream_t s) {
  const int tpw = NW / SPLITK;
  const unsigned grid = static_cast<unsigned>((d.n_tiles + tpw - 1) / tpw);
  const size_t lds = lds_bytes_mfma(chunk_groups(d.n_groups, m), m, NW, SETS);  // T = 1
  hipLaunchKernelGGL((pmpd_gemm_layer_mfma_kernel<B, SETS, NW, SPLITK>), dim3(grid), dim3(NW * 64), lds, s, d,
                     static_cast<const _Float16*>(x), m, y);
  return hipGetLastError();
}

template <int B, int SETS>
static hipError_t launch_layer_mfma_bs(const LayerDesc& d, const void* x, int m, float* y, hipStream_t s) {
  const int cg = chunk_groups(d.n_groups, m);
  int splitk = 1;
  while (splitk < 8 && static_cast<int64_t>(d.n_tiles) * splitk < 2048 && cg / (splitk * 2) >= 4) splitk *= 2;
  switch (splitk) {
    case 1: return launch_layer_mfma<B, SETS, 4, 1>(d, x, m, y, s);
    case 2: return launch_layer_mfma<B, SETS, 4, 2>(d, x, m, y, s);
    case 4: return launch_layer_mfma<B, SETS, 4, 4>(d, x, m, y, s);
    default: return launch_layer_mfma<B, SETS, 8, 8>(d, x, m, y, s);
  }
}

template <int B>
static hipError_t launch_layer_mfma_b(const LayerDesc& d, const void* x, int m, float* y, hipStream_t s) {
  return m <= 4 ? launch_layer_mfma_bs<B, 1>(d, x, m, y, s) : launch_layer_mfma_bs<B, 2>(d, x, m, y, s);
}

// defined in pmpd_prefill.hip
hipError_t launch_prefill_layer(const LayerDesc& d, int b, const void* X, int m, float* Y, hipStream_t s);
hipError_t launch_prefill_stack(const pmpd_stack* st, int b, const void* X, int m, float* Y, hipStream_t s);

static int32_t linear_entry(const char* who, const pmpd_layer_t* layer, int32_t b, const void* x, int32_t m, int32_t max_m,
                            float* y, void* stream) {
  int32_t rc = check_bits(b, who);
  if (rc) return rc;
  rc = check_layer(layer, b, who);
  if (rc) return rc;
  if (m < 1 || m > max_m) return fail(PMPD_EINVAL, "%s: batch %d outside 1..%d", who, m, max_m);
  if (!x || !y) return fail(PMPD_EINVAL, "%s: x or y is NULL", who);
  if (reinterpret_cast<uintptr_t>(x) % 16) return fail(PMPD_EALIGN, "%s: x not 16-byte aligned", who);
  if (reinterpret_cast<uintptr_t>(y) % 4) return fail(PMPD_EALIGN, "%s: y not 4-byte aligned", who);
  const LayerDesc d = make_desc(*layer, 0, 0);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (m > PMPD_MAX_BATCH) {  // compute-bound shape: MFMA tile kernel
    e = launch_prefill_layer(d, b, x, m, y, s);
  } else if (m > 1) {  // skinny batch: unpack once, MFMA multiply-accumulate
    e = b == 4 ? launch_layer_mfma_b<4>(d, x, m, y, s)
        : b == 3 ? launch_layer_mfma_b<3>(d, x, m, y, s)
                 : launch_layer_mfma_b<2>(d, x, m, y, s);
  } else {  // batch 1: VALU dot2 with x in SGPRs
    e = b == 4 ? launch_layer_b<4>(d, x, y, s)
        : b == 3 ? launch_layer_b<3>(d, x, y, s)
                 : launch_layer_b<2>(d, x, y, s);
  }
  if (e != hipSuccess) return hip_fail(e, who);
  return PMPD_OK;
}

}  // namespace pmpd

using namespace pmpd;

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

static void build_items(const std::vector<LayerDesc>& layers, int tiles_per_wg, std::vector<WorkItem>& out) {
  // Longest rows first: the last workgroups to start are the short ones, which trims the tail.
  std::vector<int> order(layers.size());
  for (size_t i = 0; i < order.size(); ++i) order[i] = static_cast<int>(i);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return layers[a].in_f > layers[b].in_f; });
  out.clear();
  for (int li : order)
    for (int t = 0; t < layers[li].n_tiles; t += tiles_per_wg) out.push_back(WorkItem{li, t});
}

static size_t stack_bytes(size_t n_layers, const size_t (&n_items)[kNumItemLists]) {
  size_t b = align_up(n_layers * sizeof(LayerDesc), 256);
  for (int q = 0; q < kNumItemLists; ++q) b += align_up(n_items[q] * sizeof(WorkItem), 256);
  return b;
}

// Stack kernel variants (PMPD_STACK_VARIANT="v4,v3,v2" overrides the per-bit-width defaults):
//   0  dot2, 4 waves x 1 tile, whole K            1  dot2, 4 waves on 1 tile, K split 4 ways
//   2  MFMA, 4 waves x 1 tile                     3  MFMA, 4 waves x 2 tiles
//   4  MFMA, 2 waves x 2 tiles                    5  dot2, 4 waves on 2 tiles, K split 2 ways
//   6  dot2, 8 waves on 1 tile, K split 8 ways    7  dot2, 8 waves on 2 tiles, K split 4 ways
//   8  dot2, 8 waves on 4 tiles, K split 2 ways   9  dot2, 2 waves on 1 tile, K split 2 ways
static constexpr int kNumVariants = 10;
// which work list (tiles per workgroup: list 0 = 4, 1 = 1, 2 = 8, 3 = 2) each variant walks
static constexpr int kVariantList[kNumVariants] = {0, 1, 0, 2, 0, 3, 1, 3, 0, 1};
// Defaults measured on the 7B-shaped and the mobile-scale stacks: at b = 4 and 3 the kernel is
// bound by the memory system and four waves that split one tile's K stream fastest; at b = 2 the
// VALU co-limits, so the per-workgroup staging is spread over more rows (4 tiles per workgroup)
// when the stack has enough tiles to keep every CU busy that way, else over 2.
static void pick_variants(pmpd_stack* st) {
  st->variant[4] = 1;
  st->variant[3] = 1;
  st->variant[2] = st->items[0].size() >= 4096 ? 0 : 5;
  const char* e = std::getenv("PMPD_STACK_VARIANT");
  if (e) {
    int v[3];
    if (std::sscanf(e, "%d,%d,%d", &v[0], &v[1], &v[2]) == 3) {
      for (int i = 0; i < 3; ++i)
        if (v[i] >= 0 && v[i] < kNumVariants) st->variant[4 - i] = v[i];
    }
  }
}

static int32_t check_stack_args(const pmpd_layer_t* layers, int32_t n, const char* who) {
  if (!layers) return fail(PMPD_EINVAL, "%s: layers is NULL", who);
  if (n < 1 || n > 65536) return fail(PMPD_EINVAL, "%s: n_layers %d outside 1..65536", who, n);
  for (int i = 0; i < n; ++i) {
    int32_t rc = check_layer(&layers[i], 4, who);
    if (rc) return rc;
  }
  return PMPD_OK;
}

template <int B>
static hipError_t launch_stack(const pmpd_stack* st, const void* xv, float* y, hipStream_t s) {
  const int v = st->variant[B];
  const int q = kVariantList[v];
  const unsigned grid = static_cast<unsigned>(st->items[q].size());
  const _Float16* x = static_cast<const _Float16*>(xv);
  const int max_groups = st->max_in / kGroup;
  const int cg = chunk_groups(max_groups, 1);
  switch (v) {
    case 0:
      hipLaunchKernelGGL((pmpd_gemv_stack_kernel<B, 4, 1>), dim3(grid), dim3(256), lds_bytes(max_groups, 4), s,
                         st->d_layers, st->d_items[q], x, y);
      break;
    case 1:
      hipLaunchKernelGGL((pmpd_gemv_stack_kernel<B, 4, 4>), dim3(grid), dim3(256), lds_bytes(max_groups, 4), s,
                         st->d_layers, st->d_items[q], x, y);
      break;
    case 5:
      hipLaunchKernelGGL((pmpd_gemv_stack_kernel<B, 4, 2>), dim3(grid), dim3(256), lds_bytes(max_groups, 4), s,
                         st->d_layers, st->d_items[q], x, y);
      break;
    case 6:
      hipLaunchKernelGGL((pmpd_gemv_stack_kernel<B, 8, 8>), dim3(grid), dim3(512), lds_bytes(max_groups, 8), s,
                         st->d_layers, st->d_items[q], x, y);
      break;
    case 7:
      hipLaunchKernelGGL((pmpd_gemv_stack_kernel<B, 8, 4>), dim3(grid), dim3(512), lds_bytes(max_groups, 8), s,
                         st->d_layers, st->d_items[q], x, y);
      break;
    case 8:
      hipLaunchKernelGGL((pmpd_gemv_stack_kernel<B, 8, 2>), dim3(grid), dim3(512), lds_bytes(max_groups, 8), s,
                         st->d_layers, st->d_items[q], x, y);
      break;
    case 9:
      hipLaunchKernelGGL((pmpd_gemv_stack_kernel<B, 2, 2>), dim3(grid), dim3(128), lds_bytes(max_groups, 2), s,
                         st->d_layers, st->d_items[q], x, y);
      break;
    case 2:
      hipLaunchKernelGGL((pmpd_gemv_stack_mfma_kernel<B, 1, 4, 1>), dim3(grid), dim3(256), lds_bytes_mfma(cg, 1, 4, 1), s,
                         st->d_layers, st->d_items[q], x, y);
      break;
    case 3:
      hipLaunchKernelGGL((pmpd_gemv_stack_mfma_kernel<B, 2, 4, 1>), dim3(grid), dim3(256), lds_bytes_mfma(cg, 1, 4, 2), s,
                         st->d_layers, st->d_items[q], x, y);
      break;
    default:
      hipLaunchKernelGGL((pmpd_gemv_stack_mfma_kernel<B, 2, 2, 1>), dim3(grid), dim3(128), lds_bytes_mfma(cg, 1, 2, 2), s,
                         st->d_layers, st->d_items[q], x, y);
      break;
  }
  return hipGetLastError();
}

template <int B, int T>
static hipError_t launch_stack_batch_t(const pmpd_stack* st, const _Float16* x, int m, float* y, hipStream_t s) {
  const int q = T == 2 ? 2 : 0;  // work list with 4*T tiles per workgroup
  const unsigned grid = static_cast<unsigned>(st->items[q].size());
  const int cg = chunk_groups(st->max_in / kGroup, m);
  if (m <= 4) {
    hipLaunchKernelGGL((pmpd_gemm_stack_mfma_kernel<B, 1, T, 4>), dim3(grid), dim3(256), lds_bytes_mfma(cg, m, 4, T), s,
                       st->d_layers, st->d_items[q], x, m, y);
  } else {
    hipLaunchKernelGGL((pmpd_gemm_stack_mfma_kernel<B, 2, T, 4>), dim3(grid), dim3(256), lds_bytes_mfma(cg, m, 4, 2 * T), s,
                       st->d_layers, st->d_items[q], x, m, y);
  }
  return hipGetLastError();
}

// Two row tiles per wave halve the LDS operand traffic per weight.  With more than 4 vectors
// (two accumulator sets) that always pays; with up to 4 it only pays when the stack has enough
// tiles to fill the machine with 8-tile workgroups (measured on the 7B and mobile-scale stacks).
template <int B>
static hipError_t launch_stack_batch(const pmpd_stack* st, const void* xv, int m, float* y, hipStream_t s) {
  const _Float16* x = static_cast<const _Float16*>(xv);
  const bool two_tiles = m > 4 || st->items[2].size() >= 2048;
  return two_tiles ? launch_stack_batch_t<B, 2>(st, x, m, y, s) : launch_stack_batch_t<B, 1>(st, x, m, y, s);
}

extern "C" {

int32_t pmpd_gemv(const pmpd_layer_t* layer, int32_t b, const void* x, float* y, void* stream) {
  return linear_entry("pmpd_gemv", layer, b, x, 1, 1, y, stream);
}

int32_t pmpd_gemm(const pmpd_layer_t* layer, int32_t b, const void* X, int32_t m, float* Y, void* stream) {
  return linear_entry("pmpd_gemm", layer, b, X, m, kMaxPrefillRows, Y, stream);
}

int32_t pmpd_stack_workspace_size(const pmpd_layer_t* layers, int32_t n, size_t* bytes) {
  int32_t rc = check_stack_args(layers, n, "pmpd_stack_workspace_size");
  if (rc) return rc;
  if (!bytes) return fail(PMPD_EINVAL, "pmpd_stack_workspace_size: bytes is NULL");
  size_t items[kNumItemLists] = {};
  for (int i = 0; i < n; ++i) {
    int64_t tiles = padded_rows(layers[i].out_features) / kTile;
    for (int q = 0; q < kNumItemLists; ++q)
      items[q] += static_cast<size_t>((tiles + kStackTilesPerWg[q] - 1) / kStackTilesPerWg[q]);
  }
  *bytes = stack_bytes(static_cast<size_t>(n), items);
  return PMPD_OK;
}

int32_t pmpd_stack_create(const pmpd_layer_t* layers, int32_t n, const int64_t* x_offset, const int64_t* y_offset,
                          void* workspace, size_t workspace_bytes, pmpd_stack_t** out) {
  int32_t rc = check_stack_args(layers, n, "pmpd_stack_create");
  if (rc) return rc;
  if (!x_offset || !y_offset || !workspace || !out) return fail(PMPD_EINVAL, "pmpd_stack_create: NULL argument");
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(PMPD_EALIGN, "pmpd_stack_create: workspace not 256-byte aligned");
  for (int i = 0; i < n; ++i) {
    if (x_offset[i] < 0 || x_offset[i] % 8) return fail(PMPD_EALIGN, "pmpd_stack_create: x_offset[%d] must be a non-negative multiple of 8", i);
    if (y_offset[i] < 0) return fail(PMPD_EINVAL, "pmpd_stack_create: y_offset[%d] is negative", i);
  }
  auto* st = new pmpd_stack;
  for (int i = 0; i < n; ++i) {
    st->layers.push_back(make_desc(layers[i], x_offset[i], y_offset[i]));
    st->max_in = std::max(st->max_in, layers[i].in_features);
  }
  size_t counts[kNumItemLists];
  for (int q = 0; q < kNumItemLists; ++q) {
    build_items(st->layers, kStackTilesPerWg[q], st->items[q]);
    counts[q] = st->items[q].size();
  }
  const size_t need = stack_bytes(st->layers.size(), counts);
  if (workspace_bytes < need) {
    delete st;
    return fail(PMPD_ESIZE, "pmpd_stack_create: workspace %zu bytes, need %zu", workspace_bytes, need);
  }
  char* w = static_cast<char*>(workspace);
  hipError_t e = hipMemcpy(w, st->layers.data(), st->layers.size() * sizeof(LayerDesc), hipMemcpyHostToDevice);
  st->d_layers = reinterpret_cast<const LayerDesc*>(w);
  w += align_up(st->layers.size() * sizeof(LayerDesc), 256);
  for (int q = 0; q < kNumItemLists && e == hipSuccess; ++q) {
    e = hipMemcpy(w, st->items[q].data(), st->items[q].size() * sizeof(WorkItem), hipMemcpyHostToDevice);
    st->d_items[q] = reinterpret_cast<const WorkItem*>(w);
    w += align_up(st->items[q].size() * sizeof(WorkItem), 256);
  }
  if (e != hipSuccess) {
    delete st;
    return hip_fail(e, "pmpd_stack_create copy");
  }
  pick_variants(st);
  *out = st;
  return PMPD_OK;
}

void pmpd_stack_destroy(pmpd_stack_t* stack) { delete stack; }

int32_t pmpd_decode_step(const pmpd_stack_t* stack, int32_t b, const void* x_base, float* y_base, void* stream) {
  int32_t rc = check_bits(b, "pmpd_decode_step");
  if (rc) return rc;
  if (!stack || !x_base || !y_base) return fail(PMPD_EINVAL, "pmpd_decode_step: NULL argument");
  if (reinterpret_cast<uintptr_t>(x_base) % 16) return fail(PMPD_EALIGN, "pmpd_decode_step: x_base not 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(y_base) % 4) return fail(PMPD_EALIGN, "pmpd_decode_step: y_base not 4-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = b == 4 ? launch_stack<4>(stack, x_base, y_base, s)
                 : b == 3 ? launch_stack<3>(stack, x_base, y_base, s)
                          : launch_stack<2>(stack, x_base, y_base, s);
  if (e != hipSuccess) return hip_fail(e, "pmpd_decode_step launch");
  return PMPD_OK;
}

int32_t pmpd_batch_step(const pmpd_stack_t* stack, int32_t b, const void* x_base, int32_t m, float* y_base,
                        void* stream) {
  int32_t rc = check_bits(b, "pmpd_batch_step");
  if (rc) return rc;
  if (!stack || !x_base || !y_base) return fail(PMPD_EINVAL, "pmpd_batch_step: NULL argument");
  if (m < 1 || m > kMaxPrefillRows) return fail(PMPD_EINVAL, "pmpd_batch_step: m %d outside 1..%d", m, kMaxPrefillRows);
  if (reinterpret_cast<uintptr_t>(x_base) % 16) return fail(PMPD_EALIGN, "pmpd_batch_step: x_base not 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(y_base) % 4) return fail(PMPD_EALIGN, "pmpd_batch_step: y_base not 4-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e;
  if (m == 1) {
    return pmpd_decode_step(stack, b, x_base, y_base, stream);
  } else if (m <= PMPD_MAX_BATCH) {
    e = b == 4 ? launch_stack_batch<4>(stack, x_base, m, y_base, s)
        : b == 3 ? launch_stack_batch<3>(stack, x_base, m, y_base, s)
                 : launch_stack_batch<2>(stack, x_base, m, y_base, s);
  } else {
    e = launch_prefill_stack(stack, b, x_base, m, y_base, s);
  }
  if (e != hipSuccess) return hip_fail(e, "pmpd_batch_step launch");
  return PMPD_OK;
}

int32_t pmpd_prefill_step(const pmpd_stack_t* stack, int32_t b, const void* x_base, int32_t m, float* y_base,
                          void* stream) {
  return pmpd_batch_step(stack, b, x_base, m, y_base, stream);
}

int32_t pmpd_decode_run(const pmpd_stack_t* stack, const pmpd_schedule_t* schedule, int32_t step0, int32_t n_steps,
                        const void* x_base, int64_t x_step_stride, float* y_base, int64_t y_step_stride, void* stream) {
  if (!stack || !schedule || !x_base || !y_base) return fail(PMPD_EINVAL, "pmpd_decode_run: NULL argument");
  if (step0 < 0 || n_steps < 0) return fail(PMPD_EINVAL, "pmpd_decode_run: negative step index or count");
  if (x_step_stride < 0 || y_step_stride < 0 || x_step_stride % 8) return fail(PMPD_EALIGN, "pmpd_decode_run: strides must be non-negative and x_step_stride a multiple of 8");
  // Validate every step's bit-width before the first launch.
  for (int32_t k = 0; k < n_steps; ++k) {
    int32_t b = 0;
    int32_t rc = pmpd_schedule_bits(schedule, step0 + k, &b);
    if (rc) return rc;
    rc = check_bits(b, "pmpd_decode_run");
    if (rc) return rc;
  }
  for (int32_t k = 0; k < n_steps; ++k) {
    int32_t b = 0;
    pmpd_schedule_bits(schedule, step0 + k, &b);
    const _Float16* x = static_cast<const _Float16*>(x_base) + static_cast<int64_t>(k) * x_step_stride;
    float* y = y_base + static_cast<int64_t>(k) * y_step_stride;
    int32_t rc = pmpd_decode_step(stack, b, x, y, stream);
    if (rc) return rc;
  }
  return PMPD_OK;
}

}  // extern "C"
