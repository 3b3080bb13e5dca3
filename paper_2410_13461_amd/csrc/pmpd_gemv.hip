// HIP kernels (gfx950, wave64) and launchers for the PMPD decode linear layers (batch 1..8).
//
// The multiply-accumulate runs on the scaled fp8 x fp4 matrix instruction
// v_mfma_scale_f32_16x16x128_f8f6f4; the VALU only interleaves and masks plane bits.
//
// Weights.  A 2-bit pair of code bits (p, p') in the two low bits of a nibble IS the fp4 (e2m1)
// number p + p'/2, so the merged plane words (pair_words) are an fp4 operand as they stand.  The
// 4-bit aligned code is q~ = q_b 2^(4-b) = 8 (p0 + p1/2) + 2 (p2 + p3/2): one MFMA per pair, the
// factors 8 and 2 ride on the block scale of the weight operand.  A b-bit pass leaves out the
// planes it does not read (b = 3: the lower pair becomes the single bit p2; b = 2: no lower pair).
//
// Activations.  The other operand is fp8 (e4m3).  Each fp16 x is split exactly into three pieces
//     x = 2^e0 m0 + 2^(e0-4) m1 + 2^(e0-8) m2,   m0, m1, m2 in e4m3,
// with one exponent e0 per 32 columns, applied by the instruction as the block scale of the
// activation operand.  (m0 = x / 2^e0 rounded to 4 significant bits; the residual is an fp16 number
// with at most 7 significant bits, and so on.)  The pieces sit in rows of the 16-row operand, so
// one MFMA multiplies 16 weight rows x 128 columns with all three pieces and the lane adds the
// three partial sums.
//
// Magnitude classes.  The instruction sums the 32 products of one scale block in a fixed-point
// window of 14 bits below the leading bit of the block's largest product (measured: smaller bits
// are dropped; different blocks and the C input are added exactly).  A product here has 6
// significant bits, so the sum is exact when the elements of a block span at most 8 binades.
// Each 32-column block of x is therefore split into two vectors with disjoint support: class A
// holds the elements within 8 binades of the block's largest magnitude, class B the rest, scaled
// by its own largest magnitude.  Elements more than 16 binades below their block's largest lose
// their low bits (below 2^-21 of the largest product of the block).  The split is done once per
// workgroup and K-chunk while the first weight loads are in flight.
//
// Rows of the activation operand.  The 16 rows are four slots of four rows; slot q carries the
// three pieces of one class of one vector in rows 4 q .. 4 q + 2 (row 4 q + 3 is not used): slot
// 2 v + c of operand set s holds class c of vector 2 s + v.  Batch 1 fills two slots of one set,
// a batch of m vectors fills 2 m slots of ceil(m / 2) sets; the weights are read and unpacked once
// for all of them.
//
// Operand geometry (checked on gfx950): the fp8 operand's lane i + 16 kb holds row i, columns
// 16 kb .. 16 kb + 15 and 64 + 16 kb .. 64 + 16 kb + 15; the scale of its columns 32 c .. 32 c + 31
// is byte 0 of the scale register of lane i + 16 c.  The fp4 operand's lane j + 16 kb holds
// column j (= weight row j of the 16-row block) for K = 32 kb .. 32 kb + 31, eight nibbles per
// register.  D[i][j] sits in lane j + 16 (i / 4), register i % 4.
//
// D[i][j] sits in lane j + 16 (i / 4), register i % 4: lane l receives, from the MFMA over weight
// rows 16 t .. 16 t + 15 of the tile, the three partial sums of slot l / 16 and weight row
// 16 t + l % 16.  It scales them with that row's (scale, min) word, which it loaded itself (the
// words of a (tile, group) are stored in the order [l % 16][t], 16 bytes per lane), and the two
// classes of a vector, 16 lanes apart, are added once at the end.
//
// Per group (128 columns), row and class:  sum_i W_b x = s_g (D + 2^(3-b) X_g) + a_g X_g,
// D = sum q~ x, X_g = sum of the class's x over the group: scale and minimum are applied once per
// 128 weights.
// No atomics and a fixed summation order: results are run-to-run identical.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "pmpd_common.hpp"
#include "pmpd_device.hpp"
#include "pmpd_sumword.hpp"

#ifndef PMPD_BATCH_WIDE_WAVES
#define PMPD_BATCH_WIDE_WAVES 3  // waves per SIMD the kernels for 5..8 vectors are compiled for
#endif

namespace pmpd {

typedef short short2_t __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

// LDS image of the split activations, per vector and group: for each of the two magnitude
// classes 3 pieces x 128 fp8 in operand order (stride kPieceStride) and 16 bytes of block exponents ([piece][32-column
// block], 12 used) and one fp32 group sum.
constexpr int kPieceStride = 144;              // 128 fp8 of one piece + 16 bytes so that the three pieces of a
                                              // group start in different LDS banks
constexpr int kPieceBytes = 3 * kPieceStride;  // one class
constexpr int kGroupPieceBytes = 2 * kPieceBytes;  // both classes of one group
constexpr int kScaleBytes = 16;    // one class
constexpr int kImageBytes = 2 * (kPieceBytes + kScaleBytes + 4);

// Groups per K-chunk: the whole row when the m images fit in the LDS budget (36 KiB for up to 4
// vectors, so that four workgroups share a CU; 64 KiB above), else as many groups as fit.
__host__ __device__ inline int chunk_groups(int n_groups, int m) {
  const int fit = ((m <= 4 ? 36 : 64) * 1024) / (m * kImageBytes);
  return n_groups < fit ? n_groups : fit;
}

__host__ __device__ inline size_t lds_bytes(int chunk, int m, int n_waves, int accs_per_lane) {
  return static_cast<size_t>(m) * chunk * kImageBytes + static_cast<size_t>(n_waves) * accs_per_lane * 64 * 4;
}

// Where the parts of the image of vector j live, for a chunk capacity of cg groups and m vectors.
struct ImageLayout {
  char* pieces;   // [m][cg][2 classes][3 pieces][kPieceStride]: six operand rows of a group in six bank phases
  char* scales;   // [m][2][cg][16]
  float* xsum;    // [m][2][cg]
  float* red;     // split-K meeting point
  int cg;
  __device__ __forceinline__ ImageLayout(void* lds, int cg_, int m) : cg(cg_) {
    pieces = static_cast<char*>(lds);
    scales = pieces + m * 2 * cg * kPieceBytes;
    xsum = reinterpret_cast<float*>(scales + m * 2 * cg * kScaleBytes);
    red = xsum + m * 2 * cg;
  }
  __device__ __forceinline__ int piece_off(int j, int cls) const { return j * cg * kGroupPieceBytes + cls * kPieceBytes; }
  __device__ __forceinline__ int scale_off(int j, int cls) const { return (j * 2 + cls) * cg * kScaleBytes; }
  __device__ __forceinline__ int xsum_off(int j, int cls) const { return (j * 2 + cls) * cg; }
};

// Four fp16 -> four e4m3 bytes, each divided by `scale` (a power of two), round to nearest even.
__device__ __forceinline__ uint32_t to_fp8x4(half2_t lo, half2_t hi, float scale) {
  short2_t r = {0, 0};
  r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(r, lo, scale, false);
  r = __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(r, hi, scale, true);
  return __builtin_bit_cast(uint32_t, r);
}

// Largest magnitude (fp16 bit pattern without sign) over the 32 columns a quad of threads owns.
__device__ __forceinline__ uint32_t quad_max_magnitude(const uint32_t (&w)[4]) {
  ushort2_t mx = __builtin_bit_cast(ushort2_t, w[0] & 0x7FFF7FFFu);
#pragma unroll
  for (int q = 1; q < 4; ++q) mx = __builtin_elementwise_max(mx, __builtin_bit_cast(ushort2_t, w[q] & 0x7FFF7FFFu));
  uint32_t mag = mx.x > mx.y ? mx.x : mx.y;
  uint32_t o = dpp_u32<kQuadSwap1>(mag);
  mag = mag > o ? mag : o;
  o = dpp_u32<kQuadSwap2>(mag);
  return mag > o ? mag : o;
}

// Three e4m3 pieces of 8 fp16 values (4 column pairs in w) whose largest exponent field in the
// 32-column block is E, written to dst (piece stride kPieceStride) in operand order: bytes 0..3 =
// columns 0,2,4,6, bytes 4..7 = columns 1,3,5,7 (the order of the nibbles in the weight words).
// Every |x| of the block is below 2^(E-14), so x / 2^(E-22) is below 256 and fits e4m3 (largest
// finite value 448) without overflow.  The block exponents go to sdst[0], [4], [8] (e8m0 bytes of
// 2^(E-22), 2^(E-26), 2^(E-30)).
__device__ __forceinline__ void split_pieces(const uint32_t (&w)[4], uint32_t E, char* dst, char* sdst, int quad_lane) {
  const float sc0 = __builtin_bit_cast(float, (E + 105u) << 23);  // 2^(E-22)
  const float sc1 = __builtin_bit_cast(float, (E + 101u) << 23);  // 2^(E-26)
  const float sc2 = __builtin_bit_cast(float, (E + 97u) << 23);   // 2^(E-30)
  uint32_t p0[2], p1[2], p2[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {  // q = 0: even columns, q = 1: odd columns
    const uint32_t sel = q == 0 ? 0x05040100u : 0x07060302u;
    half2_t a = __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(w[1], w[0], sel));
    half2_t b = __builtin_bit_cast(half2_t, __builtin_amdgcn_perm(w[3], w[2], sel));
    p0[q] = to_fp8x4(a, b, sc0);
    a -= __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(p0[q], sc0, false);  // exact
    b -= __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(p0[q], sc0, true);
    p1[q] = to_fp8x4(a, b, sc1);
    a -= __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(p1[q], sc1, false);
    b -= __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(p1[q], sc1, true);
    p2[q] = to_fp8x4(a, b, sc2);
  }
  *reinterpret_cast<uint2*>(dst) = make_uint2(p0[0], p0[1]);
  *reinterpret_cast<uint2*>(dst + kPieceStride) = make_uint2(p1[0], p1[1]);
  *reinterpret_cast<uint2*>(dst + 2 * kPieceStride) = make_uint2(p2[0], p2[1]);
  // thread p of the quad writes the block exponent of piece p
  if (quad_lane < 3) sdst[4 * quad_lane] = static_cast<char>(E + 105u - 4u * quad_lane);
}

// Split groups [c0, c0 + cn) of activation vector j into the two classes' pieces, block
// exponents and group sums, by NT threads (whole waves) of which the caller is number tid.
// Thread idx handles columns 8 idx .. 8 idx + 7 of the range; a quad of threads owns one
// 32-column block, a row of 16 threads one group.
// Where a layer's activations come from: an fp16 vector, or the output of an earlier layer of the same
// launch, scaled by `gain` and rounded to fp16 (round to nearest even) on the way in: the sums of its
// `parts` K-parts (y64), read again (at most `spin_limit` times, then *timed_out is set) until complete.
struct XSource {
  const _Float16* x16;
  const unsigned long long* y64;
  float gain;
  int parts;
  uint32_t spin_limit;
  uint32_t* timed_out;
};
__device__ __forceinline__ XSource x_from_fp16(const _Float16* p) { return XSource{p, nullptr, 1.f, 0, 0, nullptr}; }

__device__ __forceinline__ uint32_t pack_half2(float a, float b) {
  const half2_t h = {static_cast<_Float16>(a), static_cast<_Float16>(b)};
  return __builtin_bit_cast(uint32_t, h);
}

template <int NT>
__device__ __forceinline__ void stage_x(const XSource& src, int c0, int cn, const ImageLayout& im, int j, int tid) {
  const int n16 = cn * 16;
  for (int idx = tid; idx < n16; idx += NT) {
    uint32_t w[4];
    if (src.y64) {
      // sums other workgroups of this launch add to: agent-scope loads read the coherent copy
      unsigned long long* yg = const_cast<unsigned long long*>(src.y64) + (c0 * 16 + idx) * 8;
      unsigned long long s8[8];
      for (uint32_t tries = 0;;) {
        bool complete = true;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          s8[e] = __hip_atomic_load(yg + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          complete = complete && sum_complete(s8[e], src.parts);
        }
        if (complete) break;
        if (++tries >= src.spin_limit) {
          __hip_atomic_store(src.timed_out, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
        __builtin_amdgcn_s_sleep(8);
      }
      float v8[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v8[e] = sum_value(s8[e], src.parts) * src.gain;
#pragma unroll
      for (int q = 0; q < 4; ++q) w[q] = pack_half2(v8[2 * q], v8[2 * q + 1]);
    } else {
      const uint4 v = (reinterpret_cast<const uint4*>(src.x16) + c0 * 16)[idx];
      w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    }
    const uint32_t EA = quad_max_magnitude(w) >> 10;  // exponent field of the block's largest |x|
    // class B: magnitude below 2^(EA-7-15), i.e. bit pattern below (EA-7) << 10
    const uint32_t thr = (EA > 7u ? EA - 7u : 0u) << 10;
    const ushort2_t thr2 = {static_cast<unsigned short>(thr), static_cast<unsigned short>(thr)};
    uint32_t wa[4], wb[4];
    float xsa = 0.f, xsb = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const ushort2_t mag = __builtin_bit_cast(ushort2_t, w[q] & 0x7FFF7FFFu);
      const short2_t below = __builtin_bit_cast(short2_t, static_cast<ushort2_t>(mag - thr2)) >> 15;  // all ones iff class B
      const uint32_t mb = __builtin_bit_cast(uint32_t, below);
      wa[q] = w[q] & ~mb;
      wb[q] = w[q] & mb;
      xsa = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, wa[q]), half2_t{1, 1}, xsa, false);
      xsb = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, wb[q]), half2_t{1, 1}, xsb, false);
    }
    const uint32_t EB = quad_max_magnitude(wb) >> 10;
    const int g = idx >> 4, c8 = idx & 15;
    const int lead = idx & 3;
    split_pieces(wa, EA, im.pieces + im.piece_off(j, 0) + g * kGroupPieceBytes + c8 * 8,
                 im.scales + im.scale_off(j, 0) + g * kScaleBytes + (c8 >> 2), lead);
    split_pieces(wb, EB, im.pieces + im.piece_off(j, 1) + g * kGroupPieceBytes + c8 * 8,
                 im.scales + im.scale_off(j, 1) + g * kScaleBytes + (c8 >> 2), lead);
    xsa += dpp_f32<kQuadSwap1>(xsa);
    xsb += dpp_f32<kQuadSwap1>(xsb);
    xsa += dpp_f32<kQuadSwap2>(xsa);
    xsb += dpp_f32<kQuadSwap2>(xsb);
    xsa += dpp_f32<kRowHalfMirror>(xsa);
    xsb += dpp_f32<kRowHalfMirror>(xsb);
    xsa += dpp_f32<kRowMirror>(xsa);
    xsb += dpp_f32<kRowMirror>(xsb);
    if (c8 == 0) {
      im.xsum[im.xsum_off(j, 0) + g] = xsa;
      im.xsum[im.xsum_off(j, 1) + g] = xsb;
    }
  }
}

__device__ __forceinline__ i32x8 fp4_operand(const uint32_t (&w)[4]) {
  return i32x8{static_cast<int>(w[0]), static_cast<int>(w[1]), static_cast<int>(w[2]), static_cast<int>(w[3]), 0, 0, 0, 0};
}

// One activation operand set: the fp8 registers and the block-scale register of the lane.
struct XOperand {
  i32x8 a;
  int scale;
};

// X x (the weights of 16-row block t of the lane's plane words pl) for the bit-width B: sum of
// q~ x over the group, per operand row.  wscale holds the e8m0 bytes of 2^3 (byte 0, upper
// pair) and 2^1 (byte 1, lower pair).  SETS operand sets share the unpacked weight operand.
template <int B, int SETS>
__device__ __forceinline__ void mfma_block(const XOperand (&X)[SETS], const u32x4 (&pl)[B], int t, int wscale,
                                           float4_t (&acc)[SETS]) {
  uint32_t w[4];
  pair_words(word_of(pl[0], t), word_of(pl[1], t), w);
  i32x8 op = fp4_operand(w);
  const float4_t zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < SETS; ++s)
    acc[s] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(X[s].a, op, zero, 0 /*A: e4m3*/, 4 /*B: e2m1*/, 0, X[s].scale, 0,
                                                              wscale);
  if constexpr (B >= 3) {
    if constexpr (B == 4) pair_words(word_of(pl[2], t), word_of(pl[3], t), w);
    else single_words(word_of(pl[2], t), w);
    op = fp4_operand(w);
#pragma unroll
    for (int s = 0; s < SETS; ++s)
      acc[s] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(X[s].a, op, acc[s], 0, 4, 0, X[s].scale, 1, wscale);
  }
}

__device__ __forceinline__ i32x8 read_fp8_operand(const char* p) {
  const u32x4 lo = *reinterpret_cast<const u32x4*>(p);
  const u32x4 hi = *reinterpret_cast<const u32x4*>(p + 64);
  return i32x8{static_cast<int>(lo.x), static_cast<int>(lo.y), static_cast<int>(lo.z), static_cast<int>(lo.w),
               static_cast<int>(hi.x), static_cast<int>(hi.y), static_cast<int>(hi.z), static_cast<int>(hi.w)};
}

template <int B>
constexpr float half_step() { return B == 4 ? 0.5f : B == 3 ? 1.0f : 2.0f; }  // 2^(3-b)

// =====================================================================================
// The groups a workgroup walks (the whole row unless K is split over workgroups) and the chunk
// capacity the LDS image was sized for.
struct KRange {
  int begin, end, chunk;
};

// A lane's addresses into the stored words of one 64-row tile: word [g * 64] of plane k is the
// lane's 16 bytes of group g, word [g * 16] of sp the (scale, min) words of rows l % 16 + 16 t,
// t = 0..3 (the 16 bytes at [l % 16] of the group's 64 words).
template <int B>
struct TileWords {
  global_u32x4_ptr pp[B];
  global_u32x4_ptr sp;
  __device__ __forceinline__ TileWords(const LayerDesc& L, int tile, int lane) {
    const int64_t tbase = (static_cast<int64_t>(tile) * L.n_groups) * 64 + lane;
#pragma unroll
    for (int k = 0; k < B; ++k) pp[k] = (global_u32x4_ptr)(L.plane[k]) + tbase;
    sp = (global_u32x4_ptr)(L.sa) + (tbase - lane) / 4 + (lane & 15);
  }
  // Weights are read exactly once per pass: nontemporal loads keep them from displacing anything
  // in the caches.
  __device__ __forceinline__ void load(u32x4 (&dst)[B], u32x4& dsa, int g) const {
#pragma unroll
    for (int k = 0; k < B; ++k) dst[k] = __builtin_nontemporal_load(&pp[k][g * 64]);
    dsa = sp[g * 16];
  }
};

// Where a lane finds its operands in the LDS image.  Row i = lane % 16 of the activation operand
// is piece i % 4 of slot i / 4; the lane receives the sums of slot lane / 16.  Slot 2 v + c =
// class c of vector 2 s + v.
template <int SETS>
struct OperandOffsets {
  int a[SETS], s[SETS], x[SETS];
  __device__ __forceinline__ OperandOffsets(const ImageLayout& im, int lane, int m) {
    const int piece = (lane & 3) == 3 ? 0 : (lane & 3);  // row 4 q + 3 is never read back
    const int in_slot = (lane & 15) >> 2, out_slot = lane >> 4;
#pragma unroll
    for (int q = 0; q < SETS; ++q) {
      int vi = 2 * q + (in_slot >> 1);
      vi = vi < m ? vi : m - 1;  // slots of absent vectors repeat the last one; their sums are not stored
      a[q] = im.piece_off(vi, in_slot & 1) + piece * kPieceStride + (lane >> 4) * 16;
      s[q] = im.scale_off(vi, in_slot & 1) + piece * 4 + (lane >> 4);
      int vo = 2 * q + (out_slot >> 1);
      vo = vo < m ? vo : m - 1;
      x[q] = im.xsum_off(vo, out_slot & 1);
    }
  }
};

// yacc += (the weights of one group of the tile) x (the split activations of group gr of the image).
template <int B, int SETS>
__device__ __forceinline__ void consume_group(const ImageLayout& im, const OperandOffsets<SETS>& off, int gr, const u32x4 (&pl)[B],
                                              const u32x4& csa, int wscale, float (&yacc)[SETS][4]) {
  XOperand X[SETS];
  float xg[SETS];
#pragma unroll
  for (int s = 0; s < SETS; ++s) {
    X[s].a = read_fp8_operand(im.pieces + off.a[s] + gr * kGroupPieceBytes);
    X[s].scale = static_cast<unsigned char>(im.scales[off.s[s] + gr * kScaleBytes]);
    xg[s] = im.xsum[off.x[s] + gr];
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    float4_t acc[SETS];
    mfma_block<B, SETS>(X, pl, t, wscale, acc);
    const uint32_t w = word_of(csa, t);
    const float sc = half_bits_to_float(w & 0xffffu);
    const float offs = fmaf(sc, half_step<B>(), half_bits_to_float(w >> 16));
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
      const float d = (acc[s][0] + acc[s][1]) + acc[s][2];
      yacc[s][t] = fmaf(sc, d, yacc[s][t]);
      yacc[s][t] = fmaf(offs, xg[s], yacc[s][t]);
    }
  }
}

__device__ __forceinline__ int weight_scale_register() {
  int wscale = 0x00008082;  // e8m0 bytes of 2^3 (byte 0, upper plane pair) and 2^1 (byte 1, lower pair)
  asm volatile("" : "+v"(wscale));
  return wscale;
}

// One workgroup: NW / SPLITK consecutive row tiles starting at tile0, each split over SPLITK waves
// along K, for m <= 2 SETS activation vectors.  K is walked in chunks whose split activations fit
// in LDS.  x: [m][in_f] fp16, y: [m][out_f] fp32.
template <int B, int SETS, int NW, int SPLITK>
__device__ __forceinline__ void run_tiles(const LayerDesc& L, int tile0, const _Float16* __restrict__ x, int m, float* __restrict__ y,
                                          uint4* lds_raw, KRange kr) {
  static_assert(NW % SPLITK == 0, "waves must divide evenly over the K splits");
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const ImageLayout im(lds_raw, kr.chunk, m);

  const int tile = tile0 + wave / SPLITK;
  const int ks = wave % SPLITK;
  const bool active = tile < L.n_tiles;
  const TileWords<B> tw(L, active ? tile : 0, lane);
  const OperandOffsets<SETS> off(im, lane, m);
  const int out_slot = lane >> 4;
  const int wscale = weight_scale_register();

  float yacc[SETS][4];
#pragma unroll
  for (int s = 0; s < SETS; ++s)
#pragma unroll
    for (int t = 0; t < 4; ++t) yacc[s][t] = 0.f;

  for (int c0 = kr.begin; c0 < kr.end; c0 += im.cg) {
    const int cn = (kr.end - c0 < im.cg) ? (kr.end - c0) : im.cg;
    const int g0 = c0 + cn * ks / SPLITK, g1 = c0 + cn * (ks + 1) / SPLITK;
    const bool work = active && g0 < g1;
    // The next group's plane words are in flight while the current group is consumed.  Past the
    // end of the range the last group is reloaded (a cache hit) instead of branching around the
    // loads.  Two register sets alternate (the loop is unrolled by two).
    u32x4 pa[B], pb[B], sa_a = {0, 0, 0, 0}, sa_b = {0, 0, 0, 0};
    auto load = [&](u32x4 (&dst)[B], u32x4& dsa, int g) { tw.load(dst, dsa, g < g1 ? g : g1 - 1); };
    // The first group's loads do not depend on the activations: issue them before the workgroup
    // splits x, so that their latency overlaps the staging and the barrier.
    if (work) load(pa, sa_a, g0);
    if (c0 != kr.begin) __syncthreads();  // the previous chunk's image has been consumed
    for (int j = 0; j < m; ++j)
      stage_x<NW * 64>(x_from_fp16(x + static_cast<int64_t>(j) * L.in_f), c0, cn, im, j, threadIdx.x);
    __syncthreads();
    if (work) {
      for (int gc = g0; gc < g1; gc += 2) {
        load(pb, sa_b, gc + 1);
        consume_group<B, SETS>(im, off, gc - c0, pa, sa_a, wscale, yacc);
        load(pa, sa_a, gc + 2);
        if (gc + 1 < g1) consume_group<B, SETS>(im, off, gc + 1 - c0, pb, sa_b, wscale, yacc);
      }
    }
  }
  // the two classes of a vector sit 16 lanes apart: add them (fixed order: A + B)
#pragma unroll
  for (int s = 0; s < SETS; ++s)
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float other = __shfl_xor(yacc[s][t], 16);
      yacc[s][t] = (out_slot & 1) ? other + yacc[s][t] : yacc[s][t] + other;
    }
  if constexpr (SPLITK > 1) {
    __syncthreads();
#pragma unroll
    for (int s = 0; s < SETS; ++s)
#pragma unroll
      for (int t = 0; t < 4; ++t) im.red[((s * 4 + t) * NW + wave) * 64 + lane] = yacc[s][t];
    __syncthreads();
    if (ks == 0) {
#pragma unroll
      for (int s = 0; s < SETS; ++s)
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          float sum = yacc[s][t];
#pragma unroll
          for (int q = 1; q < SPLITK; ++q) sum += im.red[((s * 4 + t) * NW + wave + q) * 64 + lane];
          yacc[s][t] = sum;
        }
    }
  }
  if (ks == 0 && active && (out_slot & 1) == 0) {
#pragma unroll
    for (int s = 0; s < SETS; ++s) {
      const int vo = 2 * s + (out_slot >> 1);
      if (vo < m) {
        float* yo = y + static_cast<int64_t>(vo) * L.out_f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int row = tile * 64 + 16 * t + (lane & 15);
          if (row < L.out_f) yo[row] = yacc[s][t];
        }
      }
    }
  }
}

// Waves per SIMD the kernels are compiled for: 4 for one or two operand sets, fewer above.
template <int SETS>
constexpr int waves_per_simd() { return SETS <= 2 ? 4 : PMPD_BATCH_WIDE_WAVES; }

template <int B, int SETS, int NW, int SPLITK>
__global__ __launch_bounds__(NW * 64, waves_per_simd<SETS>()) void pmpd_stack_kernel(
    const LayerDesc* __restrict__ layers, const WorkItem* __restrict__ items, const _Float16* __restrict__ x_base, int m,
    float* __restrict__ y_base) {
  extern __shared__ uint4 lds[];
  const WorkItem it = items[blockIdx.x];
  const LayerDesc L = layers[it.layer];
  run_tiles<B, SETS, NW, SPLITK>(L, it.tile0, x_base + static_cast<int64_t>(m) * L.x_off, m,
                                 y_base + static_cast<int64_t>(m) * L.y_off, lds, KRange{0, L.n_groups, chunk_groups(L.n_groups, m)});
}

template <int B, int SETS, int NW, int SPLITK>
__global__ __launch_bounds__(NW * 64, waves_per_simd<SETS>()) void pmpd_layer_kernel(LayerDesc L,
                                                                                    const _Float16* __restrict__ x, int m,
                                                                                    float* __restrict__ y) {
  extern __shared__ uint4 lds[];
  run_tiles<B, SETS, NW, SPLITK>(L, static_cast<int>(blockIdx.x) * (NW / SPLITK), x, m, y, lds,
                                 KRange{0, L.n_groups, chunk_groups(L.n_groups, m)});
}

// =====================================================================================
// Dependency-ordered step in one cooperative launch.  The layers of a step are grouped into
// stages; a layer of stage s may take its input from the output of a layer of an earlier stage
// (x = fp16(gain * y)).  An item is one 64-row tile and one K-part of at least 8 groups (8: two
// groups per wave, all of an item's weights in registers before its x is there); the parts of a
// layer are as small as that allows while its stage still has no more items than the chip holds
// workgroups, so that every stage, however few rows it has, spreads over the whole chip in one
// round.  The items of the step form one list in stage order; the grid is persistent and
// workgroup w takes items w, w + gridDim, ... of it: the deal goes on across stage ends, so the
// workgroups a short stage leaves out are already waiting, weights loaded, for the stage after.
// There is no barrier between stages.  Every output row is a 64-bit word that counts the K-parts
// added to it (see part_word): an item waits for exactly the words it reads, the 128 * groups
// outputs of the source layer that make up its K-part, and for nothing else, and a producer's
// single atomic add both delivers its part and announces it.  The wait cannot deadlock: all
// workgroups are resident (cooperative launch), each takes its items in list order, and the
// first unfinished item of the list depends only on finished ones.  It is bounded all the same
// (spin_limit rounds), and a wait that runs out only sets `timed_out`.
// The words of the first two groups of every wave's quarter of an item's K-part are requested as
// soon as the wave's part in the item before is over, so that the weights of the next stage stream
// while the results of this one travel.  A wave's loads return in the order they were issued, so it
// sees x only once its own weights are there; the product needs those anyway.
// The sums are read with agent-scope loads (coherent across the chip's L2 slices); y is written
// by whoever completes it: the producer itself where a layer has one K-part, a sweep over the
// sums after the last stage otherwise.
struct OrderedSync {
  uint32_t timed_out;
};

struct ChainDesc {
  int64_t src_y_off;     // elements from the start of the sums of the producing layer's output; -1: input from x_base
  float gain;
  int32_t n_parts;       // K-parts of part_groups groups each (the last one may be shorter)
  int32_t part_groups;
  int32_t src_parts;     // K-parts of the producing layer: its sums are complete when they count that many
};

constexpr int kOrderedWaves = 4;           // one quarter of the K-part each
constexpr int kOrderedThreads = kOrderedWaves * 64;
constexpr int kOrderedWgPerCu = 4;         // 16 waves per compute unit, 128 registers each
constexpr int kOrderedPartGroups = 8;      // smallest K-part: two groups per wave, all in registers before x is there
constexpr int kOrderedMaxPartGroups = 32;  // largest K-part the LDS image is sized for
constexpr int kItemPartShift = 20;  // WorkItem::tile0 = tile | part << 20

template <int B>
__global__ __launch_bounds__(kOrderedThreads, kOrderedWgPerCu) void pmpd_ordered_kernel(
    const LayerDesc* __restrict__ layers, const ChainDesc* __restrict__ chains, const WorkItem* __restrict__ items,
    int n_items, const _Float16* __restrict__ x_base, float* __restrict__ y_base, unsigned long long* __restrict__ sums,
    OrderedSync* sync, uint32_t spin_limit, int n_layers) {
  extern __shared__ uint4 lds[];
  const uint32_t n_wg = gridDim.x;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const ImageLayout im(lds, kOrderedMaxPartGroups, 1);
  const OperandOffsets<1> off(im, lane, 1);
  const int wscale = weight_scale_register();

  // The tables an item needs (the item, then its layer and chain records) are two dependent reads.
  // They are taken ahead of time, so that neither sits between the end of one item and the first
  // weight loads of the next: while an item runs, the records of the next and the item after that
  // are requested, each from values that arrived an item earlier.  A request is one load per lane
  // (lane k holds word k of the record), so a whole record waits in one vector register and is
  // moved to scalar registers lane by lane when it is needed.
  static_assert(sizeof(LayerDesc) == 18 * 4 && sizeof(ChainDesc) == 6 * 4, "records are read one 32-bit word per lane");
  auto request_records = [&](int layer) {  // lanes 0..17: LayerDesc, lanes 32..37: ChainDesc
    const uint32_t* pl = reinterpret_cast<const uint32_t*>(layers + (layer < 0 ? 0 : layer));
    const uint32_t* pc = reinterpret_cast<const uint32_t*>(chains + (layer < 0 ? 0 : layer));
    return lane < 32 ? pl[lane < 18 ? lane : 0] : pc[lane < 38 ? lane - 32 : 0];
  };
  auto request_item = [&](int i) {  // lanes 0, 1
    return reinterpret_cast<const uint32_t*>(items + (i < n_items ? i : 0))[lane & 1];
  };
  auto word = [](uint32_t v, int k) { return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), k)); };
  auto take_records = [&](uint32_t records, LayerDesc& L, ChainDesc& c) {
    uint32_t w[18], v[6];
#pragma unroll
    for (int k = 0; k < 18; ++k) w[k] = word(records, k);
#pragma unroll
    for (int k = 0; k < 6; ++k) v[k] = word(records, 32 + k);
    __builtin_memcpy(&L, w, sizeof(L));
    __builtin_memcpy(&c, v, sizeof(c));
  };
  // The K-part of an item, and the quarter of it this wave multiplies.
  struct Range {
    int g0, g1;
  };
  auto part_of = [](const WorkItem& wi, const LayerDesc& Li, const ChainDesc& ci) {
    const int p0 = (wi.tile0 >> kItemPartShift) * ci.part_groups;
    return Range{p0, p0 + ci.part_groups < Li.n_groups ? p0 + ci.part_groups : Li.n_groups};
  };
  auto quarter_of = [&](const Range& p) {
    const int cn = p.g1 - p.g0;
    return Range{p.g0 + cn * wave / kOrderedWaves, p.g0 + cn * (wave + 1) / kOrderedWaves};
  };
  // The words of the first two groups of this wave's quarter, on their way from the moment the
  // wave's part in the item before is over.
  u32x4 pa[B], pb[B], sa_a = {0, 0, 0, 0}, sa_b = {0, 0, 0, 0};
  auto request_weights = [&](const WorkItem& wi, const LayerDesc& Li, const ChainDesc& ci) {
    if (wi.layer < 0) return;
    const Range q = quarter_of(part_of(wi, Li, ci));
    if (q.g0 >= q.g1) return;
    const TileWords<B> tw(Li, wi.tile0 & ((1 << kItemPartShift) - 1), lane);
    tw.load(pa, sa_a, q.g0);
    if (q.g0 + 1 < q.g1) tw.load(pb, sa_b, q.g0 + 1);
  };
  // One item.  Barriers: every wave has consumed the image of the item before, and the sums this
  // item reads have been seen complete once; the image of x is complete; the four partial sums are
  // in LDS.  Wave 0 adds them and delivers the rows.
  auto run_item = [&](const WorkItem& wi, const LayerDesc& Li, const ChainDesc& ci) {
    const int tile = wi.tile0 & ((1 << kItemPartShift) - 1);
    const Range part = part_of(wi, Li, ci);
    XSource src = x_from_fp16(x_base + Li.x_off);
    if (ci.src_y_off >= 0) {
      src = XSource{nullptr, sums + ci.src_y_off, ci.gain, ci.src_parts, spin_limit, &sync->timed_out};
      // One thread per 64 source rows polls the first of them: few readers while the producers are
      // still at work.  The other rows follow within a fraction of a microsecond, and every word is
      // checked again where it is read.
      const int n_rows = (part.g1 - part.g0) * kGroup;
      for (int r = threadIdx.x * 64; r < n_rows; r += kOrderedThreads * 64) {
        const unsigned long long* w = src.y64 + part.g0 * kGroup + r;
        uint32_t polls = 0;
        while (!sum_complete(__hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), ci.src_parts)) {
          if (++polls >= spin_limit) {
            __hip_atomic_store(&sync->timed_out, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
          }
          __builtin_amdgcn_s_sleep(16);
        }
      }
    }
    __syncthreads();
    stage_x<kOrderedThreads>(src, part.g0, part.g1 - part.g0, im, 0, threadIdx.x);
    __syncthreads();
    float yacc[1][4] = {{0.f, 0.f, 0.f, 0.f}};
    const Range q = quarter_of(part);
    if (q.g0 < q.g1) {
      const TileWords<B> tw(Li, tile, lane);
      for (int gc = q.g0; gc < q.g1; gc += 2) {
        if (gc > q.g0 && gc + 1 < q.g1) tw.load(pb, sa_b, gc + 1);
        consume_group<B, 1>(im, off, gc - part.g0, pa, sa_a, wscale, yacc);
        if (gc + 2 < q.g1) tw.load(pa, sa_a, gc + 2);
        if (gc + 1 < q.g1) consume_group<B, 1>(im, off, gc + 1 - part.g0, pb, sa_b, wscale, yacc);
      }
    }
    // the two classes sit 16 lanes apart: add them (fixed order: A + B)
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float other = __shfl_xor(yacc[0][t], 16);
      yacc[0][t] = (lane & 16) ? other + yacc[0][t] : yacc[0][t] + other;
      if (wave != 0) im.red[(t * kOrderedWaves + wave) * 64 + lane] = yacc[0][t];
    }
    __syncthreads();
    if (wave == 0 && lane < 16) {
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float sum = yacc[0][t];
#pragma unroll
        for (int k = 1; k < kOrderedWaves; ++k) sum += im.red[(t * kOrderedWaves + k) * 64 + lane];
        const int row = tile * 64 + 16 * t + lane;
        if (row < Li.out_f) {
          if (ci.n_parts > 1) {
            __hip_atomic_fetch_add(&sums[Li.y_off + row], part_word(sum), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          } else {  // the row is this workgroup's alone
            y_base[Li.y_off + row] = sum;
            __hip_atomic_store(&sums[Li.y_off + row], whole_word(sum), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        }
      }
    }
    // The rows are what the next stage waits for: they enter the compute unit's memory pipeline
    // before the next item's weight requests (ten 1 KiB loads per wave) queue up in it.
    __syncthreads();
  };

  const int first = static_cast<int>(blockIdx.x), step = static_cast<int>(n_wg);
  WorkItem it = first < n_items ? items[first] : WorkItem{-1, 0};
  WorkItem it_next = first + step < n_items ? items[first + step] : WorkItem{-1, 0};
  LayerDesc L;
  ChainDesc c;
  take_records(request_records(it.layer), L, c);
  request_weights(it, L, c);
  for (int i = first; i < n_items; i += step) {
    const uint32_t records = request_records(it_next.layer);
    const uint32_t after = request_item(i + 2 * step);
    if (it.layer >= 0) run_item(it, L, c);
    it = it_next;
    it_next = i + 2 * step < n_items ? WorkItem{static_cast<int32_t>(word(after, 0)), static_cast<int32_t>(word(after, 1))} : WorkItem{-1, 0};
    take_records(records, L, c);
    request_weights(it, L, c);
  }
  // y of the layers with several K-parts, from their sums as they become complete.
  for (int li = 0; li < n_layers; ++li) {
    const int n_parts = chains[li].n_parts;
    if (n_parts <= 1) continue;
    const LayerDesc& Ld = layers[li];
    for (int row = blockIdx.x * blockDim.x + threadIdx.x; row < Ld.out_f; row += gridDim.x * blockDim.x) {
      unsigned long long w = __hip_atomic_load(sums + Ld.y_off + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      for (uint32_t polls = 0; !sum_complete(w, n_parts);) {
        if (++polls >= spin_limit) {
          __hip_atomic_store(&sync->timed_out, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
        __builtin_amdgcn_s_sleep(16);
        w = __hip_atomic_load(sums + Ld.y_off + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      y_base[Ld.y_off + row] = sum_value(w, n_parts);
    }
  }
}

__global__ void pmpd_ordered_reset_kernel(unsigned long long* sums, int64_t n_sums) {
  const int64_t tid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x, n_threads = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t i = tid; i < n_sums; i += n_threads) sums[i] = 0;
}

// Read-only stream over a buffer: the HBM ceiling the decode kernels are held against.  Each
// workgroup reads one contiguous share with four 16-byte nontemporal loads per thread in flight.
__global__ __launch_bounds__(256) void pmpd_read_stream_kernel(const u32x4* __restrict__ p, size_t vec_per_block,
                                                              uint32_t* __restrict__ sink) {
  const u32x4* base = p + static_cast<size_t>(blockIdx.x) * vec_per_block;
  u32x4 acc = {0, 0, 0, 0};
  for (size_t i = threadIdx.x; i < vec_per_block; i += 1024) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(&base[i + u * 256]);
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u];
  }
  const uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
  if (r == 0x9e3779b9u) sink[0] = r;  // keeps the loads alive; the store almost never happens
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

// Launch shapes.  A stack has thousands of row tiles; a single layer (or a short stack) has few
// and splits K over the waves of a workgroup to put more waves on the machine: 2 or 4 ways with
// four waves, 8 or 16 ways with one tile per workgroup of 8 or 16 waves.
static int pick_splitk(int64_t n_tiles, int groups_per_pass, int max_split) {
  // Split K until about 2048 waves exist or a wave would get fewer than 2 groups.
  int splitk = 1;
  while (splitk < max_split && n_tiles * splitk < 2048 && groups_per_pass / (splitk * 2) >= 2) splitk *= 2;
  return splitk;
}

template <int B, int SETS, int NW, int SPLITK>
static hipError_t launch_layer(const LayerDesc& d, const void* x, int m, float* y, hipStream_t s) {
  const int tpw = NW / SPLITK;
  const unsigned grid = static_cast<unsigned>((d.n_tiles + tpw - 1) / tpw);
  const size_t lds = lds_bytes(chunk_groups(d.n_groups, m), m, NW, SETS * 4);
  hipLaunchKernelGGL((pmpd_layer_kernel<B, SETS, NW, SPLITK>), dim3(grid), dim3(NW * 64), lds, s, d,
                     static_cast<const _Float16*>(x), m, y);
  return hipGetLastError();
}

template <int B, int SETS>
static hipError_t launch_layer_s(const LayerDesc& d, const void* x, int m, float* y, hipStream_t s) {
  switch (pick_splitk(d.n_tiles, chunk_groups(d.n_groups, m), SETS == 1 ? 16 : 4)) {
    case 1: return launch_layer<B, SETS, 4, 1>(d, x, m, y, s);
    case 2: return launch_layer<B, SETS, 4, 2>(d, x, m, y, s);
    case 4: return launch_layer<B, SETS, 4, 4>(d, x, m, y, s);
    case 8:
      if constexpr (SETS == 1) return launch_layer<B, 1, 8, 8>(d, x, m, y, s);
    default:
      if constexpr (SETS == 1) return launch_layer<B, 1, 16, 16>(d, x, m, y, s);
      return launch_layer<B, SETS, 4, 4>(d, x, m, y, s);
  }
}

template <int B>
static hipError_t launch_layer_b(const LayerDesc& d, const void* x, int m, float* y, hipStream_t s) {
  switch ((m + 1) / 2) {
    case 1: return launch_layer_s<B, 1>(d, x, m, y, s);
    case 2: return launch_layer_s<B, 2>(d, x, m, y, s);
    case 3: return launch_layer_s<B, 3>(d, x, m, y, s);
    default: return launch_layer_s<B, 4>(d, x, m, y, s);
  }
}

// defined in pmpd_prefill.hip
hipError_t launch_prefill_layer(const LayerDesc& d, int b, const void* X, int m, float* Y, hipStream_t s);
hipError_t launch_prefill_stack(const pmpd_stack* st, int b, const void* X, int m, float* Y, hipStream_t s);
// defined in pmpd_skinny.hip
hipError_t launch_skinny_stack(const pmpd_stack* st, int b, const void* X, int m, float* Y, hipStream_t s);
constexpr int kSkinnyMinBatch = 3, kSkinnyMaxBatch = PMPD_MAX_STACK_BATCH;  // batches the int8 kernel takes over a stack
// defined in pmpd_block16.hip
hipError_t launch_block16_stack(const pmpd_stack* st, int b, const void* X, int m, float* Y, hipStream_t s);
hipError_t launch_block16_layer(const LayerDesc& d, int b, const void* X, int m, float* Y, hipStream_t s);
// Which of the two takes a batch over a stack (measured on the 7B-shaped and the mobile-scale stack): the fp16 kernel
// costs the same whatever the batch, the int8 kernel grows with every four vectors; they meet at 5 to 8 vectors,
// where the fp16 kernel wins at b = 4 (the int8 kernel waits for memory there) and loses at b = 3 and 2.
static bool block16_takes(int m, int b) { return m >= 9 || (m >= 5 && b == 4); }

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
  if (m > PMPD_MAX_BATCH && m <= kSkinnyMaxBatch) {  // one 16-token block: codes as fp16 subnormals, weights read once
    e = launch_block16_layer(d, b, x, m, y, s);
  } else if (m > PMPD_MAX_BATCH) {  // compute-bound shape: fp16 MFMA tile kernel
    // the kernel addresses X with 32-bit byte offsets from the layer's first activation
    if (static_cast<uint64_t>(m) * static_cast<uint64_t>(d.in_f) * 2u >= (uint64_t{1} << 32))
      return fail(PMPD_EINVAL, "%s: m x in_features = %d x %d: X of one layer must stay below 4 GiB", who, m, d.in_f);
    e = launch_prefill_layer(d, b, x, m, y, s);
  } else {  // memory-bound shapes: unpack once for all vectors
    e = b == 4 ? launch_layer_b<4>(d, x, m, y, s)
        : b == 3 ? launch_layer_b<3>(d, x, m, y, s)
                 : launch_layer_b<2>(d, x, m, y, s);
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

// Launch shapes of the one-launch decode step (pmpd_stack_variant reports the one chosen for a
// bit-width, pmpd_stack_set_variant overrides it):
//   0  4 waves x 1 tile each, whole K       1  4 waves on 1 tile, K split 4 ways
//   2  4 waves on 2 tiles, K split 2 ways   3  8 waves on 1 tile, K split 8 ways
//   4  16 waves on 1 tile, K split 16 ways
static constexpr int kNumVariants = 5;
// which work list (tiles per workgroup: list 0 = 4, 1 = 1, 2 = 2) each variant walks
static constexpr int kVariantList[kNumVariants] = {0, 1, 2, 1, 1};
static void pick_variants(pmpd_stack* st) {
  // Measured on the 7B-, 13B-shaped and mobile-scale stacks and on 64 copies of one 4096 x 4096
  // layer: shapes 0 and 2 are within 2 to 5 % of each other.  Whole-K waves (shape 0) split x once for
  // four tiles; shape 2 puts twice as many workgroups on the machine.  Stacks with at least 4096
  // four-tile workgroups: 0 at b = 4 and 3, 2 at b = 2.  Smaller stacks: 2 at b = 4, 0 at b = 3 and 2
  // (at b = 3 shape 2 loses 2 % on the mobile-scale stack and 5 % on the 64 copies).  Short
  // stacks (the layers of one dependency stage, say) split K further, like single layers.
  const bool big = st->items[0].size() >= 4096;
  st->variant[4] = big ? 0 : 2;
  st->variant[3] = 0;
  st->variant[2] = big ? 2 : 0;
  const int64_t n_tiles = static_cast<int64_t>(st->items[1].size());
  int min_groups = st->max_in / kGroup;
  for (const LayerDesc& d : st->layers) min_groups = std::min(min_groups, d.n_groups);
  const int split = pick_splitk(n_tiles, std::min(min_groups, chunk_groups(st->max_in / kGroup, 1)), 16);
  if (split >= 4) {
    const int v = split == 4 ? 1 : split == 8 ? 3 : 4;
    st->variant[4] = st->variant[3] = st->variant[2] = v;
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
  const int nw = v == 3 ? 8 : v == 4 ? 16 : 4;
  const size_t lds = lds_bytes(chunk_groups(st->max_in / kGroup, 1), 1, nw, 4);
  switch (v) {
    case 0:
      hipLaunchKernelGGL((pmpd_stack_kernel<B, 1, 4, 1>), dim3(grid), dim3(256), lds, s, st->d_layers, st->d_items[q], x, 1, y);
      break;
    case 2:
      hipLaunchKernelGGL((pmpd_stack_kernel<B, 1, 4, 2>), dim3(grid), dim3(256), lds, s, st->d_layers, st->d_items[q], x, 1, y);
      break;
    case 3:
      hipLaunchKernelGGL((pmpd_stack_kernel<B, 1, 8, 8>), dim3(grid), dim3(512), lds, s, st->d_layers, st->d_items[q], x, 1, y);
      break;
    case 4:
      hipLaunchKernelGGL((pmpd_stack_kernel<B, 1, 16, 16>), dim3(grid), dim3(1024), lds, s, st->d_layers, st->d_items[q], x, 1, y);
      break;
    default:
      hipLaunchKernelGGL((pmpd_stack_kernel<B, 1, 4, 4>), dim3(grid), dim3(256), lds, s, st->d_layers, st->d_items[q], x, 1, y);
      break;
  }
  return hipGetLastError();
}

// Skinny batches over a stack: 4 waves, one tile each over the whole K (work list 0).
template <int B, int SETS>
static hipError_t launch_stack_batch_s(const pmpd_stack* st, const _Float16* x, int m, float* y, hipStream_t s) {
  const unsigned grid = static_cast<unsigned>(st->items[0].size());
  const size_t lds = lds_bytes(chunk_groups(st->max_in / kGroup, m), m, 4, 0);
  hipLaunchKernelGGL((pmpd_stack_kernel<B, SETS, 4, 1>), dim3(grid), dim3(256), lds, s, st->d_layers, st->d_items[0], x, m, y);
  return hipGetLastError();
}

template <int B>
static hipError_t launch_stack_batch(const pmpd_stack* st, const void* xv, int m, float* y, hipStream_t s) {
  const _Float16* x = static_cast<const _Float16*>(xv);
  switch ((m + 1) / 2) {
    case 1: return launch_stack_batch_s<B, 1>(st, x, m, y, s);
    case 2: return launch_stack_batch_s<B, 2>(st, x, m, y, s);
    case 3: return launch_stack_batch_s<B, 3>(st, x, m, y, s);
    default: return launch_stack_batch_s<B, 4>(st, x, m, y, s);
  }
}

// ---------------------------------------------------------------- ordered step ----
struct pmpd_ordered {
  const pmpd_stack* stack = nullptr;
  std::vector<ChainDesc> chains;
  std::vector<WorkItem> items;
  const ChainDesc* d_chains = nullptr;
  const WorkItem* d_items = nullptr;
  OrderedSync* d_sync = nullptr;
  unsigned long long* d_sums = nullptr;  // fixed-point row sums, laid out like y
  int64_t n_sums = 0;
  int grid = 0;  // workgroups of the launch: what the chip holds at once, or one per item if that is fewer
  uint32_t spin_limit = 1u << 20;
};

static int32_t check_chain(const pmpd_stack* st, const pmpd_chain_t* chain, int* n_stages_out) {
  if (!st || !chain) return fail(PMPD_EINVAL, "pmpd_ordered: NULL argument");
  const int n = static_cast<int>(st->layers.size());
  int n_stages = 0;
  for (int i = 0; i < n; ++i) {
    if (chain[i].stage < 0 || chain[i].stage >= 65536) return fail(PMPD_EINVAL, "pmpd_ordered: stage %d of layer %d outside 0..65535", chain[i].stage, i);
    n_stages = std::max(n_stages, chain[i].stage + 1);
    const int src = chain[i].source;
    if (src == -1) continue;
    if (src < 0 || src >= n) return fail(PMPD_EINVAL, "pmpd_ordered: source %d of layer %d is not a layer", src, i);
    if (chain[src].stage >= chain[i].stage) return fail(PMPD_EINVAL, "pmpd_ordered: layer %d (stage %d) reads layer %d of stage %d, which is not earlier", i, chain[i].stage, src, chain[src].stage);
    if (st->layers[src].out_f != st->layers[i].in_f) return fail(PMPD_EINVAL, "pmpd_ordered: layer %d has %d inputs but its source %d has %d outputs", i, st->layers[i].in_f, src, st->layers[src].out_f);
    if (st->layers[src].y_off % 4) return fail(PMPD_EALIGN, "pmpd_ordered: y_offset of source layer %d must be a multiple of 4", src);
    if (!(chain[i].gain == chain[i].gain) || chain[i].gain - chain[i].gain != 0.f) return fail(PMPD_EINVAL, "pmpd_ordered: gain of layer %d is not finite", i);
  }
  *n_stages_out = n_stages;
  return PMPD_OK;
}

// K-part size (in groups) of every layer: as close to kOrderedPartGroups as keeps the items of the
// layer's stage within `slots` workgroups (a stage that takes two items of some workgroups takes
// twice as long to deliver), and a row within kMaxParts parts; never above kOrderedMaxPartGroups.
static std::vector<int> ordered_part_groups(const pmpd_stack* st, const pmpd_chain_t* chain, int n_stages, int slots) {
  std::vector<int64_t> stage_tiles(static_cast<size_t>(n_stages), 0);
  for (size_t i = 0; i < st->layers.size(); ++i) stage_tiles[static_cast<size_t>(chain[i].stage)] += st->layers[i].n_tiles;
  std::vector<int> pg(st->layers.size());
  for (size_t i = 0; i < st->layers.size(); ++i) {
    const int G = st->layers[i].n_groups;
    const int64_t tiles = std::max<int64_t>(1, stage_tiles[static_cast<size_t>(chain[i].stage)]);
    int parts = static_cast<int>(std::max<int64_t>(1, std::min<int64_t>((G + kOrderedPartGroups - 1) / kOrderedPartGroups, slots / tiles)));
    parts = std::min(parts, kMaxParts);  // what the count bits of a sum can hold
    pg[i] = std::min((G + parts - 1) / parts, kOrderedMaxPartGroups);
  }
  return pg;
}

// Workgroup slots the parts are planned for: kOrderedWgPerCu workgroups per compute unit.
static int ordered_slots() {
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess || prop.multiProcessorCount < 1)
    return kOrderedWgPerCu * 256;
  return kOrderedWgPerCu * prop.multiProcessorCount;
}

static int parts_of(int n_groups, int part_groups) { return (n_groups + part_groups - 1) / part_groups; }

// Items of an ordered step (per stage and in all) and the length of its y (= of the sums).
struct OrderedCounts {
  std::vector<size_t> stage_items;
  size_t n_items = 0, max_stage_items = 0, n_sums = 0;
};
static OrderedCounts ordered_counts(const pmpd_stack* st, const pmpd_chain_t* chain, int n_stages, const std::vector<int>& pg) {
  OrderedCounts c;
  c.stage_items.assign(static_cast<size_t>(n_stages), 0);
  for (size_t i = 0; i < st->layers.size(); ++i) {
    const LayerDesc& d = st->layers[i];
    const size_t n = static_cast<size_t>(d.n_tiles) * static_cast<size_t>(parts_of(d.n_groups, pg[i]));
    c.stage_items[static_cast<size_t>(chain[i].stage)] += n;
    c.n_items += n;
    c.n_sums = std::max(c.n_sums, static_cast<size_t>(d.y_off) + static_cast<size_t>(d.out_f));
  }
  for (size_t n : c.stage_items) c.max_stage_items = std::max(c.max_stage_items, n);
  return c;
}

// Workgroups of the kernel for bit-width B that the device holds at once.
template <int B>
static hipError_t ordered_capacity(int* slots) {
  int per_cu = 0, dev = 0;
  hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, pmpd_ordered_kernel<B>, kOrderedThreads,
                                                              lds_bytes(kOrderedMaxPartGroups, 1, kOrderedWaves, 4));
  hipDeviceProp_t prop;
  if (e != hipSuccess || (e = hipGetDevice(&dev)) != hipSuccess || (e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
  *slots = std::min(per_cu, kOrderedWgPerCu) * prop.multiProcessorCount;
  return hipSuccess;
}

// The item list gives every stage a whole number of rounds of the grid (empty items fill up), so
// that workgroup w meets item w of every stage.  `grid_bound`: the largest grid the list may be built for.
static size_t ordered_bytes(const pmpd_stack* st, const OrderedCounts& c, size_t grid_bound) {
  const size_t list_bound = c.n_items + c.stage_items.size() * std::min(grid_bound, std::max<size_t>(1, c.max_stage_items));
  return align_up(st->layers.size() * sizeof(ChainDesc), 256) + align_up(list_bound * sizeof(WorkItem), 256) +
         align_up(sizeof(OrderedSync), 256) + align_up(c.n_sums * sizeof(unsigned long long), 256);
}

template <int B>
static hipError_t launch_ordered(const pmpd_ordered* o, const void* x, float* y, hipStream_t s) {
  const pmpd_stack* st = o->stack;
  const size_t lds = lds_bytes(kOrderedMaxPartGroups, 1, kOrderedWaves, 4);
  hipLaunchKernelGGL(pmpd_ordered_reset_kernel, dim3(1024), dim3(256), 0, s, o->d_sums, o->n_sums);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const LayerDesc* layers = st->d_layers;
  const _Float16* xb = static_cast<const _Float16*>(x);
  int n_items = static_cast<int>(o->items.size());
  uint32_t spin = o->spin_limit;
  int n_layers = static_cast<int>(st->layers.size());
  void* args[] = {&layers, const_cast<ChainDesc**>(&o->d_chains), const_cast<WorkItem**>(&o->d_items), &n_items, &xb, &y,
                  const_cast<unsigned long long**>(&o->d_sums), const_cast<OrderedSync**>(&o->d_sync), &spin, &n_layers};
  // a cooperative launch is refused, not queued, when the grid does not fit the device at once
  return hipLaunchCooperativeKernel(reinterpret_cast<const void*>(&pmpd_ordered_kernel<B>), dim3(o->grid), dim3(kOrderedThreads),
                                    args, static_cast<unsigned>(lds), s);
}

extern "C" {

int32_t pmpd_ordered_workspace_size(const pmpd_stack_t* stack, const pmpd_chain_t* chain, size_t* bytes) {
  int n_stages = 0;
  int32_t rc = check_chain(stack, chain, &n_stages);
  if (rc) return rc;
  if (!bytes) return fail(PMPD_EINVAL, "pmpd_ordered_workspace_size: bytes is NULL");
  const std::vector<int> pg = ordered_part_groups(stack, chain, n_stages, ordered_slots());
  *bytes = ordered_bytes(stack, ordered_counts(stack, chain, n_stages, pg), static_cast<size_t>(ordered_slots()));
  return PMPD_OK;
}

int32_t pmpd_ordered_create(const pmpd_stack_t* stack, const pmpd_chain_t* chain, void* workspace, size_t workspace_bytes,
                            pmpd_ordered_t** out) {
  int n_stages = 0;
  int32_t rc = check_chain(stack, chain, &n_stages);
  if (rc) return rc;
  if (!workspace || !out) return fail(PMPD_EINVAL, "pmpd_ordered_create: NULL argument");
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(PMPD_EALIGN, "pmpd_ordered_create: workspace not 256-byte aligned");
  const size_t n_layers = stack->layers.size();
  const std::vector<int> pg = ordered_part_groups(stack, chain, n_stages, ordered_slots());
  const OrderedCounts counts = ordered_counts(stack, chain, n_stages, pg);
  const size_t need = ordered_bytes(stack, counts, static_cast<size_t>(ordered_slots()));
  if (workspace_bytes < need) return fail(PMPD_ESIZE, "pmpd_ordered_create: workspace %zu bytes, need %zu", workspace_bytes, need);
  // the kernel indexes the list with int, two rounds of the grid beyond the current item
  if (counts.n_items + static_cast<size_t>(n_stages) * static_cast<size_t>(ordered_slots()) > (size_t{1} << 30))
    return fail(PMPD_EINVAL, "pmpd_ordered_create: too many work items");
  int slots[3] = {0, 0, 0};
  hipError_t e = ordered_capacity<2>(&slots[0]);
  if (e == hipSuccess) e = ordered_capacity<3>(&slots[1]);
  if (e == hipSuccess) e = ordered_capacity<4>(&slots[2]);
  if (e != hipSuccess) return hip_fail(e, "pmpd_ordered_create occupancy");
  const int capacity = std::min(std::min(slots[0], std::min(slots[1], slots[2])), ordered_slots());
  if (capacity < 1) return fail(PMPD_EINVAL, "pmpd_ordered_create: the device holds no workgroup of the kernel");
  auto* o = new pmpd_ordered;
  o->stack = stack;
  o->n_sums = static_cast<int64_t>(counts.n_sums);
  o->grid = static_cast<int>(std::min<size_t>(static_cast<size_t>(capacity), std::max<size_t>(1, counts.max_stage_items)));
  for (size_t i = 0; i < n_layers; ++i) {
    const LayerDesc& d = stack->layers[i];
    const int src = chain[i].source;
    const int parts = parts_of(d.n_groups, pg[i]);
    if (d.n_tiles >= (1 << kItemPartShift) || parts >= (1 << (31 - kItemPartShift))) {
      delete o;
      return fail(PMPD_EINVAL, "pmpd_ordered_create: layer %zu is too large for the item encoding", i);
    }
    if (parts > kMaxParts) {  // the count bits of a sum word hold at most kMaxParts
      delete o;
      return fail(PMPD_EINVAL, "pmpd_ordered_create: layer %zu has %d input features; rows longer than %d cannot be split into at most %d parts",
                  i, d.in_f, kMaxParts * kOrderedMaxPartGroups * kGroup, kMaxParts);
    }
    const int src_parts = src >= 0 ? parts_of(stack->layers[src].n_groups, pg[src]) : 0;
    o->chains.push_back(ChainDesc{src < 0 ? int64_t{-1} : stack->layers[src].y_off, chain[i].gain, parts, pg[i], src_parts});
  }
  // (tile, K-part) items, stage by stage; inside a stage long rows first
  std::vector<int> order(n_layers);
  for (size_t i = 0; i < n_layers; ++i) order[i] = static_cast<int>(i);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
    if (chain[a].stage != chain[b].stage) return chain[a].stage < chain[b].stage;
    return stack->layers[a].in_f > stack->layers[b].in_f;
  });
  int stage = -1;
  for (int li : order) {
    if (chain[li].stage != stage)  // a new stage starts a new round
      while (o->items.size() % static_cast<size_t>(o->grid)) o->items.push_back(WorkItem{-1, 0});
    stage = chain[li].stage;
    const int parts = o->chains[li].n_parts;
    for (int t = 0; t < stack->layers[li].n_tiles; ++t)
      for (int q = 0; q < parts; ++q) o->items.push_back(WorkItem{li, t | (q << kItemPartShift)});
  }
  char* w = static_cast<char*>(workspace);
  e = hipMemcpy(w, o->chains.data(), n_layers * sizeof(ChainDesc), hipMemcpyHostToDevice);  // the list fits: see ordered_bytes
  o->d_chains = reinterpret_cast<const ChainDesc*>(w);
  w += align_up(n_layers * sizeof(ChainDesc), 256);
  if (e == hipSuccess) e = hipMemcpy(w, o->items.data(), o->items.size() * sizeof(WorkItem), hipMemcpyHostToDevice);
  o->d_items = reinterpret_cast<const WorkItem*>(w);
  w += align_up(o->items.size() * sizeof(WorkItem), 256);
  o->d_sync = reinterpret_cast<OrderedSync*>(w);
  const size_t sync_bytes = sizeof(OrderedSync);
  if (e == hipSuccess) e = hipMemset(w, 0, sync_bytes);
  w += align_up(sync_bytes, 256);
  o->d_sums = reinterpret_cast<unsigned long long*>(w);
  if (e != hipSuccess) {
    delete o;
    return hip_fail(e, "pmpd_ordered_create copy");
  }
  *out = o;
  return PMPD_OK;
}

void pmpd_ordered_destroy(pmpd_ordered_t* ordered) { delete ordered; }

int32_t pmpd_ordered_set_spin_limit(pmpd_ordered_t* ordered, uint32_t polls) {
  if (!ordered || polls == 0) return fail(PMPD_EINVAL, "pmpd_ordered_set_spin_limit: bad argument");
  ordered->spin_limit = polls;
  return PMPD_OK;
}

int32_t pmpd_ordered_step(const pmpd_ordered_t* ordered, int32_t b, const void* x_base, float* y_base, void* stream) {
  int32_t rc = check_bits(b, "pmpd_ordered_step");
  if (rc) return rc;
  if (!ordered || !x_base || !y_base) return fail(PMPD_EINVAL, "pmpd_ordered_step: NULL argument");
  if (reinterpret_cast<uintptr_t>(x_base) % 16) return fail(PMPD_EALIGN, "pmpd_ordered_step: x_base not 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(y_base) % 16) return fail(PMPD_EALIGN, "pmpd_ordered_step: y_base not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = b == 4 ? launch_ordered<4>(ordered, x_base, y_base, s)
                 : b == 3 ? launch_ordered<3>(ordered, x_base, y_base, s)
                          : launch_ordered<2>(ordered, x_base, y_base, s);
  if (e != hipSuccess) return hip_fail(e, "pmpd_ordered_step launch");
  return PMPD_OK;
}

int32_t pmpd_ordered_status(const pmpd_ordered_t* ordered, int32_t* timed_out) {
  if (!ordered || !timed_out) return fail(PMPD_EINVAL, "pmpd_ordered_status: NULL argument");
  uint32_t flag = 0;
  hipError_t e = hipMemcpy(&flag, &ordered->d_sync->timed_out, sizeof(flag), hipMemcpyDeviceToHost);
  if (e == hipSuccess && flag) e = hipMemset(&ordered->d_sync->timed_out, 0, sizeof(flag));
  if (e != hipSuccess) return hip_fail(e, "pmpd_ordered_status");
  *timed_out = static_cast<int32_t>(flag);
  return PMPD_OK;
}

}  // extern "C"

extern "C" {

int32_t pmpd_read_stream(const void* src, size_t bytes, uint32_t* sink, size_t* bytes_read, void* stream) {
  if (!src || !sink || !bytes_read) return fail(PMPD_EINVAL, "pmpd_read_stream: NULL argument");
  if (reinterpret_cast<uintptr_t>(src) % 16) return fail(PMPD_EALIGN, "pmpd_read_stream: src not 16-byte aligned");
  constexpr size_t kBlocks = 8192, kStep = 1024;  // 16-byte vectors read per workgroup iteration
  const size_t per_block = bytes / 16 / kBlocks / kStep * kStep;
  if (per_block == 0) return fail(PMPD_EINVAL, "pmpd_read_stream: buffer smaller than %zu bytes", kBlocks * kStep * 16);
  hipLaunchKernelGGL(pmpd_read_stream_kernel, dim3(kBlocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(src), per_block, sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hip_fail(e, "pmpd_read_stream launch");
  *bytes_read = per_block * kBlocks * 16;
  return PMPD_OK;
}

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
    w += align_up(counts[q] * sizeof(WorkItem), 256);
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

int32_t pmpd_stack_variant(const pmpd_stack_t* stack, int32_t b, int32_t* variant) {
  int32_t rc = check_bits(b, "pmpd_stack_variant");
  if (rc) return rc;
  if (!stack || !variant) return fail(PMPD_EINVAL, "pmpd_stack_variant: NULL argument");
  *variant = stack->variant[b];
  return PMPD_OK;
}

int32_t pmpd_stack_set_variant(pmpd_stack_t* stack, int32_t b, int32_t variant) {
  int32_t rc = check_bits(b, "pmpd_stack_set_variant");
  if (rc) return rc;
  if (!stack) return fail(PMPD_EINVAL, "pmpd_stack_set_variant: NULL stack");
  if (variant < 0 || variant >= kNumVariants) return fail(PMPD_EINVAL, "pmpd_stack_set_variant: variant %d outside 0..%d", variant, kNumVariants - 1);
  stack->variant[b] = variant;
  return PMPD_OK;
}

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
  } else if (m <= kSkinnyMaxBatch && block16_takes(m, b)) {
    e = launch_block16_stack(stack, b, x_base, m, y_base, s);
  } else if (m >= kSkinnyMinBatch && m <= kSkinnyMaxBatch) {
    e = launch_skinny_stack(stack, b, x_base, m, y_base, s);
  } else if (m <= PMPD_MAX_BATCH) {
    e = b == 4 ? launch_stack_batch<4>(stack, x_base, m, y_base, s)
        : b == 3 ? launch_stack_batch<3>(stack, x_base, m, y_base, s)
                 : launch_stack_batch<2>(stack, x_base, m, y_base, s);
  } else {
    if (static_cast<uint64_t>(m) * static_cast<uint64_t>(stack->max_in) * 2u >= (uint64_t{1} << 32))
      return fail(PMPD_EINVAL, "pmpd_batch_step: m x in_features = %d x %d: X of one layer must stay below 4 GiB", m, stack->max_in);
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
