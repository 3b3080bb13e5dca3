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
// exponents and group sums, by the whole workgroup.  Thread idx handles columns 8 idx ..
// 8 idx + 7 of the range; a quad of threads owns one 32-column block, a row of 16 threads one
// group.
// Where a layer's activations come from: an fp16 vector, or the output of an earlier layer of the same
// launch, scaled by `gain` and rounded to fp16 (round to nearest even) on the way in: its fp32 values
// (y32), or its 64-bit fixed-point sums (y64) when that layer's K-parts meet by integer atomics.
struct XSource {
  const _Float16* x16;
  const float* y32;
  const unsigned long long* y64;
  float gain;
};
__device__ __forceinline__ XSource x_from_fp16(const _Float16* p) { return XSource{p, nullptr, nullptr, 1.f}; }

// Sums of K-parts that meet across workgroups are kept as 64-bit fixed-point numbers with 32 fractional
// bits: integer addition is associative, so atomic adds in any order of arrival give the same bits (no
// floating-point atomics, no partial-sum buffers, nobody has to arrive last).  |v| must stay below 2^31;
// what lies below 2^-32 is dropped (a row's sum over 13824 products of fp16 inputs stays below 2^28).
__device__ __forceinline__ unsigned long long to_fixed(float v) {
  const float fl = floorf(v);
  const int hi = static_cast<int>(fl);
  const uint32_t lo = static_cast<uint32_t>((v - fl) * 4294967296.0f);  // v - floor(v) is exact, in [0, 1)
  return (static_cast<unsigned long long>(static_cast<uint32_t>(hi)) << 32) | lo;
}
__device__ __forceinline__ float fixed_to_float(unsigned long long f) {
  const int hi = static_cast<int>(static_cast<uint32_t>(f >> 32));
  const uint32_t lo = static_cast<uint32_t>(f);
  return fmaf(static_cast<float>(lo), 2.3283064365386963e-10f, static_cast<float>(hi));  // one rounding, wherever it is used
}

__device__ __forceinline__ uint32_t pack_half2(float a, float b) {
  const half2_t h = {static_cast<_Float16>(a), static_cast<_Float16>(b)};
  return __builtin_bit_cast(uint32_t, h);
}

template <int NW>
__device__ __forceinline__ void stage_x(const XSource& src, int c0, int cn, const ImageLayout& im, int j) {
  const int n16 = cn * 16;
  for (int idx = threadIdx.x; idx < n16; idx += NW * 64) {
    uint32_t w[4];
    if (src.y64) {
      // fixed-point sums other workgroups of this launch have added to: agent-scope loads read the coherent copy
      unsigned long long* yg = const_cast<unsigned long long*>(src.y64) + (c0 * 16 + idx) * 8;
      float v8[8];
#pragma unroll
      for (int e = 0; e < 8; ++e)
        v8[e] = fixed_to_float(__hip_atomic_load(yg + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) * src.gain;
#pragma unroll
      for (int q = 0; q < 4; ++q) w[q] = pack_half2(v8[2 * q], v8[2 * q + 1]);
    } else if (src.y32) {
      // written by other workgroups of this launch: agent-scope loads read the coherent copy
      float* yg = const_cast<float*>(src.y32) + (c0 * 16 + idx) * 8;
      float v8[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) v8[e] = __hip_atomic_load(yg + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) * src.gain;
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
// One workgroup: NW / SPLITK consecutive row tiles starting at tile0, each split over SPLITK waves
// along K, for m <= 2 SETS activation vectors.  K is walked in chunks whose split activations fit
// in LDS.  x: [m][in_f] fp16, y: [m][out_f] fp32.
struct NoHook {
  __device__ __forceinline__ void operator()() const {}
};

// The groups a workgroup walks (the whole row unless K is split over workgroups) and the chunk
// capacity the LDS image was sized for.
struct KRange {
  int begin, end, chunk;
};

// before_staging() runs in every thread after the first weight loads have been issued and before x
// is read: the dependency-ordered kernel waits there for the producers of x.  ORDERED also issues
// the loads of the first two groups before that point instead of one, and stores y with agent-scope
// (write-through) stores, so that workgroups of the same launch can read it without a cache flush.
template <int B, int SETS, int NW, int SPLITK, bool ORDERED = false, typename Hook = NoHook>
__device__ __forceinline__ void run_tiles(const LayerDesc& L, int tile0, const XSource& x, int m, float* __restrict__ y,
                                          uint4* lds_raw, KRange kr, Hook before_staging = Hook(),
                                          unsigned long long* y64 = nullptr) {
  static_assert(NW % SPLITK == 0, "waves must divide evenly over the K splits");
  static_assert(!ORDERED || SETS == 1, "chained inputs are batch-1 only");
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int G = L.n_groups;
  const ImageLayout im(lds_raw, kr.chunk, m);

  const int tile = tile0 + wave / SPLITK;
  const int ks = wave % SPLITK;
  const bool active = tile < L.n_tiles;
  const int64_t tbase = (static_cast<int64_t>(active ? tile : 0) * G) * 64 + lane;  // + g*64 per group
  global_u32x4_ptr pp[B];
#pragma unroll
  for (int k = 0; k < B; ++k) pp[k] = (global_u32x4_ptr)(L.plane[k]) + tbase;
  // (scale, min) words of rows l % 16 + 16 t, t = 0..3: the 16 bytes at [l % 16] of the group's 64 words
  global_u32x4_ptr sp = (global_u32x4_ptr)(L.sa) + (tbase - lane) / 4 + (lane & 15);  // + g*16 per group

  // Operand addressing.  Row i = lane % 16 of the activation operand is piece i % 4 of slot i / 4;
  // the lane receives the sums of slot lane / 16.  Slot 2 v + c = class c of vector 2 s + v.
  const int piece = (lane & 3) == 3 ? 0 : (lane & 3);  // row 4 q + 3 is never read back
  const int in_slot = (lane & 15) >> 2, out_slot = lane >> 4;
  int a_off[SETS], s_off[SETS], x_off[SETS];
#pragma unroll
  for (int s = 0; s < SETS; ++s) {
    int vi = 2 * s + (in_slot >> 1);
    vi = vi < m ? vi : m - 1;  // slots of absent vectors repeat the last one; their sums are not stored
    a_off[s] = im.piece_off(vi, in_slot & 1) + piece * kPieceStride + (lane >> 4) * 16;
    s_off[s] = im.scale_off(vi, in_slot & 1) + piece * 4 + (lane >> 4);
    int vo = 2 * s + (out_slot >> 1);
    vo = vo < m ? vo : m - 1;
    x_off[s] = im.xsum_off(vo, out_slot & 1);
  }
  int wscale = 0x00008082;
  asm volatile("" : "+v"(wscale));

  float yacc[SETS][4];
#pragma unroll
  for (int s = 0; s < SETS; ++s)
#pragma unroll
    for (int t = 0; t < 4; ++t) yacc[s][t] = 0.f;

  for (int c0 = kr.begin; c0 < kr.end; c0 += im.cg) {
    const int cn = (kr.end - c0 < im.cg) ? (kr.end - c0) : im.cg;
    const int g0 = c0 + cn * ks / SPLITK, g1 = c0 + cn * (ks + 1) / SPLITK;
    const bool work = active && g0 < g1;
    // The next group's plane words are in flight while the current group is consumed.  Weights
    // are read exactly once per pass: nontemporal loads keep them from displacing anything in
    // the caches.  Past the end of the range the last group is reloaded (a cache hit) instead
    // of branching around the loads.  Two register sets alternate (the loop is unrolled by two).
    u32x4 pa[B], pb[B], sa_a = {0, 0, 0, 0}, sa_b = {0, 0, 0, 0};
    auto load = [&](u32x4 (&dst)[B], u32x4& dsa, int g) {
      const int gl = g < g1 ? g : g1 - 1;
#pragma unroll
      for (int k = 0; k < B; ++k) dst[k] = __builtin_nontemporal_load(&pp[k][gl * 64]);
      dsa = sp[gl * 16];
    };
    // The first group's loads do not depend on the activations: issue them before the workgroup
    // splits x, so that their latency overlaps the staging and the barrier.
    if (work) load(pa, sa_a, g0);
    if (ORDERED && work) load(pb, sa_b, g0 + 1);
    if (c0 == kr.begin) before_staging();
    else __syncthreads();  // the previous chunk's image has been consumed
    for (int j = 0; j < m; ++j) {
      XSource xj = x;
      if (xj.x16) xj.x16 += static_cast<int64_t>(j) * L.in_f;
      stage_x<NW>(xj, c0, cn, im, j);
    }
    __syncthreads();
    if (work) {
      auto consume = [&](const u32x4 (&pl)[B], const u32x4& csa, int g) {
        const int gr = g - c0;
        XOperand X[SETS];
        float xg[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) {
          X[s].a = read_fp8_operand(im.pieces + a_off[s] + gr * kGroupPieceBytes);
          X[s].scale = static_cast<unsigned char>(im.scales[s_off[s] + gr * kScaleBytes]);
          xg[s] = im.xsum[x_off[s] + gr];
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          float4_t acc[SETS];
          mfma_block<B, SETS>(X, pl, t, wscale, acc);
          const uint32_t w = word_of(csa, t);
          const float sc = half_bits_to_float(w & 0xffffu);
          const float off = fmaf(sc, half_step<B>(), half_bits_to_float(w >> 16));
#pragma unroll
          for (int s = 0; s < SETS; ++s) {
            const float d = (acc[s][0] + acc[s][1]) + acc[s][2];
            yacc[s][t] = fmaf(sc, d, yacc[s][t]);
            yacc[s][t] = fmaf(off, xg[s], yacc[s][t]);
          }
        }
      };
      for (int gc = g0; gc < g1; gc += 2) {
        if (!ORDERED || gc > g0) load(pb, sa_b, gc + 1);
        consume(pa, sa_a, gc);
        load(pa, sa_a, gc + 2);
        if (gc + 1 < g1) consume(pb, sa_b, gc + 1);
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
          if (row < L.out_f) {
            if constexpr (ORDERED) {
              // one K-part among several: add it to the row's fixed-point sum; else the row is this workgroup's alone
              if (y64) __hip_atomic_fetch_add(&y64[row], to_fixed(yacc[s][t]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              else __hip_atomic_store(&yo[row], yacc[s][t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else {
              yo[row] = yacc[s][t];
            }
          }
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
  run_tiles<B, SETS, NW, SPLITK>(L, it.tile0, x_from_fp16(x_base + static_cast<int64_t>(m) * L.x_off), m,
                                 y_base + static_cast<int64_t>(m) * L.y_off, lds, KRange{0, L.n_groups, chunk_groups(L.n_groups, m)});
}

template <int B, int SETS, int NW, int SPLITK>
__global__ __launch_bounds__(NW * 64, waves_per_simd<SETS>()) void pmpd_layer_kernel(LayerDesc L,
                                                                                    const _Float16* __restrict__ x, int m,
                                                                                    float* __restrict__ y) {
  extern __shared__ uint4 lds[];
  run_tiles<B, SETS, NW, SPLITK>(L, static_cast<int>(blockIdx.x) * (NW / SPLITK), x_from_fp16(x), m, y, lds,
                                 KRange{0, L.n_groups, chunk_groups(L.n_groups, m)});
}

// =====================================================================================
// Dependency-ordered step in one cooperative launch.  The layers of a step are grouped into
// stages; a layer of stage s may take its input from the output of a layer of an earlier stage
// (x = fp16(gain * y)).  The grid is persistent: for every stage each workgroup takes the items
// blockIdx, blockIdx + gridDim, ... of that stage, issues the weight loads of its first item, and
// only then waits until every workgroup has finished the previous stage: weights stream while the
// barrier settles, x is read after it.
// An item is one 64-row tile and one K-part of at least 8 groups (8: two groups per wave, all of
// them in flight before the wait); the parts of a layer are as small as that allows while its
// stage still has no more items than the chip holds workgroups, so that every stage, however few
// rows it has, spreads over the whole chip in one round.  The K-parts of a row meet in a 64-bit
// fixed-point sum (32 fractional bits) that every part adds to with an integer atomic: integer
// addition is associative, so the result does not depend on the order of arrival, there are no
// floating-point atomics, no buffers of partial sums, and nobody has to wait to be last.  Layers
// chained to such a layer read the sums; y of those layers is written from them after the last
// stage.  A layer with a single K-part writes y directly.
// Only y and the sums cross workgroups; they are written and read with agent-scope accesses
// (coherent across the chip's L2 slices), so the barrier needs no cache write-back or invalidate.  The launch is cooperative, so all workgroups are resident and the wait ends; it is
// bounded all the same (spin_limit polls), and a wait that runs out only sets sync->timed_out.
// Counters of the stage barrier.  Workgroup w adds to sub-counter w % 16 of the stage; the last
// one of each sub-counter adds to the stage's top counter, and the last of those publishes the
// stage number in the 32 copies of `stage_done`, the only words the waiting workgroups poll
// (workgroup w reads copy w % 32): the polls (a thousand readers) and the arrivals (a thousand
// read-modify-writes) never meet on one cache line, and no line has more than a few dozen readers.
constexpr int kSyncLine = 64;   // uint32 per 256-byte line
constexpr int kSubCounters = 16;
constexpr int kFlagCopies = 32;  // copies of the polled word, one 256-byte line each: 32 times fewer readers per line
struct OrderedSync {
  uint32_t stage_done[kFlagCopies * kSyncLine];  // [copy][0]: stages completed in this step (monotonic), polled
  uint32_t timed_out;
  uint32_t pad1[kSyncLine - 1];
  uint32_t counters[1];  // [n_stages][kSubCounters + 1][kSyncLine / 4] arrival counters, then [tiles] K-parts finished
};
constexpr int kStageCounterWords = (kSubCounters + 1) * (kSyncLine / 4);  // 16 uint32 (64 bytes) apart

struct ChainDesc {
  int64_t src_y_off;     // elements from y_base (or from the fixed-point sums) of the producing layer's output; -1: input from x_base
  float gain;
  int32_t n_parts;       // K-parts of part_groups groups each (the last one may be shorter); > 1: the parts meet in fixed point
  int32_t part_groups;
  int32_t src_fixed;     // the producing layer has more than one K-part: read its fixed-point sums
};

// Wait until every vector memory operation of this wave, stores included, has been acknowledged
// (s_waitcnt vmcnt(0); gfx9 encoding: vmcnt in bits 3:0 and 15:14, the other counters left at their
// maxima).  For the agent-scope (write-through) stores used here that is when they are visible to
// the other workgroups; a release fence would add a write-back of the whole L2 that nothing needs.
__device__ __forceinline__ void wait_for_own_stores() { __builtin_amdgcn_s_waitcnt(0x0F70); }

constexpr int kOrderedWaves = 4;
constexpr int kOrderedPartGroups = 8;      // smallest K-part: two groups per wave, all in flight before the wait
constexpr int kOrderedMaxPartGroups = 32;  // largest K-part the LDS image is sized for
constexpr int kItemPartShift = 20;  // WorkItem::tile0 = tile | part << 20

template <int B>
__global__ __launch_bounds__(kOrderedWaves * 64, 4) void pmpd_ordered_kernel(
    const LayerDesc* __restrict__ layers, const ChainDesc* __restrict__ chains, const WorkItem* __restrict__ items,
    const int32_t* __restrict__ stage_begin, int n_stages, const _Float16* __restrict__ x_base, float* __restrict__ y_base,
    unsigned long long* __restrict__ sums, OrderedSync* sync, uint32_t spin_limit, int n_layers) {
  extern __shared__ uint4 lds[];
  const uint32_t n_wg = gridDim.x;
  uint32_t* arrived = sync->counters;  // + s * kStageCounterWords + k * 16
  for (int s = 0; s < n_stages; ++s) {
    bool waited = s == 0;
    auto wait_for_previous_stage = [&]() {
      if (waited) return;
      waited = true;
      if (threadIdx.x == 0) {
        uint32_t polls = 0;
        while (__hip_atomic_load(&sync->stage_done[(blockIdx.x % kFlagCopies) * kSyncLine], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) <
               static_cast<uint32_t>(s)) {
          if (++polls >= spin_limit) {
            __hip_atomic_store(&sync->timed_out, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
          }
          __builtin_amdgcn_s_sleep(32);  // about a microsecond between polls (a thousand readers of one word); shorter intervals measured no faster
        }
      }
      __syncthreads();
    };
    for (int i = stage_begin[s] + static_cast<int>(blockIdx.x); i < stage_begin[s + 1]; i += static_cast<int>(n_wg)) {
      const WorkItem it = items[i];
      const LayerDesc L = layers[it.layer];
      const ChainDesc c = chains[it.layer];
      const int tile = it.tile0 & ((1 << kItemPartShift) - 1), part = it.tile0 >> kItemPartShift;
      const XSource src = c.src_y_off < 0 ? x_from_fp16(x_base + L.x_off)
                          : c.src_fixed   ? XSource{nullptr, nullptr, sums + c.src_y_off, c.gain}
                                          : XSource{nullptr, y_base + c.src_y_off, nullptr, c.gain};
      const int g0 = part * c.part_groups;
      const int g1 = g0 + c.part_groups < L.n_groups ? g0 + c.part_groups : L.n_groups;
      // a layer with one K-part writes y itself; the parts of the others add to the rows' fixed-point sums
      run_tiles<B, 1, kOrderedWaves, kOrderedWaves, true>(L, tile, src, 1, y_base + L.y_off, lds, KRange{g0, g1, kOrderedMaxPartGroups},
                                                         wait_for_previous_stage, c.n_parts > 1 ? sums + L.y_off : nullptr);
      __syncthreads();  // the LDS image is reused by the next item
    }
    // every wave waits until its own (write-through) stores and atomic adds of stage s are acknowledged, then
    // the workgroup is counted
    wait_for_own_stores();
    __syncthreads();
    if (threadIdx.x == 0) {
      const uint32_t k = blockIdx.x % kSubCounters;
      const uint32_t in_sub = (n_wg - k + kSubCounters - 1) / kSubCounters;  // workgroups that share sub-counter k
      uint32_t* cnt = arrived + s * kStageCounterWords;
      if (__hip_atomic_fetch_add(&cnt[k * 16], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == in_sub) {
        const uint32_t n_sub = n_wg < kSubCounters ? n_wg : kSubCounters;
        if (__hip_atomic_fetch_add(&cnt[kSubCounters * 16], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1 == n_sub)
          for (int q = 0; q < kFlagCopies; ++q)
            __hip_atomic_store(&sync->stage_done[q * kSyncLine], static_cast<uint32_t>(s + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  // After the last stage: y of the layers whose K-parts met in fixed point (the same conversion the
  // chained layers used when they read those sums).
  if (threadIdx.x == 0) {
    uint32_t polls = 0;
    while (__hip_atomic_load(&sync->stage_done[(blockIdx.x % kFlagCopies) * kSyncLine], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) <
           static_cast<uint32_t>(n_stages)) {
      if (++polls >= spin_limit) {
        __hip_atomic_store(&sync->timed_out, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(32);
    }
  }
  __syncthreads();
  for (int li = 0; li < n_layers; ++li) {
    if (chains[li].n_parts <= 1) continue;
    const LayerDesc& L = layers[li];
    for (int row = blockIdx.x * blockDim.x + threadIdx.x; row < L.out_f; row += gridDim.x * blockDim.x)
      y_base[L.y_off + row] = fixed_to_float(__hip_atomic_load(sums + L.y_off + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  }
}

__global__ void pmpd_ordered_reset_kernel(OrderedSync* sync, int n_counters, unsigned long long* sums, int64_t n_sums) {
  const int64_t tid = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x, n_threads = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t i = tid; i < n_counters; i += n_threads) sync->counters[i] = 0;
  for (int64_t i = tid; i < n_sums; i += n_threads) sums[i] = 0;
  if (blockIdx.x == 0 && threadIdx.x < kFlagCopies) sync->stage_done[threadIdx.x * kSyncLine] = 0;
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
  if (m > PMPD_MAX_BATCH) {  // compute-bound shape: fp16 MFMA tile kernel
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

// Launch shapes of the one-launch decode step (PMPD_STACK_VARIANT="v4,v3,v2" overrides the
// per-bit-width defaults):
//   0  4 waves x 1 tile each, whole K       1  4 waves on 1 tile, K split 4 ways
//   2  4 waves on 2 tiles, K split 2 ways   3  8 waves on 1 tile, K split 8 ways
//   4  16 waves on 1 tile, K split 16 ways
static constexpr int kNumVariants = 5;
// which work list (tiles per workgroup: list 0 = 4, 1 = 1, 2 = 2) each variant walks
static constexpr int kVariantList[kNumVariants] = {0, 1, 2, 1, 1};
static void pick_variants(pmpd_stack* st) {
  // Measured on the 7B-, 13B-shaped and mobile-scale stacks: shapes 0..2 are within 2 % of each
  // other.  Whole-K waves (shape 0) split x once for four tiles and win at b = 4 and 3 when the
  // stack has enough four-tile workgroups to fill the machine several times; shape 2 otherwise
  // and at b = 2, where the split of x weighs more against the shorter weight stream.  Short
  // stacks (the layers of one dependency stage, say) split K further, like single layers.
  const bool big = st->items[0].size() >= 4096;
  st->variant[4] = big ? 0 : 2;
  st->variant[3] = big ? 0 : 2;
  st->variant[2] = 2;
  const int64_t n_tiles = static_cast<int64_t>(st->items[1].size());
  int min_groups = st->max_in / kGroup;
  for (const LayerDesc& d : st->layers) min_groups = std::min(min_groups, d.n_groups);
  const int split = pick_splitk(n_tiles, std::min(min_groups, chunk_groups(st->max_in / kGroup, 1)), 16);
  if (split >= 4) {
    const int v = split == 4 ? 1 : split == 8 ? 3 : 4;
    st->variant[4] = st->variant[3] = st->variant[2] = v;
  }
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
  std::vector<int32_t> stage_begin;
  const ChainDesc* d_chains = nullptr;
  const WorkItem* d_items = nullptr;
  const int32_t* d_stage_begin = nullptr;
  OrderedSync* d_sync = nullptr;
  unsigned long long* d_sums = nullptr;  // fixed-point row sums, laid out like y
  int64_t n_sums = 0;
  int n_counters = 0;
  int n_stages = 0;
  int max_stage_items = 0;
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
// layer's stage within `slots` workgroups, never above kOrderedMaxPartGroups.
static std::vector<int> ordered_part_groups(const pmpd_stack* st, const pmpd_chain_t* chain, int n_stages, int slots) {
  std::vector<int64_t> stage_tiles(static_cast<size_t>(n_stages), 0);
  for (size_t i = 0; i < st->layers.size(); ++i) stage_tiles[static_cast<size_t>(chain[i].stage)] += st->layers[i].n_tiles;
  std::vector<int> pg(st->layers.size());
  for (size_t i = 0; i < st->layers.size(); ++i) {
    const int G = st->layers[i].n_groups;
    const int64_t tiles = std::max<int64_t>(1, stage_tiles[static_cast<size_t>(chain[i].stage)]);
    int parts = static_cast<int>(std::max<int64_t>(1, std::min<int64_t>((G + kOrderedPartGroups - 1) / kOrderedPartGroups, slots / tiles)));
    int groups = (G + parts - 1) / parts;
    groups = std::min(groups, kOrderedMaxPartGroups);
    pg[i] = groups;
  }
  return pg;
}

static int parts_of(int n_groups, int part_groups) { return (n_groups + part_groups - 1) / part_groups; }

// items an ordered step of this stack needs, and the length of its y (= of the fixed-point sums)
static void ordered_counts(const pmpd_stack* st, const std::vector<int>& pg, size_t* n_items, size_t* n_sums) {
  *n_items = *n_sums = 0;
  for (size_t i = 0; i < st->layers.size(); ++i) {
    const LayerDesc& d = st->layers[i];
    *n_items += static_cast<size_t>(d.n_tiles) * static_cast<size_t>(parts_of(d.n_groups, pg[i]));
    *n_sums = std::max(*n_sums, static_cast<size_t>(d.y_off) + static_cast<size_t>(d.out_f));
  }
}

// Workgroup slots the ordered kernel is planned for: four workgroups of four waves per compute unit.
static int ordered_slots() {
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess || prop.multiProcessorCount < 1) return 1024;
  return 4 * prop.multiProcessorCount;
}

static size_t ordered_bytes(const pmpd_stack* st, const std::vector<int>& pg, size_t n_stages) {
  size_t n_items, n_sums;
  ordered_counts(st, pg, &n_items, &n_sums);
  return align_up(st->layers.size() * sizeof(ChainDesc), 256) + align_up(n_items * sizeof(WorkItem), 256) +
         align_up((n_stages + 1) * sizeof(int32_t), 256) +
         align_up(sizeof(OrderedSync) + n_stages * kStageCounterWords * sizeof(uint32_t), 256) +
         align_up(n_sums * sizeof(unsigned long long), 256);
}

template <int B>
static hipError_t launch_ordered(const pmpd_ordered* o, const void* x, float* y, hipStream_t s) {
  const pmpd_stack* st = o->stack;
  const size_t lds = lds_bytes(kOrderedMaxPartGroups, 1, kOrderedWaves, 4);
  int per_cu = 0, dev = 0;
  hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, pmpd_ordered_kernel<B>, kOrderedWaves * 64, lds);
  if (e != hipSuccess) return e;
  hipDeviceProp_t prop;
  if ((e = hipGetDevice(&dev)) != hipSuccess || (e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
  int grid = std::min(per_cu, 4) * prop.multiProcessorCount;
  if (grid < 1) return hipErrorCooperativeLaunchTooLarge;
  grid = std::min(grid, o->max_stage_items);
  hipLaunchKernelGGL(pmpd_ordered_reset_kernel, dim3(1024), dim3(256), 0, s, o->d_sync, o->n_counters, o->d_sums, o->n_sums);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const LayerDesc* layers = st->d_layers;
  const _Float16* xb = static_cast<const _Float16*>(x);
  int n_stages = o->n_stages;
  uint32_t spin = o->spin_limit;
  int n_layers = static_cast<int>(st->layers.size());
  void* args[] = {&layers, const_cast<ChainDesc**>(&o->d_chains), const_cast<WorkItem**>(&o->d_items),
                  const_cast<int32_t**>(&o->d_stage_begin), &n_stages, &xb, &y, const_cast<unsigned long long**>(&o->d_sums),
                  const_cast<OrderedSync**>(&o->d_sync), &spin, &n_layers};
  return hipLaunchCooperativeKernel(reinterpret_cast<const void*>(&pmpd_ordered_kernel<B>), dim3(grid), dim3(kOrderedWaves * 64),
                                    args, static_cast<unsigned>(lds), s);
}

extern "C" {

int32_t pmpd_ordered_workspace_size(const pmpd_stack_t* stack, const pmpd_chain_t* chain, size_t* bytes) {
  int n_stages = 0;
  int32_t rc = check_chain(stack, chain, &n_stages);
  if (rc) return rc;
  if (!bytes) return fail(PMPD_EINVAL, "pmpd_ordered_workspace_size: bytes is NULL");
  *bytes = ordered_bytes(stack, ordered_part_groups(stack, chain, n_stages, ordered_slots()), static_cast<size_t>(n_stages));
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
  const size_t need = ordered_bytes(stack, pg, static_cast<size_t>(n_stages));
  if (workspace_bytes < need) return fail(PMPD_ESIZE, "pmpd_ordered_create: workspace %zu bytes, need %zu", workspace_bytes, need);
  size_t n_items, n_sums;
  ordered_counts(stack, pg, &n_items, &n_sums);
  if (n_items > static_cast<size_t>(INT32_MAX)) return fail(PMPD_EINVAL, "pmpd_ordered_create: too many work items");
  auto* o = new pmpd_ordered;
  o->stack = stack;
  o->n_stages = n_stages;
  o->n_counters = static_cast<int>(static_cast<size_t>(n_stages) * kStageCounterWords);
  o->n_sums = static_cast<int64_t>(n_sums);
  for (size_t i = 0; i < n_layers; ++i) {
    const LayerDesc& d = stack->layers[i];
    const int src = chain[i].source;
    const int parts = parts_of(d.n_groups, pg[i]);
    if (d.n_tiles >= (1 << kItemPartShift) || parts >= (1 << (31 - kItemPartShift))) {
      delete o;
      return fail(PMPD_EINVAL, "pmpd_ordered_create: layer %zu is too large for the item encoding", i);
    }
    const int src_fixed = src >= 0 && parts_of(stack->layers[src].n_groups, pg[src]) > 1;
    o->chains.push_back(ChainDesc{src < 0 ? int64_t{-1} : stack->layers[src].y_off, chain[i].gain, parts, pg[i], src_fixed});
  }
  // (tile, K-part) items, stage by stage; inside a stage long rows first
  std::vector<int> order(n_layers);
  for (size_t i = 0; i < n_layers; ++i) order[i] = static_cast<int>(i);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
    if (chain[a].stage != chain[b].stage) return chain[a].stage < chain[b].stage;
    return stack->layers[a].in_f > stack->layers[b].in_f;
  });
  o->stage_begin.assign(static_cast<size_t>(n_stages) + 1, 0);
  for (int li : order) {
    const int parts = o->chains[li].n_parts;
    for (int t = 0; t < stack->layers[li].n_tiles; ++t)
      for (int q = 0; q < parts; ++q) o->items.push_back(WorkItem{li, t | (q << kItemPartShift)});
    o->stage_begin[static_cast<size_t>(chain[li].stage) + 1] = static_cast<int32_t>(o->items.size());
  }
  for (int sidx = 1; sidx <= n_stages; ++sidx)  // stages without layers stay empty
    o->stage_begin[sidx] = std::max(o->stage_begin[sidx], o->stage_begin[sidx - 1]);
  for (int sidx = 0; sidx < n_stages; ++sidx)
    o->max_stage_items = std::max(o->max_stage_items, o->stage_begin[sidx + 1] - o->stage_begin[sidx]);
  char* w = static_cast<char*>(workspace);
  hipError_t e = hipMemcpy(w, o->chains.data(), n_layers * sizeof(ChainDesc), hipMemcpyHostToDevice);
  o->d_chains = reinterpret_cast<const ChainDesc*>(w);
  w += align_up(n_layers * sizeof(ChainDesc), 256);
  if (e == hipSuccess) e = hipMemcpy(w, o->items.data(), o->items.size() * sizeof(WorkItem), hipMemcpyHostToDevice);
  o->d_items = reinterpret_cast<const WorkItem*>(w);
  w += align_up(n_items * sizeof(WorkItem), 256);
  if (e == hipSuccess) e = hipMemcpy(w, o->stage_begin.data(), o->stage_begin.size() * sizeof(int32_t), hipMemcpyHostToDevice);
  o->d_stage_begin = reinterpret_cast<const int32_t*>(w);
  w += align_up(o->stage_begin.size() * sizeof(int32_t), 256);
  o->d_sync = reinterpret_cast<OrderedSync*>(w);
  const size_t sync_bytes = sizeof(OrderedSync) + static_cast<size_t>(n_stages) * kStageCounterWords * sizeof(uint32_t);
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
  } else if (m >= kSkinnyMinBatch && m <= kSkinnyMaxBatch) {
    e = launch_skinny_stack(stack, b, x_base, m, y_base, s);
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
