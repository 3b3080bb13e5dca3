// Prefill / large-batch linear layers on the matrix cores (gfx950):
//     Y[j][r] = sum_i W_b[r][i] X[j][i],   j < m  (m in the hundreds: the prompt tokens)
// The paper runs the prefill phase at a (higher) weight precision of the same nested store
// (Section 4.1; Algorithm 1, line 10) and notes that prefill is compute-bound (Section 1), so
// here the contraction goes to v_mfma_f32_16x16x32_f16 and the bit-plane unpack is amortised
// over a 128-token block of X.
//
// The weights never touch LDS.  In the storage format lane 16 kb + j of a wave holds, in word t
// of its 16 bytes of a plane, 32 columns (32 kb .. 32 kb + 31 of the group) of row 16 t + j.  The
// B operand of the 16x16x32 MFMA wants, in lane 16 kb + j, column j of B for K = 8 kb .. 8 kb + 7:
// taking weight row 16 t + j as column j and the lane's columns 32 kb + 8 s .. 32 kb + 8 s + 7 as
// its K slice (s = 0..3), the lane's own words are four operands per t after dequantisation,
//     w = fp16(a_g + s_g * (q~ + 2^(3-b)))    (exact code, then one fused multiply-add),
// with the K index of MFMA s meaning column 32 kb + 8 s + e of the group for K = 8 kb + e.  The A
// operand (rows = 16 tokens) follows the same K order: lane 16 kb + i reads the 16 bytes at
// columns 32 kb + 8 s of token i from the X tile in LDS.
//
// Workgroup = 8 waves; wave w owns row tile tile0 + w (64 weight rows) and all 128 tokens of the
// block: 8 x 4 accumulator blocks of 16 x 16 (128 registers).  Per group of 128 columns a wave
// dequantises its 128 weights per lane once and issues 128 MFMAs; the workgroup shares one X tile
// (128 tokens x 128 columns, double-buffered in LDS, rows padded to 272 bytes so that the 16-byte
// operand reads of 16 consecutive lanes fall into different banks).  Plane words, (scale, min)
// words and the X tile of the next group are loaded while the current one is multiplied.
// The weight is rounded to fp16 once (relative error 2^-11 per weight, about 3e-4 relative L2
// on y, inside the 1e-3 bar); the decode kernels keep exact codes instead because there the
// per-group scaling is free.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "pmpd_common.hpp"
#include "pmpd_device.hpp"

namespace pmpd {

constexpr int kPfWaves = 8;             // waves (= 64-row tiles) per workgroup
constexpr int kPfTokens = 128;          // rows of X per workgroup
constexpr int kPfThreads = kPfWaves * 64;
constexpr int kPfMB = kPfTokens / 16;   // 16-token MFMA blocks
constexpr int kPfXStride = 128 + 8;     // halves per X row in LDS (272 bytes)
constexpr size_t kPrefillLds = 2 * static_cast<size_t>(kPfTokens) * kPfXStride * 2;
constexpr int kPfXV = kPfTokens * 16 / kPfThreads;  // uint4 of the X tile per thread

__device__ __forceinline__ half2_t h2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ uint32_t u32(half2_t v) { return __builtin_bit_cast(uint32_t, v); }

// 4-bit aligned codes q~ of one 32-bit word of each plane (32 columns of one row): word v holds
// columns 8 v .. 8 v + 7, nibbles 0,4 / 1,5 / 2,6 / 3,7 = column pairs (0,1) / (2,3) / (4,5) / (6,7).
template <int B>
__device__ __forceinline__ void code_words(const u32x4 (&pl)[B], int t, uint32_t (&code)[4]) {
  uint32_t hi[4], lo[4];
  pair_words(word_of(pl[0], t), word_of(pl[1], t), hi);
  if constexpr (B == 4) pair_words(word_of(pl[2], t), word_of(pl[3], t), lo);
  if constexpr (B == 3) single_words(word_of(pl[2], t), lo);
#pragma unroll
  for (int v = 0; v < 4; ++v) code[v] = (B == 2) ? (hi[v] << 2) : ((hi[v] << 2) | lo[v]);
}

// One workgroup: tokens [mtile * 128, +128) x the 8 row tiles from tile0 of one layer.
template <int B>
__device__ __forceinline__ void prefill_tile(const LayerDesc& L, const _Float16* __restrict__ X, int m_rows,
                                             float* __restrict__ Y, int mtile, int tile0, _Float16* lds) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int G = L.n_groups;
  const int in_f = L.in_f;
  const int m0 = mtile * kPfTokens;

  // this wave's row tile (clamped: rows past the end are never stored)
  const int tile = tile0 + wave;
  const int tl = tile < L.n_tiles ? tile : L.n_tiles - 1;
  const int64_t tbase = (static_cast<int64_t>(tl) * G) * 64;
  global_u32x4_ptr pp[B];
#pragma unroll
  for (int k = 0; k < B; ++k) pp[k] = (global_u32x4_ptr)(L.plane[k]) + tbase + lane;  // + g*64
  global_u32x4_ptr sp = (global_u32x4_ptr)(L.sa) + tbase / 4 + (lane & 15);         // + g*16

  // X tile copy: 128 rows x 16 uint4; thread handles (row, c) = (idx / 16, idx % 16), idx = tid + 512 i,
  // i.e. rows tid / 16 + 32 i, the same 16 bytes of each
  const int xrow = tid >> 4, xc = tid & 15;
  const uint4* xg = reinterpret_cast<const uint4*>(X) + xc;  // + token * in_f / 8 + g * 16
  const int64_t xrow_stride = static_cast<int64_t>(in_f / 8);
  const int xdst = xrow * kPfXStride + xc * 8;
  auto load_x = [&](uint4 (&xr)[kPfXV], int g) {
#pragma unroll
    for (int i = 0; i < kPfXV; ++i) {
      const int token = m0 + xrow + 32 * i;
      xr[i] = token < m_rows ? xg[token * xrow_stride + g * 16] : make_uint4(0, 0, 0, 0);
    }
  };
  auto store_x = [&](const uint4 (&xr)[kPfXV], _Float16* buf) {
#pragma unroll
    for (int i = 0; i < kPfXV; ++i) *reinterpret_cast<uint4*>(buf + xdst + 32 * i * kPfXStride) = xr[i];
  };
  // A operand of this lane: token 16 mb + lane % 16, columns 32 (lane / 16) + 8 s
  const int a_off = (lane & 15) * kPfXStride + (lane >> 4) * 32;

  float4_t acc[kPfMB][4];
#pragma unroll
  for (int mb = 0; mb < kPfMB; ++mb)
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[mb][t] = float4_t{0.f, 0.f, 0.f, 0.f};

  constexpr float kOff = (B == 4) ? 0.5f : (B == 3) ? 1.0f : 2.0f;  // 2^(3-b)
  const half2_t cL = {static_cast<_Float16>(kOff - 1024.0f), static_cast<_Float16>(kOff - 1024.0f)};
  const half2_t cH = {static_cast<_Float16>(kOff - 64.0f), static_cast<_Float16>(kOff - 64.0f)};
  const half2_t sixteenth = {static_cast<_Float16>(0.0625f), static_cast<_Float16>(0.0625f)};
  const uint32_t maskL = opaque_sgpr(0x000F000Fu), maskH = opaque_sgpr(0x00F000F0u);
  uint32_t magic = 0x64006400u;  // fp16 pair (1024, 1024)
  asm volatile("" : "+v"(magic));

  // group 0: plane words and X tile
  u32x4 pc[B], sac;
#pragma unroll
  for (int k = 0; k < B; ++k) pc[k] = pp[k][0];
  sac = sp[0];
  {
    uint4 xr[kPfXV];
    load_x(xr, 0);
    store_x(xr, lds);
  }
  __syncthreads();

  for (int g = 0; g < G; ++g) {
    const _Float16* xs = lds + (g & 1) * (kPfTokens * kPfXStride);
    _Float16* xn = lds + ((g + 1) & 1) * (kPfTokens * kPfXStride);
    // ---- codes of the lane's 4 x 32 weights, scale / min pairs of its 4 rows
    uint32_t code[4][4];
    half2_t s2[4], a2[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      code_words<B>(pc, t, code[t]);
      const uint32_t w = word_of(sac, t);
      const _Float16 sv = __builtin_bit_cast(_Float16, static_cast<uint16_t>(w & 0xffffu));
      const _Float16 av = __builtin_bit_cast(_Float16, static_cast<uint16_t>(w >> 16));
      s2[t] = half2_t{sv, sv};
      a2[t] = half2_t{av, av};
    }
    // ---- the plane words are consumed: the loads of the next group reuse their registers and fly
    // while this group is multiplied; its X tile goes to the other LDS buffer after the first K-step
    const int gn = g + 1 < G ? g + 1 : g;
    uint4 xr[kPfXV];
    load_x(xr, gn);
#pragma unroll
    for (int k = 0; k < B; ++k) pc[k] = pp[k][gn * 64];
    sac = sp[gn * 16];
    // ---- 4 K-steps of 32: dequantise the 4 B operands, then 8 x 4 MFMAs
    half8_t af = *reinterpret_cast<const half8_t*>(xs + a_off);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      half8_t bw[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const uint32_t w = code[t][s], w8 = w >> 8;
        // exact codes q~ + 2^(3-b): low-nibble pairs carry 1024 + q~, high-nibble pairs 1024 + 16 q~
        const half2_t q0 = h2(and_or(w, maskL, magic)) + cL;
        const half2_t q1 = __builtin_elementwise_fma(h2(and_or(w, maskH, magic)), sixteenth, cH);
        const half2_t q2 = h2(and_or(w8, maskL, magic)) + cL;
        const half2_t q3 = __builtin_elementwise_fma(h2(and_or(w8, maskH, magic)), sixteenth, cH);
        u32x4 o;
        o.x = u32(__builtin_elementwise_fma(q0, s2[t], a2[t]));
        o.y = u32(__builtin_elementwise_fma(q1, s2[t], a2[t]));
        o.z = u32(__builtin_elementwise_fma(q2, s2[t], a2[t]));
        o.w = u32(__builtin_elementwise_fma(q3, s2[t], a2[t]));
        bw[t] = __builtin_bit_cast(half8_t, o);
      }
#pragma unroll
      for (int mb = 0; mb < kPfMB; ++mb) {
        const half8_t a_cur = af;
        // the operand of the next MFMA block is read from LDS before the MFMAs of this one issue
        const int nmb = mb + 1 < kPfMB ? mb + 1 : 0, ns = mb + 1 < kPfMB ? s : s + 1;
        if (ns < 4) af = *reinterpret_cast<const half8_t*>(xs + a_off + nmb * 16 * kPfXStride + ns * 8);
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[mb][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a_cur, bw[t], acc[mb][t], 0, 0, 0);
      }
      if (s == 0) store_x(xr, xn);
      __builtin_amdgcn_sched_barrier(0);  // keep the dequantised operands of one K-step live at a time
    }
    __syncthreads();
  }

  // ---- store: D[i][j] of a 16 x 16 block sits in lane j + 16 (i / 4), register i % 4
  if (tile < L.n_tiles) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int col = tile * 64 + 16 * t + (lane & 15);
      if (col < L.out_f) {
#pragma unroll
        for (int mb = 0; mb < kPfMB; ++mb)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int row = m0 + 16 * mb + 4 * (lane >> 4) + r;
            if (row < m_rows) Y[static_cast<int64_t>(row) * L.out_f + col] = acc[mb][t][r];
          }
      }
    }
  }
}

template <int B>
__global__ __launch_bounds__(kPfThreads, 2) void pmpd_prefill_layer_kernel(LayerDesc L, const _Float16* __restrict__ X, int m,
                                                                     float* __restrict__ Y, int m_tiles) {
  extern __shared__ uint4 lds_raw[];
  const int mtile = static_cast<int>(blockIdx.x) % m_tiles;
  const int ntile = static_cast<int>(blockIdx.x) / m_tiles;
  prefill_tile<B>(L, X, m, Y, mtile, ntile * kPfWaves, reinterpret_cast<_Float16*>(lds_raw));
}

template <int B>
__global__ __launch_bounds__(kPfThreads, 2) void pmpd_prefill_stack_kernel(const LayerDesc* __restrict__ layers,
                                                                     const WorkItem* __restrict__ items,
                                                                     const _Float16* __restrict__ x_base, int m,
                                                                     float* __restrict__ y_base, int m_tiles) {
  extern __shared__ uint4 lds_raw[];
  const int mtile = static_cast<int>(blockIdx.x) % m_tiles;
  const WorkItem it = items[static_cast<int>(blockIdx.x) / m_tiles];
  const LayerDesc L = layers[it.layer];
  prefill_tile<B>(L, x_base + static_cast<int64_t>(m) * L.x_off, m, y_base + static_cast<int64_t>(m) * L.y_off, mtile,
                  it.tile0, reinterpret_cast<_Float16*>(lds_raw));
}

// The X tile needs more than the 64 KiB of dynamic LDS a kernel gets by default.
template <typename K>
static hipError_t allow_lds(K kernel) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             static_cast<int>(kPrefillLds));
}

// Launchers used by the C entry points (defined in pmpd_gemv.hip).
hipError_t launch_prefill_layer(const LayerDesc& d, int b, const void* X, int m, float* Y, hipStream_t s) {
  const int m_tiles = (m + kPfTokens - 1) / kPfTokens;
  const int n_tiles = (d.n_tiles + kPfWaves - 1) / kPfWaves;
  const unsigned grid = static_cast<unsigned>(m_tiles) * static_cast<unsigned>(n_tiles);
  const _Float16* x = static_cast<const _Float16*>(X);
  hipError_t e = b == 4 ? allow_lds(&pmpd_prefill_layer_kernel<4>)
                 : b == 3 ? allow_lds(&pmpd_prefill_layer_kernel<3>)
                          : allow_lds(&pmpd_prefill_layer_kernel<2>);
  if (e != hipSuccess) return e;
  if (b == 4) hipLaunchKernelGGL((pmpd_prefill_layer_kernel<4>), dim3(grid), dim3(kPfThreads), kPrefillLds, s, d, x, m, Y, m_tiles);
  else if (b == 3) hipLaunchKernelGGL((pmpd_prefill_layer_kernel<3>), dim3(grid), dim3(kPfThreads), kPrefillLds, s, d, x, m, Y, m_tiles);
  else hipLaunchKernelGGL((pmpd_prefill_layer_kernel<2>), dim3(grid), dim3(kPfThreads), kPrefillLds, s, d, x, m, Y, m_tiles);
  return hipGetLastError();
}

hipError_t launch_prefill_stack(const pmpd_stack* st, int b, const void* X, int m, float* Y, hipStream_t s) {
  const int m_tiles = (m + kPfTokens - 1) / kPfTokens;
  const size_t n_items = st->items[kPrefillItemList].size();
  const unsigned grid = static_cast<unsigned>(m_tiles) * static_cast<unsigned>(n_items);
  const _Float16* x = static_cast<const _Float16*>(X);
  const WorkItem* items = st->d_items[kPrefillItemList];
  hipError_t e = b == 4 ? allow_lds(&pmpd_prefill_stack_kernel<4>)
                 : b == 3 ? allow_lds(&pmpd_prefill_stack_kernel<3>)
                          : allow_lds(&pmpd_prefill_stack_kernel<2>);
  if (e != hipSuccess) return e;
  if (b == 4) hipLaunchKernelGGL((pmpd_prefill_stack_kernel<4>), dim3(grid), dim3(kPfThreads), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles);
  else if (b == 3) hipLaunchKernelGGL((pmpd_prefill_stack_kernel<3>), dim3(grid), dim3(kPfThreads), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles);
  else hipLaunchKernelGGL((pmpd_prefill_stack_kernel<2>), dim3(grid), dim3(kPfThreads), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles);
  return hipGetLastError();
}

}  // namespace pmpd
