// Prefill / large-batch linear layers on the matrix cores (gfx950):
//     Y[j][r] = sum_i W_b[r][i] X[j][i],   j < m  (m in the hundreds: the prompt tokens)
// The paper runs the prefill phase at a (higher) weight precision of the same nested store
// (Section 4.1; Algorithm 1, line 10) and notes that prefill is compute-bound (Section 1), so
// here the contraction goes to v_mfma_f32_32x32x16_f16 and the bit-plane unpack is amortised
// over a 256-row block of X.
//
// Workgroup = 2 x 2 waves, output tile 256 (rows of X) x 128 (rows of W), K walked in steps of
// 64 columns (half a quantisation group).  Per step:
//   * all threads copy the 256 x 64 fp16 tile of X to LDS (global loads issued one step ahead);
//   * the weights of the step are unpacked one 32-bit word of each plane per thread (32 columns
//     of one row; the same pair merge as the decode kernels, then the two 2-bit pairs are joined
//     into 4-bit codes q~), turned into fp16 values  w = fp16(a_g + s_g * (q~ + 2^(3-b)))  with
//     packed fp16 math, and written to LDS as a 128 x 64 tile with K contiguous;
//   * each wave multiplies its 128 x 64 quarter with 4 x 2 blocks of 32x32x16 MFMAs (fp32
//     accumulate, 128 accumulator registers), reading the operand fragments of the next 16
//     columns from LDS before it issues the MFMAs of the current ones.
// Measured alternatives (13B-shaped stack, m = 512, b = 4): 64x64 wave tiles with 4 or 8 waves
// 880-925 TFLOP/s, this shape 965 TFLOP/s; a register-only MFMA loop reaches 2.1-2.3 PFLOP/s on
// the same box.
// Rows of both LDS tiles are padded to 144 bytes so that the 16-byte operand reads of 16
// consecutive lanes fall into 64 different banks.
// The weight is rounded to fp16 once (relative error 2^-11 per weight, about 3e-4 relative L2
// on y, inside the 1e-3 bar); the decode kernels keep exact integer codes instead because there
// the per-group scaling is free.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "pmpd_common.hpp"
#include "pmpd_device.hpp"

namespace pmpd {

typedef float float16_t __attribute__((ext_vector_type(16)));

#ifndef PMPD_PREFILL_WM
#define PMPD_PREFILL_WM 2  // wave rows per workgroup
#endif
#ifndef PMPD_PREFILL_MB
#define PMPD_PREFILL_MB 4  // 32-row MFMA blocks per wave along the rows of X
#endif
constexpr int kPWM = PMPD_PREFILL_WM;
constexpr int kPMB = PMPD_PREFILL_MB;
constexpr int kPWaveM = 32 * kPMB;      // rows of X per wave
constexpr int kPM = kPWaveM * kPWM;     // rows of X per workgroup
constexpr int kPN = 128;          // rows of W per workgroup (two 64-row storage tiles)
constexpr int kPK = 64;           // columns per step
constexpr int kPStride = kPK + 8; // halves per LDS row (144 bytes)
constexpr int kPThreads = 128 * kPWM;  // WM x 2 waves
constexpr size_t kPrefillLds = static_cast<size_t>(kPM + kPN) * kPStride * 2;

__device__ __forceinline__ half2_t h2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ uint32_t u32(half2_t v) { return __builtin_bit_cast(uint32_t, v); }

// One workgroup: the (64 WM) x 128 output tile (mtile, ntile) of one layer.
template <int B>
__device__ __forceinline__ void prefill_tile(const LayerDesc& L, const _Float16* __restrict__ X, int m_rows,
                                             float* __restrict__ Y, int mtile, int tile0, _Float16* lds) {
  static_assert(kPWM == 2, "the unpack mapping below assumes 256 threads");
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;  // which block of the output this wave multiplies
  // unpack share of this thread: storage tile ut, 32-column slice up of the 64-column step,
  // row 16 ur_t + ur_j of the tile (one 32-bit word of each plane, consecutive over the lanes)
  const int ut = wave >> 1, up = wave & 1;
  const int ur_j = lane >> 2, ur_t = lane & 3;
  const int G = L.n_groups;
  const int in_f = L.in_f;
  _Float16* Xs = lds;
  _Float16* Ws = lds + kPM * kPStride;

  const int m0 = mtile * kPM;
  // storage tile this wave unpacks (clamped: rows past the end are never stored)
  int T = tile0 + ut;
  T = T < L.n_tiles ? T : L.n_tiles - 1;
  const int64_t tbase = (static_cast<int64_t>(T) * G) * 64;  // (tile, group 0) in 16-byte units
  global_u32_ptr pw[B];
#pragma unroll
  for (int k = 0; k < B; ++k) pw[k] = (global_u32_ptr)(L.plane[k]) + tbase * 4 + (16 * up + ur_j) * 4 + ur_t;
  global_u32_ptr sp = (global_u32_ptr)(L.sa) + tbase + 4 * ur_j + ur_t;  // = lane: rows in [j][t] order

  // X tile copy: kPM rows x 8 uint4; thread t handles (row, c) = ((t + T i) / 8, (t + T i) % 8), T threads
  constexpr int kXV = kPM * 8 / kPThreads;  // uint4 of the X tile per thread
  const uint4* xg[kXV];
  bool xok[kXV];
  int xdst[kXV];
#pragma unroll
  for (int i = 0; i < kXV; ++i) {
    const int idx = tid + kPThreads * i;
    const int row = idx >> 3, c = idx & 7;
    xok[i] = (m0 + row) < m_rows;
    const int rr = xok[i] ? (m0 + row) : 0;
    xg[i] = reinterpret_cast<const uint4*>(X + static_cast<int64_t>(rr) * in_f) + c;
    xdst[i] = row * kPStride + c * 8;
  }

  float16_t acc[kPMB][2];
#pragma unroll
  for (int a = 0; a < kPMB; ++a)
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b2][r] = 0.f;

  constexpr float kOff = (B == 4) ? 0.5f : (B == 3) ? 1.0f : 2.0f;  // 2^(3-b)
  const half2_t cL = {static_cast<_Float16>(kOff - 1024.0f), static_cast<_Float16>(kOff - 1024.0f)};
  const half2_t cH = {static_cast<_Float16>(kOff - 64.0f), static_cast<_Float16>(kOff - 64.0f)};
  const half2_t sixteenth = {static_cast<_Float16>(0.0625f), static_cast<_Float16>(0.0625f)};

  const int n_steps = G * 2;
  // register-staged loads of step 0
  uint4 xr[kXV];
  uint32_t pr[B];
  uint32_t sar;
#pragma unroll
  for (int i = 0; i < kXV; ++i) xr[i] = xok[i] ? xg[i][0] : make_uint4(0, 0, 0, 0);
#pragma unroll
  for (int k = 0; k < B; ++k) pr[k] = pw[k][0];
  sar = sp[0];

  for (int step = 0; step < n_steps; ++step) {
    if (step) __syncthreads();  // the previous step's MFMAs have read the tiles
    // ---- X tile to LDS
#pragma unroll
    for (int i = 0; i < kXV; ++i) *reinterpret_cast<uint4*>(Xs + xdst[i]) = xr[i];
    // ---- unpack, dequantise, W tile to LDS
    {
      const half2_t s2 = {__builtin_bit_cast(_Float16, static_cast<uint16_t>(sar & 0xffffu)),
                          __builtin_bit_cast(_Float16, static_cast<uint16_t>(sar & 0xffffu))};
      const half2_t a2 = {__builtin_bit_cast(_Float16, static_cast<uint16_t>(sar >> 16)),
                          __builtin_bit_cast(_Float16, static_cast<uint16_t>(sar >> 16))};
      _Float16* wrow = Ws + (ut * 64 + 16 * ur_t + ur_j) * kPStride + up * 32;
      // 4-bit aligned codes q~ of the thread's 32 columns: word v holds columns 8 v .. 8 v + 7,
      // nibbles 0,4 / 1,5 / 2,6 / 3,7 = column pairs (0,1) / (2,3) / (4,5) / (6,7)
      uint32_t code[4];
      {
        uint32_t hi[4], lo[4];
        pair_words(pr[0], pr[1], hi);
        if constexpr (B == 4) pair_words(pr[2], pr[3], lo);
        if constexpr (B == 3) single_words(pr[2], lo);
#pragma unroll
        for (int v = 0; v < 4; ++v) code[v] = (B == 2) ? (hi[v] << 2) : ((hi[v] << 2) | lo[v]);
      }
      const uint32_t maskL = opaque_sgpr(0x000F000Fu), maskH = opaque_sgpr(0x00F000F0u);
      uint32_t magic = 0x64006400u;  // fp16 pair (1024, 1024)
      asm volatile("" : "+v"(magic));
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const uint32_t w = code[v], w8 = w >> 8;
        // exact codes q~ + 2^(3-b): low-nibble pairs carry 1024 + q~, high-nibble pairs 1024 + 16 q~
        const half2_t q0 = h2(and_or(w, maskL, magic)) + cL;
        const half2_t q1 = __builtin_elementwise_fma(h2(and_or(w, maskH, magic)), sixteenth, cH);
        const half2_t q2 = h2(and_or(w8, maskL, magic)) + cL;
        const half2_t q3 = __builtin_elementwise_fma(h2(and_or(w8, maskH, magic)), sixteenth, cH);
        u32x4 o;
        o.x = u32(__builtin_elementwise_fma(q0, s2, a2));
        o.y = u32(__builtin_elementwise_fma(q1, s2, a2));
        o.z = u32(__builtin_elementwise_fma(q2, s2, a2));
        o.w = u32(__builtin_elementwise_fma(q3, s2, a2));
        *reinterpret_cast<u32x4*>(wrow + v * 8) = o;
      }
    }
    __syncthreads();
    // ---- loads of the next step fly while this step multiplies
    if (step + 1 < n_steps) {
      const int ns = step + 1;
      const int g = ns >> 1, kh = ns & 1;
#pragma unroll
      for (int i = 0; i < kXV; ++i) xr[i] = xok[i] ? xg[i][ns * 8] : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int k = 0; k < B; ++k) pr[k] = pw[k][g * 256 + kh * 128];
      sar = sp[g * 64];
    }
    // ---- 64 x 64 x 64 per wave; the operand fragments of the next 16 columns are read from LDS
    // before the MFMAs of the current ones are issued, so the matrix pipe does not wait on LDS.
    {
      const _Float16* xa = Xs + (wm * kPWaveM + (lane & 31)) * kPStride + 8 * (lane >> 5);
      const _Float16* wb = Ws + (wn * 64 + (lane & 31)) * kPStride + 8 * (lane >> 5);
      half8_t af[2][kPMB], bf[2][2];
#pragma unroll
      for (int a = 0; a < kPMB; ++a) af[0][a] = *reinterpret_cast<const half8_t*>(xa + a * 32 * kPStride);
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) bf[0][b2] = *reinterpret_cast<const half8_t*>(wb + b2 * 32 * kPStride);
#pragma unroll
      for (int kk = 0; kk < kPK / 16; ++kk) {
        const int cur = kk & 1, nxt = cur ^ 1;
        if (kk + 1 < kPK / 16) {
#pragma unroll
          for (int a = 0; a < kPMB; ++a)
            af[nxt][a] = *reinterpret_cast<const half8_t*>(xa + a * 32 * kPStride + (kk + 1) * 16);
#pragma unroll
          for (int b2 = 0; b2 < 2; ++b2)
            bf[nxt][b2] = *reinterpret_cast<const half8_t*>(wb + b2 * 32 * kPStride + (kk + 1) * 16);
        }
#pragma unroll
        for (int a = 0; a < kPMB; ++a)
#pragma unroll
          for (int b2 = 0; b2 < 2; ++b2)
            acc[a][b2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[cur][a], bf[cur][b2], acc[a][b2], 0, 0, 0);
      }
    }
  }

  // ---- store: D[i][j] of a 32 x 32 block sits in lane l = j + 32 * ((i / 4) % 2), register (i / 8) * 4 + i % 4
  const int n0 = tile0 * 64;
#pragma unroll
  for (int a = 0; a < kPMB; ++a)
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2) {
      const int col = n0 + wn * 64 + b2 * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * kPWaveM + a * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (row < m_rows && col < L.out_f) Y[static_cast<int64_t>(row) * L.out_f + col] = acc[a][b2][r];
      }
    }
}

template <int B>
__global__ __launch_bounds__(kPThreads, 2) void pmpd_prefill_layer_kernel(LayerDesc L, const _Float16* __restrict__ X, int m,
                                                                    float* __restrict__ Y, int m_tiles) {
  extern __shared__ uint4 lds_raw[];
  const int mtile = static_cast<int>(blockIdx.x) % m_tiles;
  const int ntile = static_cast<int>(blockIdx.x) / m_tiles;
  prefill_tile<B>(L, X, m, Y, mtile, ntile * 2, reinterpret_cast<_Float16*>(lds_raw));
}

template <int B>
__global__ __launch_bounds__(kPThreads, 2) void pmpd_prefill_stack_kernel(const LayerDesc* __restrict__ layers,
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

// Launchers used by the C entry points (defined in pmpd_gemv.hip).
hipError_t launch_prefill_layer(const LayerDesc& d, int b, const void* X, int m, float* Y, hipStream_t s) {
  const int m_tiles = (m + kPM - 1) / kPM;
  const int n_tiles = (d.n_tiles + 1) / 2;
  const unsigned grid = static_cast<unsigned>(m_tiles) * static_cast<unsigned>(n_tiles);
  const _Float16* x = static_cast<const _Float16*>(X);
  if (b == 4) hipLaunchKernelGGL((pmpd_prefill_layer_kernel<4>), dim3(grid), dim3(kPThreads), kPrefillLds, s, d, x, m, Y, m_tiles);
  else if (b == 3) hipLaunchKernelGGL((pmpd_prefill_layer_kernel<3>), dim3(grid), dim3(kPThreads), kPrefillLds, s, d, x, m, Y, m_tiles);
  else hipLaunchKernelGGL((pmpd_prefill_layer_kernel<2>), dim3(grid), dim3(kPThreads), kPrefillLds, s, d, x, m, Y, m_tiles);
  return hipGetLastError();
}

hipError_t launch_prefill_stack(const pmpd_stack* st, int b, const void* X, int m, float* Y, hipStream_t s) {
  const int m_tiles = (m + kPM - 1) / kPM;
  const size_t n_items = st->items[kPrefillItemList].size();
  const unsigned grid = static_cast<unsigned>(m_tiles) * static_cast<unsigned>(n_items);
  const _Float16* x = static_cast<const _Float16*>(X);
  const WorkItem* items = st->d_items[kPrefillItemList];
  if (b == 4) hipLaunchKernelGGL((pmpd_prefill_stack_kernel<4>), dim3(grid), dim3(kPThreads), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles);
  else if (b == 3) hipLaunchKernelGGL((pmpd_prefill_stack_kernel<3>), dim3(grid), dim3(kPThreads), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles);
  else hipLaunchKernelGGL((pmpd_prefill_stack_kernel<2>), dim3(grid), dim3(kPThreads), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles);
  return hipGetLastError();
}

}  // namespace pmpd
