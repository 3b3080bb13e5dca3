// Prefill / large-batch linear layers on the matrix cores (gfx950):
//     Y[j][r] = sum_i W_b[r][i] X[j][i],   j < m  (m in the hundreds: the prompt tokens)
// The paper runs the prefill phase at a (higher) weight precision of the same nested store
// (Section 4.1; Algorithm 1, line 10) and notes that prefill is compute-bound (Section 1), so
// here the contraction goes to v_mfma_f32_32x32x16_f16 and the bit-plane unpack is amortised
// over a 128-row block of X.
//
// Workgroup = 4 waves, output tile 128 (rows of X) x 128 (rows of W), K walked in steps of 64
// columns (half a quantisation group).  Per step:
//   * 256 threads copy the 128 x 64 fp16 tile of X to LDS;
//   * the weights of the step are unpacked by the lane that owns the row (same storage format
//     and bit tricks as the decode kernels: lane l of a wave <-> row l of a 64-row tile), turned
//     into fp16 values  w = fp16(a_g + s_g * (q~ + 2^(3-b)))  with packed fp16 math, and written to
//     LDS as a 128 x 64 tile with K contiguous;
//   * each wave multiplies its 64 x 64 quarter with 2 x 2 blocks of 32x32x16 MFMAs, fp32 accumulate.
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

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int kPM = 128;          // rows of X per workgroup
constexpr int kPN = 128;          // rows of W per workgroup (two 64-row storage tiles)
constexpr int kPK = 64;           // columns per step
constexpr int kPStride = kPK + 8; // halves per LDS row (144 bytes)
constexpr size_t kPrefillLds = static_cast<size_t>(kPM + kPN) * kPStride * 2;

__device__ __forceinline__ half2_t h2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ uint32_t u32(half2_t v) { return __builtin_bit_cast(uint32_t, v); }

// One workgroup: the 128 x 128 output tile (mtile, ntile) of one layer.
template <int B>
__device__ __forceinline__ void prefill_tile(const LayerDesc& L, const _Float16* __restrict__ X, int m_rows,
                                             float* __restrict__ Y, int mtile, int tile0, _Float16* lds) {
  const UnpackConsts<B> uc;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;  // which 64 x 64 quarter this wave multiplies
  const int ut = wave >> 1, up = wave & 1;  // which storage tile / which 32-column word it unpacks
  const int G = L.n_groups;
  const int in_f = L.in_f;
  _Float16* Xs = lds;
  _Float16* Ws = lds + kPM * kPStride;

  const int m0 = mtile * kPM;
  // storage tile this wave unpacks (clamped: rows past the end are never stored)
  int T = tile0 + ut;
  T = T < L.n_tiles ? T : L.n_tiles - 1;
  const int64_t tbase = (static_cast<int64_t>(T) * G) * 64 + lane;  // (tile, group 0, lane) in 16-byte units
  global_u32_ptr pw[B];
#pragma unroll
  for (int k = 0; k < B; ++k) pw[k] = (global_u32_ptr)(L.plane[k]) + tbase * 4;
  global_u32_ptr sp = (global_u32_ptr)(L.sa) + tbase;

  // X tile copy: 128 rows x 8 uint4; thread t handles (row, c) = ((t + 256 i) / 8, (t + 256 i) % 8)
  const uint4* xg[4];
  bool xok[4];
  int xdst[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int idx = tid + 256 * i;
    const int row = idx >> 3, c = idx & 7;
    xok[i] = (m0 + row) < m_rows;
    const int rr = xok[i] ? (m0 + row) : 0;
    xg[i] = reinterpret_cast<const uint4*>(X + static_cast<int64_t>(rr) * in_f) + c;
    xdst[i] = row * kPStride + c * 8;
  }

  float16_t acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
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
  uint4 xr[4];
  uint32_t pr[B];
  uint32_t sar;
#pragma unroll
  for (int i = 0; i < 4; ++i) xr[i] = xok[i] ? xg[i][0] : make_uint4(0, 0, 0, 0);
#pragma unroll
  for (int k = 0; k < B; ++k) pr[k] = pw[k][up];
  sar = sp[0];

  for (int step = 0; step < n_steps; ++step) {
    if (step) __syncthreads();  // the previous step's MFMAs have read the tiles
    // ---- X tile to LDS
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<uint4*>(Xs + xdst[i]) = xr[i];
    // ---- unpack, dequantise, W tile to LDS
    {
      const half2_t s2 = {__builtin_bit_cast(_Float16, static_cast<uint16_t>(sar & 0xffffu)),
                          __builtin_bit_cast(_Float16, static_cast<uint16_t>(sar & 0xffffu))};
      const half2_t a2 = {__builtin_bit_cast(_Float16, static_cast<uint16_t>(sar >> 16)),
                          __builtin_bit_cast(_Float16, static_cast<uint16_t>(sar >> 16))};
      _Float16* wrow = Ws + (ut * 64 + lane) * kPStride + up * 32;
#pragma unroll
      for (int mm = 0; mm < 4; ++mm) {
        uint32_t u = merge_planes<B>(uc, pr, mm);
        uint32_t w = (mm == 0) ? u : __builtin_amdgcn_alignbit(u, u, mm);
        uint32_t w8 = w >> 8;
        // exact codes q~ + 2^(3-b): low-nibble pairs carry 1024 + q~, high-nibble pairs 1024 + 16 q~
        const half2_t q0 = h2(and_or(w, uc.maskL, uc.magic)) + cL;
        const half2_t q1 = __builtin_elementwise_fma(h2(and_or(w, uc.maskH, uc.magic)), sixteenth, cH);
        const half2_t q2 = h2(and_or(w8, uc.maskL, uc.magic)) + cL;
        const half2_t q3 = __builtin_elementwise_fma(h2(and_or(w8, uc.maskH, uc.magic)), sixteenth, cH);
        u32x4 o;
        o.x = u32(__builtin_elementwise_fma(q0, s2, a2));
        o.y = u32(__builtin_elementwise_fma(q1, s2, a2));
        o.z = u32(__builtin_elementwise_fma(q2, s2, a2));
        o.w = u32(__builtin_elementwise_fma(q3, s2, a2));
        *reinterpret_cast<u32x4*>(wrow + mm * 8) = o;
      }
    }
    __syncthreads();
    // ---- loads of the next step fly while this step multiplies
    if (step + 1 < n_steps) {
      const int ns = step + 1;
      const int g = ns >> 1, kh = ns & 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) xr[i] = xok[i] ? xg[i][ns * 8] : make_uint4(0, 0, 0, 0);
#pragma unroll
      for (int k = 0; k < B; ++k) pr[k] = pw[k][g * 256 + kh * 2 + up];
      sar = sp[g * 64];
    }
    // ---- 64 x 64 x 64 per wave
#pragma unroll
    for (int kk = 0; kk < kPK / 16; ++kk) {
      half8_t af[2], bf[2];
      const int koff = kk * 16 + 8 * (lane >> 5);
#pragma unroll
      for (int a = 0; a < 2; ++a)
        af[a] = *reinterpret_cast<const half8_t*>(Xs + (wm * 64 + a * 32 + (lane & 31)) * kPStride + koff);
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2)
        bf[b2] = *reinterpret_cast<const half8_t*>(Ws + (wn * 64 + b2 * 32 + (lane & 31)) * kPStride + koff);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b2 = 0; b2 < 2; ++b2)
          acc[a][b2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[a], bf[b2], acc[a][b2], 0, 0, 0);
    }
  }

  // ---- store: D[i][j] of a 32 x 32 block sits in lane l = j + 32 * ((i / 4) % 2), register (i / 8) * 4 + i % 4
  const int n0 = tile0 * 64;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2) {
      const int col = n0 + wn * 64 + b2 * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * 64 + a * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (row < m_rows && col < L.out_f) Y[static_cast<int64_t>(row) * L.out_f + col] = acc[a][b2][r];
      }
    }
}

template <int B>
__global__ __launch_bounds__(256, 2) void pmpd_prefill_layer_kernel(LayerDesc L, const _Float16* __restrict__ X, int m,
                                                                    float* __restrict__ Y, int m_tiles) {
  extern __shared__ uint4 lds_raw[];
  const int mtile = static_cast<int>(blockIdx.x) % m_tiles;
  const int ntile = static_cast<int>(blockIdx.x) / m_tiles;
  prefill_tile<B>(L, X, m, Y, mtile, ntile * 2, reinterpret_cast<_Float16*>(lds_raw));
}

template <int B>
__global__ __launch_bounds__(256, 2) void pmpd_prefill_stack_kernel(const LayerDesc* __restrict__ layers,
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
  if (b == 4) hipLaunchKernelGGL((pmpd_prefill_layer_kernel<4>), dim3(grid), dim3(256), kPrefillLds, s, d, x, m, Y, m_tiles);
  else if (b == 3) hipLaunchKernelGGL((pmpd_prefill_layer_kernel<3>), dim3(grid), dim3(256), kPrefillLds, s, d, x, m, Y, m_tiles);
  else hipLaunchKernelGGL((pmpd_prefill_layer_kernel<2>), dim3(grid), dim3(256), kPrefillLds, s, d, x, m, Y, m_tiles);
  return hipGetLastError();
}

hipError_t launch_prefill_stack(const pmpd_stack* st, int b, const void* X, int m, float* Y, hipStream_t s) {
  const int m_tiles = (m + kPM - 1) / kPM;
  const size_t n_items = st->items[kPrefillItemList].size();
  const unsigned grid = static_cast<unsigned>(m_tiles) * static_cast<unsigned>(n_items);
  const _Float16* x = static_cast<const _Float16*>(X);
  const WorkItem* items = st->d_items[kPrefillItemList];
  if (b == 4) hipLaunchKernelGGL((pmpd_prefill_stack_kernel<4>), dim3(grid), dim3(256), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles);
  else if (b == 3) hipLaunchKernelGGL((pmpd_prefill_stack_kernel<3>), dim3(grid), dim3(256), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles);
  else hipLaunchKernelGGL((pmpd_prefill_stack_kernel<2>), dim3(grid), dim3(256), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles);
  return hipGetLastError();
}

}  // namespace pmpd
