// Prefill / large-batch linear layers on the matrix cores (gfx950):
//     Y[j][r] = sum_i W_b[r][i] X[j][i],   j < m  (m in the hundreds: the prompt tokens)
// The paper runs the prefill phase at a (higher) weight precision of the same nested store
// (Section 4.1; Algorithm 1, line 10) and notes that prefill is compute-bound (Section 1), so
// here the contraction goes to v_mfma_f32_16x16x32_f16 and the bit-plane unpack is amortised
// over a 128-token block of X.
//
// The weights never touch LDS.  In the storage format lane 16 kb + j of a wave holds, in word t
// of its 16 bytes of a plane, 32 columns (32 kb .. 32 kb + 31 of the group) of row 16 t + j.  The
// first operand of the 16x16x32 MFMA wants, in lane 16 kb + j, row j for K = 8 kb .. 8 kb + 7:
// taking weight row 16 t + j as row j and the lane's columns 32 kb + 8 s .. 32 kb + 8 s + 7 as
// its K slice (s = 0..3), the lane's own words are four operands per t after dequantisation,
//     w = fp16(a_g + s_g * (q~ + 2^(3-b)))    (exact code, then one fused multiply-add),
// with the K index of MFMA s meaning column 32 kb + 8 s + e of the group for K = 8 kb + e.  The
// second operand (columns = 16 tokens) follows the same K order: lane 16 kb + i reads the 16 bytes at
// columns 32 kb + 8 s of token i from the X tile in LDS.
//
// Workgroup = 4 waves; wave w owns row tile tile0 + w (64 weight rows) and all 128 tokens of the
// block: 8 x 4 accumulator blocks of 16 x 16 (128 registers).  Per group of 128 columns a wave
// dequantises its 128 weights per lane once and issues 128 MFMAs; the workgroup shares one X tile
// (128 tokens x 128 columns, double-buffered in LDS in a swizzled layout whose 16-byte operand reads
// are free of bank conflicts).  Plane words, (scale, min) words and the X tile of the next group are
// loaded while the current one is multiplied.
// The weight is rounded to fp16 once (relative error 2^-11 per weight, about 3e-4 relative L2
// on y, inside the 1e-3 bar); the decode kernels keep exact codes instead because there the
// per-group scaling is free.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "pmpd_common.hpp"
#include "pmpd_device.hpp"

namespace pmpd {

constexpr int kPfWaves = 4;             // waves (= 64-row tiles) per workgroup; two workgroups share a compute unit
constexpr int kPfTokens = 128;          // rows of X per workgroup
constexpr int kPfThreads = kPfWaves * 64;
constexpr int kPfMB = kPfTokens / 16;   // 16-token MFMA blocks
constexpr int kPfRowBytes = 256;        // one token's 128 columns of a group in LDS
constexpr int kPfTileBytes = kPfTokens * kPfRowBytes;
constexpr size_t kPrefillLds = 2 * static_cast<size_t>(kPfTileBytes);
constexpr int kPfXV = kPfTokens * 16 / kPfThreads;  // 16-byte pieces of the X tile per thread

__device__ __forceinline__ half2_t h2(uint32_t v) { return __builtin_bit_cast(half2_t, v); }
__device__ __forceinline__ uint32_t u32(half2_t v) { return __builtin_bit_cast(uint32_t, v); }

// X tile in LDS: token row r holds its 16 chunks of 16 bytes (8 columns) at chunk position c ^ swz(r).
// A ds_read_b128 serves 16 lanes per cycle, and not 16 consecutive ones: the groups are lanes
// {0-3, 12-15, 20-27}, {4-11, 16-19, 28-31} and the same plus 32 (measured on gfx950 with the bank-conflict
// counter, one pair of active lanes per dispatch).  The MFMA operand read has lane 16 kb + i fetch chunk
// 4 kb + s of token i, so a group mixes chunks 4 kb + s and 4 (kb ^ 1) + s: with
//     swz(i) = i for i < 4,  i + 4 for 4 <= i < 12,  i - 8 for i >= 12     (i = r % 16)
// tokens {0-3, 12-15} get the values 0..7 and tokens {4-11} the values 8..15; both sets are closed under
// ^ 4, so the sixteen lanes of every group land in sixteen different 16-byte bank columns (4 cycles per
// read instead of 8 with rows padded to 272 bytes).  The tile's 16-byte stores (16 consecutive lanes =
// one row, rows 4 k .. 4 k + 3 per wave) are conflict-free as well.
__device__ __forceinline__ int pf_swz(int r) {
  const int hi = (r >> 2) & 3;
  return (r & 3) | (((0x78 >> (2 * hi)) & 3) << 2);  // hi: 0, 1, 2, 3 -> 0, 2, 3, 1
}

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

typedef __attribute__((address_space(3))) void* lds_ptr_t;
__device__ __forceinline__ lds_ptr_t to_lds(const void* p) {
  return reinterpret_cast<lds_ptr_t>(static_cast<uint32_t>(reinterpret_cast<uintptr_t>(p)));  // low half of a generic LDS address
}

// One workgroup: tokens [mtile * 128, +128) x the 8 row tiles from tile0 of one layer.
//
// A wave alternates between a VALU phase (dequantise the four B operands of a K-step: 56 instructions, plus
// 88 once per group to merge the plane words) and a matrix phase (32 MFMAs fed by 8 LDS reads).  Measured on
// gfx950 with two-wave probes: one 16x16x32 MFMA per 16 cycles and SIMD, and two VALU instructions of the
// SIMD's other wave ride under each MFMA for free; but the hardware serves the older wave of a SIMD first
// and a workgroup barrier per group keeps a workgroup's waves in step, so two waves of ONE workgroup on a
// SIMD run their VALU phases together and then queue for the matrix pipe together.  A workgroup is therefore
// four waves, one per SIMD, and two workgroups share a compute unit: the two waves of a SIMD belong to
// different workgroups, no barrier couples them, and their phases drift apart and overlap.
// Global loads: the plane words of group g + 2 are requested right after those of group g + 1 have been
// merged, at the end of group g (their registers are free then), and have a whole group to arrive.  The X
// tile goes from global memory straight to LDS (no registers, no LDS store instructions), requested one
// group ahead, right after the barrier that frees its buffer; every wave waits for its own loads before
// the barrier that ends the next group.  A wait for loads is always a wait for ALL of the wave's loads
// (the counter is not tracked across the loop's back edge), so new loads are only issued after that wait.
template <int B>
__device__ __forceinline__ void prefill_tile(const LayerDesc& L, const _Float16* __restrict__ X, int m_rows,
                                             float* __restrict__ Y, int mtile, int tile0, char* lds) {
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
  // Addresses are a wave-uniform 64-bit base (scalar registers) plus a 32-bit byte offset per lane, so that
  // a pointer costs no vector registers: plane words of group g at plane[k] + (tbase + 64 g) 16 + 16 lane,
  // (scale, min) words at sa + (tbase / 4 + 16 g) 16 + 16 (lane % 16).
  const uint32_t plane_lane = static_cast<uint32_t>(lane) * 16u, sa_lane = static_cast<uint32_t>(lane & 15) * 16u;
  auto uniform = [](const void* p) {  // the same pointer, known to the compiler as wave-uniform
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v)), hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
    return reinterpret_cast<const char*>((static_cast<uint64_t>(hi) << 32) | lo);
  };
  const char* pbase[B];
#pragma unroll
  for (int k = 0; k < B; ++k) pbase[k] = uniform(static_cast<const char*>(L.plane[k]) + tbase * 16);
  const char* sbase = uniform(static_cast<const char*>(L.sa) + tbase * 4);

  // X tile: a wave's load instruction i fills the four token rows 4 (wave + 8 i) .. + 3 of the tile, 1 KiB
  // that the hardware places at consecutive LDS addresses in lane order: lane l is position l % 16 of row
  // 4 (wave + 8 i) + l / 16 and therefore fetches the chunk that the swizzle puts there.  Rows 32 i apart
  // share r % 16, so the lane's chunk is the same for its four loads.  Tokens past the end repeat the last
  // one (their outputs are never stored).  Byte offsets from X fit 32 bits (checked by the launcher).
  const int xrow = 4 * wave + (lane >> 4);
  const int xchunk = (lane & 15) ^ pf_swz(xrow);
  uint32_t xoff[kPfXV];
#pragma unroll
  for (int i = 0; i < kPfXV; ++i) {
    int token = m0 + xrow + 4 * kPfWaves * i;
    token = token < m_rows ? token : m_rows - 1;
    xoff[i] = static_cast<uint32_t>(token) * static_cast<uint32_t>(in_f) * 2u + static_cast<uint32_t>(xchunk) * 16u;
  }
  const char* xbase = uniform(X);
  auto request_x = [&](int g, char* buf) {
    const char* xg = xbase + g * (kGroup * 2);
#pragma unroll
    for (int i = 0; i < kPfXV; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(xg + xoff[i]),
                                       to_lds(buf + (4 * wave + 4 * kPfWaves * i) * kPfRowBytes), 16, 0, 0);
  };
  // A operand of this lane for K-step s: token 16 mb + lane % 16, chunk 4 (lane / 16) + s
  const int a_row = (lane & 15) * kPfRowBytes;
  const int a_col = (4 * (lane >> 4)) ^ pf_swz(lane & 15);  // chunk position of K-step s: a_col ^ s

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

  u32x4 pc[B], sac;           // plane words and (scale, min) words of the group that is merged next
  uint32_t code[4][4];        // codes of the group being dequantised: [16-row block][K-step]
  half2_t sa[4];              // (scale, min) of the lane's four rows
  u32x4 bw[4];                // B operands of one K-step

  // Once per group: codes of the lane's 4 x 32 weights, scale / min pairs of its 4 rows.
  auto merge = [&]() {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      code_words<B>(pc, t, code[t]);
      sa[t] = h2(word_of(sac, t));
    }
  };
  auto request_planes = [&](int g) {
    const int gn = g < G ? g : G - 1;
#pragma unroll
    for (int k = 0; k < B; ++k) pc[k] = *(global_u32x4_ptr)(pbase[k] + gn * 1024 + plane_lane);
    sac = *(global_u32x4_ptr)(sbase + gn * 256 + sa_lane);
  };
  // VALU phase: the four B operands of K-step s.  Exact codes q~ + 2^(3-b) (low-nibble pairs carry 1024 + q~,
  // high-nibble pairs 1024 + 16 q~), then one fused multiply-add with the row's scale and minimum, which
  // the instruction's operand selects broadcast from the two halves of one register.
  auto dequant = [&](int s) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const uint32_t w = code[t][s], w8 = w >> 8;
      const half2_t sc = {sa[t].x, sa[t].x}, mn = {sa[t].y, sa[t].y};
      const half2_t q0 = h2(and_or(w, maskL, magic)) + cL;
      const half2_t q1 = __builtin_elementwise_fma(h2(and_or(w, maskH, magic)), sixteenth, cH);
      const half2_t q2 = h2(and_or(w8, maskL, magic)) + cL;
      const half2_t q3 = __builtin_elementwise_fma(h2(and_or(w8, maskH, magic)), sixteenth, cH);
      bw[t].x = u32(__builtin_elementwise_fma(q0, sc, mn));
      bw[t].y = u32(__builtin_elementwise_fma(q1, sc, mn));
      bw[t].z = u32(__builtin_elementwise_fma(q2, sc, mn));
      bw[t].w = u32(__builtin_elementwise_fma(q3, sc, mn));
    }
  };
  // Matrix phase: 8 token blocks x 4 row blocks.  The A operands are read from LDS three blocks ahead into
  // a ring of four.  LDS reads complete in order, so before the MFMAs of block mb it is enough to wait until
  // at most the reads issued after block mb's are outstanding.  The compiler's own wait insertion does not do
  // that here (it waits for every read, the one just issued included, which puts most of an LDS latency in
  // front of every other block), so the reads and their waits are written out: the read is an asm statement
  // whose result the compiler takes as available at once, and the wait is an asm statement that "modifies"
  // the operand registers, so that the MFMAs that use them cannot be moved in front of it.  No other LDS or
  // scalar-memory access is outstanding during the phase.
  auto multiply = [&](int s, const char* xs) {
    const uint32_t ap = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(xs + a_row + ((a_col ^ s) << 4)));  // LDS address
    half8_t af[4];
#define PMPD_PF_READ(dst, block) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(ap), "n"((block) * 16 * kPfRowBytes))
    PMPD_PF_READ(af[0], 0);
    PMPD_PF_READ(af[1], 1);
    PMPD_PF_READ(af[2], 2);
#pragma unroll
    for (int mb = 0; mb < kPfMB; ++mb) {
      half8_t& a = af[mb & 3];
      // reads issued so far: min(mb + 3, 8); those after block mb's may stay outstanding
      if (mb + 3 <= kPfMB) asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(a));
      else if (mb + 2 == kPfMB) asm volatile("s_waitcnt lgkmcnt(1)" : "+v"(a));
      else asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a));
#pragma unroll
      for (int t = 0; t < 4; ++t)
        acc[mb][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, bw[t]), a, acc[mb][t], 0, 0, 0);
      switch (mb) {  // the read for three blocks on (offsets are immediates)
        case 0: PMPD_PF_READ(af[3], 3); break;
        case 1: PMPD_PF_READ(af[0], 4); break;
        case 2: PMPD_PF_READ(af[1], 5); break;
        case 3: PMPD_PF_READ(af[2], 6); break;
        case 4: PMPD_PF_READ(af[3], 7); break;
        default: break;
      }
    }
#undef PMPD_PF_READ
  };
  auto phase_end = []() { __builtin_amdgcn_sched_barrier(0); };  // phases stay apart in the instruction stream

  // All of a wave's outstanding loads have arrived (the LDS writes of its X loads included).
  auto loads_landed = []() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), other counters untouched
    __builtin_amdgcn_sched_barrier(0);
  };

  // group 0: X tile to buffer 0, plane words merged; group 1 requested
  request_x(0, lds);
  request_planes(0);
  merge();
  loads_landed();
  request_planes(1);
  __syncthreads();
  if (G > 1) request_x(1, lds + kPfTileBytes);

  for (int g = 0; g < G; ++g) {
    const char* xs = lds + (g & 1) * kPfTileBytes;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      dequant(s);
      phase_end();
      multiply(s, xs);
      phase_end();
    }
    // The loads of group g + 1 (plane words, then X tile) were issued a group ago: merge the plane words, make
    // sure the X tile has landed, and only then issue new loads, so that no wait ever covers a fresh load.
    merge();
    loads_landed();
    request_planes(g + 2);
    __syncthreads();  // every wave's part of X tile g + 1 is in LDS, and buffer g % 2 is free
    if (g + 2 < G) request_x(g + 2, lds + (g & 1) * kPfTileBytes);
  }

  // ---- store.  The weights are the first MFMA operand (rows i of D = weight rows) and X the second (columns
  // j = tokens): D[i][j] sits in lane j + 16 (i / 4), register i % 4, so a lane holds four consecutive
  // output features of one token, 16 bytes of Y.  They go out as one 16-byte store where Y allows it (written
  // once, never read here: nontemporal).
  if (tile < L.n_tiles) {
    const bool wide = (reinterpret_cast<uintptr_t>(Y) % 16 == 0) && (L.out_f % 4 == 0);
#pragma unroll
    for (int mb = 0; mb < kPfMB; ++mb) {
      const int row = m0 + 16 * mb + (lane & 15);
      if (row >= m_rows) continue;
      float* yrow = Y + static_cast<int64_t>(row) * L.out_f;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int col = tile * 64 + 16 * t + 4 * (lane >> 4);
        if (wide) {
          if (col < L.out_f) __builtin_nontemporal_store(acc[mb][t], reinterpret_cast<float4_t*>(yrow + col));
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (col + r < L.out_f) yrow[col + r] = acc[mb][t][r];
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
  prefill_tile<B>(L, X, m, Y, mtile, ntile * kPfWaves, reinterpret_cast<char*>(lds_raw));
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
                  it.tile0, reinterpret_cast<char*>(lds_raw));
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
  constexpr int kList = 0;  // work list of 4-tile items: one 64-row tile per wave
  static_assert(kStackTilesPerWg[kList] == kPfWaves, "one tile per wave");
  const size_t n_items = st->items[kList].size();
  const unsigned grid = static_cast<unsigned>(m_tiles) * static_cast<unsigned>(n_items);
  const _Float16* x = static_cast<const _Float16*>(X);
  const WorkItem* items = st->d_items[kList];
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
