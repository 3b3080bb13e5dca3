// Unquantised fp16 matrix-vector reference (gfx950): y = W x with W fp16 [out][in] row-major,
// x fp16, fp32 accumulation, fp32 y.  The paper quotes its linear-layer speedups against fp16
// kernels on the same device (Section 5.2, Table 3); this file gives that denominator for this
// device, held to the same standard as the quantised path: a list of layers in one launch, weights
// read once with 128-bit streaming loads, x staged in LDS, nothing but the loads on the critical
// path (2 bytes per weight: HBM-bound).
//
// Work split: a workgroup of 4 waves takes 32 consecutive rows of one layer; a wave takes 4 rows at
// a time (two passes), its 64 lanes striding over the row in 16-byte chunks, so one wave-wide load
// covers 512 consecutive columns of one row and eight loads are in flight per wave.  The lane sums
// meet in a butterfly of cross-lane adds; the order of additions is fixed, results are deterministic.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <vector>

#include "pmpd_common.hpp"

namespace pmpd {
namespace {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));

constexpr int kRefWaves = 4;
constexpr int kRefRowsPerPass = 4;
constexpr int kRefPasses = 2;
constexpr int kRefRowsPerWg = kRefWaves * kRefRowsPerPass * kRefPasses;  // 32
constexpr int kRefMaxIn = 32768;  // the x image has to fit 64 KiB of LDS

struct RefDesc {
  const void* w;
  int64_t x_off;  // fp16 elements from x_base
  int64_t y_off;  // fp32 elements from y_base
  int32_t out_f;
  int32_t in_f;
};
static_assert(sizeof(RefDesc) == 32, "RefDesc is read by the kernel with this layout");

struct RefItem {
  int32_t layer;
  int32_t row0;
};

__device__ __forceinline__ float dot8(const h8& w, const h8& x, float acc) {
  acc = __builtin_amdgcn_fdot2(h2{w[0], w[1]}, h2{x[0], x[1]}, acc, false);
  acc = __builtin_amdgcn_fdot2(h2{w[2], w[3]}, h2{x[2], x[3]}, acc, false);
  acc = __builtin_amdgcn_fdot2(h2{w[4], w[5]}, h2{x[4], x[5]}, acc, false);
  acc = __builtin_amdgcn_fdot2(h2{w[6], w[7]}, h2{x[6], x[7]}, acc, false);
  return acc;
}

__device__ __forceinline__ void ref_rows(const RefDesc& L, int row0, const _Float16* x_base, float* y_base, char* lds) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = L.in_f >> 3;  // 16-byte chunks per row
  h8* xs = reinterpret_cast<h8*>(lds);
  const h8* xg = reinterpret_cast<const h8*>(x_base + L.x_off);
  for (int i = tid; i < n; i += kRefWaves * 64) xs[i] = xg[i];
  __syncthreads();
  const h8* w = static_cast<const h8*>(L.w);
#pragma unroll 1
  for (int pass = 0; pass < kRefPasses; ++pass) {
    const int r0 = row0 + (wave * kRefPasses + pass) * kRefRowsPerPass;
    if (r0 >= L.out_f) break;
    const h8* wr[kRefRowsPerPass];
    float acc[kRefRowsPerPass];
#pragma unroll
    for (int k = 0; k < kRefRowsPerPass; ++k) {
      const int r = min(r0 + k, L.out_f - 1);  // rows past the end repeat the last one; never stored
      wr[k] = w + static_cast<int64_t>(r) * n;
      acc[k] = 0.f;
    }
    int c = lane;
    for (; c + 64 < n; c += 128) {
      h8 a[kRefRowsPerPass], b[kRefRowsPerPass];
#pragma unroll
      for (int k = 0; k < kRefRowsPerPass; ++k) a[k] = __builtin_nontemporal_load(wr[k] + c);
#pragma unroll
      for (int k = 0; k < kRefRowsPerPass; ++k) b[k] = __builtin_nontemporal_load(wr[k] + c + 64);
      const h8 xa = xs[c], xb = xs[c + 64];
#pragma unroll
      for (int k = 0; k < kRefRowsPerPass; ++k) acc[k] = dot8(b[k], xb, dot8(a[k], xa, acc[k]));
    }
    if (c < n) {
      h8 a[kRefRowsPerPass];
#pragma unroll
      for (int k = 0; k < kRefRowsPerPass; ++k) a[k] = __builtin_nontemporal_load(wr[k] + c);
      const h8 xa = xs[c];
#pragma unroll
      for (int k = 0; k < kRefRowsPerPass; ++k) acc[k] = dot8(a[k], xa, acc[k]);
    }
#pragma unroll
    for (int k = 0; k < kRefRowsPerPass; ++k) {
#pragma unroll
      for (int d = 32; d >= 1; d >>= 1) acc[k] += __shfl_xor(acc[k], d, 64);
    }
    if (lane < kRefRowsPerPass && r0 + lane < L.out_f) {
      const float v = lane == 0 ? acc[0] : lane == 1 ? acc[1] : lane == 2 ? acc[2] : acc[3];
      y_base[L.y_off + r0 + lane] = v;
    }
  }
}

__global__ __launch_bounds__(kRefWaves * 64) void fp16_stack_kernel(const RefDesc* __restrict__ layers,
                                                                    const RefItem* __restrict__ items,
                                                                    const _Float16* __restrict__ x_base,
                                                                    float* __restrict__ y_base) {
  extern __shared__ __align__(16) char lds[];
  const RefItem it = items[blockIdx.x];
  const RefDesc L = layers[it.layer];
  ref_rows(L, it.row0, x_base, y_base, lds);
}

__global__ __launch_bounds__(kRefWaves * 64) void fp16_layer_kernel(RefDesc L, const _Float16* __restrict__ x_base,
                                                                    float* __restrict__ y_base) {
  extern __shared__ __align__(16) char lds[];
  ref_rows(L, static_cast<int>(blockIdx.x) * kRefRowsPerWg, x_base, y_base, lds);
}

size_t ref_align(size_t v) { return (v + 255) / 256 * 256; }

int32_t ref_hip_fail(hipError_t e, const char* what) {
  return fail(PMPD_EHIP, "%s: %s", what, hipGetErrorString(e));
}

int32_t check_ref_shape(int32_t out_f, int32_t in_f, const char* who) {
  if (out_f < 1) return fail(PMPD_EINVAL, "%s: out_features %d < 1", who, out_f);
  if (in_f < kGroup || in_f % kGroup) return fail(PMPD_EINVAL, "%s: in_features %d is not a positive multiple of %d", who, in_f, kGroup);
  if (in_f > kRefMaxIn) return fail(PMPD_EINVAL, "%s: in_features %d above %d", who, in_f, kRefMaxIn);
  return PMPD_OK;
}

int32_t check_ref_layers(const pmpd_fp16_layer_t* layers, int32_t n, const char* who) {
  if (!layers) return fail(PMPD_EINVAL, "%s: NULL layers", who);
  if (n < 1) return fail(PMPD_EINVAL, "%s: n_layers %d < 1", who, n);
  for (int i = 0; i < n; ++i) {
    int32_t rc = check_ref_shape(layers[i].out_features, layers[i].in_features, who);
    if (rc) return rc;
    if (!layers[i].weight) return fail(PMPD_EINVAL, "%s: layer %d has a NULL weight pointer", who, i);
    if (reinterpret_cast<uintptr_t>(layers[i].weight) % 16) return fail(PMPD_EALIGN, "%s: layer %d weight not 16-byte aligned", who, i);
  }
  return PMPD_OK;
}

size_t ref_items(const pmpd_fp16_layer_t* layers, int32_t n) {
  size_t k = 0;
  for (int i = 0; i < n; ++i) k += (layers[i].out_features + kRefRowsPerWg - 1) / kRefRowsPerWg;
  return k;
}

}  // namespace
}  // namespace pmpd

struct pmpd_fp16_stack {
  const pmpd::RefDesc* d_layers = nullptr;
  const pmpd::RefItem* d_items = nullptr;
  size_t n_items = 0;
  int max_in = 0;
};

using namespace pmpd;

extern "C" {

int32_t pmpd_fp16_gemv(const void* weight, int32_t out_features, int32_t in_features, const void* x, float* y,
                       void* stream) {
  int32_t rc = check_ref_shape(out_features, in_features, "pmpd_fp16_gemv");
  if (rc) return rc;
  if (!weight || !x || !y) return fail(PMPD_EINVAL, "pmpd_fp16_gemv: NULL argument");
  if (reinterpret_cast<uintptr_t>(weight) % 16 || reinterpret_cast<uintptr_t>(x) % 16)
    return fail(PMPD_EALIGN, "pmpd_fp16_gemv: weight and x must be 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(y) % 4) return fail(PMPD_EALIGN, "pmpd_fp16_gemv: y not 4-byte aligned");
  RefDesc L{weight, 0, 0, out_features, in_features};
  const unsigned grid = (out_features + kRefRowsPerWg - 1) / kRefRowsPerWg;
  fp16_layer_kernel<<<grid, kRefWaves * 64, static_cast<size_t>(in_features) * 2, static_cast<hipStream_t>(stream)>>>(
      L, static_cast<const _Float16*>(x), y);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return ref_hip_fail(e, "pmpd_fp16_gemv launch");
  return PMPD_OK;
}

int32_t pmpd_fp16_stack_workspace_size(const pmpd_fp16_layer_t* layers, int32_t n_layers, size_t* bytes) {
  int32_t rc = check_ref_layers(layers, n_layers, "pmpd_fp16_stack_workspace_size");
  if (rc) return rc;
  if (!bytes) return fail(PMPD_EINVAL, "pmpd_fp16_stack_workspace_size: NULL bytes");
  *bytes = ref_align(static_cast<size_t>(n_layers) * sizeof(RefDesc)) + ref_align(ref_items(layers, n_layers) * sizeof(RefItem));
  return PMPD_OK;
}

int32_t pmpd_fp16_stack_create(const pmpd_fp16_layer_t* layers, int32_t n_layers, const int64_t* x_offset,
                               const int64_t* y_offset, void* workspace, size_t workspace_bytes,
                               pmpd_fp16_stack_t** out) {
  int32_t rc = check_ref_layers(layers, n_layers, "pmpd_fp16_stack_create");
  if (rc) return rc;
  if (!x_offset || !y_offset || !workspace || !out) return fail(PMPD_EINVAL, "pmpd_fp16_stack_create: NULL argument");
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(PMPD_EALIGN, "pmpd_fp16_stack_create: workspace not 256-byte aligned");
  for (int i = 0; i < n_layers; ++i) {
    if (x_offset[i] < 0 || x_offset[i] % 8) return fail(PMPD_EALIGN, "pmpd_fp16_stack_create: x_offset[%d] must be a non-negative multiple of 8", i);
    if (y_offset[i] < 0) return fail(PMPD_EINVAL, "pmpd_fp16_stack_create: y_offset[%d] is negative", i);
  }
  std::vector<RefDesc> descs;
  std::vector<RefItem> items;
  int max_in = 0;
  for (int i = 0; i < n_layers; ++i) {
    descs.push_back(RefDesc{layers[i].weight, x_offset[i], y_offset[i], layers[i].out_features, layers[i].in_features});
    for (int r = 0; r < layers[i].out_features; r += kRefRowsPerWg) items.push_back(RefItem{i, r});
    max_in = std::max(max_in, layers[i].in_features);
  }
  const size_t need = ref_align(descs.size() * sizeof(RefDesc)) + ref_align(items.size() * sizeof(RefItem));
  if (workspace_bytes < need) return fail(PMPD_ESIZE, "pmpd_fp16_stack_create: workspace %zu bytes, need %zu", workspace_bytes, need);
  char* w = static_cast<char*>(workspace);
  char* wi = w + ref_align(descs.size() * sizeof(RefDesc));
  hipError_t e = hipMemcpy(w, descs.data(), descs.size() * sizeof(RefDesc), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMemcpy(wi, items.data(), items.size() * sizeof(RefItem), hipMemcpyHostToDevice);
  if (e != hipSuccess) return ref_hip_fail(e, "pmpd_fp16_stack_create copy");
  auto* st = new pmpd_fp16_stack;
  st->d_layers = reinterpret_cast<const RefDesc*>(w);
  st->d_items = reinterpret_cast<const RefItem*>(wi);
  st->n_items = items.size();
  st->max_in = max_in;
  *out = st;
  return PMPD_OK;
}

void pmpd_fp16_stack_destroy(pmpd_fp16_stack_t* stack) { delete stack; }

int32_t pmpd_fp16_step(const pmpd_fp16_stack_t* stack, const void* x_base, float* y_base, void* stream) {
  if (!stack || !x_base || !y_base) return fail(PMPD_EINVAL, "pmpd_fp16_step: NULL argument");
  if (reinterpret_cast<uintptr_t>(x_base) % 16) return fail(PMPD_EALIGN, "pmpd_fp16_step: x_base not 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(y_base) % 4) return fail(PMPD_EALIGN, "pmpd_fp16_step: y_base not 4-byte aligned");
  fp16_stack_kernel<<<static_cast<unsigned>(stack->n_items), kRefWaves * 64, static_cast<size_t>(stack->max_in) * 2,
                      static_cast<hipStream_t>(stream)>>>(stack->d_layers, stack->d_items,
                                                          static_cast<const _Float16*>(x_base), y_base);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return ref_hip_fail(e, "pmpd_fp16_step launch");
  return PMPD_OK;
}

}  // extern "C"
