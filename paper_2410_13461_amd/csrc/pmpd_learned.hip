// Forward pass of the learned precision-switching scheduler (Section 4.3 "Task-Agnostic Learned
// Scheduler"; Appendix A.1 "Learned Scheduler Details", A.1.1), gfx950.  Run once per prompt, after the prefill and before decoding
// (Algorithm 1, deployment stage):
//     scores_t = q . K_t / sqrt(D_k)      K fp16 [T][D_k]: key cache of one attention block
//     p        = softmax_t(scores)
//     O        = sum_t p_t V_t            V fp16 [T][D_v]: value cache of the same block
//     hid      = relu(W1 O + b1)          fp32 parameters, one hidden layer
//     probs    = softmax(W2 hid + b2)     class c = candidate switch point c of the static grid
// The work is two streaming passes over the caches (2 (D_k + D_v) T bytes: HBM-bound) and a tiny
// network; all arithmetic in fp32, every reduction in a fixed order (no atomics), so the result does
// not depend on the launch shape.  Five small kernels on the caller's stream, no host synchronisation:
//   scores  one wave per key row, 16-byte streaming loads, q in LDS
//   mix     grid = (512-column blocks of V) x (row chunks): every workgroup recomputes the softmax
//           statistics from the T scores (L2-resident), weighs its rows, writes one partial row
//   reduce  O[c] = sum over chunks, in a fixed order
//   hidden  one wave per hidden unit
//   head    one workgroup: logits, softmax, first index of the largest probability
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <mutex>

#include "pmpd_common.hpp"

// Work area of pmpd_learned_forward_static: the scores, the partial rows, O and the hidden layer of one
// call, for callers that may not allocate.  Every GPU the library runs on holds its own copy, at its
// own address, until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the address that kernels get is the one that call returns.
static __device__ __align__(256) unsigned char scratch[PMPD_LEARNED_STATIC_BYTES];

namespace pmpd {
namespace {

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kLsMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kLsMaxDevices] = {};

int32_t scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(PMPD_EHIP, "pmpd_learned_forward_static: hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kLsMaxDevices) return fail(PMPD_EHIP, "pmpd_learned_forward_static: device index %d outside 0..%d", dev, kLsMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(PMPD_EHIP, "pmpd_learned_forward_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return PMPD_OK;
}

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kLsThreads = 256;
constexpr int kLsWaves = 4;
constexpr int kLsMaxChunks = 128;
constexpr int kLsMinRowsPerChunk = 8;
constexpr int kLsMaxDk = 16384;   // q as fp32 in 64 KiB of LDS
constexpr int kLsMaxDv = 65536;
constexpr int kLsMaxHidden = 65536;
constexpr int kLsMaxClasses = 1024;
constexpr int kLsMaxT = 1 << 22;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, 64));
  return v;
}

__global__ __launch_bounds__(kLsThreads) void learned_scores_kernel(const h8* __restrict__ K, const float* __restrict__ q,
                                                                    int T, int d_k, float scale, float* __restrict__ s) {
  extern __shared__ __align__(16) float ql[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < d_k; i += kLsThreads) ql[i] = q[i];
  __syncthreads();
  const f4* q4 = reinterpret_cast<const f4*>(ql);
  const int n = d_k >> 3;
  for (int t = blockIdx.x * kLsWaves + wave; t < T; t += gridDim.x * kLsWaves) {
    const h8* row = K + static_cast<int64_t>(t) * n;
    float acc = 0.f;
#pragma unroll 4
    for (int c = lane; c < n; c += 64) {
      const h8 k = __builtin_nontemporal_load(row + c);
      const f4 a = q4[2 * c], b = q4[2 * c + 1];
      acc += static_cast<float>(k[0]) * a.x;
      acc += static_cast<float>(k[1]) * a.y;
      acc += static_cast<float>(k[2]) * a.z;
      acc += static_cast<float>(k[3]) * a.w;
      acc += static_cast<float>(k[4]) * b.x;
      acc += static_cast<float>(k[5]) * b.y;
      acc += static_cast<float>(k[6]) * b.z;
      acc += static_cast<float>(k[7]) * b.w;
    }
    acc = wave_sum(acc);
    if (lane == 0) s[t] = acc * scale;
  }
}

// Softmax statistics of s[0..T): every thread of the workgroup gets (max, 1 / sum exp(s - max)).
__device__ __forceinline__ void softmax_stats(const float* __restrict__ s, int T, float* sh, float& m, float& inv) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float v = -INFINITY;
  for (int t = tid; t < T; t += kLsThreads) v = fmaxf(v, s[t]);
  v = wave_max(v);
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  m = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
  __syncthreads();
  float l = 0.f;
  for (int t = tid; t < T; t += kLsThreads) l += expf(s[t] - m);
  l = wave_sum(l);
  if (lane == 0) sh[wave] = l;
  __syncthreads();
  inv = 1.f / (((sh[0] + sh[1]) + sh[2]) + sh[3]);
}

__device__ __forceinline__ void axpy8(float (&acc)[8], float w, const h8& v) {
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] += w * static_cast<float>(v[i]);
}

__global__ __launch_bounds__(kLsThreads) void learned_mix_kernel(const h8* __restrict__ V, const float* __restrict__ s, int T,
                                                                 int d_v, int rows_per_chunk, float* __restrict__ partial) {
  __shared__ float sh[kLsWaves];
  __shared__ __align__(16) float comb[kLsWaves][64][8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float m, inv;
  softmax_stats(s, T, sh, m, inv);
  const int nv = d_v >> 3;
  const int cc = blockIdx.x * 64 + lane;
  const int t0 = blockIdx.y * rows_per_chunk, t1 = min(T, t0 + rows_per_chunk);
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (cc < nv) {
    const h8* col = V + cc;
    int t = t0 + wave;
    for (; t + 3 * kLsWaves < t1; t += 4 * kLsWaves) {  // four rows in flight per wave
      const h8 v0 = __builtin_nontemporal_load(col + static_cast<int64_t>(t) * nv);
      const h8 v1 = __builtin_nontemporal_load(col + static_cast<int64_t>(t + kLsWaves) * nv);
      const h8 v2 = __builtin_nontemporal_load(col + static_cast<int64_t>(t + 2 * kLsWaves) * nv);
      const h8 v3 = __builtin_nontemporal_load(col + static_cast<int64_t>(t + 3 * kLsWaves) * nv);
      axpy8(acc, expf(s[t] - m) * inv, v0);
      axpy8(acc, expf(s[t + kLsWaves] - m) * inv, v1);
      axpy8(acc, expf(s[t + 2 * kLsWaves] - m) * inv, v2);
      axpy8(acc, expf(s[t + 3 * kLsWaves] - m) * inv, v3);
    }
    for (; t < t1; t += kLsWaves) axpy8(acc, expf(s[t] - m) * inv, __builtin_nontemporal_load(col + static_cast<int64_t>(t) * nv));
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) comb[wave][lane][i] = acc[i];
  __syncthreads();
  if (wave == 0 && cc < nv) {
    f4 lo, hi;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      lo[i] = ((comb[0][lane][i] + comb[1][lane][i]) + comb[2][lane][i]) + comb[3][lane][i];
      hi[i] = ((comb[0][lane][4 + i] + comb[1][lane][4 + i]) + comb[2][lane][4 + i]) + comb[3][lane][4 + i];
    }
    f4* dst = reinterpret_cast<f4*>(partial + static_cast<int64_t>(blockIdx.y) * d_v + static_cast<int64_t>(cc) * 8);
    dst[0] = lo;
    dst[1] = hi;
  }
}

// O[c] = sum of the chunks' partial rows.  A workgroup takes 64 columns; its four waves each add every
// fourth chunk in ascending order (eight loads in flight), then the four sums are added in wave order.
__global__ __launch_bounds__(kLsThreads) void learned_reduce_kernel(const float* __restrict__ partial, int n_chunks, int d_v,
                                                                    float* __restrict__ O, float* __restrict__ context) {
  __shared__ float part[kLsWaves][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float acc = 0.f;
  if (c < d_v) {
    const float* p = partial + c;
    int k = wave;
    for (; k + 7 * kLsWaves < n_chunks; k += 8 * kLsWaves) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = p[static_cast<int64_t>(k + u * kLsWaves) * d_v];
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += v[u];
    }
    for (; k < n_chunks; k += kLsWaves) acc += p[static_cast<int64_t>(k) * d_v];
  }
  part[wave][lane] = acc;
  __syncthreads();
  if (wave == 0 && c < d_v) {
    const float o = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
    O[c] = o;
    if (context) context[c] = o;
  }
}

__global__ __launch_bounds__(kLsThreads) void learned_hidden_kernel(const float* __restrict__ W1, const float* __restrict__ b1,
                                                                    const float* __restrict__ O, int hidden, int d_v,
                                                                    float* __restrict__ hid) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * kLsWaves + wave;
  if (j >= hidden) return;
  const f4* w = reinterpret_cast<const f4*>(W1 + static_cast<int64_t>(j) * d_v);
  const f4* o = reinterpret_cast<const f4*>(O);
  float acc = 0.f;
#pragma unroll 4
  for (int c = lane; c < (d_v >> 2); c += 64) {
    const f4 a = w[c], b = o[c];
    acc += a.x * b.x;
    acc += a.y * b.y;
    acc += a.z * b.z;
    acc += a.w * b.w;
  }
  acc = wave_sum(acc);
  if (lane == 0) hid[j] = fmaxf(acc + b1[j], 0.f);
}

__global__ __launch_bounds__(kLsThreads) void learned_head_kernel(const float* __restrict__ W2, const float* __restrict__ b2,
                                                                  const float* __restrict__ hid, int hidden, int n_classes,
                                                                  float* __restrict__ probs, int32_t* __restrict__ cls) {
  __shared__ float z[kLsMaxClasses];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int k = wave; k < n_classes; k += kLsWaves) {
    const float* w = W2 + static_cast<int64_t>(k) * hidden;
    float acc = 0.f;
    for (int j = lane; j < hidden; j += 64) acc += w[j] * hid[j];
    acc = wave_sum(acc);
    if (lane == 0) z[k] = acc + b2[k];
  }
  __syncthreads();
  if (tid == 0) {  // a handful of classes: one lane, one fixed order
    float m = z[0];
    for (int k = 1; k < n_classes; ++k) m = fmaxf(m, z[k]);
    float l = 0.f;
    for (int k = 0; k < n_classes; ++k) l += expf(z[k] - m);
    const float inv = 1.f / l;
    int best = 0;
    float pb = -1.f;
    for (int k = 0; k < n_classes; ++k) {
      const float p = expf(z[k] - m) * inv;
      probs[k] = p;
      if (p > pb) {  // strict: the first of equal probabilities wins
        pb = p;
        best = k;
      }
    }
    cls[0] = best;
  }
}

size_t ls_align(size_t v) { return (v + 255) / 256 * 256; }

int ls_chunks(int T) { return std::max(1, std::min(kLsMaxChunks, (T + kLsMinRowsPerChunk - 1) / kLsMinRowsPerChunk)); }

struct LsPlan {
  int n_chunks, rows_per_chunk;
  size_t off_s, off_partial, off_o, off_h, bytes;
};

LsPlan ls_plan(const pmpd_learned_t& net, int T) {
  LsPlan p;
  const int want = ls_chunks(T);
  p.rows_per_chunk = (T + want - 1) / want;
  p.n_chunks = (T + p.rows_per_chunk - 1) / p.rows_per_chunk;  // no empty chunk
  p.off_s = 0;
  p.off_partial = ls_align(static_cast<size_t>(T) * 4);
  p.off_o = p.off_partial + ls_align(static_cast<size_t>(p.n_chunks) * net.d_v * 4);
  p.off_h = p.off_o + ls_align(static_cast<size_t>(net.d_v) * 4);
  p.bytes = p.off_h + ls_align(static_cast<size_t>(net.hidden) * 4);
  return p;
}

int32_t check_net(const pmpd_learned_t* net, int32_t T, bool need_pointers, const char* who) {
  if (!net) return fail(PMPD_EINVAL, "%s: NULL network", who);
  if (net->d_k < 8 || net->d_k % 8 || net->d_k > kLsMaxDk) return fail(PMPD_EINVAL, "%s: d_k %d must be a multiple of 8 in 8..%d", who, net->d_k, kLsMaxDk);
  if (net->d_v < 8 || net->d_v % 8 || net->d_v > kLsMaxDv) return fail(PMPD_EINVAL, "%s: d_v %d must be a multiple of 8 in 8..%d", who, net->d_v, kLsMaxDv);
  if (net->hidden < 1 || net->hidden > kLsMaxHidden) return fail(PMPD_EINVAL, "%s: hidden %d outside 1..%d", who, net->hidden, kLsMaxHidden);
  if (net->n_classes < 2 || net->n_classes > kLsMaxClasses) return fail(PMPD_EINVAL, "%s: n_classes %d outside 2..%d", who, net->n_classes, kLsMaxClasses);
  if (T < 1 || T > kLsMaxT) return fail(PMPD_EINVAL, "%s: T %d outside 1..%d", who, T, kLsMaxT);
  if (need_pointers) {
    if (!net->query || !net->w1 || !net->b1 || !net->w2 || !net->b2) return fail(PMPD_EINVAL, "%s: NULL parameter pointer", who);
    if (reinterpret_cast<uintptr_t>(net->w1) % 16) return fail(PMPD_EALIGN, "%s: w1 not 16-byte aligned", who);
    if (reinterpret_cast<uintptr_t>(net->query) % 4 || reinterpret_cast<uintptr_t>(net->b1) % 4 ||
        reinterpret_cast<uintptr_t>(net->w2) % 4 || reinterpret_cast<uintptr_t>(net->b2) % 4)
      return fail(PMPD_EALIGN, "%s: fp32 parameters must be 4-byte aligned", who);
  }
  return PMPD_OK;
}

}  // namespace
}  // namespace pmpd

using namespace pmpd;

extern "C" {

int32_t pmpd_learned_workspace_size(const pmpd_learned_t* net, int32_t T, size_t* bytes) {
  int32_t rc = check_net(net, T, false, "pmpd_learned_workspace_size");
  if (rc) return rc;
  if (!bytes) return fail(PMPD_EINVAL, "pmpd_learned_workspace_size: NULL bytes");
  *bytes = ls_plan(*net, T).bytes;
  return PMPD_OK;
}

// The argument checks both entry points share (everything but the work area).
static int32_t check_forward_args(const pmpd_learned_t* net, const void* K, const void* V, int32_t T, const float* context,
                                  const float* probs, const int32_t* cls, const char* who) {
  int32_t rc = check_net(net, T, true, who);
  if (rc) return rc;
  if (!K || !V || !probs || !cls) return fail(PMPD_EINVAL, "%s: NULL argument", who);
  if (reinterpret_cast<uintptr_t>(K) % 16 || reinterpret_cast<uintptr_t>(V) % 16)
    return fail(PMPD_EALIGN, "%s: K and V must be 16-byte aligned", who);
  if (reinterpret_cast<uintptr_t>(probs) % 4 || reinterpret_cast<uintptr_t>(cls) % 4 || reinterpret_cast<uintptr_t>(context) % 4)
    return fail(PMPD_EALIGN, "%s: outputs must be 4-byte aligned", who);
  return PMPD_OK;
}

// The five launches, with the work area at `workspace` (device address, p.bytes long).  Every word
// of the work area that is read has been written by an earlier kernel of the same call.
static int32_t launch_forward(const pmpd_learned_t* net, const LsPlan& p, const void* K, const void* V, int32_t T, void* workspace,
                              float* context, float* probs, int32_t* cls, void* stream, const char* who) {
  char* w = static_cast<char*>(workspace);
  float* s = reinterpret_cast<float*>(w + p.off_s);
  float* partial = reinterpret_cast<float*>(w + p.off_partial);
  float* O = reinterpret_cast<float*>(w + p.off_o);
  float* hid = reinterpret_cast<float*>(w + p.off_h);
  hipStream_t st = static_cast<hipStream_t>(stream);

  const unsigned g1 = static_cast<unsigned>(std::min((T + kLsWaves - 1) / kLsWaves, 2048));
  learned_scores_kernel<<<g1, kLsThreads, static_cast<size_t>(net->d_k) * 4, st>>>(
      static_cast<const h8*>(K), net->query, T, net->d_k, 1.0f / std::sqrt(static_cast<float>(net->d_k)), s);
  const dim3 g2((net->d_v / 8 + 63) / 64, p.n_chunks);
  learned_mix_kernel<<<g2, kLsThreads, 0, st>>>(static_cast<const h8*>(V), s, T, net->d_v, p.rows_per_chunk, partial);
  learned_reduce_kernel<<<(net->d_v + 63) / 64, kLsThreads, 0, st>>>(partial, p.n_chunks, net->d_v, O, context);
  learned_hidden_kernel<<<(net->hidden + kLsWaves - 1) / kLsWaves, kLsThreads, 0, st>>>(net->w1, net->b1, O, net->hidden, net->d_v, hid);
  learned_head_kernel<<<1, kLsThreads, 0, st>>>(net->w2, net->b2, hid, net->hidden, net->n_classes, probs, cls);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(PMPD_EHIP, "%s launch: %s", who, hipGetErrorString(e));
  return PMPD_OK;
}

int32_t pmpd_learned_forward(const pmpd_learned_t* net, const void* K, const void* V, int32_t T, void* workspace,
                             size_t workspace_bytes, float* context, float* probs, int32_t* cls, void* stream) {
  int32_t rc = check_forward_args(net, K, V, T, context, probs, cls, "pmpd_learned_forward");
  if (rc) return rc;
  if (!workspace) return fail(PMPD_EINVAL, "pmpd_learned_forward: NULL argument");
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(PMPD_EALIGN, "pmpd_learned_forward: workspace not 256-byte aligned");
  const LsPlan p = ls_plan(*net, T);
  if (workspace_bytes < p.bytes) return fail(PMPD_ESIZE, "pmpd_learned_forward: workspace %zu bytes, need %zu", workspace_bytes, p.bytes);
  return launch_forward(net, p, K, V, T, workspace, context, probs, cls, stream, "pmpd_learned_forward");
}

int32_t pmpd_learned_forward_static(const pmpd_learned_t* net, const void* K, const void* V, int32_t T, float* context,
                                    float* probs, int32_t* cls, void* stream) {
  int32_t rc = check_forward_args(net, K, V, T, context, probs, cls, "pmpd_learned_forward_static");
  if (rc) return rc;
  const LsPlan p = ls_plan(*net, T);
  if (p.bytes > static_cast<size_t>(PMPD_LEARNED_STATIC_BYTES))
    return fail(PMPD_ESIZE, "pmpd_learned_forward_static: this call needs %zu bytes of work area, the built-in one holds %zu; use pmpd_learned_forward",
                p.bytes, static_cast<size_t>(PMPD_LEARNED_STATIC_BYTES));
  void* work = nullptr;
  rc = scratch_of_current_device(&work);
  if (rc) return rc;
  return launch_forward(net, p, K, V, T, work, context, probs, cls, stream, "pmpd_learned_forward_static");
}

int32_t pmpd_schedule_from_class(int32_t high, int32_t low, int32_t cls, int32_t max_steps, int32_t n_points,
                                 pmpd_schedule_t** out) {
  if (!out) return fail(PMPD_EINVAL, "pmpd_schedule_from_class: NULL out");
  if (n_points < 2 || n_points > 4096) return fail(PMPD_EINVAL, "pmpd_schedule_from_class: n_points %d outside 2..4096", n_points);
  if (cls < 0 || cls >= n_points) return fail(PMPD_EINVAL, "pmpd_schedule_from_class: class %d outside 0..%d", cls, n_points - 1);
  int32_t grid[4096];
  int32_t rc = pmpd_schedule_grid(max_steps, n_points, grid);
  if (rc) return rc;
  const int32_t P[2] = {high, low}, S[2] = {0, grid[cls]};
  return pmpd_schedule_create(P, S, 2, max_steps, out);
}

}  // extern "C"
