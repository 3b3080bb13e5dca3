/*
 * pmpd.h -- C ABI of the MI355X (gfx950) library for the decode-phase linear layers of
 * Progressive Mixed-Precision Decoding (PMPD).
 *
 * The paper (Section 4.2, Algorithm 1 deployment stage) decodes token i with the model
 * variant m_p whose weight precision p is chosen per step by a precision-switching
 * scheduler; all variants are read from ONE nested weight store so that switching costs
 * no extra memory (Section 2.1; Section 5 "PMPD Implementation Details").  At batch 1 the
 * linear layers are memory-bound matrix-vector products (Section 1; Section 5.2 "GPU
 * Evaluation"), so a b-bit step should move only b bits per weight.
 *
 * This library implements that path for b in {4,3,2}:
 *     q_b = q4 >> (4-b)                       nested code (top b bits of the 4-bit code)
 *     W_b = a_g + s_g * 2^(4-b) * (q_b + 0.5) group g = 128 consecutive input features
 *     y   = W_b x                             fp16 x, fp32 accumulation, fp32 y
 * The weights are stored once as 4 bit-planes (plane 0 = most significant bit); a b-bit
 * pass reads planes 0..b-1 and the (scale, min) words only.
 *
 * Conventions
 *   - Every function returns an int32 status: PMPD_OK or a negative PMPD_E* code;
 *     pmpd_last_error() gives a thread-local message for the last failure.
 *   - "host" / "device" on a pointer says where the memory lives.  The library never
 *     allocates, frees or keeps device memory: every device buffer is the caller's and
 *     must outlive the calls that use it.  Objects returned by *_create are host objects
 *     owned by the library until *_destroy.
 *   - Device work is enqueued on the caller's HIP stream (passed as void*, NULL = the
 *     default stream) and is asynchronous; there is no hidden synchronisation.
 *   - Activations must be finite fp16 numbers (subnormals included).  With Inf or NaN among them the
 *     outputs are unspecified; no call reads or writes out of bounds because of them.
 *   - Arguments are validated on the host before anything is launched, so every error
 *     path can be exercised without a GPU.  There is no CPU fallback: a call that needs
 *     the GPU fails with PMPD_EHIP when none is usable.
 *
 * Storage format ("tile-plane"), shared by pack, unpack and the kernels:
 *   rows padded to a multiple of 64; row r -> tile T = r/64, position rr = r%64 = 16*t + j
 *   (t 0..3, j 0..15); feature i -> group g = i/128, position e = i%128 = 32*kb + 8*v + c
 *   (kb 0..3, v 0..3, c 0..7); n = c/2 + 4*(c%2); G = in_features/128.
 *   plane k: uint32 words; weight (r,i) is bit
 *              4n+1, 4n+3, 4n, 4n+2            for v = 0..3 when k is 0 or 2
 *              4n, 4n+2, (4n+31) mod 32, 4n+1  for v = 0..3 when k is 1 or 3
 *            of word ((T*G + g)*64 + 16*kb + j)*4 + t      -> plane_bytes = padded_rows*in/8
 *   scale_min: uint32 word (T*G + g)*64 + 4*j + t = fp16 scale (low half) | fp16 min (high half)
 *   A wave of 64 lanes reads one contiguous 1 KiB chunk per (tile, group, plane): lane 16*kb + j
 *   gets, in word t, 32 columns of row 16*t + j.  Merging the words of planes (0,1) and of planes
 *   (2,3) with one bit-select and a mask gives words of eight nibbles 00pp' (the two bits of a
 *   pair): operands of the gfx950 fp4 matrix instruction as they stand, and two shifts away from
 *   4-bit codes for the fp16 path.
 */
#ifndef PMPD_H_
#define PMPD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PMPD_OK 0
#define PMPD_EINVAL (-1)  /* null pointer, bad shape, bit-width outside {2,3,4}, bad count */
#define PMPD_EALIGN (-2)  /* a buffer is not aligned as documented */
#define PMPD_ESCHED (-3)  /* schedule violates Eq. 2-3 (range / precedence) */
#define PMPD_EHIP (-4)    /* HIP runtime failure or no usable GPU */
#define PMPD_ESIZE (-5)   /* caller-provided buffer too small */

#define PMPD_GROUP 128     /* input features per quantisation group */
#define PMPD_ROW_TILE 64   /* rows per storage tile (one per lane of a wave) */
#define PMPD_MAX_BATCH 8   /* rows of X up to which pmpd_gemm takes its skinny path */
#define PMPD_MAX_STACK_BATCH 16 /* rows of X up to which pmpd_batch_step takes its skinny path */
#define PMPD_MAX_ROWS 65536 /* rows of X accepted by pmpd_gemm / pmpd_prefill_step */

/* One packed linear layer.  Plain data; the pointers are the caller's (device memory for
 * pmpd_gemv / pmpd_gemm / stacks, host memory for pmpd_unpack).  planes[k] must be 16-byte
 * aligned, scale_min 4-byte aligned.  planes[b..3] are never read by a b-bit call and may be
 * NULL for it. */
typedef struct pmpd_layer {
  int32_t out_features;
  int32_t in_features; /* multiple of 128 */
  int32_t group_size;  /* must be 128 */
  int32_t reserved;    /* must be 0 */
  const void* planes[4];
  const void* scale_min;
} pmpd_layer_t;

typedef struct pmpd_stack pmpd_stack_t;       /* a list of layers prepared for one-launch decode steps */
typedef struct pmpd_schedule pmpd_schedule_t; /* precision-switching schedule <P, S> */

/* Error reporting (library plumbing, no counterpart in the paper): a fixed English name for a
 * status code, and the message of the calling thread's last failed call (valid until its next call). */
const char* pmpd_strerror(int32_t status);
const char* pmpd_last_error(void);

/* Bytes of one plane and of the scale_min array for a layer of this shape: the nested store of
 * Section 2.1 / Section 5 "PMPD Implementation Details" holds every precision in the memory of the
 * highest one (4 planes of out*in/8 bytes, rows padded to 64) plus one (scale, min) word per group. */
int32_t pmpd_packed_size(int32_t out_features, int32_t in_features, int32_t group_size,
                         size_t* plane_bytes, size_t* scale_min_bytes);

/* Offline stage (Algorithm 1, line 1 hands over quantised variants; this turns 4-bit codes
 * into the nested store).  All pointers host.  q4: row-major [out][in], values 0..15.
 * scale, minv: fp16 bit patterns, row-major [out][in/128].  planes[k], scale_min: host
 * buffers of the sizes pmpd_packed_size reports; fully overwritten (padding rows zero). */
int32_t pmpd_pack(const uint8_t* q4, const uint16_t* scale, const uint16_t* minv, int32_t out_features,
                  int32_t in_features, int32_t group_size, void* const planes[4], void* scale_min);

/* Host inverse of pmpd_pack for the top b planes: qb_out[r][i] = q4[r][i] >> (4-b), b in 1..4: the
 * lower-precision model is a prefix of the stored one (Section 2.1, nested quantisation; Section 5
 * "PMPD Implementation Details").  Reads host_layer->planes[0..b-1] only.  All pointers host. */
int32_t pmpd_unpack(const pmpd_layer_t* host_layer, int32_t b, uint8_t* qb_out);

/* y = W_b x for one layer (the decode-phase linear layer, Algorithm 1 line 16).
 * x: device, fp16 [in], 16-byte aligned.  y: device, fp32 [out].  b in {2,3,4}. */
int32_t pmpd_gemv(const pmpd_layer_t* layer, int32_t b, const void* x, float* y, void* stream);

/* Y[j][r] = sum_i W_b[r][i] X[j][i] for 1 <= m <= PMPD_MAX_ROWS.
 * m <= PMPD_MAX_BATCH: memory-bound path (the one pmpd_gemv takes), the weights are read once and
 *   codes and activations enter the matrix cores exactly (fp32 accumulation).
 * PMPD_MAX_BATCH < m <= PMPD_MAX_STACK_BATCH: still read once and exact: the 4-bit codes meet the fp16
 *   activations on the fp16 matrix cores as fp16 subnormals (fp32 accumulation).
 * m >  PMPD_MAX_STACK_BATCH: the compute-bound prefill shape (Section 4.1: prefill runs at its own,
 *   higher precision of the same store): the weights are dequantised to fp16 (one rounding) and
 *   the contraction runs on the matrix cores with fp32 accumulation.
 * X: device, fp16 row-major [m][in], 16-byte aligned.  Y: device, fp32 row-major [m][out]. */
int32_t pmpd_gemm(const pmpd_layer_t* layer, int32_t b, const void* X, int32_t m, float* Y, void* stream);

/* ---- a stack of layers decoded with one launch per step --------------------------------- *
 * The paper observes that per-kernel CPU launch work becomes the bottleneck once the layers
 * are this fast (Section 5.2 "GPU Evaluation"); a stack runs every linear layer of a decode
 * step in one launch.  Layer l reads x_base + x_offset[l] (fp16 elements, offset multiple of 8)
 * and writes y_base + y_offset[l] (fp32 elements).  The layers are independent of each other.
 * The stack's device-side tables live in a caller-provided device workspace of at least
 * pmpd_stack_workspace_size() bytes (256-byte aligned), which must stay untouched while the
 * stack exists.  pmpd_stack_create copies the tables there synchronously. */
int32_t pmpd_stack_workspace_size(const pmpd_layer_t* layers, int32_t n_layers, size_t* bytes);
int32_t pmpd_stack_create(const pmpd_layer_t* layers, int32_t n_layers, const int64_t* x_offset,
                          const int64_t* y_offset, void* workspace, size_t workspace_bytes,
                          pmpd_stack_t** out);
void pmpd_stack_destroy(pmpd_stack_t* stack);

/* Launch shape of pmpd_decode_step on this stack at bit-width b (chosen by pmpd_stack_create from
 * the number of row tiles and the row lengths; it affects speed and summation order, never which
 * planes are read):
 *   0  workgroup = 4 waves x 1 tile each, whole K     1  4 waves on 1 tile, K split 4 ways
 *   2  4 waves on 2 tiles, K split 2 ways            3  8 waves on 1 tile, K split 8 ways
 *   4  16 waves on 1 tile, K split 16 ways
 * pmpd_stack_variant reads it (so that a test can state which shape it checked, and a benchmark
 * which one it timed); pmpd_stack_set_variant overrides it for later steps on this stack (tuning
 * and tests; every shape computes the linear layers of Algorithm 1 line 16 for any stack).  Host only. */
int32_t pmpd_stack_variant(const pmpd_stack_t* stack, int32_t b, int32_t* variant);
int32_t pmpd_stack_set_variant(pmpd_stack_t* stack, int32_t b, int32_t variant);

/* One decode step: every layer of the stack at bit-width b, one kernel launch. */
int32_t pmpd_decode_step(const pmpd_stack_t* stack, int32_t b, const void* x_base, float* y_base,
                         void* stream);

/* m tokens through every layer of the stack in one launch:
 *     Y_l[j][r] = sum_i W_b,l[r][i] X_l[j][i],  j < m,  for every layer l,
 * X_l = x_base + m*x_offset[l] (fp16 row-major [m][in_l]), Y_l = y_base + m*y_offset[l] (fp32
 * row-major [m][out_l]).  m == 1 is pmpd_decode_step; 2 <= m <= PMPD_MAX_STACK_BATCH reads and unpacks
 * the weights once for all m vectors (skinny batches; the paper itself stays at batch 1, Section 5.2):
 * 3 to 8 vectors (3, 4 at b = 4) enter the int8 matrix cores as three base-256 digits of a 23-bit fixed-point
 * number per group of 128 (values within 2^-11 of the group's largest are exact, smaller ones are rounded at
 * 2^-23 of it), the codes exactly, with int32 sums; 9 to 16 vectors (from 5 at b = 4) go to the fp16 matrix
 * cores as they are, against the 4-bit codes as fp16 subnormals (exact products, fp32 sums);
 * larger m is the compute-bound prefill shape on the matrix cores (Algorithm 1 line 10, Section 4.1).
 * pmpd_prefill_step is the same call under the paper's name for that phase. */
int32_t pmpd_batch_step(const pmpd_stack_t* stack, int32_t b, const void* x_base, int32_t m, float* y_base,
                        void* stream);
int32_t pmpd_prefill_step(const pmpd_stack_t* stack, int32_t b, const void* x_base, int32_t m, float* y_base,
                          void* stream);

/* ---- precision-switching schedule (Section 4.2, Eq. 1-3; Algorithm 1 lines 14 and 20) ----- *
 * precisions[0..n-1] strictly decreasing bit-widths; st[j] = index of the first decode step
 * run at precisions[j].  Requirements: st[0] == 0 (decoding starts at the allocated decode
 * precision), 0 <= st[j] <= max_steps, st non-decreasing (a higher precision never starts after
 * a lower one, Eq. 3).  st[j] == max_steps means "never reached".  Violations -> PMPD_ESCHED. */
int32_t pmpd_schedule_create(const int32_t* precisions, const int32_t* st, int32_t n, int32_t max_steps,
                             pmpd_schedule_t** out);
void pmpd_schedule_destroy(pmpd_schedule_t* schedule);
/* Bit-width of decode step `step` (>= 0): the lowest precision whose switch point is <= step. */
int32_t pmpd_schedule_bits(const pmpd_schedule_t* schedule, int32_t step, int32_t* b_out);
/* Mean bit-width over steps 0..n_steps-1 (Section 5 "Baselines"); negative on error. */
double pmpd_schedule_avg_bits(const pmpd_schedule_t* schedule, int32_t n_steps);

/* ---- static scheduler: offline search for <P, S> (Section 4.3; Algorithm 1 line 4) ---------- *
 * Candidate switch points: points[k] = round(k * max_steps / (n_points - 1)), k = 0 .. n_points-1
 * (0, OL/(N-1), ..., OL; halves round up).  2 <= n_points <= max_steps + 1. */
int32_t pmpd_schedule_grid(int32_t max_steps, int32_t n_points, int32_t* points);
/* Number of progressive schedules: sum over r of C(max_steps, r) * C(n_precisions - 1, r); -1 on error. */
int64_t pmpd_schedule_count(int32_t max_steps, int32_t n_precisions);
/* Quality of a schedule as the caller measures it (the paper: mean task score over a validation
 * set); called on the host, higher is better. */
typedef double (*pmpd_quality_fn)(const int32_t* precisions, const int32_t* st, int32_t n, void* user);
/* Among the schedules with st[0] = 0, st non-decreasing and every st[j] on the candidate grid whose
 * quality is >= q_ref - eps (Eq. 2), the one with the fewest high-precision tokens (Eq. 1): lowest
 * average bit-width over max_steps steps, ties to the lexicographically smallest st.  quality() is
 * only called for schedules that would beat the best one found so far; *evaluated_out counts the
 * calls.  PMPD_ESCHED when no schedule on the grid reaches the quality bar. */
int32_t pmpd_schedule_search(const int32_t* precisions, int32_t n, int32_t max_steps, int32_t n_points,
                             pmpd_quality_fn quality, void* user, double q_ref, double eps, int32_t* st_out,
                             double* avg_bits_out, int64_t* evaluated_out);

/* Steps step0 .. step0+n_steps-1 of a decode run, each at the schedule's bit-width (which must
 * be in {2,3,4}).  Step k reads x_base + (k-step0)*x_step_stride and writes
 * y_base + (k-step0)*y_step_stride (strides in elements; 0 reuses the same buffers). */
int32_t pmpd_decode_run(const pmpd_stack_t* stack, const pmpd_schedule_t* schedule, int32_t step0,
                        int32_t n_steps, const void* x_base, int64_t x_step_stride, float* y_base,
                        int64_t y_step_stride, void* stream);

/* ---- a decode step in dependency order, one launch ------------------------------------------ *
 * In a real decoder the linear layers of a step depend on each other ((q,k,v) -> o -> (up,gate) ->
 * down, block after block); launched one kernel per stage, the step is bound by launch overhead,
 * which the paper observes for its own kernels and leaves to future work (Section 5.2 "GPU
 * Evaluation").  Here the whole step is one cooperative launch: the layers of the stack are
 * assigned to stages, the workgroups stay resident and take their tiles stage after stage; a tile
 * waits only for the outputs it reads (every output word counts the partial sums added to it), and
 * the weights of a workgroup's next tile are requested before it waits for that tile's inputs.
 * chain[l] (host, one per layer of the stack): stage of layer l (layers of one stage are independent);
 * source = -1: the layer reads x_base + x_offset[l] as in pmpd_decode_step; source = k: it reads
 * fp16(gain * y_k), the output of layer k of an earlier stage (out_features(k) == in_features(l),
 * y_offset[k] a multiple of 4); gain stands for the elementwise glue between the layers, which is
 * not part of this library.  Every layer still writes its full fp32 output at y_base + y_offset[l].
 * Where a layer's rows are long enough to be split over workgroups, the parts meet in 64-bit
 * fixed-point sums (32 fractional bits, integer atomic adds: the same bits whatever the order of
 * arrival).  Each part's sum is clamped to +-(2^21 - 1) (a NaN counts as the lower bound); sums of
 * that size do not occur with fp16 activations of a decoder and weights below 1.  A layer whose
 * rows are not split passes its fp32 outputs on unchanged.
 * The tables and sums (8 bytes per output of the stack) live in a caller-provided device
 * workspace (256-byte aligned, untouched while the object exists); calls on one object must not
 * overlap.  y_base must be 16-byte aligned.
 * The wait for inputs is bounded: if it runs out (it cannot while the launch is cooperative,
 * unless the limit is set very low) the step still ends and pmpd_ordered_status reports it. */
typedef struct pmpd_chain {
  int32_t stage;
  int32_t source;
  float gain;
} pmpd_chain_t;
typedef struct pmpd_ordered pmpd_ordered_t;
int32_t pmpd_ordered_workspace_size(const pmpd_stack_t* stack, const pmpd_chain_t* chain, size_t* bytes);
int32_t pmpd_ordered_create(const pmpd_stack_t* stack, const pmpd_chain_t* chain, void* workspace,
                            size_t workspace_bytes, pmpd_ordered_t** out); /* the stack must outlive it */
void pmpd_ordered_destroy(pmpd_ordered_t* ordered);
int32_t pmpd_ordered_step(const pmpd_ordered_t* ordered, int32_t b, const void* x_base, float* y_base,
                          void* stream);
/* Synchronous: *timed_out = 1 if a wait for inputs ran out since the last call (then cleared). */
int32_t pmpd_ordered_status(const pmpd_ordered_t* ordered, int32_t* timed_out);
/* Polls per wait before it gives up (default 2^20, about a second). */
int32_t pmpd_ordered_set_spin_limit(pmpd_ordered_t* ordered, uint32_t polls);

/* ---- learned scheduler: forward pass (Section 4.3 "Task-Agnostic Learned Scheduler"; Appendix A.1.1) *
 * Run once per prompt between prefill and decoding (Algorithm 1, deployment stage):
 *     p = softmax_t(q . K_t / sqrt(d_k)),  O = sum_t p_t V_t,
 *     probs = softmax(W2 relu(W1 O + b1) + b2),  class = first index of the largest probability;
 * class c stands for candidate switch point c of the grid of pmpd_schedule_grid with n_classes points.
 * K: device fp16 [T][d_k], V: device fp16 [T][d_v] (the key / value cache of one attention block, heads
 * side by side), both 16-byte aligned; d_k, d_v multiples of 8, d_k <= 16384, d_v <= 65536; 1 <= T <= 2^22;
 * hidden <= 65536; 2 <= n_classes <= 1024.  Parameters: device fp32, row-major, w1 16-byte aligned.
 * Outputs (device): probs fp32 [n_classes], cls int32 [1], context = O fp32 [d_v] or NULL.  All arithmetic
 * in fp32 with fixed reduction orders.  workspace: device, 256-byte aligned, pmpd_learned_workspace_size
 * bytes, free for reuse once the call's work on the stream has finished.  Asynchronous like the rest. */
typedef struct pmpd_learned {
  int32_t d_k, d_v, hidden, n_classes;
  const float* query; /* [d_k] */
  const float* w1;    /* [hidden][d_v] */
  const float* b1;    /* [hidden] */
  const float* w2;    /* [n_classes][hidden] */
  const float* b2;    /* [n_classes] */
} pmpd_learned_t;
int32_t pmpd_learned_workspace_size(const pmpd_learned_t* net, int32_t T, size_t* bytes);
int32_t pmpd_learned_forward(const pmpd_learned_t* net, const void* K, const void* V, int32_t T, void* workspace,
                             size_t workspace_bytes, float* context, float* probs, int32_t* cls, void* stream);
/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid it): pmpd_learned_forward with its work area inside the library, a device
 * array of PMPD_LEARNED_STATIC_BYTES that every GPU the library runs on holds until the process ends.
 * The call itself calls no hipMalloc, hipFree or other allocating routine; inputs and
 * outputs are still the caller's and everything else is as for pmpd_learned_forward, whose results it
 * reproduces bit for bit.  A call whose pmpd_learned_workspace_size exceeds PMPD_LEARNED_STATIC_BYTES
 * is refused with PMPD_ESIZE (d_v = 4096: T up to about 500 000).  All calls on one GPU share the one
 * work area: calls that overlap there (different streams, different threads) race and must be
 * serialised by the caller; calls in stream order on one stream are safe, and nothing a call reads of
 * the work area is left over from an earlier call. */
#define PMPD_LEARNED_STATIC_BYTES (4u << 20)
int32_t pmpd_learned_forward_static(const pmpd_learned_t* net, const void* K, const void* V, int32_t T, float* context,
                                    float* probs, int32_t* cls, void* stream);

/* Two-precision schedule from a predicted class: `high` bits for steps 0 .. points[cls]-1 and `low` bits
 * from step points[cls] on, points = pmpd_schedule_grid(max_steps, n_points) (host only). */
int32_t pmpd_schedule_from_class(int32_t high, int32_t low, int32_t cls, int32_t max_steps, int32_t n_points,
                                 pmpd_schedule_t** out);

/* ---- unquantised fp16 reference --------------------------------------------------------- *
 * The paper states its linear-layer speedups relative to fp16 kernels on the same device
 * (Section 5.2 "GPU Evaluation", Table 3).  These calls are that reference on this device:
 * y = W x with W fp16 [out][in] row-major (device, 16-byte aligned, in_features a multiple of
 * 128 and at most 32768), x fp16, fp32 accumulation, fp32 y; 2 bytes per weight are read, once.
 * pmpd_fp16_gemv runs one layer; a pmpd_fp16_stack_t runs a list of layers in one launch with the
 * same conventions as pmpd_stack_t (tables in a caller-provided 256-byte aligned device workspace,
 * per-layer offsets into x_base in fp16 elements, multiples of 8, and into y_base in fp32 elements). */
typedef struct pmpd_fp16_layer {
  int32_t out_features;
  int32_t in_features;
  const void* weight; /* device */
} pmpd_fp16_layer_t;
typedef struct pmpd_fp16_stack pmpd_fp16_stack_t;
int32_t pmpd_fp16_gemv(const void* weight, int32_t out_features, int32_t in_features, const void* x, float* y,
                       void* stream);
int32_t pmpd_fp16_stack_workspace_size(const pmpd_fp16_layer_t* layers, int32_t n_layers, size_t* bytes);
int32_t pmpd_fp16_stack_create(const pmpd_fp16_layer_t* layers, int32_t n_layers, const int64_t* x_offset,
                               const int64_t* y_offset, void* workspace, size_t workspace_bytes,
                               pmpd_fp16_stack_t** out);
void pmpd_fp16_stack_destroy(pmpd_fp16_stack_t* stack);
int32_t pmpd_fp16_step(const pmpd_fp16_stack_t* stack, const void* x_base, float* y_base, void* stream);

/* ---- measurement aid ------------------------------------------------------------------- *
 * Streams `bytes` (rounded down to a multiple of 128 MiB; *bytes_read says how many) of device memory
 * at src (16-byte aligned) through a read-only kernel: the HBM rate a plain read reaches on this
 * device, against which the decode kernels' effective rate is held (the paper's Section 5.2 reasons
 * about the same bound: decode linear layers are limited by weight transfers).  sink: device, 4 bytes. */
int32_t pmpd_read_stream(const void* src, size_t bytes, uint32_t* sink, size_t* bytes_read, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PMPD_H_ */
