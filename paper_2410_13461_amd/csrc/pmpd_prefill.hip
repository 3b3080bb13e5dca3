// Prefill / large-batch linear layers on the matrix cores (gfx950):
//     Y[j][r] = sum_i W_b[r][i] X[j][i],   j < m  (m in the hundreds: the prompt tokens)
// The paper runs the prefill phase at a (higher) weight precision of the same nested store
// (Section 4.1; Algorithm 1, line 10) and notes that prefill is compute-bound (Section 1), so
// here the contraction goes to v_mfma_f32_16x16x32_f16 and the bit-plane unpack is amortised
// over a 256-token block of X.
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
// The weight is rounded to fp16 once (relative error 2^-11 per weight, about 3e-4 relative L2
// on y, inside the 1e-3 bar); the decode kernels keep exact codes instead because there the
// per-group scaling is free.
//
// Shape of the kernel.  A workgroup is four waves, one per SIMD, and it is alone on its compute unit; the grid is
// one round of the chip and every workgroup walks through its share of the work items (four row tiles x 256
// tokens each) as one sequence of groups, so that loads run ahead across item boundaries and only a workgroup's
// first item has a prologue.  Wave w
// owns row tile tile0 + w (64 weight rows) and all 256 tokens of the block: 16 x 4 accumulator blocks of
// 16 x 16, the 256 accumulation registers of a lane.  Per group of 128 columns it issues 256 MFMAs (4 K-steps
// x 16 token blocks x 4 row blocks) and dequantises its 128 weights per lane once, so the VALU work per MFMA
// is half of what a 128-token block would need.  The four waves share one X tile per group (256 tokens x 128
// columns, 64 KiB, double-buffered in LDS).
//
// One wave per SIMD has nobody to hide behind, so the instruction stream is laid out by hand.  Measured on
// gfx950: back-to-back independent 16x16x32 MFMAs issue every 16 cycles, and about two other instructions
// of the same wave fit between two of them without delaying the second; everything else costs time.  The
// stream is therefore MFMA, <= 2 VALU, MFMA, <= 2 VALU, ... with the whole of the remaining work cut into
// such pieces:
//   * the dequantisation of the operands of the NEXT K-step (28 units of one or two instructions per K-step),
//   * the merge of the plane words of the NEXT group into 4-bit codes (7 pieces per 16-row block, one row
//     block per K-step),
//   * one LDS read per token block, three blocks ahead of its use, with a counted wait,
//   * the global loads: the 16 loads of the next X tile spread over K-steps 0..2 (so that they have K-step 3
//     to land), the plane words of the group after next issued last, in K-step 3, into the registers the merge
//     has just finished with.  The end of a group waits until at most those last loads are outstanding: the
//     X tile is then complete, and plane words get a whole group to arrive.
// Register sets alternate with the parity of the group (the loop body is written out for both), so nothing
// is copied between groups.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "pmpd_common.hpp"
#include "pmpd_device.hpp"
#include "pmpd_prefill_deal.hpp"

namespace pmpd {

constexpr int kPfWaves = 4;             // waves (= 64-row tiles) per workgroup, one per SIMD
constexpr int kPfTokens = 256;          // rows of X per workgroup
constexpr int kPfThreads = kPfWaves * 64;
constexpr int kPfMB = kPfTokens / 16;   // 16-token MFMA blocks
constexpr int kPfRowBytes = 256;        // one token's 128 columns of a group in LDS
constexpr int kPfTileBytes = kPfTokens * kPfRowBytes;
constexpr size_t kPrefillLds = 2 * static_cast<size_t>(kPfTileBytes);
constexpr int kPfXV = kPfTokens * 16 / kPfThreads;  // 16-byte pieces of the X tile per thread
static_assert(kPfMB == 16 && kPfXV == 16, "the schedule below is written out for 16 token blocks and 16 X loads per wave");

__device__ __forceinline__ uint32_t u32(half2_t v) { return __builtin_bit_cast(uint32_t, v); }

// X tile in LDS: token row r holds its 16 chunks of 16 bytes (8 columns) at chunk position c ^ swz(r).
// A ds_read_b128 serves 16 lanes per cycle, and not 16 consecutive ones: the groups are lanes
// {0-3, 12-15, 20-27}, {4-11, 16-19, 28-31} and the same plus 32 (measured on gfx950 with the bank-conflict
// counter, one pair of active lanes per dispatch).  The MFMA operand read has lane 16 kb + i fetch chunk
// 4 kb + s of token i, so a group mixes chunks 4 kb + s and 4 (kb ^ 1) + s: with
//     swz(i) = i for i < 4,  i + 4 for 4 <= i < 12,  i - 8 for i >= 12     (i = r % 16)
// tokens {0-3, 12-15} get the values 0..7 and tokens {4-11} the values 8..15; both sets are closed under
// ^ 4, so the sixteen lanes of every group land in sixteen different 16-byte bank columns (4 cycles per
// read instead of 8 with rows padded to 272 bytes).
__device__ __forceinline__ int pf_swz(int r) {
  const int hi = (r >> 2) & 3;
  return (r & 3) | (((0x78 >> (2 * hi)) & 3) << 2);  // hi: 0, 1, 2, 3 -> 0, 2, 3, 1
}

typedef __attribute__((address_space(3))) void* lds_ptr_t;
__device__ __forceinline__ lds_ptr_t to_lds(const void* p) {
  return reinterpret_cast<lds_ptr_t>(static_cast<uint32_t>(reinterpret_cast<uintptr_t>(p)));  // low half of a generic LDS address
}

// the accumulation registers by name, for clobber lists
#define PMPD_PF_ALL_ACC \
  "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", "a10", "a11", "a12", "a13", "a14", "a15", "a16", \
  "a17", "a18", "a19", "a20", "a21", "a22", "a23", "a24", "a25", "a26", "a27", "a28", "a29", "a30", "a31", "a32", \
  "a33", "a34", "a35", "a36", "a37", "a38", "a39", "a40", "a41", "a42", "a43", "a44", "a45", "a46", "a47", "a48", \
  "a49", "a50", "a51", "a52", "a53", "a54", "a55", "a56", "a57", "a58", "a59", "a60", "a61", "a62", "a63", "a64", \
  "a65", "a66", "a67", "a68", "a69", "a70", "a71", "a72", "a73", "a74", "a75", "a76", "a77", "a78", "a79", "a80", \
  "a81", "a82", "a83", "a84", "a85", "a86", "a87", "a88", "a89", "a90", "a91", "a92", "a93", "a94", "a95", "a96", \
  "a97", "a98", "a99", "a100", "a101", "a102", "a103", "a104", "a105", "a106", "a107", "a108", "a109", "a110", \
  "a111", "a112", "a113", "a114", "a115", "a116", "a117", "a118", "a119", "a120", "a121", "a122", "a123", "a124", \
  "a125", "a126", "a127", "a128", "a129", "a130", "a131", "a132", "a133", "a134", "a135", "a136", "a137", "a138", \
  "a139", "a140", "a141", "a142", "a143", "a144", "a145", "a146", "a147", "a148", "a149", "a150", "a151", "a152", \
  "a153", "a154", "a155", "a156", "a157", "a158", "a159", "a160", "a161", "a162", "a163", "a164", "a165", "a166", \
  "a167", "a168", "a169", "a170", "a171", "a172", "a173", "a174", "a175", "a176", "a177", "a178", "a179", "a180", \
  "a181", "a182", "a183", "a184", "a185", "a186", "a187", "a188", "a189", "a190", "a191", "a192", "a193", "a194", \
  "a195", "a196", "a197", "a198", "a199", "a200", "a201", "a202", "a203", "a204", "a205", "a206", "a207", "a208", \
  "a209", "a210", "a211", "a212", "a213", "a214", "a215", "a216", "a217", "a218", "a219", "a220", "a221", "a222", \
  "a223", "a224", "a225", "a226", "a227", "a228", "a229", "a230", "a231", "a232", "a233", "a234", "a235", "a236", \
  "a237", "a238", "a239", "a240", "a241", "a242", "a243", "a244", "a245", "a246", "a247", "a248", "a249", "a250", \
  "a251", "a252", "a253", "a254", "a255"

// What the kernel needs to know of a work item: four consecutive 64-row tiles of one layer (one per wave).
struct PfItem {
  LayerDesc L;
  const _Float16* X;  // the layer's activations, row-major [m][in_f]
  float* Y;           // the layer's outputs, row-major [m][out_f]
  int tile0;
};
// Items of a stack: entry idx of the work list (longest rows first).
struct PfStackSource {
  const LayerDesc* layers;
  const WorkItem* items;
  const _Float16* x_base;
  float* y_base;
  int m;
  __device__ __forceinline__ PfItem get(int idx) const {
    const WorkItem it = items[idx];
    PfItem r;
    r.L = layers[it.layer];
    r.X = x_base + static_cast<int64_t>(m) * r.L.x_off;
    r.Y = y_base + static_cast<int64_t>(m) * r.L.y_off;
    r.tile0 = it.tile0;
    return r;
  }
};
// Items of one layer: entry idx is its idx-th block of four tiles.
struct PfLayerSource {
  LayerDesc L;
  const _Float16* X;
  float* Y;
  __device__ __forceinline__ PfItem get(int idx) const { return PfItem{L, X, Y, idx * kPfWaves}; }
};

// One workgroup: token block mtile (256 tokens) of the work items first, first + stride, ... (n_mine of them), one
// after the other, as ONE sequence of groups: the loads run ahead of the MFMAs across item boundaries (the X tile
// by one group, the plane words by three), so only the first item of a workgroup has a prologue, and the stores of
// an item's results are followed at once by the next item's MFMAs.  Three cursors walk the sequence of (item, group)
// pairs, each with the buffer resources of its own item: one for the plane loads, one for the X loads, one for the
// MFMAs; they move between groups, never inside one.  All cursor state is wave-uniform.
template <int B, typename Source>
__device__ __forceinline__ void prefill_run(const Source& src, int m_rows, int mtile, int first, int stride, int n_mine,
                                            char* lds) {
  if (n_mine <= 0) return;  // (the launchers never start such a workgroup)
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int m0 = mtile * kPfTokens;

  // All loads go through buffer resources (a base and a byte count in scalar registers) with a 32-bit byte offset
  // per lane and a scalar offset for the group, so that an address costs neither vector registers nor vector
  // instructions: plane k of this wave's tile is the 1 KiB per group at plane[k] + (tbase + 64 g) 16, lane l
  // taking bytes 16 l..; its (scale, min) words are the 256 bytes per group at sa + (tbase / 4 + 16 g) 16, lane l
  // taking bytes 16 (l % 16)...  A read past a resource's end would return zero instead of faulting.
  constexpr int kRsrcFlags = 0x00020000;  // raw buffer, 32-bit data format
  const uint32_t plane_lane = static_cast<uint32_t>(lane) * 16u, sa_lane = static_cast<uint32_t>(lane & 15) * 16u;

  // ---- plane cursor: item kp, group gp of its Gp
  int kp = 0, gp = 0, Gp = 1;
  __amdgpu_buffer_rsrc_t pr[B], sr;
  auto plane_item = [&](int k) {
    const PfItem it = src.get(first + k * stride);
    const int tile = it.tile0 + wave;  // this wave's row tile (clamped: rows past the end are never stored)
    const int tl = tile < it.L.n_tiles ? tile : it.L.n_tiles - 1;
    Gp = it.L.n_groups;
    const int64_t tbase = (static_cast<int64_t>(tl) * Gp) * 64;
#pragma unroll
    for (int q = 0; q < B; ++q)
      pr[q] = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(static_cast<const char*>(it.L.plane[q]) + tbase * 16), 0, Gp * 1024, kRsrcFlags);
    sr = __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(static_cast<const char*>(it.L.sa) + tbase * 4), 0, Gp * 256, kRsrcFlags);
  };
  // to the next group; past the last group of the last item the cursor stays where it is (loads repeat, unused)
  auto plane_next = [&]() {
    if (gp + 1 < Gp) {
      ++gp;
    } else if (kp + 1 < n_mine) {
      ++kp;
      gp = 0;
      plane_item(kp);
    }
  };

  // ---- X cursor: item kx, group gx of its Gx.  X tile: a wave's load instruction i fills the four token rows
  // 4 (wave + 4 i) .. + 3 of the tile, 1 KiB that the hardware places at consecutive LDS addresses in lane order: lane
  // l is position l % 16 of row 4 (wave + 4 i) + l / 16 and therefore fetches the chunk that the swizzle puts there.
  // Rows 16 i apart share r % 16, so the lane's chunk is the same for its sixteen loads.  Tokens past the end repeat
  // the last one (their outputs are never stored).  The byte count of X fits 32 bits (checked by the launcher).
  int kx = 0, gx = 0, Gx = 1;
  __amdgpu_buffer_rsrc_t xr;
  uint32_t xoff[kPfXV];
  const int xrow = 4 * wave + (lane >> 4);
  const uint32_t xchunk16 = static_cast<uint32_t>((lane & 15) ^ pf_swz(xrow)) * 16u;
  auto x_item = [&](int k) {
    const PfItem it = src.get(first + k * stride);
    Gx = it.L.n_groups;
    const uint32_t row_bytes = static_cast<uint32_t>(it.L.in_f) * 2u;
    xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16*>(it.X), 0, static_cast<int>(static_cast<uint32_t>(m_rows) * row_bytes), kRsrcFlags);
#pragma unroll
    for (int i = 0; i < kPfXV; ++i) {
      int token = m0 + xrow + 4 * kPfWaves * i;
      token = token < m_rows ? token : m_rows - 1;
      xoff[i] = static_cast<uint32_t>(token) * row_bytes + xchunk16;
    }
  };
  auto x_next = [&]() {
    if (gx + 1 < Gx) {
      ++gx;
    } else if (kx + 1 < n_mine) {
      ++kx;
      gx = 0;
      x_item(kx);
    }
  };
  // load i of the X tile the cursor points to, into the buffer at LDS address buf
  auto load_x = [&](int i, uint32_t buf) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, reinterpret_cast<lds_ptr_t>(buf + (4 * wave + 4 * kPfWaves * i) * kPfRowBytes), 16,
                                             xoff[i], gx * (kGroup * 2), 0, 0);
  };
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds));  // low half of a generic LDS address

  // ---- MFMA cursor: item kc, group gc of its Gc, and where the item's results go
  int kc = 0, gc = 0, Gc = 1, c_tile = 0, c_ntiles = 0, c_out = 0;
  float* c_y = nullptr;
  auto mfma_item = [&](int k) {
    const PfItem it = src.get(first + k * stride);
    Gc = it.L.n_groups;
    c_tile = it.tile0 + wave;
    c_ntiles = it.L.n_tiles;
    c_out = it.L.out_f;
    c_y = it.Y;
  };

  // A operand of this lane for K-step s: token 16 mb + lane % 16, chunk 4 (lane / 16) + s
  const int a_row = (lane & 15) * kPfRowBytes;
  const int a_col = (4 * (lane >> 4)) ^ pf_swz(lane & 15);  // chunk position of K-step s: a_col ^ s

  // The 256 accumulators of this lane (16 token blocks x 4 row blocks x 4) are the accumulation registers a0..a255,
  // named outright in the MFMA, clear and read instructions below: block (mb, t) is a[16 mb + 4 t .. + 3].  The
  // compiler is told once that they are written; it has no reason to use them itself (its own values fit the
  // ordinary registers of a one-wave-per-SIMD kernel), and then the accumulators never move.  (As C++ variables
  // they do: with all 256 live, the register allocator shuttles them between the two register files.)
  asm volatile("" ::: PMPD_PF_ALL_ACC);
#pragma unroll
  for (int i = 0; i < 16 * kPfMB; ++i) asm volatile("v_accvgpr_write_b32 a[%0], 0" ::"n"(i));

  constexpr float kOff = (B == 4) ? 0.5f : (B == 3) ? 1.0f : 2.0f;  // 2^(3-b)
  const half2_t cL2 = {static_cast<_Float16>(kOff - 1024.0f), static_cast<_Float16>(kOff - 1024.0f)};
  const half2_t cH2 = {static_cast<_Float16>(kOff - 64.0f), static_cast<_Float16>(kOff - 64.0f)};
  const half2_t sixteenth2 = {static_cast<_Float16>(0.0625f), static_cast<_Float16>(0.0625f)};
  const uint32_t cL = opaque_sgpr(u32(cL2)), sixteenth = opaque_sgpr(u32(sixteenth2));
  uint32_t cH = u32(cH2);
  asm volatile("" : "+v"(cH));
  const uint32_t maskL = opaque_sgpr(0x000F000Fu), maskH = opaque_sgpr(0x00F000F0u);
  const uint32_t odd = opaque_sgpr(0xAAAAAAAAu), even = opaque_sgpr(0x55555555u), top = opaque_sgpr(0xCCCCCCCCu);
  uint32_t magic = 0x64006400u;  // fp16 pair (1024, 1024)
  asm volatile("" : "+v"(magic));

  // Register sets, indexed by the parity of a group: pcs[q], sacs[q] receive plane words and (scale, min) words of
  // groups of parity q; code[q], sa[q] are the merged codes and the (scale, min) pairs of such a group.  The
  // operands of K-step s are in bw[s % 2].
  u32x4 pcs[2][B], sacs[2];
  uint32_t code[2][4][4];     // [parity][16-row block][K-step]
  uint32_t sa[2][4];          // (scale, min) of the lane's four rows, two fp16
  uint32_t bw[2][4][4];       // [K-step parity][16-row block][register of the operand]

  // the words of the group the plane cursor points to, into register set q
  auto load_plane = [&](int q, int k) { pcs[q][k] = __builtin_amdgcn_raw_buffer_load_b128(pr[k], plane_lane, gp * 1024, 0); };
  auto load_sa = [&](int q) { sacs[q] = __builtin_amdgcn_raw_buffer_load_b128(sr, sa_lane, gp * 256, 0); };
  // Everything that rides under the MFMAs is written as asm statements, one instruction each: such statements keep
  // their order, so the instruction stream is the one written here and the compiler only assigns registers.
  // Measured on gfx950 with one wave per SIMD: two VALU instructions after an MFMA do not delay the next MFMA, a
  // third costs 12 cycles; an LDS read rides free if no VALU instruction shares its slot.  A statement that reads
  // what the statement before it wrote would get a wait state from the compiler, so the two instructions of a slot
  // are always independent of each other.
#define PMPD_V2(op, d, a) asm volatile(op " %0, %1" : "=v"(d) : "v"(a))
#define PMPD_VN(op, d, n, a) asm volatile(op " %0, %1, %2" : "=v"(d) : "n"(n), "v"(a))
#define PMPD_VS(op, d, sreg, a) asm volatile(op " %0, %1, %2" : "=v"(d) : "s"(sreg), "v"(a))
#define PMPD_BFI(d, mask, a, b) asm volatile("v_bfi_b32 %0, %1, %2, %3" : "=v"(d) : "s"(mask), "v"(a), "v"(b))
#define PMPD_ROTL(d, a, n) asm volatile("v_alignbit_b32 %0, %1, %1, %2" : "=v"(d) : "v"(a), "n"(32 - (n)))
  // Merge of 16-row block t of the plane words pcs[q] into the four code words code[q][t][0..3] (eight 4-bit
  // aligned codes q~ each: columns 8 v .. 8 v + 7 of the lane's 32, nibbles 0,4 / 1,5 / 2,6 / 3,7 = column pairs
  // (0,1) / (2,3) / (4,5) / (6,7)), in seven pairs of instructions.  With r1 = odd bits of plane 0 and even bits
  // of plane 1, r2 the other way round (s1, s2 the same from planes 2, 3), the upper two bits of the nibbles of
  // words 0..3 are r1 << 2, r1, rotl(r2, 3), r2 << 1 under the mask 0xCCCCCCCC and the lower two s1, s1 >> 2,
  // rotl(s2, 1), s2 >> 1 under its complement: one bit-field insert joins the two.  With three planes the
  // lower halves come from plane 2 alone (its odd bits for words 0, 1, its even bits for words 2, 3: the bit
  // that the complement mask keeps is then the plane's, the other is zero); with two planes they are zero.
  uint32_t m_r1, m_r2, m_s1, m_s2, m_a, m_b, m_c, m_d;
  auto merge_pair = [&](int q, int t, int k) {
    switch (k) {
      case 0:
        PMPD_BFI(m_r1, odd, word_of(pcs[q][0], t), word_of(pcs[q][1], t));
        PMPD_BFI(m_r2, odd, word_of(pcs[q][1], t), word_of(pcs[q][0], t));
        break;
      case 1:
        if constexpr (B == 4) {
          PMPD_BFI(m_s1, odd, word_of(pcs[q][2], t), word_of(pcs[q][3], t));
          PMPD_BFI(m_s2, odd, word_of(pcs[q][3], t), word_of(pcs[q][2], t));
        } else if constexpr (B == 3) {
          PMPD_VS("v_and_b32", m_s1, odd, word_of(pcs[q][2], t));
          PMPD_VS("v_and_b32", m_s2, even, word_of(pcs[q][2], t));
        }
        break;
      case 2:
        PMPD_VN("v_lshlrev_b32", m_a, 2, m_r1);
        if constexpr (B != 2) PMPD_VN("v_lshrrev_b32", m_b, 2, m_s1);
        break;
      case 3:
        if constexpr (B == 2) {
          PMPD_VS("v_and_b32", code[q][t][0], top, m_a);
          PMPD_VS("v_and_b32", code[q][t][1], top, m_r1);
        } else {
          PMPD_BFI(code[q][t][0], top, m_a, m_s1);
          PMPD_BFI(code[q][t][1], top, m_r1, m_b);
        }
        break;
      case 4:
        PMPD_ROTL(m_c, m_r2, 3);
        if constexpr (B == 4) PMPD_ROTL(m_d, m_s2, 1);
        if constexpr (B == 3) PMPD_VN("v_lshlrev_b32", m_d, 1, m_s2);
        break;
      case 5:
        PMPD_VN("v_lshlrev_b32", m_a, 1, m_r2);
        if constexpr (B != 2) PMPD_VN("v_lshrrev_b32", m_b, 1, m_s2);
        break;
      default:
        if constexpr (B == 2) {
          PMPD_VS("v_and_b32", code[q][t][2], top, m_c);
          PMPD_VS("v_and_b32", code[q][t][3], top, m_a);
        } else {
          PMPD_BFI(code[q][t][2], top, m_c, m_d);
          PMPD_BFI(code[q][t][3], top, m_a, m_b);
        }
        sa[q][t] = word_of(sacs[q], t);  // the row's (scale, min); no instruction
        break;
    }
  };
  // The operand of 16-row block t for K-step s of a group of parity q: sixteen weights of the lane -> four registers
  // w[t][0..3], in seven units of at most two instructions (u = 0..2: code nibbles 0,4,1,5, registers 0, 1; u = 3:
  // the shift that brings nibbles 2,6,3,7 down; u = 4..6: registers 2, 3).  Exact codes q~ + 2^(3-b): low-nibble
  // pairs carry 1024 + q~, high-nibble pairs 1024 + 16 q~; then one fused multiply-add with the row's scale and
  // minimum, which the instruction's operand selects broadcast from the two halves of one register.
  uint32_t d_w, d_a0, d_a1, d_q0, d_q1;
  auto dequant_unit = [&](int q, int s, int t, int u, uint32_t (&w)[4][4]) {
    const int half = u >= 3;
    switch (u) {
      case 3:
        PMPD_VN("v_lshrrev_b32", d_w, 8, code[q][t][s]);
        break;
      case 0:
      case 4: {
        const uint32_t c = half ? d_w : code[q][t][s];
        asm volatile("v_and_or_b32 %0, %1, %2, %3" : "=v"(d_a0) : "v"(c), "s"(maskL), "v"(magic));
        asm volatile("v_and_or_b32 %0, %1, %2, %3" : "=v"(d_a1) : "v"(c), "s"(maskH), "v"(magic));
        break;
      }
      case 1:
      case 5:
        asm volatile("v_pk_add_f16 %0, %1, %2" : "=v"(d_q0) : "v"(d_a0), "s"(cL));
        asm volatile("v_pk_fma_f16 %0, %1, %2, %3" : "=v"(d_q1) : "v"(d_a1), "s"(sixteenth), "v"(cH));
        break;
      default:
        asm volatile("v_pk_fma_f16 %0, %1, %2, %2 op_sel:[0,0,1] op_sel_hi:[1,0,1]" : "=v"(w[t][2 * half]) : "v"(d_q0), "v"(sa[q][t]));
        asm volatile("v_pk_fma_f16 %0, %1, %2, %2 op_sel:[0,0,1] op_sel_hi:[1,0,1]" : "=v"(w[t][2 * half + 1]) : "v"(d_q1), "v"(sa[q][t]));
        break;
    }
  };

  // K-step s of group g (X tile in LDS buffer xs, operands `cur`): 64 MFMAs, 16 token blocks x 4 row blocks.  The
  // slots after the first and the second MFMA of a token block carry the 28 units of the operands `nxt` of K-step
  // ns of the group of parity nq; the slot after the third carries, in the first seven token blocks, the merge of
  // row block s of the plane words of parity mq (the next group's); the slot after the fourth has no VALU work:
  // there goes the LDS read of the X operand three token blocks ahead (a ring of four; LDS reads complete in
  // order, so before block mb it is enough to wait until at most the reads issued after block mb's are
  // outstanding: nothing else uses that counter meanwhile), and in some blocks one global load: in K-steps 0..2
  // every third block a load of X tile g + 1 into the other buffer xn (16 in all); in K-step 3 the last three
  // blocks load the plane words and (scale, min) words of group g + 3 into the set of parity mq, which the merge
  // has finished with by then.
  auto step = [&](int s, const char* xs, uint32_t xn, const uint32_t (&cur)[4][4], int nq, int ns, uint32_t (&nxt)[4][4], int mq) {
    const uint32_t ap = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(xs + a_row + ((a_col ^ s) << 4)));  // LDS address
    half8_t af[4];
    u32x4 cw[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) cw[t] = u32x4{cur[t][0], cur[t][1], cur[t][2], cur[t][3]};
#define PMPD_PF_READ(dst, block) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(ap), "n"((block) * 16 * kPfRowBytes))
#define PMPD_PF_MFMA(t)                                                                                           \
  asm volatile("v_mfma_f32_16x16x32_f16 a[%2:%3], %0, %1, a[%2:%3]" ::"v"(cw[t]), "v"(a), "n"(16 * mb + 4 * (t)), \
               "n"(16 * mb + 4 * (t) + 3))
    PMPD_PF_READ(af[0], 0);
    PMPD_PF_READ(af[1], 1);
    PMPD_PF_READ(af[2], 2);
#pragma unroll
    for (int mb = 0; mb < kPfMB; ++mb) {
      half8_t& a = af[mb & 3];
      if (mb + 3 <= kPfMB) asm volatile("s_waitcnt lgkmcnt(2)");
      else if (mb + 2 == kPfMB) asm volatile("s_waitcnt lgkmcnt(1)");
      else asm volatile("s_waitcnt lgkmcnt(0)");
      PMPD_PF_MFMA(0);
      if (2 * mb < 28) dequant_unit(nq, ns, (2 * mb) / 7, (2 * mb) % 7, nxt);
      PMPD_PF_MFMA(1);
      if (2 * mb + 1 < 28) dequant_unit(nq, ns, (2 * mb + 1) / 7, (2 * mb + 1) % 7, nxt);
      PMPD_PF_MFMA(2);
      if (mb < 7) merge_pair(mq, s, mb);
      PMPD_PF_MFMA(3);
      switch (mb) {  // the read for three blocks on (offsets are immediates)
        case 0: PMPD_PF_READ(af[3], 3); break;
        case 1: PMPD_PF_READ(af[0], 4); break;
        case 2: PMPD_PF_READ(af[1], 5); break;
        case 3: PMPD_PF_READ(af[2], 6); break;
        case 4: PMPD_PF_READ(af[3], 7); break;
        case 5: PMPD_PF_READ(af[0], 8); break;
        case 6: PMPD_PF_READ(af[1], 9); break;
        case 7: PMPD_PF_READ(af[2], 10); break;
        case 8: PMPD_PF_READ(af[3], 11); break;
        case 9: PMPD_PF_READ(af[0], 12); break;
        case 10: PMPD_PF_READ(af[1], 13); break;
        case 11: PMPD_PF_READ(af[2], 14); break;
        case 12: PMPD_PF_READ(af[3], 15); break;
        default: break;
      }
      if (s < 3) {
        if (mb % 3 == 0 && mb < 15) load_x(5 * s + mb / 3, xn);
        if (s == 2 && mb == 15) load_x(15, xn);
      } else {
        if (mb == 13) {
          load_plane(mq, 0);
          load_plane(mq, 1);
        }
        if (mb == 14 && B > 2) {
          load_plane(mq, 2);
          if constexpr (B > 3) load_plane(mq, 3);
        }
        if (mb == 15) load_sa(mq);
      }
    }
#undef PMPD_PF_READ
#undef PMPD_PF_MFMA
  };

  // Results of the item the MFMA cursor has just finished: the weights are the first MFMA operand (rows i of D =
  // weight rows) and X the second (columns j = tokens), so D[i][j] sits in lane j + 16 (i / 4), register i % 4: a
  // lane holds four consecutive output features of one token, 16 bytes of Y, which go out as one 16-byte store where
  // Y allows it.  (Plain stores: the write-back caches absorb the burst; nontemporal ones measured 4 % slower.)  Every
  // accumulator is cleared right after it is read.  The MFMAs that wrote them are at least a barrier away.
  auto store_item = [&]() {
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    const bool mine = c_tile < c_ntiles;
    const bool wide = (reinterpret_cast<uintptr_t>(c_y) % 16 == 0) && (c_out % 4 == 0);
#pragma unroll
    for (int mb = 0; mb < kPfMB; ++mb) {
      const int row = m0 + 16 * mb + (lane & 15);
      float* yrow = c_y + static_cast<int64_t>(row) * c_out;
      const bool row_ok = mine && row < m_rows;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int col = c_tile * 64 + 16 * t + 4 * (lane >> 4);
        float4_t d;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(d[r]) : "n"(16 * mb + 4 * t + r));
          asm volatile("v_accvgpr_write_b32 a[%0], 0" ::"n"(16 * mb + 4 * t + r));
        }
        if (row_ok) {
          if (wide) {
            if (col < c_out) *reinterpret_cast<float4_t*>(yrow + col) = d;
          } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (col + r < c_out) yrow[col + r] = d[r];
          }
        }
      }
    }
  };

  // Before the first group: X tile of group 0 to buffer 0; plane words of group 0 merged and the operands of its
  // K-step 0 made; plane words of groups 1 and 2 in their sets; the plane cursor three groups ahead, the X cursor
  // one.  Nothing is outstanding afterwards.
  mfma_item(0);
  x_item(0);
  plane_item(0);
#pragma unroll
  for (int i = 0; i < kPfXV; ++i) load_x(i, lds0);
  x_next();
#pragma unroll
  for (int k = 0; k < B; ++k) load_plane(0, k);
  load_sa(0);
  plane_next();
#pragma unroll
  for (int k = 0; k < B; ++k) load_plane(1, k);
  load_sa(1);
  plane_next();
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int k = 0; k < 7; ++k) merge_pair(0, t, k);
#pragma unroll
  for (int k = 0; k < B; ++k) load_plane(0, k);
  load_sa(0);
  plane_next();
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int u = 0; u < 7; ++u) dequant_unit(0, 0, t, u, bw[0]);
  __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0), other counters untouched
  __syncthreads();

  // One group of the sequence, of parity p (groups are counted through all items).  On entry: codes of this group in
  // code[p], operands of its K-step 0 in bw[0], plane words of the next group in pcs[1 - p] (arrived), those of the
  // one after on their way to pcs[p] or there, this group's X tile in LDS buffer p; the X cursor points to the next
  // group, the plane cursor three groups ahead.  Returns false after the last group of the last item.
  auto group = [&](auto parity) -> bool {
    constexpr int p = decltype(parity)::value;
    const char* xs = lds + p * kPfTileBytes;
    // (opaque: the sixteen destination addresses of the X loads are then computed where they are used, one scalar
    // add each, instead of being kept in sixteen scalar registers per buffer)
    const uint32_t xn = opaque_sgpr(lds0 + (1 - p) * kPfTileBytes);
    step(0, xs, xn, bw[0], p, 1, bw[1], 1 - p);
    step(1, xs, xn, bw[1], p, 2, bw[0], 1 - p);
    step(2, xs, xn, bw[0], p, 3, bw[1], 1 - p);
    step(3, xs, xn, bw[1], 1 - p, 0, bw[0], 1 - p);
    // Loads complete in order: with at most the B + 1 loads of K-step 3 outstanding, this wave's part of the next X
    // tile is in LDS and the plane words of the group after next are in their registers.
    if constexpr (B == 4) __builtin_amdgcn_s_waitcnt(0x0F75);  // vmcnt(5), other counters untouched
    if constexpr (B == 3) __builtin_amdgcn_s_waitcnt(0x0F74);
    if constexpr (B == 2) __builtin_amdgcn_s_waitcnt(0x0F73);
    __syncthreads();  // everybody's part of the next X tile is in LDS; buffer p is free
    x_next();
    plane_next();
    if (++gc == Gc) {
      store_item();
      if (++kc == n_mine) return false;
      gc = 0;
      mfma_item(kc);
    }
    return true;
  };
  while (group(std::integral_constant<int, 0>{}) && group(std::integral_constant<int, 1>{})) {
  }
#undef PMPD_V2
#undef PMPD_VN
#undef PMPD_VS
#undef PMPD_BFI
#undef PMPD_ROTL
}

// Which token block and which items a workgroup takes: pf_share (pmpd_prefill_deal.hpp).
template <int B>
__global__ __launch_bounds__(kPfThreads, 1) void pmpd_prefill_layer_kernel(LayerDesc L, const _Float16* __restrict__ X, int m,
                                                                     float* __restrict__ Y, int m_tiles, int n_items,
                                                                     int per_block, int per_xcd) {
  extern __shared__ uint4 lds_raw[];
  const PfShare sh = pf_share(static_cast<int>(blockIdx.x), n_items, m_tiles, per_block, per_xcd);
  const PfLayerSource src{L, X, Y};
  prefill_run<B>(src, m, sh.mtile, sh.first, per_block, sh.n_mine, reinterpret_cast<char*>(lds_raw));
}

template <int B>
__global__ __launch_bounds__(kPfThreads, 1) void pmpd_prefill_stack_kernel(const LayerDesc* __restrict__ layers,
                                                                     const WorkItem* __restrict__ items,
                                                                     const _Float16* __restrict__ x_base, int m,
                                                                     float* __restrict__ y_base, int m_tiles, int n_items,
                                                                     int per_block, int per_xcd) {
  extern __shared__ uint4 lds_raw[];
  const PfShare sh = pf_share(static_cast<int>(blockIdx.x), n_items, m_tiles, per_block, per_xcd);
  const PfStackSource src{layers, items, x_base, y_base, m};
  prefill_run<B>(src, m, sh.mtile, sh.first, per_block, sh.n_mine, reinterpret_cast<char*>(lds_raw));
}

// The X tile needs more than the 64 KiB of dynamic LDS a kernel gets by default.
template <typename K>
static hipError_t allow_lds(K kernel) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             static_cast<int>(kPrefillLds));
}

// Grid for n_items items and m_tiles token blocks on the current device (pf_grid, pmpd_prefill_deal.hpp).
static hipError_t prefill_grid(int n_items, int m_tiles, PfGrid* g) {
  int dev = 0, cus = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  *g = pf_grid(n_items, m_tiles, cus);
  return hipSuccess;
}

// Launchers used by the C entry points (defined in pmpd_gemv.hip).
hipError_t launch_prefill_layer(const LayerDesc& d, int b, const void* X, int m, float* Y, hipStream_t s) {
  const int m_tiles = (m + kPfTokens - 1) / kPfTokens;
  const int n_items = (d.n_tiles + kPfWaves - 1) / kPfWaves;
  PfGrid g;
  hipError_t e = prefill_grid(n_items, m_tiles, &g);
  if (e != hipSuccess) return e;
  const _Float16* x = static_cast<const _Float16*>(X);
  e = b == 4 ? allow_lds(&pmpd_prefill_layer_kernel<4>) : b == 3 ? allow_lds(&pmpd_prefill_layer_kernel<3>) : allow_lds(&pmpd_prefill_layer_kernel<2>);
  if (e != hipSuccess) return e;
  if (b == 4) hipLaunchKernelGGL((pmpd_prefill_layer_kernel<4>), dim3(g.grid), dim3(kPfThreads), kPrefillLds, s, d, x, m, Y, m_tiles, n_items, g.per_block, g.per_xcd);
  else if (b == 3) hipLaunchKernelGGL((pmpd_prefill_layer_kernel<3>), dim3(g.grid), dim3(kPfThreads), kPrefillLds, s, d, x, m, Y, m_tiles, n_items, g.per_block, g.per_xcd);
  else hipLaunchKernelGGL((pmpd_prefill_layer_kernel<2>), dim3(g.grid), dim3(kPfThreads), kPrefillLds, s, d, x, m, Y, m_tiles, n_items, g.per_block, g.per_xcd);
  return hipGetLastError();
}

hipError_t launch_prefill_stack(const pmpd_stack* st, int b, const void* X, int m, float* Y, hipStream_t s) {
  const int m_tiles = (m + kPfTokens - 1) / kPfTokens;
  constexpr int kList = 0;  // work list of 4-tile items: one 64-row tile per wave
  static_assert(kStackTilesPerWg[kList] == kPfWaves, "one tile per wave");
  const int n_items = static_cast<int>(st->items[kList].size());
  PfGrid g;
  hipError_t e = prefill_grid(n_items, m_tiles, &g);
  if (e != hipSuccess) return e;
  const _Float16* x = static_cast<const _Float16*>(X);
  const WorkItem* items = st->d_items[kList];
  e = b == 4 ? allow_lds(&pmpd_prefill_stack_kernel<4>) : b == 3 ? allow_lds(&pmpd_prefill_stack_kernel<3>) : allow_lds(&pmpd_prefill_stack_kernel<2>);
  if (e != hipSuccess) return e;
  if (b == 4) hipLaunchKernelGGL((pmpd_prefill_stack_kernel<4>), dim3(g.grid), dim3(kPfThreads), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles, n_items, g.per_block, g.per_xcd);
  else if (b == 3) hipLaunchKernelGGL((pmpd_prefill_stack_kernel<3>), dim3(g.grid), dim3(kPfThreads), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles, n_items, g.per_block, g.per_xcd);
  else hipLaunchKernelGGL((pmpd_prefill_stack_kernel<2>), dim3(g.grid), dim3(kPfThreads), kPrefillLds, s, st->d_layers, items, x, m, Y, m_tiles, n_items, g.per_block, g.per_xcd);
  return hipGetLastError();
}

}  // namespace pmpd
