// Host side of the PMPD library: error reporting, argument checks, the storage format
// (pack / unpack) and the precision-switching schedule.  Nothing here touches the GPU.
#include <algorithm>
#include <climits>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "pmpd_common.hpp"

namespace pmpd {

static thread_local char g_err[512] = "";

int32_t fail(int32_t status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return status;
}

int32_t check_shape(int32_t out_f, int32_t in_f, int32_t group) {
  if (group != kGroup) return fail(PMPD_EINVAL, "group_size must be %d (got %d)", kGroup, group);
  if (out_f <= 0) return fail(PMPD_EINVAL, "out_features must be positive (got %d)", out_f);
  if (in_f <= 0 || in_f % kGroup) return fail(PMPD_EINVAL, "in_features must be a positive multiple of %d (got %d)", kGroup, in_f);
  return PMPD_OK;
}

int32_t check_layer(const pmpd_layer_t* L, int32_t b, const char* who) {
  if (!L) return fail(PMPD_EINVAL, "%s: layer is NULL", who);
  if (b < 1 || b > 4) return fail(PMPD_EINVAL, "%s: bit-width %d outside 1..4", who, b);
  if (L->reserved != 0) return fail(PMPD_EINVAL, "%s: layer.reserved must be 0", who);
  int32_t rc = check_shape(L->out_features, L->in_features, L->group_size);
  if (rc) return rc;
  for (int k = 0; k < b; ++k) {
    if (!L->planes[k]) return fail(PMPD_EINVAL, "%s: planes[%d] is NULL but bit-width is %d", who, k, b);
    if (reinterpret_cast<uintptr_t>(L->planes[k]) % 16) return fail(PMPD_EALIGN, "%s: planes[%d] not 16-byte aligned", who, k);
  }
  if (!L->scale_min) return fail(PMPD_EINVAL, "%s: scale_min is NULL", who);
  if (reinterpret_cast<uintptr_t>(L->scale_min) % 4) return fail(PMPD_EALIGN, "%s: scale_min not 4-byte aligned", who);
  return PMPD_OK;
}

// Where plane k keeps its bit of the weight in row rr (0..63) of a tile and column e (0..127)
// of a group: the 32-bit word index inside the (tile, group) block of 256 words, and the bit.
//   rr = 16 t + j,  e = 32 kb + 8 v + c,  n = c/2 + 4 (c%2)
//   word = (16 kb + j) 4 + t
//   bit  = 4 n + {1,3,0,2}[v]            for the even planes (upper bit of a 2-bit pair)
//          (4 n + {0,2,31,1}[v]) mod 32  for the odd planes (lower bit)
struct BitHome {
  int word, bit;
};
static inline BitHome bit_home(int k, int rr, int e) {
  static const int even_off[4] = {1, 3, 0, 2}, odd_off[4] = {0, 2, 31, 1};
  const int t = rr >> 4, j = rr & 15;
  const int kb = e >> 5, v = (e >> 3) & 3, c = e & 7;
  const int n = (c >> 1) + 4 * (c & 1);
  const int off = (k & 1) ? odd_off[v] : even_off[v];
  return BitHome{(16 * kb + j) * 4 + t, (4 * n + off) & 31};
}

}  // namespace pmpd

using namespace pmpd;

extern "C" {

const char* pmpd_strerror(int32_t status) {
  switch (status) {
    case PMPD_OK: return "ok";
    case PMPD_EINVAL: return "invalid argument";
    case PMPD_EALIGN: return "misaligned buffer";
    case PMPD_ESCHED: return "invalid precision-switching schedule";
    case PMPD_EHIP: return "HIP runtime failure";
    case PMPD_ESIZE: return "buffer too small";
    default: return "unknown status";
  }
}

const char* pmpd_last_error(void) { return g_err; }

int32_t pmpd_packed_size(int32_t out_f, int32_t in_f, int32_t group, size_t* plane_bytes, size_t* sm_bytes) {
  int32_t rc = check_shape(out_f, in_f, group);
  if (rc) return rc;
  if (!plane_bytes || !sm_bytes) return fail(PMPD_EINVAL, "pmpd_packed_size: output pointer is NULL");
  int64_t rows = padded_rows(out_f);
  *plane_bytes = static_cast<size_t>(rows) * static_cast<size_t>(in_f) / 8;
  *sm_bytes = static_cast<size_t>(rows) * static_cast<size_t>(in_f / kGroup) * 4;
  return PMPD_OK;
}

int32_t pmpd_pack(const uint8_t* q4, const uint16_t* scale, const uint16_t* minv, int32_t out_f, int32_t in_f,
                  int32_t group, void* const planes[4], void* scale_min) {
  int32_t rc = check_shape(out_f, in_f, group);
  if (rc) return rc;
  if (!q4 || !scale || !minv || !planes || !scale_min) return fail(PMPD_EINVAL, "pmpd_pack: NULL argument");
  for (int k = 0; k < 4; ++k) {
    if (!planes[k]) return fail(PMPD_EINVAL, "pmpd_pack: planes[%d] is NULL", k);
    if (reinterpret_cast<uintptr_t>(planes[k]) % 4) return fail(PMPD_EALIGN, "pmpd_pack: planes[%d] not 4-byte aligned", k);
  }
  if (reinterpret_cast<uintptr_t>(scale_min) % 4) return fail(PMPD_EALIGN, "pmpd_pack: scale_min not 4-byte aligned");

  const int64_t G = in_f / kGroup;
  const int64_t n_tiles = padded_rows(out_f) / kTile;
  uint32_t* pl[4];
  for (int k = 0; k < 4; ++k) pl[k] = static_cast<uint32_t*>(planes[k]);
  uint32_t* sm = static_cast<uint32_t*>(scale_min);

  // Tiles are independent: split them over host threads.
  unsigned hw = std::thread::hardware_concurrency();
  int n_thr = static_cast<int>(std::min<int64_t>(std::max(1u, std::min(hw, 16u)), n_tiles));
  std::vector<int> bad(n_thr, 0);
  // bit_home() split into its column part and its row part
  int col_word[kGroup], col_bit[2][kGroup], row_word[kTile];
  for (int e = 0; e < kGroup; ++e) {
    col_word[e] = bit_home(0, 0, e).word;
    col_bit[0][e] = bit_home(0, 0, e).bit;
    col_bit[1][e] = bit_home(1, 0, e).bit;
  }
  for (int rr = 0; rr < kTile; ++rr) row_word[rr] = bit_home(0, rr, 0).word;
  auto work = [&](int tid) {
    std::vector<uint32_t> blk(4 * 256);
    for (int64_t T = tid; T < n_tiles; T += n_thr) {
      for (int64_t g = 0; g < G; ++g) {
        std::fill(blk.begin(), blk.end(), 0u);
        const int64_t base = (T * G + g) * kTile;  // first (scale, min) word; x4 = first plane word
        for (int rr = 0; rr < kTile; ++rr) {
          const int64_t r = T * kTile + rr;
          if (r >= out_f) {
            sm[base + 4 * (rr & 15) + (rr >> 4)] = 0;
            continue;
          }
          const uint8_t* src = q4 + r * static_cast<int64_t>(in_f) + g * kGroup;
          for (int e = 0; e < kGroup; ++e) {
            uint32_t code = src[e];
            if (code > 15) { bad[tid] = 1; code &= 15; }
            const int w = col_word[e] + row_word[rr];
            for (int k = 0; k < 4; ++k) blk[k * 256 + w] |= ((code >> (3 - k)) & 1u) << col_bit[k & 1][e];
          }
          sm[base + 4 * (rr & 15) + (rr >> 4)] =
              static_cast<uint32_t>(scale[r * G + g]) | (static_cast<uint32_t>(minv[r * G + g]) << 16);
        }
        for (int k = 0; k < 4; ++k) std::memcpy(pl[k] + base * 4, &blk[k * 256], 256 * sizeof(uint32_t));
      }
    }
  };
  std::vector<std::thread> pool;
  for (int t = 1; t < n_thr; ++t) pool.emplace_back(work, t);
  work(0);
  for (auto& t : pool) t.join();
  for (int t = 0; t < n_thr; ++t)
    if (bad[t]) return fail(PMPD_EINVAL, "pmpd_pack: a code is outside 0..15");
  return PMPD_OK;
}

int32_t pmpd_unpack(const pmpd_layer_t* L, int32_t b, uint8_t* qb_out) {
  int32_t rc = check_layer(L, b, "pmpd_unpack");
  if (rc) return rc;
  if (!qb_out) return fail(PMPD_EINVAL, "pmpd_unpack: qb_out is NULL");
  const int64_t in_f = L->in_features, out_f = L->out_features, G = in_f / kGroup;
  for (int64_t r = 0; r < out_f; ++r) {
    const int64_t T = r / kTile;
    const int rr = static_cast<int>(r % kTile);
    for (int64_t g = 0; g < G; ++g) {
      const int64_t base = (T * G + g) * kTile * 4;
      for (int e = 0; e < kGroup; ++e) {
        uint32_t code = 0;
        for (int k = 0; k < b; ++k) {
          const BitHome h = bit_home(k, rr, e);
          code = (code << 1) | ((static_cast<const uint32_t*>(L->planes[k])[base + h.word] >> h.bit) & 1u);
        }
        qb_out[r * in_f + g * kGroup + e] = static_cast<uint8_t>(code);
      }
    }
  }
  return PMPD_OK;
}

// ------------------------------------------------------------------ schedule ----
struct pmpd_schedule {
  std::vector<int32_t> precisions;
  std::vector<int32_t> st;
  int32_t max_steps;
};

int32_t pmpd_schedule_create(const int32_t* precisions, const int32_t* st, int32_t n, int32_t max_steps,
                             pmpd_schedule_t** out) {
  if (!precisions || !st || !out) return fail(PMPD_EINVAL, "pmpd_schedule_create: NULL argument");
  if (n < 1 || n > 16) return fail(PMPD_EINVAL, "pmpd_schedule_create: need 1..16 precisions (got %d)", n);
  if (max_steps < 1) return fail(PMPD_EINVAL, "pmpd_schedule_create: max_steps must be positive");
  for (int j = 0; j < n; ++j) {
    if (precisions[j] < 1 || precisions[j] > 16) return fail(PMPD_EINVAL, "pmpd_schedule_create: precision %d out of range", precisions[j]);
    if (j && precisions[j] >= precisions[j - 1]) return fail(PMPD_EINVAL, "pmpd_schedule_create: precisions must be strictly decreasing");
  }
  if (st[0] != 0) return fail(PMPD_ESCHED, "schedule: the first (highest) precision must start at step 0 (got %d)", st[0]);
  for (int j = 0; j < n; ++j) {
    if (st[j] < 0 || st[j] > max_steps) return fail(PMPD_ESCHED, "schedule: switch point %d outside [0, %d]", st[j], max_steps);
    if (j && st[j] < st[j - 1]) return fail(PMPD_ESCHED, "schedule: precedence violated, %d-bit starts at %d before %d-bit at %d", precisions[j], st[j], precisions[j - 1], st[j - 1]);
  }
  auto* s = new pmpd_schedule;
  s->precisions.assign(precisions, precisions + n);
  s->st.assign(st, st + n);
  s->max_steps = max_steps;
  *out = s;
  return PMPD_OK;
}

void pmpd_schedule_destroy(pmpd_schedule_t* s) { delete s; }

int32_t pmpd_schedule_bits(const pmpd_schedule_t* s, int32_t step, int32_t* b_out) {
  if (!s || !b_out) return fail(PMPD_EINVAL, "pmpd_schedule_bits: NULL argument");
  if (step < 0) return fail(PMPD_EINVAL, "pmpd_schedule_bits: negative step");
  // st is non-decreasing and precisions decreasing: the last reached entry is the lowest precision.
  int32_t b = s->precisions[0];
  for (size_t j = 1; j < s->st.size(); ++j)
    if (s->st[j] <= step) b = s->precisions[j];
  *b_out = b;
  return PMPD_OK;
}

double pmpd_schedule_avg_bits(const pmpd_schedule_t* s, int32_t n_steps) {
  if (!s || n_steps < 1) { fail(PMPD_EINVAL, "pmpd_schedule_avg_bits: bad argument"); return -1.0; }
  // Segment lengths instead of a per-step loop: precision j is active on [st[j], st[j+1]),
  // clipped to the first n_steps steps (st is non-decreasing, so no segment is negative).
  const size_t n = s->st.size();
  int64_t total = 0;
  for (size_t j = 0; j < n; ++j) {
    int64_t lo = std::min<int64_t>(s->st[j], n_steps);
    int64_t hi = (j + 1 < n) ? std::min<int64_t>(s->st[j + 1], n_steps) : n_steps;
    total += (hi - lo) * s->precisions[j];
  }
  return static_cast<double>(total) / static_cast<double>(n_steps);
}

// ------------------------------------------------------- static scheduler search ----
// Candidate switch points (Section 4.3): 0 and k * OL / (N - 1), k = 1 .. N - 1, rounded to the
// nearest integer step (halves up); the last one is OL itself ("never reached").
int32_t pmpd_schedule_grid(int32_t max_steps, int32_t n_points, int32_t* points) {
  if (!points) return fail(PMPD_EINVAL, "pmpd_schedule_grid: points is NULL");
  if (max_steps < 1) return fail(PMPD_EINVAL, "pmpd_schedule_grid: max_steps must be positive");
  if (n_points < 2 || n_points > max_steps + 1) return fail(PMPD_EINVAL, "pmpd_schedule_grid: need 2 <= n_points <= max_steps + 1 (got %d)", n_points);
  for (int32_t k = 0; k < n_points; ++k)
    points[k] = static_cast<int32_t>((2 * static_cast<int64_t>(k) * max_steps + (n_points - 1)) / (2 * (n_points - 1)));
  return PMPD_OK;
}

// Number of progressive schedules, sum over the number of switches r of C(OL, r) C(|P| - 1, r)
// (Section 4.3); -1 on bad arguments or overflow of int64.
int64_t pmpd_schedule_count(int32_t max_steps, int32_t n_precisions) {
  if (max_steps < 1 || n_precisions < 1 || n_precisions > 16) { fail(PMPD_EINVAL, "pmpd_schedule_count: bad argument"); return -1; }
  auto binom = [](int64_t n, int64_t k, bool& ok) -> int64_t {
    if (k < 0 || k > n) return 0;
    __int128 v = 1;
    for (int64_t i = 1; i <= k; ++i) {
      v = v * (n - k + i) / i;
      if (v > INT64_MAX) { ok = false; return 0; }
    }
    return static_cast<int64_t>(v);
  };
  bool ok = true;
  __int128 total = 0;
  for (int r = 0; r < n_precisions; ++r) {
    total += static_cast<__int128>(binom(max_steps, r, ok)) * binom(n_precisions - 1, r, ok);
    if (!ok || total > INT64_MAX) { fail(PMPD_EINVAL, "pmpd_schedule_count: result exceeds int64"); return -1; }
  }
  return static_cast<int64_t>(total);
}

// Offline optimisation of the static scheduler (Eq. 1-3 with the candidate grid of Section 4.3):
// among the schedules with st[0] = 0, st non-decreasing and st[j] on the grid whose quality is at
// least q_ref - eps, the one with the fewest tokens at high precision.  "Fewest" is taken as the
// lowest average bit-width over the max_steps steps; ties go to the schedule that leaves the
// highest precision earliest, then the next one, and so on (lexicographically smallest st).
int32_t pmpd_schedule_search(const int32_t* precisions, int32_t n, int32_t max_steps, int32_t n_points,
                             pmpd_quality_fn quality, void* user, double q_ref, double eps, int32_t* st_out,
                             double* avg_bits_out, int64_t* evaluated_out) {
  if (!precisions || !quality || !st_out) return fail(PMPD_EINVAL, "pmpd_schedule_search: NULL argument");
  if (n < 1 || n > 16) return fail(PMPD_EINVAL, "pmpd_schedule_search: need 1..16 precisions (got %d)", n);
  for (int j = 0; j < n; ++j) {
    if (precisions[j] < 1 || precisions[j] > 16) return fail(PMPD_EINVAL, "pmpd_schedule_search: precision %d out of range", precisions[j]);
    if (j && precisions[j] >= precisions[j - 1]) return fail(PMPD_EINVAL, "pmpd_schedule_search: precisions must be strictly decreasing");
  }
  std::vector<int32_t> grid(static_cast<size_t>(std::max(n_points, 2)));
  int32_t rc = pmpd_schedule_grid(max_steps, n_points, grid.data());
  if (rc) return rc;
  grid.erase(std::unique(grid.begin(), grid.end()), grid.end());

  std::vector<int32_t> idx(n, 0), st(n, 0), best;
  int64_t best_bits = -1, evaluated = 0;
  // odometer over non-decreasing index vectors idx[1..n-1] (idx[0] = 0 -> st[0] = 0)
  while (true) {
    for (int j = 0; j < n; ++j) st[j] = grid[idx[j]];
    // total bits over max_steps steps: precision j is active on [st[j], st[j+1])
    int64_t bits = 0;
    for (int j = 0; j < n; ++j) {
      const int64_t hi = j + 1 < n ? st[j + 1] : max_steps;
      bits += (hi - st[j]) * precisions[j];
    }
    const bool better = best_bits < 0 || bits < best_bits || (bits == best_bits && st < best);
    if (better) {  // the quality measurement is the expensive part: only ask when it could win
      ++evaluated;
      if (quality(precisions, st.data(), n, user) >= q_ref - eps) {
        best_bits = bits;
        best = st;
      }
    }
    int j = n - 1;
    while (j >= 1 && idx[j] == static_cast<int32_t>(grid.size()) - 1) --j;
    if (j < 1) break;
    ++idx[j];
    for (int k = j + 1; k < n; ++k) idx[k] = idx[j];
  }
  if (evaluated_out) *evaluated_out = evaluated;
  if (best_bits < 0) return fail(PMPD_ESCHED, "pmpd_schedule_search: no schedule on the grid reaches quality %g", q_ref - eps);
  for (int j = 0; j < n; ++j) st_out[j] = best[j];
  if (avg_bits_out) *avg_bits_out = static_cast<double>(best_bits) / static_cast<double>(max_steps);
  return PMPD_OK;
}

}  // extern "C"
