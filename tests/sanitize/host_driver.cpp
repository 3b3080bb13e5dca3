// Sanitizer driver for the host part of the library (pmpd_host.cpp: pack, unpack, schedule, static
// scheduler search).  Built by tests/test_sanitizers.py with -fsanitize=address,undefined together
// with pmpd_host.cpp and run as a program of its own, so that the sanitizer runtime is the first
// thing in the process.  It checks results only as far as it can without a second implementation
// (round trips, prefix property, closed forms); the point of the run is that no access goes out of
// bounds and nothing undefined happens on ragged shapes and on every error path.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "pmpd.h"

#define REQUIRE(cond)                                                       \
  do {                                                                      \
    if (!(cond)) {                                                          \
      std::fprintf(stderr, "host_driver: %s failed at line %d (%s)\n", #cond, __LINE__, pmpd_last_error()); \
      return 1;                                                             \
    }                                                                       \
  } while (0)

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static uint32_t next_u32() {  // xorshift64*: inputs only
  g_state ^= g_state >> 12;
  g_state ^= g_state << 25;
  g_state ^= g_state >> 27;
  return static_cast<uint32_t>((g_state * 0x2545F4914F6CDD1Dull) >> 32);
}

static int pack_round_trip(int out_f, int in_f) {
  const int G = in_f / PMPD_GROUP;
  std::vector<uint8_t> q4(static_cast<size_t>(out_f) * in_f);
  std::vector<uint16_t> s(static_cast<size_t>(out_f) * G), a(s.size());
  for (auto& v : q4) v = static_cast<uint8_t>(next_u32() & 15);
  for (auto& v : s) v = static_cast<uint16_t>(0x1400 + (next_u32() & 0x3ff));
  for (auto& v : a) v = static_cast<uint16_t>(0x9c00 + (next_u32() & 0x3ff));
  size_t pb = 0, sb = 0;
  REQUIRE(pmpd_packed_size(out_f, in_f, PMPD_GROUP, &pb, &sb) == PMPD_OK);
  // exact-size heap buffers: one byte past the end is caught
  std::vector<std::vector<uint32_t>> planes(4, std::vector<uint32_t>(pb / 4, 0xDEADBEEFu));
  std::vector<uint32_t> sm(sb / 4, 0xDEADBEEFu);
  void* pp[4] = {planes[0].data(), planes[1].data(), planes[2].data(), planes[3].data()};
  REQUIRE(pmpd_pack(q4.data(), s.data(), a.data(), out_f, in_f, PMPD_GROUP, pp, sm.data()) == PMPD_OK);
  std::vector<uint8_t> qb(q4.size());
  for (int b = 1; b <= 4; ++b) {
    pmpd_layer_t L;
    std::memset(&L, 0, sizeof(L));
    L.out_features = out_f;
    L.in_features = in_f;
    L.group_size = PMPD_GROUP;
    for (int k = 0; k < b; ++k) L.planes[k] = planes[k].data();  // lower planes absent
    L.scale_min = sm.data();
    REQUIRE(pmpd_unpack(&L, b, qb.data()) == PMPD_OK);
    for (size_t i = 0; i < q4.size(); ++i) REQUIRE(qb[i] == (q4[i] >> (4 - b)));
  }
  // a code outside 0..15 is refused, not written out of place
  q4[q4.size() / 2] = 16;
  REQUIRE(pmpd_pack(q4.data(), s.data(), a.data(), out_f, in_f, PMPD_GROUP, pp, sm.data()) == PMPD_EINVAL);
  return 0;
}

struct Quality {
  int min_high_steps;  // feasible iff the lowest precision starts at or after this step
  int calls;
};
static double quality_cb(const int32_t* P, const int32_t* st, int32_t n, void* user) {
  (void)P;
  Quality* q = static_cast<Quality*>(user);
  ++q->calls;
  return st[n - 1] >= q->min_high_steps ? 1.0 : 0.0;
}

int main() {
  const int shapes[][2] = {{1, 128}, {64, 128}, {65, 256}, {130, 384}, {257, 1408}};
  for (const auto& sh : shapes)
    if (pack_round_trip(sh[0], sh[1])) return 1;

  // argument errors: nothing is touched
  size_t pb = 0, sb = 0;
  REQUIRE(pmpd_packed_size(0, 128, 128, &pb, &sb) == PMPD_EINVAL);
  REQUIRE(pmpd_packed_size(64, 100, 128, &pb, &sb) == PMPD_EINVAL);
  REQUIRE(pmpd_packed_size(64, 128, 64, &pb, &sb) == PMPD_EINVAL);
  REQUIRE(pmpd_packed_size(64, 128, 128, nullptr, &sb) == PMPD_EINVAL);
  REQUIRE(pmpd_unpack(nullptr, 4, nullptr) == PMPD_EINVAL);
  REQUIRE(std::strlen(pmpd_last_error()) > 0);
  for (int st = -7; st <= 1; ++st) REQUIRE(pmpd_strerror(st) != nullptr);

  // schedule: the two workloads' closed forms and every refusal
  {
    const int32_t P[3] = {4, 3, 2}, S[3] = {0, 64, 160};
    pmpd_schedule_t* sch = nullptr;
    REQUIRE(pmpd_schedule_create(P, S, 3, 256, &sch) == PMPD_OK);
    REQUIRE(pmpd_schedule_avg_bits(sch, 256) == 2.875);
    int32_t b = 0;
    const int steps[6] = {0, 63, 64, 159, 160, 255}, want[6] = {4, 4, 3, 3, 2, 2};
    for (int i = 0; i < 6; ++i) {
      REQUIRE(pmpd_schedule_bits(sch, steps[i], &b) == PMPD_OK);
      REQUIRE(b == want[i]);
    }
    REQUIRE(pmpd_schedule_bits(sch, -1, &b) == PMPD_EINVAL);
    REQUIRE(pmpd_schedule_bits(sch, 1 << 30, &b) == PMPD_OK && b == 2);
    REQUIRE(pmpd_schedule_avg_bits(sch, 0) < 0);
    pmpd_schedule_destroy(sch);
    const int32_t bad1[3] = {1, 64, 160}, bad2[3] = {0, 160, 64}, bad3[3] = {0, 64, 257}, badP[3] = {4, 4, 2};
    REQUIRE(pmpd_schedule_create(P, bad1, 3, 256, &sch) == PMPD_ESCHED);
    REQUIRE(pmpd_schedule_create(P, bad2, 3, 256, &sch) == PMPD_ESCHED);
    REQUIRE(pmpd_schedule_create(P, bad3, 3, 256, &sch) == PMPD_ESCHED);
    REQUIRE(pmpd_schedule_create(badP, S, 3, 256, &sch) == PMPD_EINVAL);
    REQUIRE(pmpd_schedule_create(P, S, 0, 256, &sch) == PMPD_EINVAL);
    REQUIRE(pmpd_schedule_create(P, S, 17, 256, &sch) == PMPD_EINVAL);
    const int32_t P2[2] = {3, 2}, S2[2] = {0, 48};
    REQUIRE(pmpd_schedule_create(P2, S2, 2, 128, &sch) == PMPD_OK);
    REQUIRE(pmpd_schedule_avg_bits(sch, 128) == 2.375);
    pmpd_schedule_destroy(sch);
    pmpd_schedule_destroy(nullptr);
  }
  // grid, count, search
  {
    int32_t pts[9];
    REQUIRE(pmpd_schedule_grid(256, 5, pts) == PMPD_OK);
    const int32_t want[5] = {0, 64, 128, 192, 256};
    for (int k = 0; k < 5; ++k) REQUIRE(pts[k] == want[k]);
    REQUIRE(pmpd_schedule_grid(7, 8, pts) == PMPD_OK);  // n_points == max_steps + 1: every step
    for (int k = 0; k < 8; ++k) REQUIRE(pts[k] == k);
    REQUIRE(pmpd_schedule_grid(7, 9, pts) == PMPD_EINVAL);
    REQUIRE(pmpd_schedule_grid(7, 1, pts) == PMPD_EINVAL);
    REQUIRE(pmpd_schedule_count(256, 3) == 33153);
    REQUIRE(pmpd_schedule_count(0, 3) == -1);
    REQUIRE(pmpd_schedule_count(1 << 30, 16) == -1);  // overflow is reported, not wrapped
    const int32_t P[3] = {4, 3, 2};
    int32_t st[3] = {-1, -1, -1};
    double avg = 0;
    int64_t evaluated = 0;
    Quality q{128, 0};
    REQUIRE(pmpd_schedule_search(P, 3, 256, 5, quality_cb, &q, 1.0, 0.0, st, &avg, &evaluated) == PMPD_OK);
    REQUIRE(st[0] == 0 && st[1] == 0 && st[2] == 128);  // 3 bits from the start, 2 bits from step 128
    REQUIRE(avg == 2.5);
    REQUIRE(evaluated == q.calls && evaluated >= 1 && evaluated <= 15);
    Quality never{1000, 0};
    REQUIRE(pmpd_schedule_search(P, 3, 256, 5, quality_cb, &never, 1.0, 0.0, st, &avg, &evaluated) == PMPD_ESCHED);
    REQUIRE(pmpd_schedule_search(P, 3, 256, 5, nullptr, nullptr, 1.0, 0.0, st, &avg, &evaluated) == PMPD_EINVAL);
    REQUIRE(pmpd_schedule_search(P, 3, 4, 9, quality_cb, &q, 1.0, 0.0, st, &avg, &evaluated) == PMPD_EINVAL);
    // duplicated grid points (few steps, many points) collapse instead of being visited twice
    Quality any{0, 0};
    REQUIRE(pmpd_schedule_search(P, 3, 3, 4, quality_cb, &any, 1.0, 0.0, st, &avg, nullptr) == PMPD_OK);
    REQUIRE(st[0] == 0 && st[1] == 0 && st[2] == 0 && avg == 2.0);
  }
  std::puts("host_driver: ok");
  return 0;
}
