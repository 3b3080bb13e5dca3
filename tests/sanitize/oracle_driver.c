/* Sanitizer driver for the CPU oracle (oracle/pmpd_oracle.c).  Built by tests/test_sanitizers.py
 * with -fsanitize=address,undefined together with the oracle's source and run as a program of its
 * own.  Exact-size heap buffers on ragged shapes: any access outside them, any shift or conversion
 * that is undefined, ends the run.  Values are checked only through the oracle's own invariants
 * (round trip, packed == logical, nested midpoints); its pins live in tests/test_oracle_pins.py. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int64_t orc_plane_words(int64_t out_f, int64_t in_f);
int64_t orc_sa_words(int64_t out_f, int64_t in_f);
int orc_pack(const uint8_t* q4, const uint16_t* s, const uint16_t* a, int64_t out_f, int64_t in_f, uint32_t* p0, uint32_t* p1,
             uint32_t* p2, uint32_t* p3, uint32_t* sa);
int orc_unpack(const uint32_t* p0, const uint32_t* p1, const uint32_t* p2, const uint32_t* p3, int b, int64_t out_f, int64_t in_f,
               uint8_t* qb);
void orc_unpack_sa(const uint32_t* sa, int64_t out_f, int64_t in_f, uint16_t* s, uint16_t* a);
int orc_dequant(const uint8_t* q4, const uint16_t* s, const uint16_t* a, int b, int64_t out_f, int64_t in_f, double* W);
int orc_linear_logical(const uint8_t* q4, const uint16_t* s, const uint16_t* a, int b, int64_t out_f, int64_t in_f,
                       const uint16_t* x, int64_t m, double* y, double* t);
int orc_linear_packed(const uint32_t* p0, const uint32_t* p1, const uint32_t* p2, const uint32_t* p3, const uint32_t* sa, int b,
                      int64_t out_f, int64_t in_f, int64_t row0, int64_t nrows, const uint16_t* x, int64_t m, double* y, double* t);
double orc_fp16_value(uint16_t h);
int orc_schedule_valid(const int32_t* P, const int32_t* st, int32_t n, int32_t OL);
int orc_schedule_bits(const int32_t* P, const int32_t* st, int32_t n, int32_t step);
double orc_schedule_avg_bits(const int32_t* P, const int32_t* st, int32_t n, int32_t n_steps);

#define REQUIRE(cond)                                                          \
  do {                                                                         \
    if (!(cond)) {                                                             \
      fprintf(stderr, "oracle_driver: %s failed at line %d\n", #cond, __LINE__); \
      return 1;                                                                \
    }                                                                          \
  } while (0)

static uint64_t g_state = 0x243F6A8885A308D3ull;
static uint32_t next_u32(void) {
  g_state ^= g_state >> 12;
  g_state ^= g_state << 25;
  g_state ^= g_state >> 27;
  return (uint32_t)((g_state * 0x2545F4914F6CDD1Dull) >> 32);
}

static int one_shape(int64_t out_f, int64_t in_f, int64_t m) {
  int64_t G = in_f / 128, n = out_f * in_f;
  uint8_t* q4 = malloc((size_t)n);
  uint8_t* qb = malloc((size_t)n);
  uint16_t* s = malloc((size_t)(out_f * G) * 2);
  uint16_t* a = malloc((size_t)(out_f * G) * 2);
  uint16_t* s2 = malloc((size_t)(out_f * G) * 2);
  uint16_t* a2 = malloc((size_t)(out_f * G) * 2);
  uint16_t* x = malloc((size_t)(m * in_f) * 2);
  int64_t pw = orc_plane_words(out_f, in_f), sw = orc_sa_words(out_f, in_f);
  uint32_t* p[4];
  for (int k = 0; k < 4; ++k) p[k] = malloc((size_t)pw * 4);
  uint32_t* sa = malloc((size_t)sw * 4);
  double* W4 = malloc((size_t)n * 8);
  double* Wb = malloc((size_t)n * 8);
  double* y = malloc((size_t)(m * out_f) * 8);
  double* t = malloc((size_t)(m * out_f) * 8);
  double* yp = malloc((size_t)(m * out_f) * 8);
  for (int64_t i = 0; i < n; ++i) q4[i] = (uint8_t)(next_u32() & 15);
  for (int64_t i = 0; i < out_f * G; ++i) {
    s[i] = (uint16_t)(0x1400 + (next_u32() & 0x3ff)); /* about 1e-3 .. 2e-3 */
    a[i] = (uint16_t)(0x9c00 + (next_u32() & 0x3ff)); /* small negative */
  }
  for (int64_t i = 0; i < m * in_f; ++i) x[i] = (uint16_t)((next_u32() & 0x8000) | (0x3000 + (next_u32() & 0xfff)));
  REQUIRE(orc_pack(q4, s, a, out_f, in_f, p[0], p[1], p[2], p[3], sa) == 0);
  orc_unpack_sa(sa, out_f, in_f, s2, a2);
  REQUIRE(memcmp(s, s2, (size_t)(out_f * G) * 2) == 0 && memcmp(a, a2, (size_t)(out_f * G) * 2) == 0);
  REQUIRE(orc_dequant(q4, s, a, 4, out_f, in_f, W4) == 0);
  for (int b = 1; b <= 4; ++b) {
    /* planes below b are not passed at all */
    REQUIRE(orc_unpack(p[0], b > 1 ? p[1] : NULL, b > 2 ? p[2] : NULL, b > 3 ? p[3] : NULL, b, out_f, in_f, qb) == 0);
    for (int64_t i = 0; i < n; ++i) REQUIRE(qb[i] == (q4[i] >> (4 - b)));
    REQUIRE(orc_dequant(q4, s, a, b, out_f, in_f, Wb) == 0);
    for (int64_t r = 0; r < out_f; ++r)
      for (int64_t i = 0; i < in_f; ++i) {
        double sv = orc_fp16_value(s[r * G + i / 128]);
        REQUIRE(fabs(Wb[r * in_f + i] - W4[r * in_f + i]) <= sv * ((1 << (4 - b)) - 1) / 2.0 + 1e-15);
      }
    if (b < 2) continue;
    REQUIRE(orc_linear_logical(q4, s, a, b, out_f, in_f, x, m, y, t) == 0);
    REQUIRE(orc_linear_packed(p[0], p[1], b > 2 ? p[2] : NULL, b > 3 ? p[3] : NULL, sa, b, out_f, in_f, 0, out_f, x, m, yp, NULL) == 0);
    for (int64_t i = 0; i < m * out_f; ++i) REQUIRE(y[i] == yp[i] && t[i] >= fabs(y[i]));
    if (out_f > 3) { /* a row window that ends at the last row */
      REQUIRE(orc_linear_packed(p[0], p[1], b > 2 ? p[2] : NULL, b > 3 ? p[3] : NULL, sa, b, out_f, in_f, out_f - 3, 3, x, m, yp, t) == 0);
      for (int64_t j = 0; j < m; ++j)
        for (int64_t r = 0; r < 3; ++r) REQUIRE(yp[j * 3 + r] == y[j * out_f + out_f - 3 + r]);
      REQUIRE(orc_linear_packed(p[0], p[1], p[2], p[3], sa, b, out_f, in_f, out_f - 2, 3, x, m, yp, t) == -1);
    }
  }
  q4[n - 1] = 16;
  REQUIRE(orc_pack(q4, s, a, out_f, in_f, p[0], p[1], p[2], p[3], sa) == -2);
  free(q4); free(qb); free(s); free(a); free(s2); free(a2); free(x);
  for (int k = 0; k < 4; ++k) free(p[k]);
  free(sa); free(W4); free(Wb); free(y); free(t); free(yp);
  return 0;
}

int main(void) {
  if (one_shape(1, 128, 1) || one_shape(64, 128, 2) || one_shape(65, 256, 1) || one_shape(130, 384, 3)) return 1;
  /* every fp16 pattern converts without anything undefined */
  double acc = 0;
  for (uint32_t h = 0; h < 65536; ++h) {
    double v = orc_fp16_value((uint16_t)h);
    if (v == v && !isinf(v)) acc += v;
  }
  REQUIRE(acc == 0.0); /* the finite values cancel in pairs +-v */
  const int32_t P[3] = {4, 3, 2}, S[3] = {0, 64, 160}, bad[3] = {0, 160, 64};
  REQUIRE(orc_schedule_valid(P, S, 3, 256) == 1 && orc_schedule_valid(P, bad, 3, 256) == 0);
  REQUIRE(orc_schedule_bits(P, S, 3, 63) == 4 && orc_schedule_bits(P, S, 3, 64) == 3 && orc_schedule_bits(P, S, 3, 1 << 30) == 2);
  REQUIRE(orc_schedule_avg_bits(P, S, 3, 256) == 2.875);
  puts("oracle_driver: ok");
  return 0;
}
