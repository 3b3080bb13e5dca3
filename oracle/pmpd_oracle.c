/*
 * CPU oracle for the PMPD decode linear-layer path.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product path may call, link or import this file.  It shares no
 * code with the HIP library; the two only agree on the storage format, which
 * each implements on its own from the index formula written out below.
 *
 * What it computes (paper: Section 2.1 "Weight-only Quantization" and Section 5
 * "PMPD Implementation Details" for the nested multi-precision weight store;
 * Algorithm 1, deployment stage, for the per-step linear layers; Section 4.2 /
 * Eq. 1-3 for the schedule; Section 5 "Baselines" for the average bit-width):
 *
 *   nested code      q_b[r][i] = q4[r][i] >> (4 - b)                  b in {4,3,2}
 *   reconstruction   W_b[r][i] = a[r][g] + s[r][g] * 2^(4-b) * (q_b[r][i] + 0.5),  g = i / 128
 *   linear layer     y[r]      = sum_i W_b[r][i] * x[i]               (fp64, index order)
 *   error budget     T[r]      = sum_i |W_b[r][i]| * |x[i]|
 *
 * The paper does not print the quantiser; the uniform group-wise reading above
 * (bin-midpoint reconstruction, truncation nesting) is the one this build fixes.
 * Everything is plain loops in fp64: every product a + s*k*(q+0.5) is exact in
 * fp64 because s and a are fp16 values and k*(q+0.5) is a small dyadic number.
 *
 * Storage format ("tile-plane"), an interface between pack and the kernels (the paper
 * fixes none; each side implements this index formula on its own):
 *   rows are padded to a multiple of 64; row r lives in tile T = r / 64 at position
 *   rr = r % 64 = 16*t + j  (t 0..3, j 0..15);
 *   input feature i lives in group g = i / 128 at position e = i % 128 = 32*kb + 8*v + c
 *   (kb 0..3, v 0..3, c 0..7), and n = c/2 + 4*(c%2) is the nibble of column c.
 *   Plane k (k = 0 is the most significant bit of the 4-bit code) is an array of 32-bit
 *   words; the bit of weight (r, i) is bit
 *        4*n + 1, 4*n + 3, 4*n, 4*n + 2            for v = 0, 1, 2, 3   (k = 0 or 2)
 *        4*n, 4*n + 2, (4*n + 31) mod 32, 4*n + 1   for v = 0, 1, 2, 3   (k = 1 or 3)
 *   of word  ((T*G + g)*64 + 16*kb + j)*4 + t,   G = in / 128.
 *   Scale and minimum are one 32-bit word per (row, group) at index (T*G + g)*64 + 4*j + t:
 *   low 16 bits = fp16 scale, high 16 bits = fp16 minimum.
 *   A b-bit pass reads planes 0..b-1 only.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_GROUP 128
#define ORC_TILE 64

/* ---- fp16 bit pattern -> double, exact ---------------------------------- */
static double orc_half_to_double(uint16_t h) {
  int sign = (h >> 15) & 1;
  int expo = (h >> 10) & 0x1f;
  int mant = h & 0x3ff;
  double v;
  if (expo == 0) {
    v = ldexp((double)mant, -24); /* subnormal: mant * 2^-24 */
  } else if (expo == 31) {
    v = mant ? NAN : INFINITY;
  } else {
    v = ldexp((double)(1024 + mant), expo - 25);
  }
  return sign ? -v : v;
}

double orc_fp16_value(uint16_t h) { return orc_half_to_double(h); }

/* ---- storage-format index formula ---------------------------------------- */
static int64_t orc_padded_rows(int64_t out_f) { return (out_f + ORC_TILE - 1) / ORC_TILE * ORC_TILE; }

int64_t orc_plane_words(int64_t out_f, int64_t in_f) { return orc_padded_rows(out_f) * (in_f / 32); }
int64_t orc_sa_words(int64_t out_f, int64_t in_f) { return orc_padded_rows(out_f) * (in_f / ORC_GROUP); }

static int64_t orc_sa_index(int64_t r, int64_t g, int64_t G) {
  int64_t T = r / ORC_TILE;
  int rr = (int)(r % ORC_TILE);
  int t = rr / 16, j = rr % 16;
  return (T * G + g) * ORC_TILE + 4 * j + t;
}

static void orc_locate(int64_t r, int64_t i, int k, int64_t in_f, int64_t* word, int* pos) {
  int64_t G = in_f / ORC_GROUP;
  int64_t T = r / ORC_TILE;
  int rr = (int)(r % ORC_TILE);
  int t = rr / 16, j = rr % 16;
  int64_t g = i / ORC_GROUP;
  int e = (int)(i % ORC_GROUP);
  int kb = e / 32, v = (e % 32) / 8, c = e % 8;
  int n = c / 2 + 4 * (c % 2);
  int bit;
  if (k % 2 == 0) {
    switch (v) {
      case 0: bit = 4 * n + 1; break;
      case 1: bit = 4 * n + 3; break;
      case 2: bit = 4 * n; break;
      default: bit = 4 * n + 2; break;
    }
  } else {
    switch (v) {
      case 0: bit = 4 * n; break;
      case 1: bit = 4 * n + 2; break;
      case 2: bit = (4 * n + 31) % 32; break;
      default: bit = 4 * n + 1; break;
    }
  }
  *word = ((T * G + g) * ORC_TILE + 16 * kb + j) * 4 + t;
  *pos = bit;
}

/* ---- pack: 4-bit codes -> 4 bit-planes + (scale, min) words --------------- */
int orc_pack(const uint8_t* q4, const uint16_t* s, const uint16_t* a, int64_t out_f, int64_t in_f,
             uint32_t* plane0, uint32_t* plane1, uint32_t* plane2, uint32_t* plane3, uint32_t* sa) {
  if (in_f <= 0 || out_f <= 0 || in_f % ORC_GROUP) return -1;
  uint32_t* planes[4] = {plane0, plane1, plane2, plane3};
  int64_t G = in_f / ORC_GROUP;
  int64_t pw = orc_plane_words(out_f, in_f);
  for (int k = 0; k < 4; ++k) memset(planes[k], 0, (size_t)pw * 4);
  memset(sa, 0, (size_t)orc_sa_words(out_f, in_f) * 4);
  for (int64_t r = 0; r < out_f; ++r) {
    for (int64_t i = 0; i < in_f; ++i) {
      uint8_t code = q4[r * in_f + i];
      if (code > 15) return -2;
      for (int k = 0; k < 4; ++k) {
        int bit = (code >> (3 - k)) & 1; /* plane 0 carries the MSB */
        int64_t w;
        int pos;
        orc_locate(r, i, k, in_f, &w, &pos);
        if (bit) planes[k][w] |= (uint32_t)1 << pos;
      }
    }
    for (int64_t g = 0; g < G; ++g)
      sa[orc_sa_index(r, g, G)] = (uint32_t)s[r * G + g] | ((uint32_t)a[r * G + g] << 16);
  }
  return 0;
}

/* ---- unpack: top-b planes -> b-bit codes (reads planes 0..b-1 only) -------- */
int orc_unpack(const uint32_t* plane0, const uint32_t* plane1, const uint32_t* plane2,
               const uint32_t* plane3, int b, int64_t out_f, int64_t in_f, uint8_t* qb) {
  if (b < 1 || b > 4 || in_f % ORC_GROUP) return -1;
  const uint32_t* planes[4] = {plane0, plane1, plane2, plane3};
  for (int64_t r = 0; r < out_f; ++r)
    for (int64_t i = 0; i < in_f; ++i) {
      int code = 0;
      for (int k = 0; k < b; ++k) {
        int64_t w;
        int pos;
        orc_locate(r, i, k, in_f, &w, &pos);
        code = (code << 1) | (int)((planes[k][w] >> pos) & 1u);
      }
      qb[r * in_f + i] = (uint8_t)code;
    }
  return 0;
}

void orc_unpack_sa(const uint32_t* sa, int64_t out_f, int64_t in_f, uint16_t* s, uint16_t* a) {
  int64_t G = in_f / ORC_GROUP;
  for (int64_t r = 0; r < out_f; ++r)
    for (int64_t g = 0; g < G; ++g) {
      uint32_t w = sa[orc_sa_index(r, g, G)];
      s[r * G + g] = (uint16_t)(w & 0xffffu);
      a[r * G + g] = (uint16_t)(w >> 16);
    }
}

/* ---- reconstruction: W_b = a + s * 2^(4-b) * (q_b + 0.5) ------------------- */
static double orc_reconstruct(double a, double s, int qb, int b) {
  double step = s * (double)(1 << (4 - b));
  return a + step * ((double)qb + 0.5);
}

/* dense W_b from logical inputs (q4 row-major, s/a [out][in/128] fp16 bits) */
int orc_dequant(const uint8_t* q4, const uint16_t* s, const uint16_t* a, int b, int64_t out_f,
                int64_t in_f, double* W) {
  if (b < 1 || b > 4 || in_f % ORC_GROUP) return -1;
  int64_t G = in_f / ORC_GROUP;
  for (int64_t r = 0; r < out_f; ++r)
    for (int64_t i = 0; i < in_f; ++i) {
      int64_t g = i / ORC_GROUP;
      int qb = q4[r * in_f + i] >> (4 - b);
      W[r * in_f + i] =
          orc_reconstruct(orc_half_to_double(a[r * G + g]), orc_half_to_double(s[r * G + g]), qb, b);
    }
  return 0;
}

/* ---- linear layer from logical inputs:  Y[j][r] = sum_i W_b[r][i] * X[j][i] -- */
int orc_linear_logical(const uint8_t* q4, const uint16_t* s, const uint16_t* a, int b, int64_t out_f,
                       int64_t in_f, const uint16_t* x, int64_t m, double* y, double* tbudget) {
  if (b < 1 || b > 4 || in_f % ORC_GROUP) return -1;
  int64_t G = in_f / ORC_GROUP;
#pragma omp parallel for schedule(static)
  for (int64_t r = 0; r < out_f; ++r) {
    for (int64_t j = 0; j < m; ++j) {
      double acc = 0.0, tb = 0.0;
      for (int64_t i = 0; i < in_f; ++i) {
        int64_t g = i / ORC_GROUP;
        int qb = q4[r * in_f + i] >> (4 - b);
        double w = orc_reconstruct(orc_half_to_double(a[r * G + g]), orc_half_to_double(s[r * G + g]), qb, b);
        double xv = orc_half_to_double(x[j * in_f + i]);
        acc += w * xv;
        tb += fabs(w) * fabs(xv);
      }
      y[j * out_f + r] = acc;
      if (tbudget) tbudget[j * out_f + r] = tb;
    }
  }
  return 0;
}

/* ---- linear layer from the packed store, reading planes 0..b-1 only -------- *
 * Rows [row0, row0 + nrows) only, so that callers can sample a large layer.   */
int orc_linear_packed(const uint32_t* plane0, const uint32_t* plane1, const uint32_t* plane2,
                      const uint32_t* plane3, const uint32_t* sa, int b, int64_t out_f, int64_t in_f,
                      int64_t row0, int64_t nrows, const uint16_t* x, int64_t m, double* y,
                      double* tbudget) {
  if (b < 1 || b > 4 || in_f % ORC_GROUP || row0 < 0 || row0 + nrows > out_f) return -1;
  const uint32_t* planes[4] = {plane0, plane1, plane2, plane3};
  int64_t G = in_f / ORC_GROUP;
#pragma omp parallel for schedule(static)
  for (int64_t rr = 0; rr < nrows; ++rr) {
    int64_t r = row0 + rr;
    for (int64_t j = 0; j < m; ++j) {
      double acc = 0.0, tb = 0.0;
      for (int64_t i = 0; i < in_f; ++i) {
        int64_t g = i / ORC_GROUP;
        uint32_t w32 = sa[orc_sa_index(r, g, G)];
        double sv = orc_half_to_double((uint16_t)(w32 & 0xffffu));
        double av = orc_half_to_double((uint16_t)(w32 >> 16));
        int code = 0;
        for (int k = 0; k < b; ++k) {
          int64_t w;
          int pos;
          orc_locate(r, i, k, in_f, &w, &pos);
          code = (code << 1) | (int)((planes[k][w] >> pos) & 1u);
        }
        double wv = orc_reconstruct(av, sv, code, b);
        double xv = orc_half_to_double(x[j * in_f + i]);
        acc += wv * xv;
        tb += fabs(wv) * fabs(xv);
      }
      y[j * nrows + rr] = acc;
      if (tbudget) tbudget[j * nrows + rr] = tb;
    }
  }
  return 0;
}

int orc_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---- precision-switching schedule (Section 4.2, Eq. 1-3; Algorithm 1) ------- *
 * precisions[] strictly decreasing, st[j] = first decode step run at precisions[j].
 * Valid iff st[0] == 0, 0 <= st[j] <= OL and st is non-decreasing (a higher
 * precision never starts after a lower one).  Step k runs at the lowest precision
 * whose switch point has been reached.                                         */
int orc_schedule_valid(const int32_t* precisions, const int32_t* st, int32_t n, int32_t OL) {
  if (n < 1 || OL < 1) return 0;
  if (st[0] != 0) return 0;
  for (int j = 0; j < n; ++j) {
    if (precisions[j] < 1 || precisions[j] > 16) return 0;
    if (st[j] < 0 || st[j] > OL) return 0;
    if (j > 0 && precisions[j] >= precisions[j - 1]) return 0;
    if (j > 0 && st[j] < st[j - 1]) return 0;
  }
  return 1;
}

int orc_schedule_bits(const int32_t* precisions, const int32_t* st, int32_t n, int32_t step) {
  int best = precisions[0];
  for (int j = 0; j < n; ++j)
    if (st[j] <= step && precisions[j] < best) best = precisions[j];
  return best;
}

/* mean of bits(k) over k = 0 .. n_steps-1 (tokens generated at each precision) */
double orc_schedule_avg_bits(const int32_t* precisions, const int32_t* st, int32_t n, int32_t n_steps) {
  double total = 0.0;
  for (int32_t k = 0; k < n_steps; ++k) total += (double)orc_schedule_bits(precisions, st, n, k);
  return total / (double)n_steps;
}
