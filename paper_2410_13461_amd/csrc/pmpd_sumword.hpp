// 64-bit sum words of the dependency-ordered step: plain C++ shared by the kernels (device) and a
// host-side unit test, no HIP types.
//
// Sums that meet across workgroups are 64-bit words: 32 fractional bits, 27 integer bits, and in the
// top 5 bits the number of K-parts that have been added.  A part adds 2^59 + 2^53 + floor(v 2^32)
// with one integer atomic: the bias 2^53 (= 2^21 in units of one) keeps the addend's low 59 bits
// positive, so nothing is borrowed from the count, and up to 31 parts cannot carry into it.  Integer
// addition is associative: the bits do not depend on the order of arrival (no floating-point
// atomics, no partial-sum buffers), and a reader sees in the word itself whether the sum is
// complete, so no flag, acknowledgement or barrier stands between a producer's add and its
// consumers.  A part's value is clamped to +-(2^21 - 1) (a NaN becomes the lower bound), so that no
// input can damage the count; what lies below 2^-32 is dropped.
#pragma once

#include <cmath>
#include <cstdint>
#include <cstring>

#if defined(__HIPCC__)
#define PMPD_HD __host__ __device__ inline
#else
#define PMPD_HD inline
#endif

namespace pmpd {

constexpr int kCountShift = 59;
constexpr int kMaxParts = 31;
constexpr unsigned long long kPartBias = 1ull << 53;
constexpr float kPartLimit = 2097151.0f;

PMPD_HD unsigned long long part_word(float v) {
  v = fminf(fmaxf(v, -kPartLimit), kPartLimit);  // fmaxf(NaN, lower) = lower
  float fl = floorf(v);
  // v - floor(v) lies in [0, 1].  It is exact except for a negative v of magnitude below one, where
  // it is rounded to 24 bits (error at most 2^-25); for -2^-25 < v < 0 it rounds to 1.0, which then
  // carries into the integer part (the value becomes 0) instead of overflowing the conversion.
  float fr = v - fl;
  if (fr >= 1.0f) {
    fr = 0.0f;
    fl += 1.0f;
  }
  const int hi = static_cast<int>(fl);
  const uint32_t lo = static_cast<uint32_t>(fr * 4294967296.0f);  // fr <= 1 - 2^-24: in range
  return ((static_cast<unsigned long long>(static_cast<uint32_t>(hi)) << 32) | lo) + kPartBias + (1ull << kCountShift);
}

// The word of a row that has a single part carries that part as it is: its fp32 bits under a count of one.
PMPD_HD unsigned long long whole_word(float v) {
  uint32_t bits;
  memcpy(&bits, &v, sizeof(bits));
  return (1ull << kCountShift) | bits;
}

PMPD_HD bool sum_complete(unsigned long long w, int n_parts) { return static_cast<int>(w >> kCountShift) == n_parts; }

PMPD_HD float sum_value(unsigned long long w, int n_parts) {
  if (n_parts == 1) {
    const uint32_t bits = static_cast<uint32_t>(w);
    float v;
    memcpy(&v, &bits, sizeof(v));
    return v;
  }
  const unsigned long long f = (w & ((1ull << kCountShift) - 1)) - static_cast<unsigned long long>(n_parts) * kPartBias;
  const int hi = static_cast<int>(static_cast<uint32_t>(f >> 32));
  const uint32_t lo = static_cast<uint32_t>(f);
  return fmaf(static_cast<float>(lo), 2.3283064365386963e-10f, static_cast<float>(hi));  // one rounding, wherever it is used
}

}  // namespace pmpd
