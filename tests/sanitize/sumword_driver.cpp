// Host-side unit test of the 64-bit sum words of the dependency-ordered step (pmpd_sumword.hpp is
// plain C++ shared with the kernels).  Built with the sanitizers by tests/test_sanitizers.py: an
// out-of-range float-to-integer conversion, which is undefined, would be reported.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <initializer_list>
#include <limits>

#include "pmpd_sumword.hpp"

using namespace pmpd;

#define REQUIRE(cond)                                                           \
  do {                                                                          \
    if (!(cond)) {                                                              \
      std::fprintf(stderr, "sumword_driver: %s failed at line %d\n", #cond, __LINE__); \
      return 1;                                                                 \
    }                                                                           \
  } while (0)

static double decode(unsigned long long w, int n) {  // the exact value of the word's fixed-point sum
  const unsigned long long f = (w & ((1ull << kCountShift) - 1)) - static_cast<unsigned long long>(n) * kPartBias;
  const long long sf = static_cast<long long>(f << 5) >> 5;  // sign-extend 59 bits
  return std::ldexp(static_cast<double>(sf), -32);
}

int main() {
  const float tiny = std::ldexp(1.0f, -25);
  // one part: floor to 2^-32, exact for non-negative values and for values of magnitude >= 1
  const float exact[] = {0.0f, 0.5f, 1.0f, 3.25f, 1234.5678f, 2097151.0f, -1.0f, -2.5f, -1234.5678f, -2097151.0f, 1e-9f};
  for (float v : exact) {
    const unsigned long long w = part_word(v) + part_word(0.0f);
    REQUIRE(sum_complete(w, 2) && !sum_complete(w, 1) && !sum_complete(w, 3));
    const double d = decode(w, 2);
    REQUIRE(d <= static_cast<double>(v) && static_cast<double>(v) - d < std::ldexp(1.0, -32));
  }
  // negative values of magnitude below one: the fraction 1 - |v| is rounded to 24 bits
  const float small_neg[] = {-0.3f, -0.999999f, -1e-3f, -tiny * 1.5f, -0.5f};
  for (float v : small_neg) {
    const double d = decode(part_word(v) + part_word(0.0f), 2);
    REQUIRE(std::fabs(d - static_cast<double>(v)) <= std::ldexp(1.0, -25) + std::ldexp(1.0, -32));
  }
  // -2^-25 < v < 0: the fraction rounds to one and carries; the part counts as zero, nothing overflows
  const float carry[] = {-1e-9f, -tiny * 0.99f, -std::numeric_limits<float>::denorm_min(), -0.0f};
  for (float v : carry) {
    const unsigned long long w = part_word(v) + part_word(0.5f);
    REQUIRE(sum_complete(w, 2));
    REQUIRE(sum_value(w, 2) == 0.5f);
  }
  // clamping: beyond the limit, infinities, NaN (counts as the lower bound); the count is never damaged
  REQUIRE(part_word(1e30f) == part_word(kPartLimit));
  REQUIRE(part_word(std::numeric_limits<float>::infinity()) == part_word(kPartLimit));
  REQUIRE(part_word(-1e30f) == part_word(-kPartLimit));
  REQUIRE(part_word(-std::numeric_limits<float>::infinity()) == part_word(-kPartLimit));
  REQUIRE(part_word(std::numeric_limits<float>::quiet_NaN()) == part_word(-kPartLimit));
  for (float v : {kPartLimit, -kPartLimit}) {
    unsigned long long w = 0;
    for (int k = 1; k <= kMaxParts; ++k) {
      w += part_word(v);
      REQUIRE(sum_complete(w, k));
      REQUIRE(decode(w, k) == static_cast<double>(k) * v);
    }
    REQUIRE(sum_value(w, kMaxParts) == static_cast<float>(kMaxParts) * v);
  }
  // the order of arrival does not matter, and the decoded value is the correctly rounded sum
  {
    const float parts[5] = {0.125f, -7.75f, 1000.5f, -0.3f, 3e-5f};
    unsigned long long fwd = 0, bwd = 0;
    double sum = 0;
    for (int k = 0; k < 5; ++k) {
      fwd += part_word(parts[k]);
      bwd += part_word(parts[4 - k]);
      sum += parts[k];
    }
    REQUIRE(fwd == bwd && sum_complete(fwd, 5));
    REQUIRE(std::fabs(static_cast<double>(sum_value(fwd, 5)) - sum) <= 5 * std::ldexp(1.0, -25) + std::fabs(sum) * std::ldexp(1.0, -24));
  }
  // a row with a single part carries its fp32 bits unchanged
  const float whole[] = {0.0f, -0.0f, 1.5f, -3e38f, 1e-40f, std::numeric_limits<float>::infinity()};
  for (float v : whole) {
    const unsigned long long w = whole_word(v);
    REQUIRE(sum_complete(w, 1) && !sum_complete(w, 2) && !sum_complete(0, 1));
    const float back = sum_value(w, 1);
    REQUIRE(std::memcmp(&back, &v, 4) == 0);
  }
  std::puts("sumword_driver: ok");
  return 0;
}
