// Host-side check of the prefill deal (pmpd_prefill_deal.hpp): for many sizes, every (item, token block) is taken by
// exactly one workgroup, every workgroup of the grid has at least one item, the shares of a token block differ by at
// most one item, and an XCD (block index % 8) of the XCD-aware deal sees one token block only.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "pmpd_prefill_deal.hpp"

#define CHECK(c)                                                                                       \
  do {                                                                                                 \
    if (!(c)) {                                                                                        \
      std::printf("deal_driver: FAILED %s (n_items %d, m_tiles %d, cus %d)\n", #c, n_items, m_tiles, cus); \
      return 1;                                                                                        \
    }                                                                                                  \
  } while (0)

int main() {
  using namespace pmpd;
  const int item_counts[] = {1, 2, 3, 7, 31, 32, 33, 63, 64, 127, 128, 129, 255, 256, 257, 511, 516, 1000, 8320};
  const int cu_counts[] = {256, 304, 8, 7, 1};
  long cases = 0;
  for (int cus : cu_counts)
    for (int n_items : item_counts)
      for (int m_tiles = 1; m_tiles <= 20; ++m_tiles) {
        const PfGrid g = pf_grid(n_items, m_tiles, cus);
        CHECK(g.per_block >= 1 && g.grid >= 1);
        CHECK(g.per_xcd == 0 || (g.grid == static_cast<unsigned>(kXcds * g.per_xcd) && g.per_block * m_tiles == static_cast<int>(g.grid)));
        std::vector<int> taken(static_cast<size_t>(n_items) * m_tiles, 0);
        std::vector<int> lo(m_tiles, 1 << 30), hi(m_tiles, 0), xcd_block(kXcds, -1);
        for (unsigned b = 0; b < g.grid; ++b) {
          const PfShare s = pf_share(static_cast<int>(b), n_items, m_tiles, g.per_block, g.per_xcd);
          CHECK(s.mtile >= 0 && s.mtile < m_tiles && s.first >= 0 && s.n_mine >= 1);
          for (int k = 0; k < s.n_mine; ++k) {
            const int item = s.first + k * g.per_block;
            CHECK(item < n_items);
            ++taken[static_cast<size_t>(item) * m_tiles + s.mtile];
          }
          if (s.n_mine < lo[s.mtile]) lo[s.mtile] = s.n_mine;
          if (s.n_mine > hi[s.mtile]) hi[s.mtile] = s.n_mine;
          if (g.per_xcd > 0) {
            int& xb = xcd_block[b % kXcds];
            CHECK(xb == -1 || xb == s.mtile);
            xb = s.mtile;
          }
        }
        for (int t : taken) CHECK(t == 1);
        for (int t = 0; t < m_tiles; ++t) CHECK(hi[t] - lo[t] <= 1);
        ++cases;
      }
  std::printf("deal_driver: ok (%ld cases)\n", cases);
  return 0;
}
