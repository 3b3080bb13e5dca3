// How the prefill grid is sized and which work items a workgroup takes: plain C++ shared by the kernel
// (device), its launcher (host) and a host-side unit test, no HIP types.
//
// A unit of work is (item, token block): four row tiles of one layer x 256 tokens.  The grid is one round
// of the chip (one workgroup per compute unit) or one workgroup per unit where there are fewer; workgroup b
// works on one token block and on the items first, first + per_block, first + 2 per_block, ...  The item
// lists are sorted by row length, so that taking one item per round gives every workgroup the same work to
// within one item.
// Workgroups go to the 8 XCDs round-robin (b % 8), and every workgroup of an item re-reads the item's X (64
// KiB per group): what keeps that traffic inside an XCD's L2 is that the workgroups of one XCD work on the
// same token block and on neighbouring items (the same layer or the next).  So where m_tiles divides 8 and
// there are enough items (per_xcd > 0), XCD x takes token block x % m_tiles and its per_xcd workgroups take
// per_xcd consecutive items of every round; otherwise (per_xcd = 0) workgroup b simply takes token block
// b % m_tiles and items b / m_tiles + k per_block.
#pragma once

#if defined(__HIPCC__)
#define PMPD_DEAL_HD __host__ __device__ inline
#else
#define PMPD_DEAL_HD inline
#endif

namespace pmpd {

constexpr int kXcds = 8;  // gfx950: 8 XCDs, workgroups dispatched to them in turn

struct PfGrid {
  int per_block;  // workgroups (= items per round) per token block
  int per_xcd;    // > 0: workgroups per XCD of the XCD-aware deal; 0: the simple deal
  unsigned grid;  // workgroups in all
};

// cus = compute units of the device, n_items >= 1, m_tiles >= 1.
PMPD_DEAL_HD PfGrid pf_grid(int n_items, int m_tiles, int cus) {
  const int per_xcd = cus / kXcds;
  if (m_tiles <= kXcds && kXcds % m_tiles == 0 && per_xcd > 0 && n_items >= per_xcd * (kXcds / m_tiles))
    return PfGrid{per_xcd * (kXcds / m_tiles), per_xcd, static_cast<unsigned>(kXcds * per_xcd)};
  int per_block = cus / m_tiles;
  if (per_block > n_items) per_block = n_items;
  if (per_block < 1) per_block = 1;
  return PfGrid{per_block, 0, static_cast<unsigned>(m_tiles) * static_cast<unsigned>(per_block)};
}

struct PfShare {
  int mtile;   // token block
  int first;   // first item; the others follow at distances of per_block
  int n_mine;  // how many items
};

PMPD_DEAL_HD PfShare pf_share(int b, int n_items, int m_tiles, int per_block, int per_xcd) {
  PfShare s;
  if (per_xcd > 0) {
    const int x = b % kXcds;
    s.mtile = x % m_tiles;
    s.first = (x / m_tiles) * per_xcd + b / kXcds;
  } else {
    s.mtile = b % m_tiles;
    s.first = b / m_tiles;
  }
  s.n_mine = s.first < n_items ? (n_items - s.first + per_block - 1) / per_block : 0;
  return s;
}

}  // namespace pmpd
