// Shared declarations of the PMPD host library and its HIP kernels (not part of the C ABI).
#pragma once

#include <cstdarg>
#include <cstddef>
#include <cstdint>
#include <vector>

#include "pmpd.h"

namespace pmpd {

constexpr int kGroup = PMPD_GROUP;    // input features per quantisation group
constexpr int kTile = PMPD_ROW_TILE;  // rows per storage tile = lanes per wave

inline int64_t padded_rows(int64_t out_f) { return (out_f + kTile - 1) / kTile * kTile; }

// Record a message for pmpd_last_error() and hand the status back.
int32_t fail(int32_t status, const char* fmt, ...);

// Shape / pointer checks shared by the entry points (no GPU needed).
int32_t check_shape(int32_t out_f, int32_t in_f, int32_t group);
int32_t check_layer(const pmpd_layer_t* layer, int32_t b, const char* who);

// Device-side description of one layer of a stack.
struct LayerDesc {
  const void* plane[4];
  const void* sa;
  int64_t x_off;  // fp16 elements from x_base
  int64_t y_off;  // fp32 elements from y_base
  int32_t out_f;
  int32_t in_f;
  int32_t n_groups;
  int32_t n_tiles;
};
static_assert(sizeof(LayerDesc) == 72, "LayerDesc is read by the kernels with this layout");

// One workgroup's share of a decode step: `count` consecutive row tiles of one layer.
struct WorkItem {
  int32_t layer;
  int32_t tile0;
};

// Work lists of a stack, one per workgroup size in 64-row tiles.
constexpr int kNumItemLists = 4;
constexpr int kStackTilesPerWg[kNumItemLists] = {4, 1, 2, 8};
constexpr int kEightTileList = 3;  // the 8-wave batch kernels work on 8-tile (512-row) blocks

int32_t check_bits(int32_t b, const char* who);  // b in {2,3,4}
constexpr int kMaxPrefillRows = 65536;
LayerDesc make_desc(const pmpd_layer_t& L, int64_t x_off, int64_t y_off);

}  // namespace pmpd

// A list of layers prepared for one-launch steps (host object; the tables live in the caller's workspace).
struct pmpd_stack {
  std::vector<pmpd::LayerDesc> layers;
  std::vector<pmpd::WorkItem> items[pmpd::kNumItemLists];
  const pmpd::LayerDesc* d_layers = nullptr;
  const pmpd::WorkItem* d_items[pmpd::kNumItemLists] = {nullptr, nullptr, nullptr, nullptr};
  int max_in = 0;
  int variant[5] = {0, 0, 0, 0, 0};  // decode kernel variant per bit-width (index = b)
};
