// Internal: plan layout shared by the host planner and the kernels' launch code.
#pragma once
#include <cstdint>
#include <vector>

#include "purekv.h"

namespace purekv {

// One unit of prefill work: a query tile and a contiguous slice of its key-tile list.
struct WorkItem {
  int32_t qtile;       // query rows [qtile*BQ, qtile*BQ + BQ)
  int32_t list_begin;  // first position in the flat tile list
  int32_t n_tiles;     // tiles in this slice
  int32_t split;       // index of this slice within the query tile's list (0 = first)
  int32_t n_splits;    // slices of this query tile (1 = writes the output itself)
  int32_t slot;        // partial-result slot when n_splits > 1, else -1
};

// A query tile whose list is split: the merge kernel combines slots [slot0, slot0 + n_splits).
struct MergeItem {
  int32_t qtile;
  int32_t slot0;
  int32_t n_splits;
  int32_t pad;
};

struct Geometry {
  int32_t F, P, T, Nv, N;
  int32_t Hq, Hkv, G, d;
  uint32_t pattern;
  float scale;
};

}  // namespace purekv

struct purekv_plan {
  purekv::Geometry g;
  int32_t n_qtiles = 0;
  std::vector<int32_t> qtile_begin;        // [n_qtiles + 1] offsets into tiles
  std::vector<int32_t> tiles;              // key_tile * 2 + full
  std::vector<purekv::WorkItem> items;     // longest first
  std::vector<purekv::MergeItem> merges;
  int32_t n_slots = 0;
  int64_t n_full = 0;
  double mask_pairs = 0;                   // allowed (query, key) pairs per head
  // device copies (null for host-only plans)
  int32_t* d_tiles = nullptr;
  purekv::WorkItem* d_items = nullptr;
  purekv::MergeItem* d_merges = nullptr;
  int device = -1;
  int n_cu = 256;
};

namespace purekv {
// Fills every host field of `p` from p.g; `n_cu` guides how long lists are split.
void build_plan(purekv_plan& p, int n_cu);
}  // namespace purekv
