// Internal: plan layout shared by the host planner and the kernels' launch code.
#pragma once
#include <cstdint>
#include <vector>

#include "purekv.h"

namespace purekv {

constexpr int kWaves = 8;        // wavefronts per prefill workgroup
constexpr int kRowsPerWave = 32; // query rows per wavefront; PUREKV_BQ = kWaves * kRowsPerWave

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

// One (key tile, wave masks) reference of a query tile's list.
struct TileRef {
  int32_t tile;        // key tile index (keys [tile*BK, tile*BK + BK))
  uint16_t need;       // bit w: wavefront w (rows 32w..32w+31 of the query tile) has an allowed pair in this tile
  uint16_t full;       // bit w: every pair of wavefront w's rows with this tile's keys is allowed
};

// One step of a persistent workgroup's stream: stage this key tile, compute it for the wavefronts that need it.
struct StreamEntry {
  uint32_t kv_off;     // byte offset of the tile's first row within the K (and V) tensor: (kvh*N + k0)*d*2
  uint32_t masks;      // need | full << 8
  int32_t unit;        // index into the unit table when this is the first step of a unit, else -1
  int32_t last;        // 1 when this is the last step of its unit
};

// A unit = work item x query head, run by one workgroup from its first to its last stream entry.
struct Unit {
  int32_t qtile, head, split, n_splits, slot, k0_first, pad0, pad1;
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
  std::vector<purekv::TileRef> tiles;
  std::vector<purekv::WorkItem> items;     // longest first
  std::vector<purekv::MergeItem> merges;
  std::vector<purekv::Unit> units;
  std::vector<purekv::StreamEntry> stream; // all queues, back to back
  std::vector<int32_t> queue_begin;        // [n_queues + 1] offsets into stream
  std::vector<int32_t> queue_units;        // (item, head) pairs per queue, for inspection
  std::vector<int32_t> queue_units_begin;  // [n_queues + 1] offsets into queue_units (in pairs)
  int32_t n_queues = 0;
  int32_t n_slots = 0;
  int64_t n_full_wave_tiles = 0;           // (tile, wavefront) pairs flagged full
  int64_t n_wave_tiles = 0;                // (tile, wavefront) pairs computed, per query head
  double mask_pairs = 0;                   // allowed (query, key) pairs per head
  // device copies (null for host-only plans)
  purekv::StreamEntry* d_stream = nullptr;
  purekv::Unit* d_units = nullptr;
  int32_t* d_queue_begin = nullptr;
  purekv::MergeItem* d_merges = nullptr;
  int device = -1;
  int n_cu = 256;
};

namespace purekv {
// Fills every host field of `p` from p.g; `n_cu` = number of persistent workgroups (one per compute unit).
void build_plan(purekv_plan& p, int n_cu);
}  // namespace purekv
