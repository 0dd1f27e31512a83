// Internal: plan layout shared by the host planner and the kernels' launch code.
#pragma once
#include <cstdint>
#include <vector>

#include "purekv.h"

namespace purekv {

constexpr int kWaves = PUREKV_WAVES;        // wavefronts per prefill workgroup
constexpr int kBlockRows = PUREKV_BLOCK;    // query rows per wavefront
constexpr int kBlockKeys = PUREKV_BLOCK;    // keys per mask block: a key tile (PUREKV_BK keys) holds two
constexpr int kMaxSplits = 32;              // slices of one query tile's key list (the merge keeps 32 x kMaxSplits weights in LDS)

// How the allowed pairs of one (row block, key block) pair are told apart from the others.
enum BlockKind : uint32_t {
  kKindFull = PUREKV_KIND_FULL,        // every pair allowed: no element mask
  kKindCausal = PUREKV_KIND_CAUSAL,    // allowed  <=>  key <= query
  kKindPrev = PUREKV_KIND_PREV,        // allowed  <=>  key == query - P (same patch, previous frame)
  kKindGeneral = PUREKV_KIND_GENERAL,  // the full predicate of the pattern
};

// One unit of prefill work: a query tile and a contiguous slice of its key-tile list.
struct WorkItem {
  int32_t qtile;       // query rows [qtile*rows_per_qtile, (qtile+1)*rows_per_qtile)
  int32_t list_begin;  // first position in the flat tile list
  int32_t n_tiles;     // tiles in this slice
  int32_t split;       // index of this slice within the query tile's list (0 = first)
  int32_t n_splits;    // slices of this query tile (1 = writes the output itself)
  int32_t slot;        // partial-result slot when n_splits > 1, else -1
};

// A query tile whose list is split: the partial results in slots [slot0, slot0 + n_splits) are combined by the
// workgroup whose slice arrives last (per head group), inside the prefill launch.
struct MergeItem {
  int32_t qtile;
  int32_t slot0;
  int32_t n_splits;
  int32_t pad;
};

// One key tile of a query tile's list.  Bit 2*rb + kb of `need`: row block rb of the query tile has an allowed
// pair among keys [tile*BK + 32*kb, +32).  Bits 4*rb + 2*kb, +1 of `kinds`: the BlockKind of that pair of blocks.
struct TileRef {
  int32_t tile;
  uint32_t need;
  uint32_t kinds;
};

// One step of a persistent workgroup's stream: stage this key tile, compute it for the row blocks that need it.
struct StreamEntry {
  uint32_t kv_off;     // byte offset of the tile's first row within the K (and V) tensor: (kvh*kv_sh + k0*kv_st)*2
  uint32_t need;       // TileRef::need | last << 16 | first << 17 | (rows - 1) << 18 | owner << 24: last / first step
                       // of its unit (units are numbered in stream order); rows = keys of the tile that exist
                       // (1..64); owner: this step is the one step of the launch that also emits the squared
                       // norms of the tile's V rows (every (KV head, key tile) has exactly one owner step)
  uint32_t kinds;      // TileRef::kinds
  int32_t k0;          // first key of the tile
};

// A unit = work item x group of stacked query heads, run by one workgroup from its first to its last stream entry.
struct Unit {
  int32_t row0;        // first query row of the tile
  int32_t head0;       // first query head of the group (the group shares one KV head)
  int32_t n_splits;    // 1: the unit writes the output; > 1: it writes a partial result
  int32_t ws_row0;     // first row of the unit's partial result in the workspace (PUREKV_WAVES*32 rows), or -1
  // slices only: first workspace row of slice 0 of the same (query tile, head group) -- slice s lies
  // s * n_groups * PUREKV_WAVES * 32 rows further -- and the arrival counter of that (query tile, head group)
  int32_t ws_row_first;
  int32_t counter;
  int32_t pad[2];
};

struct Geometry {
  int32_t F, P, T, Nv, N;
  int32_t Hq, Hkv, G, d;
  uint32_t pattern;
  float scale;
  // Element strides of the (head, token) axes of Q, of K and V, and of O (never 0 here: packed defaults filled in).
  int64_t q_sh, q_st, kv_sh, kv_st, o_sh, o_st;
  // Workgroup shape: Gs query heads of one KV group x R row blocks of 32 rows, one wavefront each
  // (wavefront w: row block w / Gs, head w % Gs); Gs * R <= PUREKV_WAVES.
  int32_t Gs, R, n_groups;   // n_groups = Hq / Gs
};

}  // namespace purekv

struct purekv_plan {
  purekv::Geometry g;
  int32_t n_qtiles = 0;
  std::vector<int32_t> qtile_begin;        // [n_qtiles + 1] offsets into tiles
  std::vector<purekv::TileRef> tiles;
  std::vector<purekv::WorkItem> items;     // longest first
  std::vector<purekv::MergeItem> merges;
  std::vector<purekv::Unit> units;         // in stream order, plus one spare record at the end
  std::vector<purekv::StreamEntry> stream; // all queues, back to back
  std::vector<int32_t> queue_begin;        // [n_queues + 1] offsets into stream
  std::vector<int32_t> queue_units;        // (item, first head) pairs per queue, for inspection
  std::vector<int32_t> queue_units_begin;  // [n_queues + 1] offsets into queue_units (in pairs)
  int32_t n_queues = 0;
  // Window plans: only the last lse_rows rows are asked for their log-sum-exp (0: every row).  Queues
  // [lse_queue0, n_queues) hold the units of the query tiles with such rows, the others hold none of them; a plan
  // without a window (or too small to be divided) has lse_queue0 = 0.
  int32_t lse_rows = 0;
  int32_t lse_queue0 = 0;
  int32_t n_slots = 0;
  int64_t n_blocks = 0;                    // (row block, key block) pairs computed, per query head
  int64_t n_kind[4] = {0, 0, 0, 0};        // of those, per BlockKind
  double mask_pairs = 0;                   // allowed (query, key) pairs per head
  // device copies (null for host-only plans)
  purekv::StreamEntry* d_stream = nullptr;
  purekv::Unit* d_units = nullptr;
  int32_t* d_queue_begin = nullptr;
  int32_t* d_queue_unit0 = nullptr;        // [n_queues + 1] first unit of each queue
  float* d_static_scores = nullptr;        // the library's static score buffer on this plan's device (not owned)
  // Head subset (empty: every query head).  A plan over a subset lists units for the selected heads only and leaves
  // the other heads' rows of every output untouched; it keeps the stacked workgroup shape when the subset consists
  // of whole stacks, else it runs one head per workgroup (Gs = 1).
  std::vector<uint8_t> head_sel;           // [Hq], non-zero = selected
  int32_t n_heads_sel = 0;                 // selected heads (Hq when head_sel is empty)
  int device = -1;
  int n_cu = 256;
};

namespace purekv {
// Fills every host field of `p` from p.g (all but Gs, R, n_groups, which it chooses), p.head_sel and p.lse_rows;
// `n_cu` = number of persistent workgroups (one per compute unit).
void build_plan(purekv_plan& p, int n_cu);
}  // namespace purekv
