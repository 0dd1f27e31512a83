// Host planner: turns (F, P, T, pattern) into per-query-tile key-tile lists with per-wavefront masks, cuts long
// lists into slices, and deals (slice, head) units onto persistent workgroups.
// The mask follows the two ST-SpAttn paragraphs of Sec. 3.2 (spatial: first frame + own frame;
// temporal: first frame + same patch one frame back), always causal, text queries dense.
#include "plan.h"

#include <algorithm>
#include <numeric>

namespace purekv {

namespace {

// Allowed keys of query row i: j <= i with (j <= a  or  j >= lo  or  j == prev  or  j == self).
struct RowSet {
  int32_t a, lo, prev, self;
};

inline RowSet row_set(const Geometry& g, int32_t i) {
  if (g.pattern == PUREKV_PATTERN_DENSE || i >= g.Nv) return {i, 0, -1, -1};
  const int32_t f = i / g.P;
  RowSet r;
  r.a = std::min(i, g.P - 1);
  r.lo = (g.pattern & PUREKV_PATTERN_SPATIAL) ? f * g.P : i + 1;
  r.prev = ((g.pattern & PUREKV_PATTERN_TEMPORAL) && f >= 1) ? i - g.P : -1;
  r.self = (g.pattern & PUREKV_PATTERN_TEMPORAL) ? i : -1;
  return r;
}

inline bool row_hits(const RowSet& s, int32_t i, int32_t k0, int32_t k1) {
  return (k0 <= s.a) || (std::max(k0, s.lo) <= std::min(k1, i)) || (s.prev >= k0 && s.prev <= k1) ||
         (s.self >= k0 && s.self <= k1);
}

// Every key of [k0, k1] allowed (single keys of the temporal path cannot fill a tile and are ignored here).
inline bool row_full(const RowSet& s, int32_t i, int32_t k0, int32_t k1) {
  if (s.lo <= s.a + 1) return k1 <= i;
  return (k1 <= s.a) || (k0 >= s.lo && k1 <= i);
}

inline double row_pairs(const RowSet& s, int32_t i) {
  double cnt = (s.lo <= s.a + 1) ? double(i) + 1.0 : double(s.a) + 1.0 + std::max(0, i - s.lo + 1);
  if (s.prev > s.a && s.prev < s.lo) cnt += 1.0;
  if (s.self > s.a && s.self < s.lo) cnt += 1.0;
  return cnt;
}

}  // namespace

void build_plan(purekv_plan& p, int n_cu) {
  const Geometry& g = p.g;
  const int32_t BQ = PUREKV_BQ, BK = PUREKV_BK;
  p.n_cu = n_cu;
  p.n_qtiles = (g.N + BQ - 1) / BQ;
  const int32_t n_ktiles = (g.N + BK - 1) / BK;
  p.qtile_begin.assign(1, 0);
  p.tiles.clear();
  p.n_full_wave_tiles = 0;
  p.n_wave_tiles = 0;
  p.mask_pairs = 0;

  std::vector<RowSet> sets(BQ);
  for (int32_t qt = 0; qt < p.n_qtiles; ++qt) {
    const int32_t r0 = qt * BQ, r1 = std::min(r0 + BQ, g.N);  // rows [r0, r1)
    for (int32_t i = r0; i < r1; ++i) {
      sets[i - r0] = row_set(g, i);
      p.mask_pairs += row_pairs(sets[i - r0], i);
    }
    const int32_t last_tile = std::min((r1 - 1) / BK, n_ktiles - 1);  // causal: no key beyond the last row
    for (int32_t c = 0; c <= last_tile; ++c) {
      const int32_t k0 = c * BK, k1 = k0 + BK - 1;
      uint16_t need = 0, full = 0;
      for (int32_t w = 0; w < kWaves; ++w) {
        const int32_t w0 = r0 + w * kRowsPerWave, w1 = std::min(w0 + kRowsPerWave, r1);
        if (w0 >= w1) continue;
        bool any = false, all = true;
        for (int32_t i = w0; i < w1; ++i) {
          any |= row_hits(sets[i - r0], i, k0, k1);
          all &= row_full(sets[i - r0], i, k0, k1);
        }
        if (any) {
          need |= uint16_t(1u << w);
          if (all) full |= uint16_t(1u << w);
        }
      }
      if (need) {
        p.tiles.push_back({c, need, full});
        p.n_wave_tiles += __builtin_popcount(need);
        p.n_full_wave_tiles += __builtin_popcount(full);
      }
    }
    p.qtile_begin.push_back(static_cast<int32_t>(p.tiles.size()));
  }

  // ---- work items: cut lists that are long against the average load of one workgroup ----
  const double total_steps = double(p.tiles.size()) * g.Hq;
  const int32_t chunk = std::max<int32_t>(8, static_cast<int32_t>(0.8 * total_steps / std::max(1, n_cu) + 0.5));
  p.items.clear();
  p.merges.clear();
  p.n_slots = 0;
  for (int32_t qt = 0; qt < p.n_qtiles; ++qt) {
    const int32_t b = p.qtile_begin[qt], len = p.qtile_begin[qt + 1] - b;
    int32_t ns = 1;
    if (2 * len > 3 * chunk) ns = (len + chunk - 1) / chunk;
    if (ns == 1) {
      p.items.push_back({qt, b, len, 0, 1, -1});
      continue;
    }
    p.merges.push_back({qt, p.n_slots, ns, 0});
    int32_t pos = b;
    for (int32_t s = 0; s < ns; ++s) {
      const int32_t cnt = len / ns + (s < len % ns ? 1 : 0);
      p.items.push_back({qt, pos, cnt, s, ns, p.n_slots + s});
      pos += cnt;
    }
    p.n_slots += ns;
  }
  std::stable_sort(p.items.begin(), p.items.end(),
                   [](const WorkItem& x, const WorkItem& y) { return x.n_tiles > y.n_tiles; });

  // ---- deal (item, head) units onto persistent workgroups: longest first, least-loaded queue ----
  // Workgroup q runs on XCD q % 8 (round-robin dispatch); when the head counts allow it, the units of one
  // KV head stay on a fixed set of XCDs so that each L2 holds the K/V of few KV heads.
  const int64_t n_units = int64_t(p.items.size()) * g.Hq;
  p.n_queues = static_cast<int32_t>(std::min<int64_t>(std::max(1, n_cu), std::max<int64_t>(1, n_units)));
  const bool affinity = (p.n_queues % 8 == 0) && (g.Hkv % 8 == 0 || 8 % g.Hkv == 0);
  std::vector<std::vector<int32_t>> queues(p.n_queues);  // flat (item, head) pairs
  std::vector<int64_t> load(p.n_queues, 0);
  for (size_t it = 0; it < p.items.size(); ++it) {
    for (int32_t h = 0; h < g.Hq; ++h) {
      const int32_t kvh = h / g.G;
      int32_t best = -1;
      for (int32_t q = 0; q < p.n_queues; ++q) {
        if (affinity) {
          const int32_t x = q % 8;
          const bool ok = (g.Hkv >= 8) ? (x == kvh % 8) : (x % g.Hkv == kvh);
          if (!ok) continue;
        }
        if (best < 0 || load[q] < load[best]) best = q;
      }
      queues[best].push_back(static_cast<int32_t>(it));
      queues[best].push_back(h);
      load[best] += p.items[it].n_tiles + 3;
    }
  }

  p.units.clear();
  p.stream.clear();
  p.queue_begin.assign(1, 0);
  p.queue_units.clear();
  p.queue_units_begin.assign(1, 0);
  const uint32_t row_bytes = uint32_t(g.d) * 2u;
  for (int32_t q = 0; q < p.n_queues; ++q) {
    for (size_t u = 0; u + 1 < queues[q].size(); u += 2) {
      const WorkItem& w = p.items[queues[q][u]];
      const int32_t h = queues[q][u + 1], kvh = h / g.G;
      p.queue_units.push_back(queues[q][u]);
      p.queue_units.push_back(h);
      const int32_t uid = static_cast<int32_t>(p.units.size());
      p.units.push_back({w.qtile, h, w.split, w.n_splits, w.slot, 0, 0, 0});
      for (int32_t t = 0; t < w.n_tiles; ++t) {
        const TileRef& r = p.tiles[w.list_begin + t];
        StreamEntry e;
        e.kv_off = (uint32_t(kvh) * uint32_t(g.N) + uint32_t(r.tile) * BK) * row_bytes;
        e.masks = uint32_t(r.need) | (uint32_t(r.full) << 8);
        e.unit = (t == 0) ? uid : -1;
        e.last = (t == w.n_tiles - 1) ? 1 : 0;
        p.stream.push_back(e);
      }
    }
    p.queue_begin.push_back(static_cast<int32_t>(p.stream.size()));
    p.queue_units_begin.push_back(static_cast<int32_t>(p.queue_units.size() / 2));
  }
}

}  // namespace purekv
