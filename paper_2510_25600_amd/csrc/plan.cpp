// Host planner: turns (F, P, T, pattern) into per-query-tile key-tile lists and balanced work items.
// The mask follows the two ST-SpAttn paragraphs of Sec. 3.2 (spatial: first frame + own frame;
// temporal: first frame + same patch one frame back), always causal, text queries dense.
#include "plan.h"

#include <algorithm>
#include <numeric>

namespace purekv {

namespace {

// Block part of the mask for query row i: allowed keys are j <= i with (j <= a or j >= lo).
// The temporal path's single previous-frame key and self key are per-row side terms, not tiles.
struct RowSpan {
  int32_t a, lo;
};

inline RowSpan row_span(const Geometry& g, int32_t i) {
  if (g.pattern == PUREKV_PATTERN_DENSE || i >= g.Nv) return {i, 0};
  const int32_t f = i / g.P;
  RowSpan r;
  r.a = std::min(i, g.P - 1);
  r.lo = (g.pattern & PUREKV_PATTERN_SPATIAL) ? f * g.P : i + 1;
  return r;
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
  p.n_full = 0;
  p.mask_pairs = 0;

  std::vector<RowSpan> spans(BQ);
  for (int32_t qt = 0; qt < p.n_qtiles; ++qt) {
    const int32_t r0 = qt * BQ, r1 = std::min(r0 + BQ, g.N);  // rows [r0, r1)
    for (int32_t i = r0; i < r1; ++i) {
      spans[i - r0] = row_span(g, i);
      const RowSpan s = spans[i - r0];
      // pairs of the block part ...
      double cnt = (s.lo <= s.a + 1) ? double(i) + 1.0 : double(s.a) + 1.0 + std::max(0, i - s.lo + 1);
      // ... plus the side keys of the temporal path
      if (g.pattern != PUREKV_PATTERN_DENSE && i < g.Nv && (g.pattern & PUREKV_PATTERN_TEMPORAL)) {
        const int32_t f = i / g.P;
        if (f >= 2) cnt += 1.0;
        if (!(g.pattern & PUREKV_PATTERN_SPATIAL) && f >= 1) cnt += 1.0;
      }
      p.mask_pairs += cnt;
    }
    const int32_t last_tile = (r1 - 1) / BK;  // causal: no key beyond the last row
    for (int32_t c = 0; c <= last_tile && c < n_ktiles; ++c) {
      const int32_t k0 = c * BK, k1 = k0 + BK - 1;
      bool any = false, all = true;
      for (int32_t i = r0; i < r1; ++i) {
        const RowSpan s = spans[i - r0];
        const bool hit = (k0 <= s.a) || (std::max(k0, s.lo) <= std::min(k1, i));
        const bool full = (s.lo <= s.a + 1) ? (k1 <= i) : ((k1 <= s.a) || (k0 >= s.lo && k1 <= i));
        any |= hit;
        all &= full;
      }
      if (any) {
        p.tiles.push_back(c * 2 + (all ? 1 : 0));
        p.n_full += all ? 1 : 0;
      }
    }
    p.qtile_begin.push_back(static_cast<int32_t>(p.tiles.size()));
  }

  // Work items: cut lists longer than ~1.5x the average load of one workgroup slot.
  const double total = double(p.tiles.size()) * g.Hq;
  const int32_t chunk = std::max<int32_t>(16, static_cast<int32_t>(total / (2.0 * n_cu) + 0.5));
  p.items.clear();
  p.merges.clear();
  p.n_slots = 0;
  for (int32_t qt = 0; qt < p.n_qtiles; ++qt) {
    const int32_t b = p.qtile_begin[qt], len = p.qtile_begin[qt + 1] - b;
    if (len == 0) {  // cannot happen (the diagonal is always allowed); keep the item so rows get written
      p.items.push_back({qt, b, 0, 0, 1, -1});
      continue;
    }
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
}

}  // namespace purekv
