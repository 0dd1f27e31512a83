// Host planner: turns (F, P, T, pattern) into per-query-tile key-tile lists with per-block masks, cuts long
// lists into slices, and deals (slice, head group) units onto persistent workgroups.
// The mask follows the two ST-SpAttn paragraphs of Sec. 3.2 (spatial: first frame + own frame;
// temporal: first frame + same patch one frame back), always causal, text queries dense.
#include "plan.h"

#include <algorithm>
#include <cmath>
#include <cstddef>
#include <numeric>
#include <utility>

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

inline bool in_range(int32_t x, int32_t k0, int32_t k1) { return x >= k0 && x <= k1; }

// Some key of [k0, k1] is allowed.
inline bool row_hits(const RowSet& s, int32_t i, int32_t k0, int32_t k1) {
  return (k0 <= s.a) || (std::max(k0, s.lo) <= std::min(k1, i)) || in_range(s.prev, k0, k1) ||
         in_range(s.self, k0, k1);
}

// Every key of [k0, k1] is allowed; an empty range counts as allowed.  Single keys of the temporal path
// are ignored here, so the answer can be a conservative "no".
inline bool row_full(const RowSet& s, int32_t i, int32_t k0, int32_t k1) {
  if (k0 > k1) return true;
  if (s.lo <= s.a + 1) return k1 <= i;
  return (k1 <= s.a) || (k0 >= s.lo && k1 <= i);
}

// The only key of [k0, k1] that can be allowed is the previous-frame key.
inline bool row_prev_only(const RowSet& s, int32_t i, int32_t k0, int32_t k1) {
  return k0 > s.a && !(std::max(k0, s.lo) <= std::min(k1, i)) && !in_range(s.self, k0, k1);
}

inline double row_pairs(const RowSet& s, int32_t i) {
  double cnt = (s.lo <= s.a + 1) ? double(i) + 1.0 : double(s.a) + 1.0 + std::max(0, i - s.lo + 1);
  if (s.prev > s.a && s.prev < s.lo) cnt += 1.0;
  if (s.self > s.a && s.self < s.lo) cnt += 1.0;
  return cnt;
}

// Largest divisor of g that is at most `cap`.
inline int32_t largest_divisor_up_to(int32_t g, int32_t cap) {
  for (int32_t x = std::min(g, cap); x >= 1; --x)
    if (g % x == 0) return x;
  return 1;
}

}  // namespace

void build_plan(purekv_plan& p, int n_cu) {
  Geometry& g = p.g;
  const int32_t BK = PUREKV_BK;
  p.n_cu = n_cu;

  // ---- workgroup shape ----
  // Stacking the query heads of a KV group in one workgroup makes every wavefront of the workgroup need the
  // same key tiles (the mask depends on the row, not on the head), so nobody waits at the tile barriers for
  // work it does not share.  The dense pattern has little such imbalance (only the diagonal tiles): it stacks
  // only when that fills all wavefronts, else one head x 8 row blocks keeps every SIMD busy.
  {
    const int32_t gs = largest_divisor_up_to(g.G, kWaves), r = kWaves / gs;
    const bool stack = (g.pattern != PUREKV_PATTERN_DENSE && gs >= 2) || (gs * r == kWaves && gs >= 2);
    // A head subset keeps the stacked shape when it is made of whole stacks (e.g. whole KV groups); otherwise it is
    // planned head by head.
    bool whole_stacks = true;
    p.n_heads_sel = g.Hq;
    if (!p.head_sel.empty()) {
      p.n_heads_sel = 0;
      for (int32_t hq = 0; hq < g.Hq; ++hq) {
        p.n_heads_sel += p.head_sel[hq] != 0;
        whole_stacks &= (p.head_sel[hq] != 0) == (p.head_sel[hq - hq % gs] != 0);
      }
    }
    const bool use_stack = stack && whole_stacks;
    g.Gs = use_stack ? gs : 1;
    g.R = use_stack ? r : kWaves;
    g.n_groups = g.Hq / g.Gs;
  }
  auto group_selected = [&](int32_t grp) { return p.head_sel.empty() || p.head_sel[grp * g.Gs] != 0; };
  const int32_t n_groups_sel = p.n_heads_sel / g.Gs;
  const int32_t rows_per_qtile = g.R * kBlockRows;
  p.n_qtiles = (g.N + rows_per_qtile - 1) / rows_per_qtile;
  const int32_t n_ktiles = (g.N + BK - 1) / BK;
  p.qtile_begin.assign(1, 0);
  p.tiles.clear();
  p.n_blocks = 0;
  for (auto& c : p.n_kind) c = 0;
  p.mask_pairs = 0;

  std::vector<RowSet> sets(rows_per_qtile);
  for (int32_t qt = 0; qt < p.n_qtiles; ++qt) {
    const int32_t r0 = qt * rows_per_qtile, r1 = std::min(r0 + rows_per_qtile, g.N);  // rows [r0, r1)
    for (int32_t i = r0; i < r1; ++i) {
      sets[i - r0] = row_set(g, i);
      p.mask_pairs += row_pairs(sets[i - r0], i);
    }
    const int32_t last_tile = std::min((r1 - 1) / BK, n_ktiles - 1);  // causal: no key beyond the last row
    // Two shortcuts keep the planner linear in the number of listed tiles for long sequences; both only skip
    // work whose outcome is known.  (1) Rows that see every earlier key (dense pattern, text rows): a key tile that
    // ends at or before the first row of the query tile is needed in full by every row block.  (2) Video rows of a
    // sparse pattern can only see the first frame, their own frame up to themselves and their previous-frame keys:
    // tiles outside those three ranges are not examined.
    const bool all_dense_rows = g.pattern == PUREKV_PATTERN_DENSE || r0 >= g.Nv;
    const bool all_video_rows = g.pattern != PUREKV_PATTERN_DENSE && r1 <= g.Nv;
    uint32_t need_all = 0;
    int32_t blocks_all = 0;
    for (int32_t rb = 0; rb < g.R; ++rb)
      if (r0 + rb * kBlockRows < r1) need_all |= 3u << (2 * rb), blocks_all += 2;
    int32_t own_tile = 0, prev_lo = 1, prev_hi = 0;   // first tile of the own-frame range; previous-frame tiles
    if (all_video_rows) {
      const int32_t own0 = (g.pattern & PUREKV_PATTERN_SPATIAL) ? (r0 / g.P) * g.P : r0;
      own_tile = own0 / BK;
      if ((g.pattern & PUREKV_PATTERN_TEMPORAL) && r1 - 1 - g.P >= 0) {
        prev_lo = std::max(0, r0 - g.P) / BK;
        prev_hi = (r1 - 1 - g.P) / BK;
      }
    }
    const int32_t first_frame_tile = (g.P - 1) / BK;
    for (int32_t c = 0; c <= last_tile; ++c) {
      if (all_dense_rows && (c + 1) * BK - 1 <= r0) {
        p.tiles.push_back({c, need_all, 0u});   // kind "full" is 0 in every field
        p.n_blocks += blocks_all;
        p.n_kind[kKindFull] += blocks_all;
        continue;
      }
      if (all_video_rows && c > first_frame_tile && c < own_tile && !(c >= prev_lo && c <= prev_hi)) {
        c = std::min(own_tile, prev_lo > c && prev_lo <= prev_hi ? prev_lo : own_tile) - 1;   // jump to the next range
        continue;
      }
      uint32_t need = 0, kinds = 0;
      for (int32_t rb = 0; rb < g.R; ++rb) {
        const int32_t w0 = r0 + rb * kBlockRows, w1 = std::min(w0 + kBlockRows, r1);
        if (w0 >= w1) continue;  // a row block without real rows is never needed
        for (int32_t kb = 0; kb < 2; ++kb) {
          const int32_t k0 = c * BK + kb * kBlockKeys, k1 = k0 + kBlockKeys - 1;
          bool any = false, full = true, causal = true, prev = true;
          for (int32_t i = w0; i < w1; ++i) {
            const RowSet& s = sets[i - r0];
            any |= row_hits(s, i, k0, k1);
            full &= row_full(s, i, k0, k1);
            causal &= row_full(s, i, k0, std::min(k1, i));
            prev &= row_prev_only(s, i, k0, k1);
          }
          if (!any) continue;
          const uint32_t kind = full ? kKindFull : causal ? kKindCausal : prev ? kKindPrev : kKindGeneral;
          need |= 1u << (2 * rb + kb);
          kinds |= kind << (4 * rb + 2 * kb);
          ++p.n_blocks;
          ++p.n_kind[kind];
        }
      }
      if (need) p.tiles.push_back({c, need, kinds});
    }
    p.qtile_begin.push_back(static_cast<int32_t>(p.tiles.size()));
  }

  // ---- cost model (in steps of one full tile) ----
  // A tile of which every row block needs one 32-key half at most skips half of the score product; a unit
  // switch (write the finished rows, reset the state, first tile without a second product to overlap) costs
  // about one and a half steps.
  // The slice that closes a split list (its workgroup runs it last, so it normally arrives last and combines the
  // partial results of all slices) pays about two steps per slice for that (measured: a sweep of this constant on the 32-frame benchmark shape).
  constexpr double kHalfTileCost = 0.85, kUnitCost = 1.5, kMergeCostPerSlice = 2.0;
  std::vector<double> tile_cost(p.tiles.size());
  for (size_t i = 0; i < p.tiles.size(); ++i) {
    bool both = false;
    for (int32_t rb = 0; rb < g.R; ++rb) both |= ((p.tiles[i].need >> (2 * rb)) & 3u) == 3u;
    tile_cost[i] = both ? 1.0 : kHalfTileCost;
  }

  // ---- work items: cut lists that are long against the average load of one workgroup ----
  const double total_steps = double(p.tiles.size()) * n_groups_sel;
  // Slice length: 0.8 of the average load of a workgroup (measured on the 32-frame benchmark shape: shorter
  // slices balance no better after the refinement pass below and double the partial results to merge).
  const int32_t chunk = std::max<int32_t>(8, static_cast<int32_t>(0.8 * total_steps / std::max(1, n_cu) + 0.5));

  // ---- window plans: the query tiles whose rows want the log-sum-exp get workgroups of their own ----
  // Only the last lse_rows rows are asked for their log-sum-exp (the recent window of Eq. 2).  Keeping the exact row
  // sum costs the tile loop 7-10 % (two more vector instructions per pair of scores), so the query tiles that
  // hold such rows ("window tiles") are dealt to a set of workgroups of their own, sized by their share of the work,
  // and only those workgroups run the variant of the loop that keeps the sum.  A set of few workgroups needs units
  // small enough to be balanced over it: the window tiles' lists are cut into the number of slices that minimises an
  // estimate of the set's longest queue (equal units dealt evenly, a unit switch per unit, the combination charged
  // to the queue that closes a list), and the set is made large enough not to be the last to finish.
  // KV-head groups of the XCD affinity of the dealing below: workgroup q runs on XCD q % 8, and the units of a KV
  // head stay on the XCDs x with x % Hkv == kvh (Hkv < 8) or x == kvh % 8
  const int32_t affinity_groups = (p.head_sel.empty() && n_cu % 8 == 0 && (g.Hkv % 8 == 0 || 8 % g.Hkv == 0)) ? std::min(g.Hkv, 8) : 1;
  auto window_tile = [&](int32_t qt) {
    return p.lse_rows > 0 && int64_t(qt + 1) * rows_per_qtile > int64_t(g.N) - p.lse_rows;
  };
  // measured on the 32-frame benchmark shape: a step that keeps the exact sum takes 1.10 of one that does not; a
  // slice costs its workgroup about three steps more than a whole list does (partial result through to memory,
  // arrival, the look at its list's counter at the end of the queue), on top of the combination itself
  constexpr double kExactSumCost = 1.10, kSliceCost = 3.0;
  int32_t n_window_queues = 0, window_slices = 1;
  {
    double steps_w = 0;
    int64_t lists_w = 0;
    int32_t shortest = INT32_MAX;
    for (int32_t qt = 0; qt < p.n_qtiles; ++qt)
      if (window_tile(qt)) {
        const int32_t len = p.qtile_begin[qt + 1] - p.qtile_begin[qt];
        steps_w += len;
        ++lists_w;
        shortest = std::min(shortest, len);
      }
    const double cost_w = kExactSumCost * steps_w * n_groups_sel, cost_rest = (double(p.tiles.size()) - steps_w) * n_groups_sel;
    // (not when the window tiles are a large share of the work -- text rows under a sparse pattern: units cut fine
    // enough to balance a large set pay more in unit switches and combinations than the other set saves)
    if (lists_w > 0 && 4 * cost_w <= cost_w + cost_rest && n_cu >= 2 &&
        (p.n_qtiles - lists_w) * int64_t(n_groups_sel) >= n_cu) {
      const int64_t units_w = lists_w * n_groups_sel, units_rest = (p.n_qtiles - lists_w) * int64_t(n_groups_sel);
      const double len = steps_w / double(lists_w);
      // longest queue of a set of nq workgroups, and the number of slices per list that gives it
      auto window_set = [&](int32_t nq, int32_t& slices) {
        double best = 0;
        for (int32_t ns = 1; ns <= std::min<int32_t>(kMaxSplits, std::max(1, shortest / 8)); ++ns) {
          const int64_t per_queue = (units_w * ns + nq - 1) / nq;
          const double longest = double(per_queue) * (len / ns + kUnitCost + (ns > 1 ? kSliceCost : 0.0)) +
                                 (ns > 1 ? kMergeCostPerSlice * ns : 0.0);
          if (ns == 1 || longest < best) best = longest, slices = ns;
        }
        return kExactSumCost * best;
      };
      auto rest_set = [&](int32_t nq) { return (cost_rest + kUnitCost * double(units_rest)) / double(n_cu - nq); };
      // smallest set, from the window tiles' share of the work on, whose longest queue ends no later than the
      // other set's average one; failing that, the size with the smallest later end of the two
      // (a multiple of the number of KV-head groups of the XCD affinity below, so that every KV head keeps the same
      // number of workgroups in both sets)
      const int32_t nq0 = std::max<int32_t>(1, static_cast<int32_t>(cost_w / (cost_w + cost_rest) * n_cu));
      double best_end = 0;
      for (int32_t nq = (nq0 + affinity_groups - 1) / affinity_groups * affinity_groups;
           nq <= std::min<int32_t>(n_cu - 1, 2 * nq0 + 8 + affinity_groups); nq += affinity_groups) {
        int32_t slices = 1;
        const double end_w = window_set(nq, slices), end_r = rest_set(nq), end = std::max(end_w, end_r);
        if (n_window_queues == 0 || end < best_end) best_end = end, n_window_queues = nq, window_slices = slices;
        if (end_w <= end_r) break;
      }
    }
  }
  p.items.clear();
  p.merges.clear();
  p.n_slots = 0;
  for (int32_t qt = 0; qt < p.n_qtiles; ++qt) {
    const int32_t b = p.qtile_begin[qt], len = p.qtile_begin[qt + 1] - b;
    int32_t ns = 1;
    if (2 * len > 3 * chunk) ns = std::min<int32_t>((len + chunk - 1) / chunk, kMaxSplits);
    if (n_window_queues > 0 && window_tile(qt)) ns = std::min(window_slices, std::max(1, len / 8));
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
  std::vector<double> item_cost(p.items.size());
  for (size_t it = 0; it < p.items.size(); ++it) {
    double c = kUnitCost;
    for (int32_t t = 0; t < p.items[it].n_tiles; ++t) c += tile_cost[p.items[it].list_begin + t];
    if (p.items[it].n_splits > 1 && p.items[it].split == p.items[it].n_splits - 1)
      c += kMergeCostPerSlice * p.items[it].n_splits;
    item_cost[it] = c;
  }

  // ---- deal (item, head group) units onto persistent workgroups: longest first, least-loaded queue ----
  // Workgroup q runs on XCD q % 8 (round-robin dispatch); when the head counts allow it, the units of one
  // KV head stay on a fixed set of XCDs so that each L2 holds the K/V of few KV heads.
  const int64_t n_units = int64_t(p.items.size()) * n_groups_sel;
  p.n_queues = static_cast<int32_t>(std::min<int64_t>(std::max(1, n_cu), std::max<int64_t>(1, n_units)));
  auto item_class = [&](int32_t it) { return (n_window_queues > 0 && window_tile(p.items[it].qtile)) ? 1 : 0; };
  if (n_window_queues > 0) {
    int64_t units_w = 0;
    for (size_t it = 0; it < p.items.size(); ++it) units_w += item_class(static_cast<int32_t>(it)) * n_groups_sel;
    n_window_queues = static_cast<int32_t>(std::min<int64_t>(n_window_queues, units_w));
  }
  // queues [0, lse_queue0): units of the other tiles; [lse_queue0, n_queues): units of the window tiles.  A plan
  // without a window keeps one class: every workgroup keeps the exact sum when the log-sum-exp is asked for.
  p.lse_queue0 = n_window_queues > 0 ? p.n_queues - n_window_queues : 0;
  // (not for a head subset: its KV heads may be few, and every queue has to receive a unit)
  const bool affinity = p.head_sel.empty() && (p.n_queues % 8 == 0) && (g.Hkv % 8 == 0 || 8 % g.Hkv == 0);
  std::vector<std::vector<int32_t>> queues(p.n_queues);  // flat (item, group) pairs
  std::vector<double> load(p.n_queues, 0.0);
  auto deal_class = [&](int cls, int32_t q_lo, int32_t q_hi) {
    // the affinity needs the same number of queues for every KV head inside the range (the sets of a divided plan
    // are sized for that)
    const bool aff = affinity && (q_hi - q_lo) % affinity_groups == 0;
    auto allowed = [&](int32_t q, int32_t kvh) {
      if (!aff) return true;
      const int32_t x = q % 8;
      return (g.Hkv >= 8) ? (x == kvh % 8) : (x % g.Hkv == kvh);
    };
    for (size_t it = 0; it < p.items.size(); ++it) {
      if (item_class(static_cast<int32_t>(it)) != cls) continue;
      for (int32_t grp = 0; grp < g.n_groups; ++grp) {
        if (!group_selected(grp)) continue;
        const int32_t kvh = grp * g.Gs / g.G;
        int32_t best = -1;
        for (int32_t q = q_lo; q < q_hi; ++q)
          if (allowed(q, kvh) && (best < 0 || load[q] < load[best])) best = q;
        queues[best].push_back(static_cast<int32_t>(it));
        queues[best].push_back(grp);
        load[best] += item_cost[it];
      }
    }
    // Refinement: while it lowers the larger of the two loads, move a unit from the fullest queue to the emptiest
    // queue that may run it, or exchange a unit of each.
    for (int32_t round = 0; round < 8 * (q_hi - q_lo); ++round) {
      const int32_t qa = static_cast<int32_t>(std::max_element(load.begin() + q_lo, load.begin() + q_hi) - load.begin());
      double best_gain = 1e-9;
      int32_t best_q = -1;
      size_t best_u = 0, best_v = SIZE_MAX;
      for (size_t u = 0; u + 1 < queues[qa].size(); u += 2) {
        const double cu = item_cost[queues[qa][u]];
        const int32_t kvh = queues[qa][u + 1] * g.Gs / g.G;
        for (int32_t qb = q_lo; qb < q_hi; ++qb) {
          if (qb == qa || !allowed(qb, kvh)) continue;
          // move u: new pair maximum = max(load[qa] - cu, load[qb] + cu)
          double gain = load[qa] - std::max(load[qa] - cu, load[qb] + cu);
          if (gain > best_gain) {
            best_gain = gain;
            best_q = qb;
            best_u = u;
            best_v = SIZE_MAX;
          }
          for (size_t v = 0; v + 1 < queues[qb].size(); v += 2) {
            const double cv = item_cost[queues[qb][v]];
            if (cv >= cu || !allowed(qa, queues[qb][v + 1] * g.Gs / g.G)) continue;
            gain = load[qa] - std::max(load[qa] - cu + cv, load[qb] + cu - cv);
            if (gain > best_gain) {
              best_gain = gain;
              best_q = qb;
              best_u = u;
              best_v = v;
            }
          }
        }
      }
      if (best_q < 0) break;
      const int32_t ui = queues[qa][best_u], ug = queues[qa][best_u + 1];
      if (best_v == SIZE_MAX) {
        queues[qa].erase(queues[qa].begin() + best_u, queues[qa].begin() + best_u + 2);
        queues[best_q].push_back(ui);
        queues[best_q].push_back(ug);
        load[qa] -= item_cost[ui];
        load[best_q] += item_cost[ui];
      } else {
        const int32_t vi = queues[best_q][best_v], vg = queues[best_q][best_v + 1];
        queues[qa][best_u] = vi;
        queues[qa][best_u + 1] = vg;
        queues[best_q][best_v] = ui;
        queues[best_q][best_v + 1] = ug;
        load[qa] += item_cost[vi] - item_cost[ui];
        load[best_q] += item_cost[ui] - item_cost[vi];
      }
    }
  };
  if (n_window_queues > 0) {
    deal_class(0, 0, p.lse_queue0);
    deal_class(1, p.lse_queue0, p.n_queues);
  } else {
    deal_class(0, 0, p.n_queues);
  }
  // Order within a queue: slices of split lists first, except the closing slice of a list, which goes last (when it
  // ends, the other slices of its list, run first elsewhere, have normally long arrived: the workgroup that the
  // cost model charged for combining them is then the one that does); whole lists in between, longest first (item
  // indices ascend with decreasing length).
  auto order_class = [&](int32_t it) {
    const WorkItem& w = p.items[it];
    return w.n_splits == 1 ? 1 : (w.split == w.n_splits - 1 ? 2 : 0);
  };
  for (auto& qv : queues) {
    std::vector<std::pair<int32_t, int32_t>> pairs;
    for (size_t u = 0; u + 1 < qv.size(); u += 2) pairs.emplace_back(qv[u], qv[u + 1]);
    std::stable_sort(pairs.begin(), pairs.end(), [&](const std::pair<int32_t, int32_t>& x, const std::pair<int32_t, int32_t>& y) {
      const int cx = order_class(x.first), cy = order_class(y.first);
      return cx != cy ? cx < cy : x < y;
    });
    for (size_t u = 0; u < pairs.size(); ++u) {
      qv[2 * u] = pairs[u].first;
      qv[2 * u + 1] = pairs[u].second;
    }
  }

  std::vector<uint8_t> owned(size_t(g.Hkv) * size_t(n_ktiles), 0);   // (KV head, key tile) pairs that have an owner step
  p.units.clear();
  p.stream.clear();
  p.queue_begin.assign(1, 0);
  p.queue_units.clear();
  p.queue_units_begin.assign(1, 0);
  for (int32_t q = 0; q < p.n_queues; ++q) {
    for (size_t u = 0; u + 1 < queues[q].size(); u += 2) {
      const WorkItem& w = p.items[queues[q][u]];
      const int32_t grp = queues[q][u + 1], head0 = grp * g.Gs, kvh = head0 / g.G;
      p.queue_units.push_back(queues[q][u]);
      p.queue_units.push_back(head0);
      Unit un{};
      un.row0 = w.qtile * rows_per_qtile;
      un.head0 = head0;
      un.n_splits = w.n_splits;
      un.ws_row0 = w.slot >= 0 ? (w.slot * g.n_groups + grp) * (kWaves * kBlockRows) : -1;
      un.ws_row_first = w.slot >= 0 ? ((w.slot - w.split) * g.n_groups + grp) * (kWaves * kBlockRows) : -1;
      un.counter = w.slot >= 0 ? (w.slot - w.split) * g.n_groups + grp : -1;
      p.units.push_back(un);
      for (int32_t t = 0; t < w.n_tiles; ++t) {
        const TileRef& r = p.tiles[w.list_begin + t];
        StreamEntry e;
        e.kv_off = uint32_t((int64_t(kvh) * g.kv_sh + int64_t(r.tile) * BK * g.kv_st) * 2);
        const int32_t k0 = r.tile * BK, rows = std::min(BK, g.N - k0);
        uint8_t& own = owned[size_t(kvh) * size_t(n_ktiles) + size_t(r.tile)];
        e.need = r.need | ((t == w.n_tiles - 1) ? (1u << 16) : 0u) | ((t == 0) ? (1u << 17) : 0u) |
                 (uint32_t(rows - 1) << 18) | (own ? 0u : (1u << 24));
        own = 1;
        e.kinds = r.kinds;
        e.k0 = k0;
        p.stream.push_back(e);
      }
    }
    p.queue_begin.push_back(static_cast<int32_t>(p.stream.size()));
    p.queue_units_begin.push_back(static_cast<int32_t>(p.queue_units.size() / 2));
  }
  p.units.push_back(Unit{});  // spare record: the kernel fetches the record after the current unit unconditionally
}

}  // namespace purekv
