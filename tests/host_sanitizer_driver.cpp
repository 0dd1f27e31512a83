// Host-side exerciser for the planner and the argument validation, meant to be built and run under
// AddressSanitizer + UndefinedBehaviorSanitizer on a machine without a GPU.  It drives the C ABI only (host-only
// plans, inspection calls, workspace sizes, error paths) over many shapes and checks the structural invariants a
// launch relies on: lists in range, every list position covered exactly once by the work items, every (work item,
// head group) unit in exactly one queue.  A sanitizer report or a failed check ends it with a non-zero status.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <random>
#include <set>
#include <vector>

#include "purekv.h"

static long g_plans = 0;

#define CHECK(cond)                                                              \
  do {                                                                           \
    if (!(cond)) {                                                               \
      std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond);   \
      std::exit(1);                                                              \
    }                                                                            \
  } while (0)

static purekv_shape_t make_shape(int F, int ph, int pw, int T, int hq, int hkv, int d, unsigned pattern) {
  purekv_shape_t s{};
  s.n_frames = F;
  s.patch_h = ph;
  s.patch_w = pw;
  s.n_text = T;
  s.n_q_heads = hq;
  s.n_kv_heads = hkv;
  s.head_dim = d;
  s.pattern = pattern;
  s.softmax_scale = 0.f;
  return s;
}

static void inspect(purekv_plan_t* p, const purekv_shape_t& s, int n_wg, const uint8_t* head_mask) {
  ++g_plans;
  int64_t c[16];
  CHECK(purekv_plan_counts(p, c) == PUREKV_OK);
  const int64_t n = (int64_t)s.n_frames * s.patch_h * s.patch_w + s.n_text;
  const int64_t n_qtiles = c[1], n_items = c[2], n_refs = c[3], n_queues = c[6], R = c[7], gs = c[8], n_groups = c[9];
  CHECK(c[0] == n && R >= 1 && gs >= 1 && gs * R <= PUREKV_WAVES && n_groups * gs == s.n_q_heads);
  CHECK(n_qtiles == (n + R * PUREKV_BLOCK - 1) / (R * PUREKV_BLOCK));
  CHECK(n_queues >= 1 && n_queues <= n_wg);
  const int64_t n_ktiles = (n + PUREKV_BK - 1) / PUREKV_BK;
  std::vector<int64_t> begin(n_qtiles + 1, 0);
  int64_t blocks = 0;
  std::vector<int32_t> refs;
  for (int64_t qt = 0; qt < n_qtiles; ++qt) {
    const int len = purekv_plan_qtile_list(p, (int32_t)qt, nullptr, 0);
    CHECK(len >= 1);
    refs.assign(3 * (size_t)len, -1);
    CHECK(purekv_plan_qtile_list(p, (int32_t)qt, refs.data(), len) == len);
    int32_t prev = -1;
    for (int i = 0; i < len; ++i) {
      CHECK(refs[3 * i] > prev && refs[3 * i] < n_ktiles);   // ascending key tiles inside the sequence
      prev = refs[3 * i];
      const uint32_t need = (uint32_t)refs[3 * i + 1];
      CHECK(need != 0 && (need >> (2 * R)) == 0);
      blocks += __builtin_popcount(need);
      CHECK((int64_t)refs[3 * i] * PUREKV_BK <= (qt + 1) * R * PUREKV_BLOCK - 1);   // causal: no key tile past the rows
    }
    // a short buffer receives only what fits
    if (len > 1) {
      std::vector<int32_t> small(3, -7);
      CHECK(purekv_plan_qtile_list(p, (int32_t)qt, small.data(), 1) == len && small[0] == refs[0]);
    }
    begin[qt + 1] = begin[qt] + len;
  }
  CHECK(begin[n_qtiles] == n_refs && blocks == c[4]);
  CHECK(c[10] + c[11] + c[12] + c[13] == c[4]);
  // work items cover every list exactly once, slots are distinct
  std::vector<int> covered((size_t)n_refs, 0);
  std::set<int32_t> slots;
  std::vector<std::vector<int32_t>> items((size_t)n_items, std::vector<int32_t>(6));
  for (int64_t it = 0; it < n_items; ++it) {
    CHECK(purekv_plan_item(p, (int32_t)it, items[it].data()) == PUREKV_OK);
    const auto& w = items[it];
    CHECK(w[0] >= 0 && w[0] < n_qtiles && w[2] >= 1 && w[3] >= 0 && w[3] < w[4] && w[4] <= 32);
    CHECK(w[1] >= begin[w[0]] && w[1] + w[2] <= begin[w[0] + 1]);
    for (int t = 0; t < w[2]; ++t) ++covered[(size_t)w[1] + t];
    CHECK((w[5] == -1) == (w[4] == 1));
    if (w[5] >= 0) CHECK(slots.insert(w[5]).second);
  }
  for (int v : covered) CHECK(v == 1);
  int32_t bad[6];
  CHECK(purekv_plan_item(p, (int32_t)n_items, bad) == PUREKV_EINVAL && purekv_plan_item(p, -1, bad) == PUREKV_EINVAL);
  // queues: every (item, selected head group) exactly once
  std::map<std::pair<int32_t, int32_t>, int> seen;
  std::vector<int32_t> units;
  for (int64_t q = 0; q < n_queues; ++q) {
    const int len = purekv_plan_queue(p, (int32_t)q, nullptr, 0);
    CHECK(len >= 0);
    units.assign(2 * (size_t)len + 2, -1);
    CHECK(purekv_plan_queue(p, (int32_t)q, units.data(), len) == len);
    for (int u = 0; u < len; ++u) {
      CHECK(units[2 * u] >= 0 && units[2 * u] < n_items && units[2 * u + 1] >= 0 && units[2 * u + 1] < s.n_q_heads);
      CHECK(units[2 * u + 1] % gs == 0);
      if (head_mask) CHECK(head_mask[units[2 * u + 1]] != 0);
      ++seen[{units[2 * u], units[2 * u + 1]}];
    }
  }
  int64_t groups_sel = 0;
  for (int h0 = 0; h0 < s.n_q_heads; h0 += (int)gs) groups_sel += head_mask == nullptr || head_mask[h0] != 0;
  CHECK((int64_t)seen.size() == n_items * groups_sel);
  for (const auto& kv : seen) CHECK(kv.second == 1);
  CHECK(purekv_plan_queue(p, (int32_t)n_queues, nullptr, 0) == PUREKV_EINVAL);
  // steps: one record of four values each; a short buffer receives only what fits
  std::vector<int32_t> steps;
  for (int64_t q = 0; q < n_queues; ++q) {
    const int len = purekv_plan_steps(p, (int32_t)q, nullptr, 0);
    CHECK(len >= 1);
    steps.assign(4 * (size_t)len, -1);
    CHECK(purekv_plan_steps(p, (int32_t)q, steps.data(), len) == len);
    CHECK(((steps[1] >> 17) & 1) == 1 && ((steps[4 * (size_t)(len - 1) + 1] >> 16) & 1) == 1);
    for (int i = 0; i < len; ++i) CHECK(steps[4 * (size_t)i + 3] >= 0 && steps[4 * (size_t)i + 3] < n);
    int32_t one[4] = {-7, -7, -7, -7};
    CHECK(purekv_plan_steps(p, (int32_t)q, one, 1) == len && one[3] == steps[3]);
  }
  CHECK(purekv_plan_steps(p, (int32_t)n_queues, nullptr, 0) == PUREKV_EINVAL && purekv_plan_steps(p, -1, nullptr, 0) == PUREKV_EINVAL);
  CHECK(purekv_plan_steps(p, 0, nullptr, 1) == PUREKV_EINVAL);
  // sizes and counts the callers allocate by
  for (int op = -1; op <= 5; ++op)
    for (int32_t layers : {0, 1, 26})
      for (int32_t w : {0, 1, (int32_t)n})
        for (int32_t cap : {0, 1, 1690, 70000}) (void)purekv_workspace_bytes(p, op, layers, w, cap);
  CHECK(purekv_plan_kept_tile_flops(p) > 0 && purekv_plan_mask_flops(p) > 0);
  CHECK(purekv_plan_mask_flops(p) <= purekv_plan_kept_tile_flops(p) * 1.0000001);
  // a host-only plan is never launched: every compute call refuses it before touching its arguments
  void* one = reinterpret_cast<void*>(16);
  CHECK(purekv_st_spattn_prefill(p, one, one, one, one, nullptr, nullptr, 0, nullptr) == PUREKV_EINVAL);
  CHECK(purekv_lowlayer_importance(p, one, one, (const float*)one, 1, (float*)one, nullptr, 0, nullptr) == PUREKV_EINVAL);
  CHECK(purekv_topk_select(p, (const float*)one, one, 0, 1, 1, 0, (int32_t*)one, nullptr, nullptr, 0, nullptr) == PUREKV_EINVAL);
  CHECK(purekv_kv_compact(p, one, one, 0, 1, (const int32_t*)one, 1, one, one, 1, nullptr) == PUREKV_EINVAL);
  CHECK(purekv_decode_attn(p, one, one, one, 1, 1, one, one, 1 << 20, nullptr) == PUREKV_EINVAL);
  CHECK(purekv_workspace_init(p, PUREKV_OP_PREFILL, one, 1 << 20, 0, 0, 0, nullptr) == PUREKV_EINVAL);
  purekv_stack_t st{4, 1, 2, 1, 0};
  CHECK(purekv_stack_workspace_bytes(p, p, &st) == 0);
}

static void one_shape(int F, int ph, int pw, int T, int hq, int hkv, int d, int n_wg) {
  for (unsigned pattern = 0; pattern <= 3; ++pattern) {
    purekv_shape_t s = make_shape(F, ph, pw, T, hq, hkv, d, pattern);
    purekv_plan_t* p = nullptr;
    CHECK(purekv_plan_create_host(&s, n_wg, &p) == PUREKV_OK && p != nullptr);
    inspect(p, s, n_wg, nullptr);
    CHECK(purekv_plan_destroy(p) == PUREKV_OK);
    // window plans of the same shape: the same invariants, and the division of the queues
    const int64_t n = (int64_t)F * ph * pw + T;
    for (int64_t w : {(int64_t)1, (int64_t)T, n / 3, n}) {
      if (w < 1 || w > n) continue;
      p = nullptr;
      CHECK(purekv_plan_create_window_host(&s, (int32_t)w, n_wg, &p) == PUREKV_OK && p != nullptr);
      inspect(p, s, n_wg, nullptr);
      int64_t c[16];
      CHECK(purekv_plan_counts(p, c) == PUREKV_OK && c[14] == w && c[15] >= 0 && c[15] < c[6]);
      if (c[15] > 0) {   // queues before c[15] hold no query tile with a window row, the others nothing else
        const int64_t rows = c[7] * PUREKV_BLOCK;
        std::vector<int32_t> units;
        for (int64_t q = 0; q < c[6]; ++q) {
          const int len = purekv_plan_queue(p, (int32_t)q, nullptr, 0);
          units.assign(2 * (size_t)len + 2, -1);
          CHECK(purekv_plan_queue(p, (int32_t)q, units.data(), len) == len);
          for (int u = 0; u < len; ++u) {
            int32_t item[6];
            CHECK(purekv_plan_item(p, units[2 * u], item) == PUREKV_OK);
            CHECK((((int64_t)item[0] + 1) * rows > n - w) == (q >= c[15]));
          }
        }
      }
      CHECK(purekv_plan_destroy(p) == PUREKV_OK);
    }
  }
}

int main() {
  // small and odd shapes, several workgroup counts
  const int shapes[][4] = {{4, 8, 8, 32}, {3, 5, 7, 19}, {1, 9, 9, 0}, {5, 16, 16, 200}, {2, 24, 24, 1}, {9, 1, 1, 3},
                           {1, 1, 1, 0},  {1, 1, 1, 200}, {1, 6, 6, 10}, {2, 16, 16, 2100}, {10, 16, 17, 190}};
  const int heads[][2] = {{4, 2}, {7, 1}, {3, 3}, {12, 2}, {2, 1}};
  for (const auto& sh : shapes)
    for (const auto& hd : heads)
      for (int n_wg : {1, 7, 256, 1000})
        for (int d : {64, 128}) one_shape(sh[0], sh[1], sh[2], sh[3], hd[0], hd[1], d, n_wg);
  // the benchmark shapes
  one_shape(8, 24, 24, 128, 32, 8, 128, 256);
  one_shape(32, 16, 16, 256, 28, 4, 128, 256);
  one_shape(64, 16, 16, 256, 28, 4, 128, 256);
  {
    purekv_shape_t s = make_shape(128, 16, 16, 512, 28, 4, 128, PUREKV_PATTERN_ST);
    purekv_plan_t* p = nullptr;
    CHECK(purekv_plan_create_host(&s, 256, &p) == PUREKV_OK);
    inspect(p, s, 256, nullptr);
    purekv_plan_destroy(p);
  }
  // seeded random shapes and head subsets
  std::mt19937 rng(7);
  for (int it = 0; it < 60; ++it) {
    const int hkv = 1 + rng() % 4, g = 1 + rng() % 8;
    const int F = 1 + rng() % 6, ph = 1 + rng() % 12, pw = 1 + rng() % 12, T = rng() % 300;
    one_shape(F, ph, pw, T, hkv * g, hkv, (rng() & 1) ? 64 : 128, 1 + rng() % 300);
    purekv_shape_t s = make_shape(F, ph, pw, T, hkv * g, hkv, 128, 1 + rng() % 3);
    std::vector<uint8_t> mask((size_t)hkv * g);
    bool any = false;
    for (auto& m : mask) any |= (m = rng() % 3 == 0);
    purekv_plan_t* p = nullptr;
    const int rc = purekv_plan_create_heads_host(&s, mask.data(), 256, &p);
    CHECK(rc == (any ? PUREKV_OK : PUREKV_EINVAL));
    if (p) {
      inspect(p, s, 256, mask.data());
      purekv_plan_destroy(p);
    }
  }
  // strides: valid layouts plan like the packed one, invalid ones are refused
  {
    purekv_shape_t s = make_shape(3, 5, 7, 19, 4, 2, 64, 3);
    const int64_t n = 3 * 35 + 19;
    s.q_stride_head = 64, s.q_stride_tok = 8 * 64, s.kv_stride_head = 64, s.kv_stride_tok = 8 * 64;
    s.o_stride_head = 64, s.o_stride_tok = 4 * 64;
    purekv_plan_t* p = nullptr;
    CHECK(purekv_plan_create_host(&s, 256, &p) == PUREKV_OK);
    inspect(p, s, 256, nullptr);
    purekv_plan_destroy(p);
    p = nullptr;
    s.kv_stride_tok = 32;
    CHECK(purekv_plan_create_host(&s, 256, &p) == PUREKV_EINVAL && p == nullptr);
    s.kv_stride_tok = 8 * 64, s.o_stride_head = n * 64 + 4;
    CHECK(purekv_plan_create_host(&s, 256, &p) == PUREKV_EINVAL);
    s.o_stride_head = (int64_t)1 << 40;
    CHECK(purekv_plan_create_host(&s, 256, &p) == PUREKV_EINVAL);
  }
  // shape validation and the small host-only calls
  {
    purekv_plan_t* p = nullptr;
    purekv_shape_t s = make_shape(2, 4, 4, 8, 4, 2, 64, 3);
    CHECK(purekv_plan_create_host(nullptr, 256, &p) == PUREKV_EINVAL);
    CHECK(purekv_plan_create_host(&s, 256, nullptr) == PUREKV_EINVAL);
    CHECK(purekv_plan_create_host(&s, 0, &p) == PUREKV_EINVAL && purekv_plan_create_host(&s, 70000, &p) == PUREKV_EINVAL);
    s.head_dim = 96;
    CHECK(purekv_plan_create_host(&s, 256, &p) == PUREKV_EUNSUPPORTED);
    s.head_dim = 64, s.pattern = 4;
    CHECK(purekv_plan_create_host(&s, 256, &p) == PUREKV_EUNSUPPORTED);
    s.pattern = 3, s.n_frames = 1 << 20, s.patch_h = 1 << 10;
    CHECK(purekv_plan_create_host(&s, 256, &p) == PUREKV_EINVAL);
    CHECK(purekv_plan_destroy(nullptr) == PUREKV_OK);
    s = make_shape(2, 4, 4, 8, 4, 2, 64, 3);
    CHECK(purekv_plan_create_window_host(&s, 0, 256, &p) == PUREKV_EINVAL && purekv_plan_create_window_host(&s, 41, 256, &p) == PUREKV_EINVAL);
    CHECK(purekv_plan_create_window_host(&s, 8, 0, &p) == PUREKV_EINVAL && purekv_plan_create_window_host(&s, 8, 256, nullptr) == PUREKV_EINVAL);
    CHECK(purekv_plan_create_window_host(nullptr, 8, 256, &p) == PUREKV_EINVAL);
    for (int st = -7; st <= 1; ++st) CHECK(purekv_strerror(st) != nullptr && purekv_strerror(st)[0] != 0);
    for (int n = 0; n < 40000; n += 997)
      for (int pct = 0; pct <= 100; pct += 5) CHECK(purekv_budget(n, 0, pct / 100.0) == (int32_t)((int64_t)pct * n / 100));
    CHECK(purekv_budget(100, 10, 0.0 / 0.0) == -1 && purekv_budget(100, 10, 2.0) == -1 && purekv_budget(-5, 0, 0.5) == -1);
    CHECK(purekv_workspace_bytes(nullptr, 0, 0, 0, 0) == 0);
    float two[2] = {0.f, 1.f};
    uint64_t acc = 0;
    CHECK(purekv_spearman(nullptr, two, 1, 2, &acc, nullptr, nullptr) == PUREKV_EINVAL);
    CHECK(purekv_spearman(two, two, 1, 2, nullptr, nullptr, nullptr) == PUREKV_EINVAL);
    CHECK(purekv_spearman(two, two, 0, 2, &acc, nullptr, nullptr) == PUREKV_EINVAL);
    CHECK(purekv_spearman(two, two, 1, 1, &acc, nullptr, nullptr) == PUREKV_EINVAL);
    CHECK(purekv_spearman(two, two, 1, 131073, &acc, nullptr, nullptr) == PUREKV_EINVAL);
  }
  std::printf("host sanitizer driver: %ld plans inspected, all checks passed\n", g_plans);
  return 0;
}
