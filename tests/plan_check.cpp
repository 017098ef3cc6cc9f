// Host check of the attend planner's work decomposition (no GPU): every (row, key) pair of a batch is
// covered by exactly one item, split rows have a merge record, and the streaming kernel's chains hold
// every unit exactly once and are balanced (also for XCDs of unequal speed).  Built and run by
// tests/test_host_plan.py.  Exits 0 when every check held.
#include <algorithm>
#include <cstdio>
#include <map>
#include <mutex>
#include <random>
#include <vector>

#include "../paper_2605_26289_amd/csrc/plan.hpp"

static int failures = 0;
#define CHECK(cond)                                               \
  do {                                                            \
    if (!(cond)) {                                                \
      ++failures;                                                 \
      std::printf("FAILED %s (line %d)\n", #cond, __LINE__);      \
    }                                                             \
  } while (0)

static dk::PlanConfig config(int hq, int hkv) {
  dk::PlanConfig c{};
  c.n_q_heads = hq;
  c.n_kv_heads = hkv;
  c.head_dim = 128;
  c.use_mfma = true;
  c.tile_rows = 256;
  c.stream_rows = 96;
  c.kv_tile = 64;
  c.tile_wave_slots = 256 / hkv;
  c.stream_target = 256 / hkv;
  c.tile_min_chunk = 128;
  c.tile_item_cost = 5;
  c.stream_min_chunk = 512;
  c.stream_chains = 256;
  c.stream_item_cost = 512;
  for (float& x : c.xcd_speed) x = 1.f;
  return c;
}

struct Case {
  std::vector<int> n, delta;
};

// Coverage: per (entry, packed row) the key ranges of its items tile [0, visible) without gap or overlap.
static void check_cover(const dk::AttendPlan& p, const dk::PlanConfig& cfg, const std::vector<DkItem>& items, int max_rows,
                        std::map<std::pair<int, int>, std::vector<std::pair<int, int>>>* cover) {
  for (const DkItem& it : items) {
    CHECK(it.nrows > 0 && it.nrows <= max_rows && it.kv_lo < it.kv_hi && it.kv_lo % cfg.kv_tile == 0);
    CHECK(it.entry >= 0 && it.entry < (int)p.entries.size());
    (*cover)[{it.entry, it.row0}].push_back({it.kv_lo, it.kv_hi});
  }
}

static void run_case(const Case& cs, int hq, int hkv, const float* speeds, double tol) {
  const int nseq = (int)cs.n.size(), group = hq / hkv;
  int64_t cells = 4096;
  for (int b = 0; b < nseq; ++b) cells += cs.n[b] + cs.delta[b] + 512;
  dk::Pool pool(nseq, 0, cells, 256);
  std::vector<int32_t> slots(nseq), cu(nseq + 1, 0);
  for (int b = 0; b < nseq; ++b) {
    CHECK(pool.acquire(0, 0, &slots[b]) == dk::OK);
    const int32_t c2[2] = {0, cs.n[b]};
    std::vector<int64_t> dst;
    if (cs.n[b] > 0) CHECK(pool.append(1, &slots[b], c2, nullptr, &dst) == dk::OK);
    cu[b + 1] = cu[b] + cs.delta[b];
  }
  dk::PlanConfig cfg = config(hq, hkv);
  if (speeds)
    for (int x = 0; x < 8; ++x) cfg.xcd_speed[x] = speeds[x];
  dk::AttendPlan p;
  {  // the same batch with the streaming units drawn from a queue at run time: no links, units longest first, and
     // only for launches whose descriptors cannot travel in the kernel arguments
    dk::PlanConfig qcfg = cfg;
    qcfg.stream_queue = 1;
    qcfg.inline_blob_bytes = 3072;
    std::lock_guard<std::mutex> g(pool.mutex());
    CHECK(dk::build_plan(pool, qcfg, nseq, slots.data(), cu.data(), /*staged=*/true, &p) == dk::OK);
    const int64_t units = (int64_t)p.stream_items.size() * hkv;
    CHECK(p.stream_units == units);
    if (p.stream_queued) {
      CHECK(units >= 4 * (int64_t)qcfg.stream_chains && p.blob_bytes > 3072);
      CHECK(p.stream_links.empty() && p.stream_chains == qcfg.stream_chains);
      CHECK(p.off_queue % 16 == 0 && p.off_queue + 16 <= p.blob_bytes);
      for (size_t i = 1; i < p.stream_items.size(); ++i) {
        const DkItem &a = p.stream_items[i - 1], &b = p.stream_items[i];
        CHECK((int64_t)(a.kv_hi - a.kv_lo) * a.nrows >= (int64_t)(b.kv_hi - b.kv_lo) * b.nrows);
      }
    } else {
      CHECK(units < 4 * (int64_t)qcfg.stream_chains || p.entries.size() * sizeof(DkEntry) <= 3072);
    }
  }
  {
    std::lock_guard<std::mutex> g(pool.mutex());
    CHECK(dk::build_plan(pool, cfg, nseq, slots.data(), cu.data(), /*staged=*/true, &p) == dk::OK);
  }
  CHECK(!p.stream_queued);
  CHECK((int)p.entries.size() == nseq);
  std::map<std::pair<int, int>, std::vector<std::pair<int, int>>> cover;
  check_cover(p, cfg, p.tile_items, cfg.tile_rows, &cover);
  check_cover(p, cfg, p.stream_items, cfg.stream_rows, &cover);
  size_t split_tiles = 0;
  for (auto& kv : cover) {
    auto& v = kv.second;
    std::sort(v.begin(), v.end());
    CHECK(v.front().first == 0);
    for (size_t i = 1; i < v.size(); ++i) CHECK(v[i].first == v[i - 1].second);
    split_tiles += v.size() > 1;
  }
  CHECK(split_tiles == p.merges.size());
  // every row of every entry with delta > 0 belongs to one row tile, whose last key is the row's causal limit
  for (int b = 0; b < nseq; ++b) {
    const int rows = group * cs.delta[b];
    int covered = 0;
    for (auto& kv : cover)
      if (kv.first.first == b) {
        int nrows = 0;
        for (const DkItem& it : p.tile_items)
          if (it.entry == b && it.row0 == kv.first.second) nrows = it.nrows;
        for (const DkItem& it : p.stream_items)
          if (it.entry == b && it.row0 == kv.first.second) nrows = it.nrows;
        covered += nrows;
        const int last_tok = (kv.first.second + nrows - 1) / group;
        CHECK(kv.second.back().second == cs.n[b] + last_tok + 1);
      }
    CHECK(covered == rows);
  }
  // chains of the tile kernel: every item in exactly one chain, no empty chain, at most tile_wave_slots of them
  {
    const int32_t n_items = (int32_t)p.tile_items.size();
    CHECK(p.tile_chains <= std::min(n_items, cfg.tile_wave_slots) && (p.tile_chains > 0) == (n_items > 0));
    CHECK((int64_t)p.tile_links.size() == (int64_t)p.tile_chains + n_items);
    std::vector<int> hit((size_t)n_items, 0);
    std::vector<double> busy((size_t)p.tile_chains, 0.0);
    double sum = 0, longest_item = 0;
    for (int32_t c = 0; c < p.tile_chains; ++c) {
      int32_t steps = 0;
      CHECK(p.tile_links[c] >= 0);
      for (int32_t i = p.tile_links[c]; i >= 0 && steps <= n_items; i = p.tile_links[p.tile_chains + i], ++steps) {
        CHECK(i < n_items);
        if (i >= n_items) break;
        ++hit[i];
        const double cost = (p.tile_items[i].kv_hi - p.tile_items[i].kv_lo + 63) / 64 + cfg.tile_item_cost;
        busy[c] += cost;
        sum += cost;
        longest_item = std::max(longest_item, cost);
      }
      CHECK(steps <= n_items);  // no cycle
    }
    for (int32_t i = 0; i < n_items; ++i) CHECK(hit[i] == 1);
    // list scheduling: no chain ends later than the average plus one item; levelled chains with several items
    // each end within 15 % of each other
    if (p.tile_chains > 0) {
      const double worst = *std::max_element(busy.begin(), busy.end());
      CHECK(worst <= sum / p.tile_chains + longest_item + 1e-9);
      if (n_items >= 3 * p.tile_chains && p.tile_chains == cfg.tile_wave_slots) CHECK(worst <= 1.15 * sum / p.tile_chains);
    }
  }
  // chains of the streaming kernel
  const int64_t n_units = (int64_t)p.stream_items.size() * hkv;
  CHECK(p.stream_chains == (int32_t)std::min<int64_t>(n_units, cfg.stream_chains));
  CHECK((int64_t)p.stream_links.size() == p.stream_chains + n_units);
  std::vector<int> seen((size_t)n_units, 0);
  std::vector<double> done(p.stream_chains, 0.0);
  double total = 0, speed_sum = 0;
  for (int32_t c = 0; c < p.stream_chains; ++c) {
    int64_t steps = 0;
    for (int32_t u = p.stream_links[c]; u >= 0 && steps <= n_units; u = p.stream_links[p.stream_chains + u], ++steps) {
      CHECK(u < n_units);
      if (u >= n_units) break;
      ++seen[u];
      const DkItem& it = p.stream_items[u / hkv];
      done[c] += (it.kv_hi - it.kv_lo + cfg.stream_item_cost) / (double)cfg.xcd_speed[c & 7];
      total += it.kv_hi - it.kv_lo + cfg.stream_item_cost;
    }
    CHECK(steps <= n_units);  // no cycle
    speed_sum += cfg.xcd_speed[c & 7];
  }
  for (int64_t u = 0; u < n_units; ++u) CHECK(seen[u] == 1);
  if (tol > 0 && p.stream_chains > 0) {
    const double ideal = total / speed_sum, worst = *std::max_element(done.begin(), done.end());
    if (!(worst <= ideal * (1.0 + tol))) {
      ++failures;
      std::printf("FAILED balance: worst chain %.0f vs ideal %.0f (tolerance %.2f)\n", worst, ideal, tol);
    }
  }
}

int main() {
  std::mt19937 rng(2605);
  auto uni = [&](int lo, int hi) { return lo + (int)(rng() % (unsigned)(hi - lo + 1)); };
  const float skew[8] = {1.f, 0.93f, 1.f, 0.93f, 1.f, 0.93f, 1.f, 0.93f};
  {  // speculative verification: 64 slots, Delta 9, long contexts of mixed length
    Case c;
    for (int b = 0; b < 64; ++b) { c.n.push_back(uni(4096, 16384)); c.delta.push_back(9); }
    run_case(c, 32, 8, nullptr, 0.05);
    run_case(c, 32, 8, skew, 0.08);  // two units per chain: the pairs can only be matched so well
  }
  {  // decode, many short slots: more units than eight per chain
    Case c;
    for (int b = 0; b < 700; ++b) { c.n.push_back(uni(100, 3000)); c.delta.push_back(1); }
    run_case(c, 32, 8, nullptr, 0.05);
    run_case(c, 32, 8, skew, 0.05);
  }
  {  // a few very long slots: the key range is split
    Case c;
    for (int b = 0; b < 3; ++b) { c.n.push_back(uni(50000, 120000)); c.delta.push_back(uni(1, 16)); }
    run_case(c, 32, 8, nullptr, 0.25);
  }
  {  // mixed batch: tile and streaming items, empty deltas, fresh sequences
    Case c;
    const int ns[] = {0, 5, 9000, 24000, 300, 0, 7777}, ds[] = {700, 0, 512, 3, 64, 1, 17};
    for (int b = 0; b < 7; ++b) { c.n.push_back(ns[b]); c.delta.push_back(ds[b]); }
    run_case(c, 32, 8, nullptr, 0);
    run_case(c, 8, 2, nullptr, 0);
    run_case(c, 16, 16, nullptr, 0);
  }
  for (int rep = 0; rep < 20; ++rep) {  // random batches
    Case c;
    const int nseq = uni(1, 40);
    for (int b = 0; b < nseq; ++b) { c.n.push_back(uni(0, 1) ? uni(0, 20000) : uni(0, 300)); c.delta.push_back(uni(0, 3) ? uni(0, 20) : uni(0, 900)); }
    run_case(c, 32, 8, rep & 1 ? skew : nullptr, 0);
  }
  std::printf("failures %d\n", failures);
  return failures ? 1 : 0;
}
