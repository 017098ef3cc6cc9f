// Seeded traffic through the host-side radix prefix cache on the real pool (no GPU), built with
// -fsanitize=address,undefined by tests/test_host_threads.py: forks, extensions, node splits and leaf
// evictions under a tight cell budget and few donor sequences.  Checks on every turn that the cached
// length is a common prefix with something saved earlier, that the trie stays inside its budget and
// that the pool holds at least the trie's cells; at the end everything must be back in the allocator.
#include <algorithm>
#include <cstdio>
#include <random>
#include <vector>

#include "../paper_2605_26289_amd/csrc/pool.hpp"
#include "../paper_2605_26289_amd/csrc/radix.hpp"

int main() {
  int failures = 0;
  for (int seed = 0; seed < 6; ++seed) {
    std::mt19937 rng(77 + seed);
    dk::Pool pool(10, 6, 1 << 14, 16);
    {
      const int64_t budget = 120 + 20 * seed;
      dk::Radix radix(&pool, budget, 1);
      std::vector<std::vector<int32_t>> bases(4), saved;
      for (auto& b : bases)
        for (int i = 0; i < 30; ++i) b.push_back((int32_t)(rng() % 4));
      for (int it = 0; it < 400; ++it) {
        std::vector<int32_t> t = bases[rng() % bases.size()];
        t.resize(1 + rng() % 30);
        for (int extra = (int)(rng() % 25); extra > 0; --extra) t.push_back((int32_t)(rng() % 4));
        int32_t slot = -1;
        if (pool.acquire(0, 0, &slot) != dk::OK) { ++failures; continue; }
        int64_t n_past = -1;
        if (radix.begin_turn(slot, t.data(), (int64_t)t.size(), &n_past) != dk::OK) ++failures;
        int64_t best = 0;  // nothing can be cached that was never saved
        for (const auto& s : saved) {
          int64_t c = 0;
          while (c < (int64_t)std::min(s.size(), t.size()) && s[c] == t[c]) ++c;
          best = std::max(best, c);
        }
        if (n_past < 0 || n_past > std::min<int64_t>(best, (int64_t)t.size() - 1)) ++failures;
        int64_t len = -1;
        if (pool.length(slot, &len) != dk::OK || len != n_past) ++failures;
        const int32_t cu[2] = {0, (int32_t)((int64_t)t.size() - n_past)};
        std::vector<int64_t> dst;
        if (pool.append(1, &slot, cu, nullptr, &dst) != dk::OK) ++failures;
        int32_t ok = -1;
        if (radix.save(slot, t.data(), (int64_t)t.size(), &ok) != dk::OK || ok < 0) ++failures;
        if (ok == 1) saved.push_back(t);
        if (pool.release(slot) != dk::OK) ++failures;
        int64_t nodes = 0, cells = 0, donors = 0, shed = 0, held = 0, free_cells = 0;
        radix.stats(&nodes, &cells, &donors, &shed);
        pool.stats(&held, &free_cells);
        if (cells > budget || donors > 6 || held < cells || nodes < donors) ++failures;
      }
      int64_t shed = 0;
      radix.stats(nullptr, nullptr, nullptr, &shed);
      if (shed < 10) ++failures;  // the budget was meant to bite
    }
    int64_t held = -1;
    pool.stats(&held, nullptr);
    if (held != 0) ++failures;  // destroying the trie released every donor
  }
  std::printf("failures %d\n", failures);
  return failures == 0 ? 0 : 1;
}
