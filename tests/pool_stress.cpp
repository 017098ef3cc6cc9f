// Multi-threaded stress of the host-side pool (no GPU): threads acquire, append, alias, trim and release
// concurrently; built with -fsanitize=thread by tests/test_host_threads.py.  Exits 0 if every invariant held.
#include <atomic>
#include <cstdio>
#include <random>
#include <thread>
#include <vector>

#include "../paper_2605_26289_amd/csrc/pool.hpp"

int main() {
  constexpr int kSlots = 12, kThreads = 6, kIters = 3000;
  dk::Pool pool(kSlots, 4, 1 << 16, 16);
  std::atomic<int> failures{0};
  std::atomic<int> shared_donor{-1};
  // one long-lived donor everybody may alias
  int32_t donor = -1;
  if (pool.acquire(1, 0, &donor) != dk::OK) return 2;
  {
    const int32_t cu[2] = {0, 500};
    std::vector<int64_t> dst;
    if (pool.append(1, &donor, cu, nullptr, &dst) != dk::OK) return 2;
  }
  shared_donor = donor;
  auto worker = [&](int id) {
    std::mt19937 rng(1000 + id);
    for (int it = 0; it < kIters; ++it) {
      int32_t s = -1;
      const int32_t rc = pool.acquire(0, 50, &s);  // blocks up to 50 ms when the transient region is empty
      if (rc == dk::ERR_TIMEOUT) continue;
      if (rc != dk::OK) { ++failures; continue; }
      int64_t len = -1;
      if (pool.length(s, &len) != dk::OK || len != 0) ++failures;
      const int64_t m = rng() % 500;
      if (m > 0 && pool.alias(shared_donor.load(), s, 0, m) != dk::OK) ++failures;
      const int32_t add = 1 + (int32_t)(rng() % 200);
      const int32_t cu[2] = {0, add};
      std::vector<int64_t> dst;
      const int32_t ra = pool.append(1, &s, cu, nullptr, &dst);
      if (ra == dk::OK) {
        if (pool.length(s, &len) != dk::OK || len != m + add) ++failures;
        std::vector<int64_t> cells((size_t)len);
        if (pool.cells(s, cells.data(), len) != dk::OK) ++failures;
        if (pool.trim(s, m + add / 2) != dk::OK) ++failures;
        std::vector<dk::Extent> ext;
        int64_t l2 = 0;
        if (pool.extents(s, &ext, &l2) != dk::OK || l2 != m + add / 2) ++failures;
      } else if (ra != dk::ERR_NO_CELLS) {
        ++failures;
      }
      if (pool.release(s) != dk::OK) ++failures;
    }
  };
  std::vector<std::thread> ts;
  for (int i = 0; i < kThreads; ++i) ts.emplace_back(worker, i);
  for (auto& t : ts) t.join();
  int64_t held = 0, free_cells = 0;
  pool.release(donor);
  pool.stats(&held, &free_cells);
  if (held != 0) ++failures;  // everything went back
  std::printf("failures %d held %lld free %lld\n", failures.load(), (long long)held, (long long)free_cells);
  return failures.load() == 0 ? 0 : 1;
}
