// C ABI of libdeltakv (see include/deltakv.h): argument checking, host bookkeeping, descriptor
// upload and kernel launches.  Launching calls neither allocate device or pinned memory nor wait for
// the device; only dk_pool_destroy and dk_attend_times wait (for the work they are asked about).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/deltakv.h"
#include "kernels.hpp"
#include "plan.hpp"
#include "pool.hpp"
#include "radix.hpp"

namespace {

constexpr int64_t kMetaBytes = 1 << 20;  // device scratch for copy tables: 256k tokens per launch
constexpr int kMaxRing = 64;
constexpr int kDefaultRing = 8;
constexpr int64_t kMinStageBytes = 64 << 10;

// One buffer of the caller's pinned staging memory and the event that tells when its last upload is done.
struct Staging {
  char* host = nullptr;
  hipEvent_t done = nullptr;
  bool in_flight = false;
};

struct PhaseClock {
  std::chrono::steady_clock::time_point t = std::chrono::steady_clock::now();
  // microseconds since the last call (or construction)
  double lap() {
    const auto now = std::chrono::steady_clock::now();
    const double us = std::chrono::duration<double, std::micro>(now - t).count();
    t = now;
    return us;
  }
};

// Exceptions must not cross the C boundary: host containers may throw std::bad_alloc.
template <typename F>
int32_t guarded(F&& body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return DK_ERR_NO_MEMORY;
  } catch (...) {
    return DK_ERR_INVALID;
  }
}

}  // namespace

struct dk_pool {
  dk_pool_desc desc;
  dk::Pool meta;
  dk::PlanConfig cfg;
  Staging ring[kMaxRing];
  int ring_size = 0;
  int ring_next = 0;
  size_t stage_cap = 0;  // bytes per staging buffer
  int32_t variant = 0;
  std::vector<hipEvent_t> ev0, ev1;  // ring of start/stop events around the attention kernels
  int64_t ev_calls = 0;              // calls recorded since timing was switched on
  int32_t last_hip = 0;
  // host time spent inside launching calls, by phase (see dk_host_times)
  double host_us[DK_HOST_PHASES] = {};
  int64_t host_calls[2] = {0, 0};  // dk_delta_attend*, dk_kv_append
  std::mutex launch_mu;  // serialises GPU-launching calls (shared staging ring, dev_meta and plan)
  dk::AttendPlan plan;   // reused from call to call so that steady-state planning allocates nothing
  std::vector<int64_t> append_cells, append_old_len;  // likewise, for the bookkeeping of appends

  dk_pool(const dk_pool_desc& d, int32_t granule)
      : desc(d), meta(d.n_slots, d.n_session_slots, d.arena_cells, granule), granule_cells(granule) {}
  int32_t granule_cells;

  dk::ArenaView view() const {
    return {desc.k_arena, desc.v_arena, meta_arena_cells, desc.n_q_heads, desc.n_kv_heads, desc.head_dim, desc.dtype};
  }
  int64_t meta_arena_cells = 0;

  int32_t hip_fail(hipError_t e) {
    last_hip = (int32_t)e;
    return DK_ERR_HIP;
  }

  // The next staging buffer, if the upload that last used it has finished.  Never waits and never
  // allocates: DK_ERR_BUSY when every buffer is still in flight, DK_ERR_WORKSPACE when the pool was
  // created without staging memory or `bytes` exceeds one buffer.
  int32_t stage(size_t bytes, Staging** out) {
    if (ring_size == 0 || bytes > stage_cap) return DK_ERR_WORKSPACE;
    Staging& s = ring[ring_next];
    if (s.in_flight) {
      const hipError_t e = hipEventQuery(s.done);
      if (e == hipErrorNotReady) return DK_ERR_BUSY;
      if (e != hipSuccess) return hip_fail(e);
      s.in_flight = false;
    }
    ring_next = (ring_next + 1) % ring_size;
    *out = &s;
    return DK_OK;
  }

  int32_t upload(Staging* s, void* dev, size_t bytes, hipStream_t stream) {
    hipError_t e = hipMemcpyAsync(dev, s->host, bytes, hipMemcpyHostToDevice, stream);
    if (e != hipSuccess) return hip_fail(e);
    e = hipEventRecord(s->done, stream);
    if (e != hipSuccess) return hip_fail(e);
    s->in_flight = true;
    return DK_OK;
  }

  void drop_events() {
    for (int i = 0; i < ring_size; ++i)
      if (ring[i].done) (void)hipEventDestroy(ring[i].done);
    for (hipEvent_t e : ev0) (void)hipEventDestroy(e);
    for (hipEvent_t e : ev1) (void)hipEventDestroy(e);
    ring_size = 0;
    ev0.clear();
    ev1.clear();
  }
};

namespace {

bool desc_ok(const dk_pool_desc* d, int32_t* why) {
  *why = DK_ERR_INVALID;
  if (!d || d->n_slots <= 0 || d->n_session_slots < 0 || d->n_session_slots > d->n_slots) return false;
  if (d->granule_cells < 0 || d->arena_cells <= 0) return false;
  if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->head_dim <= 0) return false;
  *why = DK_ERR_UNSUPPORTED;
  if (d->n_q_heads % d->n_kv_heads) return false;
  if (d->head_dim != 64 && d->head_dim != 128) return false;
  if (d->dtype != DK_F32 && d->dtype != DK_BF16) return false;
  return true;
}

bool is_pow2(int32_t x) { return x > 0 && (x & (x - 1)) == 0; }

}  // namespace

extern "C" {

int32_t dk_meta_bytes(const dk_pool_desc* desc, int64_t* bytes_out) {
  int32_t why;
  if (!bytes_out) return DK_ERR_INVALID;
  if (!desc_ok(desc, &why)) return why;
  *bytes_out = kMetaBytes;
  return DK_OK;
}

int32_t dk_staging_bytes(const dk_pool_desc* desc, int64_t* bytes_out) {
  int32_t why;
  if (!bytes_out) return DK_ERR_INVALID;
  if (!desc_ok(desc, &why)) return why;
  const int64_t depth = desc->staging_depth ? desc->staging_depth : kDefaultRing;
  if (depth < 1 || depth > kMaxRing) return DK_ERR_INVALID;
  *bytes_out = depth * kMetaBytes;
  return DK_OK;
}

int32_t dk_pool_create(const dk_pool_desc* desc, dk_pool** pool_out) {
  return guarded([&]() -> int32_t {
    int32_t why;
    if (!pool_out) return DK_ERR_INVALID;
    *pool_out = nullptr;
    if (!desc_ok(desc, &why)) return why;
    if (!desc->k_arena || !desc->v_arena || !desc->dev_meta || desc->dev_meta_bytes < kMetaBytes) return DK_ERR_INVALID;
    if (((uintptr_t)desc->k_arena | (uintptr_t)desc->v_arena | (uintptr_t)desc->dev_meta) & 255) return DK_ERR_INVALID;
    const int32_t granule = desc->granule_cells ? desc->granule_cells : 256;
    if (desc->arena_cells / granule <= 0) return DK_ERR_INVALID;
    if (desc->arena_cells > INT32_MAX) return DK_ERR_UNSUPPORTED;
    const int32_t depth = desc->staging_depth ? desc->staging_depth : kDefaultRing;
    if (depth < 1 || depth > kMaxRing || desc->host_staging_bytes < 0) return DK_ERR_INVALID;
    if ((desc->host_staging == nullptr) != (desc->host_staging_bytes == 0)) return DK_ERR_INVALID;
    if (desc->host_staging && (((uintptr_t)desc->host_staging & 255) || desc->host_staging_bytes / depth < kMinStageBytes))
      return DK_ERR_INVALID;
    dk_pool* p = new dk_pool(*desc, granule);
    // The arena keeps the caller's stride: rows of KV head g start at g * arena_cells.
    p->meta_arena_cells = desc->arena_cells;
    if (desc->host_staging) {
      p->stage_cap = (size_t)(desc->host_staging_bytes / depth) & ~(size_t)255;
      for (int i = 0; i < depth; ++i) {
        p->ring[i].host = (char*)desc->host_staging + (size_t)i * p->stage_cap;
        const hipError_t e = hipEventCreateWithFlags(&p->ring[i].done, hipEventDisableTiming);
        if (e != hipSuccess) {
          p->drop_events();
          delete p;
          return DK_ERR_HIP;
        }
        p->ring_size = i + 1;
      }
    }
    const int32_t group = desc->n_q_heads / desc->n_kv_heads;
    dk::PlanConfig& c = p->cfg;
    c.n_q_heads = desc->n_q_heads;
    c.n_kv_heads = desc->n_kv_heads;
    c.head_dim = desc->head_dim;
    c.use_mfma = desc->dtype == DK_BF16 && desc->head_dim == 128 && is_pow2(group) && group <= 16;
    c.tile_rows = 256;
    c.stream_rows = 96;
    c.kv_tile = 64;
    // stream items: never cut a slot's keys finer than one CU's fair share of the batch (256 CUs); every extra
    // item costs a ramp-up, a partial write and merge work, and the planner's chains balance the rest
    c.stream_target = std::max(1, 256 / desc->n_kv_heads);
    c.tile_wave_slots = std::max(1, 256 / desc->n_kv_heads);
    c.tile_min_chunk = 128;
    c.tile_item_cost = 5;
    c.stream_min_chunk = 512;
    c.stream_chains = 256;
    c.stream_item_cost = 512;
    // Workgroup w of a launch runs on XCD w % 8, and on every MI355X measured the odd XCDs stream K/V 5-10 % slower
    // than the even ones while the whole chip pulls on HBM: chains planned on the host give them that much less.
    for (int x = 0; x < 8; ++x) c.xcd_speed[x] = (x & 1) ? 0.95f : 1.f;
    c.stream_queue = 1;
    c.inline_blob_bytes = dk::INLINE_BLOB_BYTES;
    *pool_out = p;
    return DK_OK;
  });
}

int32_t dk_pool_destroy(dk_pool* pool) {
  if (!pool) return DK_ERR_INVALID;
  for (int i = 0; i < pool->ring_size; ++i)
    if (pool->ring[i].in_flight) (void)hipEventSynchronize(pool->ring[i].done);
  pool->drop_events();
  delete pool;
  return DK_OK;
}

int32_t dk_set_tuning(dk_pool* pool, const char* name, double value) {
  if (!pool || !name || !(value == value)) return DK_ERR_INVALID;
  std::lock_guard<std::mutex> launch(pool->launch_mu);
  dk::PlanConfig& c = pool->cfg;
  const std::string key(name);
  const auto whole = [&](int32_t lo, int32_t hi, int32_t* dst) -> int32_t {
    if (value < lo || value > hi || value != (double)(int64_t)value) return DK_ERR_INVALID;
    *dst = (int32_t)value;
    return DK_OK;
  };
  if (key == "stream_rows") return whole(32, 96, &c.stream_rows);
  if (key == "stream_target") return whole(1, 1 << 20, &c.stream_target);
  if (key == "stream_min_chunk") return whole(64, 1 << 24, &c.stream_min_chunk);
  if (key == "stream_chains") return whole(1, 1 << 16, &c.stream_chains);
  if (key == "stream_item_cost") return whole(0, 1 << 20, &c.stream_item_cost);
  if (key == "stream_queue") return whole(0, 2, &c.stream_queue);
  if (key == "tile_wave_slots") return whole(1, 1 << 16, &c.tile_wave_slots);
  if (key == "tile_min_chunk") return whole(64, 1 << 24, &c.tile_min_chunk);
  if (key == "tile_item_cost") return whole(0, 1 << 16, &c.tile_item_cost);
  if (key.size() == 10 && key.compare(0, 9, "xcd_speed") == 0 && key[9] >= '0' && key[9] <= '7') {
    if (!(value > 0.0) || value > 100.0) return DK_ERR_INVALID;
    c.xcd_speed[key[9] - '0'] = (float)value;
    return DK_OK;
  }
  return DK_ERR_UNSUPPORTED;
}

int32_t dk_seq_acquire(dk_pool* pool, int32_t region, int64_t timeout_ms, int32_t* slot_out) {
  if (!pool) return DK_ERR_INVALID;
  return pool->meta.acquire(region, timeout_ms, slot_out);
}
int32_t dk_seq_release(dk_pool* pool, int32_t slot) { return pool ? pool->meta.release(slot) : DK_ERR_INVALID; }
int32_t dk_seq_len(dk_pool* pool, int32_t slot, int64_t* len_out) {
  return pool ? pool->meta.length(slot, len_out) : DK_ERR_INVALID;
}
int32_t dk_seq_alias(dk_pool* pool, int32_t donor, int32_t dst, int64_t p0, int64_t p1) {
  return pool ? pool->meta.alias(donor, dst, p0, p1) : DK_ERR_INVALID;
}
int32_t dk_seq_trim(dk_pool* pool, int32_t slot, int64_t new_len) {
  return pool ? pool->meta.trim(slot, new_len) : DK_ERR_INVALID;
}
int32_t dk_seq_trim_batch(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int64_t* new_len) {
  if (!pool) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t { return pool->meta.trim_batch(n_seqs, slots, new_len); });
}
int32_t dk_seq_cells(dk_pool* pool, int32_t slot, int64_t* cells_out, int64_t cap) {
  return pool ? pool->meta.cells(slot, cells_out, cap) : DK_ERR_INVALID;
}
int32_t dk_seq_stats(dk_pool* pool, int32_t slot, int64_t* segments_out, int64_t* chain_nodes_out) {
  if (!pool) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t { return pool->meta.seq_stats(slot, segments_out, chain_nodes_out); });
}
int32_t dk_pool_stats(dk_pool* pool, int64_t* held, int64_t* free_cells) {
  return pool ? pool->meta.stats(held, free_cells) : DK_ERR_INVALID;
}

}  // extern "C"

namespace {

void undo_append(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const std::vector<int64_t>& old_len) {
  for (int32_t b = 0; b < n_seqs; ++b) (void)pool->meta.trim(slots[b], old_len[b]);
}

// dk_kv_append with pool->launch_mu held.  Leaves the slots' previous lengths in pool->append_old_len.
int32_t append_locked(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                      const int32_t* n_accept, const void* k_new, const void* v_new, void* stream) {
  PhaseClock clk;
  const int64_t total = (n_seqs > 0 && cu_delta) ? cu_delta[n_seqs] : 0;
  if (total > 0 && (!k_new || !v_new)) return DK_ERR_INVALID;
  const bool inline_cells = total <= dk::KV_INLINE_MAX_TOKENS;
  const int64_t per_launch =
      std::min<int64_t>(pool->desc.dev_meta_bytes, (int64_t)pool->stage_cap) / (int64_t)sizeof(int32_t);
  if (!inline_cells && per_launch <= 0) return DK_ERR_WORKSPACE;  // long appends need staging memory
  std::vector<int64_t>& dst = pool->append_cells;
  std::vector<int64_t>& old_len = pool->append_old_len;
  int32_t rc = pool->meta.append(n_seqs, slots, cu_delta, n_accept, &dst, &old_len);
  if (rc != DK_OK) return rc;
  // From here on a failure must leave the pool as it was: the bookkeeping is rolled back.
  const auto undo = [&](int32_t status) {
    undo_append(pool, n_seqs, slots, old_len);
    return status;
  };
  hipStream_t st = (hipStream_t)stream;
  pool->host_us[DK_HOST_APPEND_BOOK] += clk.lap();
  ++pool->host_calls[1];
  if (inline_cells) {
    hipError_t e = dk::launch_kv_scatter_inline(pool->view(), pool->desc.k_arena, pool->desc.v_arena, dst.data(),
                                                (int32_t)total, k_new, v_new, st);
    pool->host_us[DK_HOST_APPEND_LAUNCH] += clk.lap();
    return e == hipSuccess ? DK_OK : undo(pool->hip_fail(e));
  }
  for (int64_t base = 0; base < total; base += per_launch) {
    const int32_t n = (int32_t)std::min<int64_t>(per_launch, total - base);
    Staging* s;
    rc = pool->stage((size_t)n * sizeof(int32_t), &s);
    // Chunks already enqueued wrote cells that the rolled-back slots no longer own: harmless, they are free.
    if (rc != DK_OK) return undo(rc);
    int32_t* h = (int32_t*)s->host;
    for (int32_t t = 0; t < n; ++t) h[t] = (int32_t)dst[base + t];
    rc = pool->upload(s, pool->desc.dev_meta, (size_t)n * sizeof(int32_t), st);
    if (rc != DK_OK) return undo(rc);
    hipError_t e = dk::launch_kv_scatter(pool->view(), pool->desc.k_arena, pool->desc.v_arena,
                                         (const int32_t*)pool->desc.dev_meta, base, n, k_new, v_new, st);
    if (e != hipSuccess) return undo(pool->hip_fail(e));
  }
  pool->host_us[DK_HOST_APPEND_LAUNCH] += clk.lap();
  return DK_OK;
}

}  // namespace

extern "C" {

int32_t dk_kv_append(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                     const int32_t* n_accept, const void* k_new, const void* v_new, void* stream) {
  if (!pool) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    std::lock_guard<std::mutex> launch(pool->launch_mu);
    return append_locked(pool, n_seqs, slots, cu_delta, n_accept, k_new, v_new, stream);
  });
}

int32_t dk_kv_reserve(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                      const int32_t* n_accept, int64_t* cells_out) {
  if (!pool) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    const int64_t total = (n_seqs > 0 && cu_delta) ? cu_delta[n_seqs] : 0;
    if (total > 0 && !cells_out) return DK_ERR_INVALID;
    std::vector<int64_t> dst;
    int32_t rc = pool->meta.append(n_seqs, slots, cu_delta, n_accept, &dst, nullptr);
    if (rc != DK_OK) return rc;
    for (int64_t t = 0; t < total; ++t) cells_out[t] = dst[t];
    return DK_OK;
  });
}

int32_t dk_seq_gather(dk_pool* pool, int32_t slot, void* k_out, void* v_out, void* stream) {
  if (!pool) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    std::lock_guard<std::mutex> launch(pool->launch_mu);
    int64_t len = 0;
    int32_t rc = pool->meta.length(slot, &len);
    if (rc != DK_OK) return rc;
    if (len == 0) return DK_OK;
    if (!k_out || !v_out) return DK_ERR_INVALID;
    std::vector<int64_t> cells(len);
    rc = pool->meta.cells(slot, cells.data(), len);
    if (rc != DK_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int64_t per_launch =
        std::min<int64_t>(pool->desc.dev_meta_bytes, (int64_t)pool->stage_cap) / (int64_t)sizeof(int32_t);
    if (per_launch <= 0) return DK_ERR_WORKSPACE;
    for (int64_t base = 0; base < len; base += per_launch) {
      const int32_t n = (int32_t)std::min<int64_t>(per_launch, len - base);
      Staging* s;
      rc = pool->stage((size_t)n * sizeof(int32_t), &s);
      if (rc != DK_OK) return rc;
      int32_t* h = (int32_t*)s->host;
      for (int32_t t = 0; t < n; ++t) h[t] = (int32_t)cells[base + t];
      rc = pool->upload(s, pool->desc.dev_meta, (size_t)n * sizeof(int32_t), st);
      if (rc != DK_OK) return rc;
      hipError_t e = dk::launch_kv_gather(pool->view(), (const int32_t*)pool->desc.dev_meta, base, n, k_out, v_out, st);
      if (e != hipSuccess) return pool->hip_fail(e);
    }
    return DK_OK;
  });
}

int32_t dk_attend_workspace_bytes(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                                  int32_t staged, int64_t* bytes_out) {
  if (!pool || !bytes_out) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    std::lock_guard<std::mutex> launch(pool->launch_mu);
    dk::AttendPlan& plan = pool->plan;
    dk::PlanConfig cfg = pool->cfg;
    if (pool->variant == 1) cfg.use_mfma = false;
    std::lock_guard<std::mutex> lk(pool->meta.mutex());
    if (staged < 0 || staged > 2) return DK_ERR_INVALID;
    int32_t rc = dk::build_plan(pool->meta, cfg, n_seqs, slots, cu_delta, staged != 0, &plan, staged == 2);
    if (rc != DK_OK) return rc;
    *bytes_out = (int64_t)plan.total_bytes;
    // dk_append_attend may also plan the batch after its append, in appended mode: the same work items over slots
    // that then have more runs of cells (at worst one per granule the append takes)
    if (staged == 2)
      *bytes_out += ((int64_t)n_seqs * 8 + plan.total_tokens / pool->granule_cells + 16) * (int64_t)sizeof(DkSeg) + 4096;
    return DK_OK;
  });
}

namespace {

// A private status of attend_locked: the call is not one whose append can be folded into the attention kernel.
constexpr int32_t kNotFoldable = 1;
// Calls above these sizes are not even planned for folding (their descriptors cannot fit the kernel arguments).
constexpr int32_t kFoldMaxSeqs = 16;
constexpr int64_t kFoldMaxTokens = 384;

// Plans the call, uploads its descriptors into `workspace` and launches the attention kernels.  pool->launch_mu
// is held.
// fold_append: the call also appends all new tokens to their slots, provided that its descriptors fit the kernel
// arguments and an MFMA kernel runs (otherwise kNotFoldable is returned and nothing has happened): the attention is
// planned on the slots as they are (staged mode), the bookkeeping follows, and the rows are written into the arena
// by the attention kernel itself.
int32_t attend_locked(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta, const void* q,
                      const void* k_new, const void* v_new, float scale, void* out, float* lse, void* workspace,
                      int64_t workspace_bytes, void* stream, bool fold_append) {
  if ((k_new == nullptr) != (v_new == nullptr)) return DK_ERR_INVALID;
  const bool staged = k_new != nullptr;
  if (fold_append && !staged) return DK_ERR_INVALID;
  PhaseClock clk;
  dk::AttendPlan& plan = pool->plan;
  dk::PlanConfig cfg = pool->cfg;
  // the MFMA kernels take the row maximum before scaling, which needs a positive finite scale
  if (pool->variant == 1 || !(scale > 0.f) || !(scale < 3.0e38f)) cfg.use_mfma = false;
  {
    std::lock_guard<std::mutex> lk(pool->meta.mutex());
    int32_t rc = dk::build_plan(pool->meta, cfg, n_seqs, slots, cu_delta, staged, &plan, fold_append);
    if (rc != DK_OK) return rc;
  }
  if (plan.total_tokens == 0) return DK_OK;
  if (!q || !out) return DK_ERR_INVALID;
  const bool inline_blob = plan.blob_bytes <= (size_t)dk::INLINE_BLOB_BYTES && !plan.stream_queued;
  if (fold_append && !(inline_blob && cfg.use_mfma && (plan.tile_chains > 0 || plan.stream_chains > 0)))
    return kNotFoldable;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < (int64_t)plan.total_bytes) return DK_ERR_WORKSPACE;
  // The bookkeeping half of a folded append.  From here on a failure must leave the pool as it was.
  std::vector<int64_t>& dst = pool->append_cells;
  std::vector<int64_t>& old_len = pool->append_old_len;
  if (fold_append) {
    const int32_t rc = pool->meta.append(n_seqs, slots, cu_delta, nullptr, &dst, &old_len);
    if (rc != DK_OK) return rc;
    ++pool->host_calls[1];
  }
  const auto fail = [&](int32_t status) {
    if (fold_append) undo_append(pool, n_seqs, slots, old_len);
    return status;
  };
  pool->host_us[DK_HOST_PLAN] += clk.lap();

  hipStream_t st = (hipStream_t)stream;
  // Small descriptor blobs travel inside the kernel arguments; larger ones go through a staging buffer into
  // the workspace.
  dk::InlineBlob blob_args{};
  char* h = (char*)&blob_args;
  Staging* s = nullptr;
  if (!inline_blob) {
    const int32_t rc = pool->stage(plan.blob_bytes, &s);
    if (rc != DK_OK) return fail(rc);
    h = s->host;
  }
  auto put = [&](size_t off, const void* src, size_t bytes) { if (bytes) std::memcpy(h + off, src, bytes); };
  put(plan.off_entries, plan.entries.data(), plan.entries.size() * sizeof(DkEntry));
  put(plan.off_segs, plan.segs.data(), plan.segs.size() * sizeof(DkSeg));
  put(plan.off_tile, plan.tile_items.data(), plan.tile_items.size() * sizeof(DkItem));
  put(plan.off_tile_links, plan.tile_links.data(), plan.tile_links.size() * sizeof(int32_t));
  put(plan.off_stream, plan.stream_items.data(), plan.stream_items.size() * sizeof(DkItem));
  put(plan.off_links, plan.stream_links.data(), plan.stream_links.size() * sizeof(int32_t));
  put(plan.off_merges, plan.merges.data(), plan.merges.size() * sizeof(DkMerge));
  if (plan.stream_queued) {  // the queue's counter: the first stream_chains units are taken when the kernel starts
    const int32_t first[4] = {plan.stream_chains, 0, 0, 0};
    put(plan.off_queue, first, sizeof(first));
  }
  if (fold_append) {
    int32_t* cells = (int32_t*)(h + plan.off_cells);
    for (int64_t t = 0; t < plan.total_tokens; ++t) cells[t] = (int32_t)dst[t];
  }
  pool->host_us[DK_HOST_STAGE] += clk.lap();
  if (!inline_blob) {
    const int32_t rc = pool->upload(s, workspace, plan.blob_bytes, st);
    if (rc != DK_OK) return fail(rc);
  }
  pool->host_us[DK_HOST_UPLOAD] += clk.lap();

  // where the kernels find the descriptors: in the workspace, or at these offsets of their own arguments
  char* ws = (char*)workspace;
  const uintptr_t desc = inline_blob ? 0 : (uintptr_t)ws;
  dk::AttendArgs a;
  a.inline_blob = inline_blob ? &blob_args : nullptr;
  a.arena = pool->view();
  a.entries = (const DkEntry*)(desc + plan.off_entries);
  a.n_entries = (int32_t)plan.entries.size();
  a.segs = (const DkSeg*)(desc + plan.off_segs);
  a.q = q;
  a.k_new = k_new;
  a.v_new = v_new;
  a.out = out;
  a.lse = lse;
  a.parts = (float*)(ws + plan.off_parts);
  a.parts_ml = a.parts + (size_t)plan.part_rows * pool->desc.n_kv_heads * pool->desc.head_dim;
  a.scale = scale;
  a.total_tokens = (int32_t)plan.total_tokens;
  a.cells = (const int32_t*)(desc + plan.off_cells);

  hipError_t e = hipSuccess;
  const bool timing = !pool->ev0.empty();
  const size_t ev_slot = timing ? (size_t)(pool->ev_calls % (int64_t)pool->ev0.size()) : 0;
  if (timing) {
    e = hipEventRecord(pool->ev0[ev_slot], st);
    if (e != hipSuccess) return fail(pool->hip_fail(e));
  }
  if (!cfg.use_mfma) {
    e = dk::launch_attend_ref(a, st);
    if (e != hipSuccess) return fail(pool->hip_fail(e));
  } else {
    // a folded append is carried out by the first MFMA kernel of the call
    a.scatter = fold_append && plan.tile_chains > 0;
    e = dk::launch_attend_tile(a, (const DkItem*)(desc + plan.off_tile), (const int32_t*)(desc + plan.off_tile_links),
                               plan.tile_chains, st);
    if (e != hipSuccess) return fail(pool->hip_fail(e));
    a.scatter = fold_append && plan.tile_chains == 0;
    int32_t stream_rows = 0;
    for (const DkItem& it : plan.stream_items) stream_rows = std::max(stream_rows, it.nrows);
    e = dk::launch_attend_stream(a, (const DkItem*)(desc + plan.off_stream), (const int32_t*)(desc + plan.off_links),
                                 plan.stream_chains, stream_rows,
                                 plan.stream_queued ? (int32_t*)(ws + plan.off_queue) : nullptr,
                                 (int32_t)plan.stream_units, st);
    if (e != hipSuccess) return fail(pool->hip_fail(e));
    a.scatter = false;
    int32_t max_rows = 0;
    for (const DkMerge& mg : plan.merges) max_rows = std::max(max_rows, mg.nrows);
    e = dk::launch_attend_merge(a, (const DkMerge*)(desc + plan.off_merges), (int32_t)plan.merges.size(), max_rows, st);
    if (e != hipSuccess) return fail(pool->hip_fail(e));
  }
  if (timing) {  // the interval covers every kernel of the call, the merge of split key ranges included
    e = hipEventRecord(pool->ev1[ev_slot], st);
    if (e != hipSuccess) return fail(pool->hip_fail(e));
    ++pool->ev_calls;
  }
  pool->host_us[DK_HOST_LAUNCH] += clk.lap();
  ++pool->host_calls[0];
  return DK_OK;
}

int32_t attend_impl(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta, const void* q,
                    const void* k_new, const void* v_new, float scale, void* out, float* lse, void* workspace,
                    int64_t workspace_bytes, void* stream) {
  std::lock_guard<std::mutex> launch(pool->launch_mu);
  return attend_locked(pool, n_seqs, slots, cu_delta, q, k_new, v_new, scale, out, lse, workspace, workspace_bytes,
                       stream, false);
}

// dk_append_attend.  A small call (its descriptors and cell table fit the kernel arguments) is one launch: the
// attention kernel writes the new rows itself.  Any other call is what dk_kv_append followed by dk_delta_attend in
// appended mode would be (measured: for large batches the copy inside the attention kernel costs about what the
// separate copy kernel does, and attending the new rows from the arena beats reading them token-major).
int32_t append_attend_impl(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                           const void* q, const void* k_new, const void* v_new, float scale, void* out, float* lse,
                           void* workspace, int64_t workspace_bytes, void* stream) {
  std::lock_guard<std::mutex> launch(pool->launch_mu);
  const int64_t total = (n_seqs > 0 && cu_delta) ? cu_delta[n_seqs] : 0;
  if (total > 0 && (!k_new || !v_new)) return DK_ERR_INVALID;
  if (n_seqs <= kFoldMaxSeqs && total <= kFoldMaxTokens) {
    const int32_t rc = attend_locked(pool, n_seqs, slots, cu_delta, q, k_new, v_new, scale, out, lse, workspace,
                                     workspace_bytes, stream, true);
    if (rc != kNotFoldable) return rc;
  }
  if (total > 0 && (!q || !out)) return DK_ERR_INVALID;
  int32_t rc = append_locked(pool, n_seqs, slots, cu_delta, nullptr, k_new, v_new, stream);
  if (rc != DK_OK) return rc;
  rc = attend_locked(pool, n_seqs, slots, cu_delta, q, nullptr, nullptr, scale, out, lse, workspace, workspace_bytes,
                     stream, false);
  // (the copy kernel already enqueued wrote cells that the rolled-back slots no longer own: harmless, they are free)
  if (rc != DK_OK) undo_append(pool, n_seqs, slots, pool->append_old_len);
  return rc;
}

}  // namespace

namespace {

// Scratch of dk_delta_attend_noalloc: descriptors and split partials of one call.  Every GPU the library
// runs on holds its own copy of this array, at its own address, until the process ends.
static __device__ __align__(256) unsigned char scratch[DK_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, resolved on first use
std::mutex g_scratch_mu;

// The array's name is only a host-side handle; what kernels and copies need is the address the current
// device gave its copy of the array.
int32_t static_scratch(dk_pool* pool, void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return pool->hip_fail(e);
  if (dev < 0 || dev >= kMaxDevices) return DK_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return pool->hip_fail(e);
    if (!ptr) return pool->hip_fail(hipErrorInvalidSymbol);
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return DK_OK;
}

}  // namespace

int32_t dk_delta_attend_noalloc(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                                const void* q, const void* k_new, const void* v_new, float scale, void* out,
                                float* lse, void* stream) {
  if (!pool) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    void* ws = nullptr;
    const int32_t rc = static_scratch(pool, &ws);
    if (rc != DK_OK) return rc;
    // a call that needs more than the array holds is turned down by the size check (DK_ERR_WORKSPACE)
    return attend_impl(pool, n_seqs, slots, cu_delta, q, k_new, v_new, scale, out, lse, ws,
                       (int64_t)DK_STATIC_SCRATCH_BYTES, stream);
  });
}

int32_t dk_append_attend(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta, const void* q,
                         const void* k_new, const void* v_new, float scale, void* out, float* lse, void* workspace,
                         int64_t workspace_bytes, void* stream) {
  if (!pool) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    return append_attend_impl(pool, n_seqs, slots, cu_delta, q, k_new, v_new, scale, out, lse, workspace,
                              workspace_bytes, stream);
  });
}

int32_t dk_delta_attend(dk_pool* pool, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta, const void* q,
                        const void* k_new, const void* v_new, float scale, void* out, float* lse, void* workspace,
                        int64_t workspace_bytes, void* stream) {
  if (!pool) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    return attend_impl(pool, n_seqs, slots, cu_delta, q, k_new, v_new, scale, out, lse, workspace, workspace_bytes,
                       stream);
  });
}

}  // extern "C"

struct dk_radix {
  dk_pool* pool;
  dk::Radix trie;
  std::mutex mu;
  dk_radix(dk_pool* p, int64_t budget, int32_t keep_last) : pool(p), trie(&p->meta, budget, keep_last) {}
};

extern "C" {

int32_t dk_radix_create(dk_pool* pool, int64_t cell_budget, int32_t keep_last, dk_radix** radix_out) {
  if (!pool || !radix_out || cell_budget <= 0 || keep_last < 0) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    *radix_out = new dk_radix(pool, cell_budget, keep_last);
    return DK_OK;
  });
}
int32_t dk_radix_destroy(dk_radix* radix) {
  if (!radix) return DK_ERR_INVALID;
  delete radix;
  return DK_OK;
}
int32_t dk_radix_begin_turn(dk_radix* radix, int32_t slot, const int32_t* tokens, int64_t n_tokens,
                            int64_t* n_past_out) {
  if (!radix) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    std::lock_guard<std::mutex> lk(radix->mu);
    return radix->trie.begin_turn(slot, tokens, n_tokens, n_past_out);
  });
}
int32_t dk_radix_save(dk_radix* radix, int32_t slot, const int32_t* tokens, int64_t n_tokens, int32_t* saved_out) {
  if (!radix) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    std::lock_guard<std::mutex> lk(radix->mu);
    return radix->trie.save(slot, tokens, n_tokens, saved_out);
  });
}
int32_t dk_radix_stats(dk_radix* radix, int64_t* nodes_out, int64_t* cells_out, int64_t* donors_out,
                       int64_t* evictions_out) {
  if (!radix) return DK_ERR_INVALID;
  std::lock_guard<std::mutex> lk(radix->mu);
  radix->trie.stats(nodes_out, cells_out, donors_out, evictions_out);
  return DK_OK;
}
int32_t dk_radix_evicted_path(dk_radix* radix, int64_t index, int32_t* tokens_out, int64_t cap, int64_t* len_out) {
  if (!radix || !len_out || cap < 0 || (cap > 0 && !tokens_out)) return DK_ERR_INVALID;
  std::lock_guard<std::mutex> lk(radix->mu);
  const int64_t n = radix->trie.evicted_path(index, tokens_out, cap);
  if (n < 0) return DK_ERR_INVALID;
  *len_out = n;
  return DK_OK;
}

int32_t dk_verify_workspace_bytes(int32_t total_rows, int64_t vocab, int32_t dtype, int64_t* bytes_out) {
  if (!bytes_out || total_rows < 0 || vocab <= 0 || vocab > INT32_MAX) return DK_ERR_INVALID;
  if (dtype != DK_F32 && dtype != DK_BF16) return DK_ERR_UNSUPPORTED;
  *bytes_out = dk::verify_workspace_bytes(total_rows, vocab, dtype);
  return DK_OK;
}

int32_t dk_verify_greedy(int32_t n_seqs, int32_t total_rows, const int32_t* cu_delta_dev, const void* logits,
                         int32_t dtype, int64_t vocab, int64_t row_stride, const int32_t* batch_tokens,
                         int32_t* argmax_out, int32_t* n_keep_out, int32_t* next_token_out, void* workspace,
                         int64_t workspace_bytes, void* stream) {
  if (n_seqs < 0 || total_rows < 0 || vocab <= 0 || vocab > INT32_MAX || row_stride < vocab) return DK_ERR_INVALID;
  if (dtype != DK_F32 && dtype != DK_BF16) return DK_ERR_UNSUPPORTED;
  if (n_seqs == 0) return DK_OK;
  if (total_rows > 65535) return DK_ERR_UNSUPPORTED;
  if (!cu_delta_dev || !n_keep_out || !next_token_out) return DK_ERR_INVALID;
  if (total_rows > 0 && (!logits || !batch_tokens)) return DK_ERR_INVALID;
  const int64_t elem = dtype == DK_BF16 ? 2 : 4;
  // rows are read with 16-byte loads
  if (((uintptr_t)logits & 15) || (row_stride * elem) % 16) return DK_ERR_UNSUPPORTED;
  if (!workspace || ((uintptr_t)workspace & 255) ||
      workspace_bytes < dk::verify_workspace_bytes(total_rows, vocab, dtype))
    return DK_ERR_WORKSPACE;
  hipError_t e = dk::launch_verify_greedy(n_seqs, total_rows, cu_delta_dev, logits, dtype, vocab, row_stride,
                                          batch_tokens, argmax_out, n_keep_out, next_token_out, workspace,
                                          (hipStream_t)stream);
  return e == hipSuccess ? DK_OK : DK_ERR_HIP;
}

int32_t dk_staging_wait(dk_pool* pool) {
  if (!pool) return DK_ERR_INVALID;
  // (The event is read under the lock and waited for outside it: other threads may go on launching.)
  hipEvent_t ev = nullptr;
  {
    std::lock_guard<std::mutex> launch(pool->launch_mu);
    if (pool->ring_size == 0) return DK_ERR_WORKSPACE;
    Staging& s = pool->ring[pool->ring_next];
    if (!s.in_flight) return DK_OK;
    ev = s.done;
  }
  const hipError_t e = hipEventSynchronize(ev);
  return e == hipSuccess ? DK_OK : pool->hip_fail(e);
}

int32_t dk_set_attend_variant(dk_pool* pool, int32_t variant) {
  if (!pool || variant < 0 || variant > 1) return DK_ERR_INVALID;
  pool->variant = variant;
  return DK_OK;
}

int32_t dk_set_attend_timing(dk_pool* pool, int32_t n_calls) {
  if (!pool || n_calls < 0 || n_calls > 256) return DK_ERR_INVALID;
  return guarded([&]() -> int32_t {
    std::lock_guard<std::mutex> launch(pool->launch_mu);
    pool->ev0.reserve(256);  // so that the push_backs below cannot throw half-way
    pool->ev1.reserve(256);
    for (hipEvent_t e : pool->ev0) (void)hipEventDestroy(e);
    for (hipEvent_t e : pool->ev1) (void)hipEventDestroy(e);
    pool->ev0.clear();
    pool->ev1.clear();
    pool->ev_calls = 0;
    for (int32_t i = 0; i < n_calls; ++i) {
      hipEvent_t a = nullptr, b = nullptr;
      hipError_t e = hipEventCreate(&a);
      if (e == hipSuccess) e = hipEventCreate(&b);
      if (e != hipSuccess) {
        if (a) (void)hipEventDestroy(a);
        return pool->hip_fail(e);
      }
      pool->ev0.push_back(a);
      pool->ev1.push_back(b);
    }
    return DK_OK;
  });
}

int32_t dk_attend_times(dk_pool* pool, float* ms_out, int32_t cap, int32_t* n_out) {
  if (!pool || !n_out || cap < 0 || (cap > 0 && !ms_out)) return DK_ERR_INVALID;
  std::lock_guard<std::mutex> launch(pool->launch_mu);
  const int64_t ring = (int64_t)pool->ev0.size();
  const int64_t have = std::min<int64_t>(std::min<int64_t>(pool->ev_calls, ring), cap);
  for (int64_t i = 0; i < have; ++i) {
    const size_t slot = (size_t)((pool->ev_calls - have + i) % ring);
    hipError_t e = hipEventSynchronize(pool->ev1[slot]);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms_out[i], pool->ev0[slot], pool->ev1[slot]);
    if (e != hipSuccess) return pool->hip_fail(e);
  }
  *n_out = (int32_t)have;
  return DK_OK;
}

int32_t dk_last_attend_ms(dk_pool* pool, float* ms_out) {
  int32_t n = 0;
  int32_t rc = dk_attend_times(pool, ms_out, 1, &n);
  if (rc != DK_OK) return rc;
  return n == 1 ? DK_OK : DK_ERR_INVALID;
}

int32_t dk_host_times(dk_pool* pool, int32_t reset, double* us_out, int64_t* calls_out) {
  if (!pool) return DK_ERR_INVALID;
  std::lock_guard<std::mutex> launch(pool->launch_mu);
  if (us_out)
    for (int i = 0; i < DK_HOST_PHASES; ++i) us_out[i] = pool->host_us[i];
  if (calls_out) {
    calls_out[0] = pool->host_calls[0];
    calls_out[1] = pool->host_calls[1];
  }
  if (reset) {
    for (double& x : pool->host_us) x = 0.0;
    pool->host_calls[0] = pool->host_calls[1] = 0;
  }
  return DK_OK;
}

const char* dk_strerror(int32_t status) {
  switch (status) {
    case DK_OK: return "ok";
    case DK_ERR_INVALID: return "invalid argument or state";
    case DK_ERR_TIMEOUT: return "no free slot within the timeout";
    case DK_ERR_NO_CELLS: return "KV arena exhausted";
    case DK_ERR_NO_SLOT: return "slot id out of range or not acquired";
    case DK_ERR_DUP_SLOT: return "slot listed twice in one batch";
    case DK_ERR_UNSUPPORTED: return "unsupported shape, dtype or alias form";
    case DK_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case DK_ERR_HIP: return "HIP runtime error";
    case DK_ERR_BUSY: return "every staging buffer is still in flight: synchronise the stream and call again";
    case DK_ERR_NO_MEMORY: return "out of host memory";
    default: return "unknown status";
  }
}

int32_t dk_last_hip_error(dk_pool* pool) { return pool ? pool->last_hip : 0; }

}  // extern "C"
