#include "plan.hpp"

#include <algorithm>
#include <functional>
#include <queue>

namespace dk {

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

namespace {
typedef PlanRowTile RowTile;
typedef PlanKeyedItem Keyed;

// Splits each row tile's visible key range [0, kv_hi) into chunks so that the items of one kernel
// have similar cost and there are about `target` of them per KV head.  All row tiles of an entry use
// the same chunk boundaries (multiples of kv_tile): the workgroups that walk one chunk of one entry
// read the same K/V tiles, so they are made neighbours in launch order (`group` = true) and, running
// at the same time on the XCD of their KV head, fetch each tile from HBM once and from L2 after that.
void cut_items(const std::vector<RowTile>& tiles, int32_t kv_tile, int32_t target, int32_t min_chunk, bool group,
               int32_t wave_slots, int32_t item_cost, std::vector<Keyed>& keyed, std::vector<int64_t>& cost, std::vector<DkItem>* items,
               std::vector<DkMerge>* merges, int64_t* part_rows) {
  if (tiles.empty()) return;
  int64_t total = 0;
  int32_t longest = 0;
  for (const RowTile& t : tiles) {
    total += t.kv_hi;
    longest = std::max(longest, t.kv_hi);
  }
  int64_t chunk = std::max<int64_t>(min_chunk, (total + target - 1) / target);
  chunk = (chunk + kv_tile - 1) / kv_tile * kv_tile;
  if (group && wave_slots > 0) {
    // Tile kernel: pick the chunk length by a small cost model instead.  `wave_slots` workgroups of a KV
    // head run at a time, so n items take ceil(n / wave_slots) rounds; a round lasts as long as an item,
    // (work / n) key tiles plus the fixed cost of an item (pipeline ramp, output store; `item_cost` key
    // tiles).  Splitting finer shortens the rounds but adds rounds, fixed costs and partial rows to merge;
    // what matters most is landing on a whole number of rounds.
    const double fixed = (double)item_cost;
    const double work = (double)total / kv_tile;
    double best = 0;
    int64_t best_chunk = 0;
    for (int32_t k = 1; k <= 512; k += (k < 16 ? 1 : k < 64 ? 4 : 16)) {
      int64_t cand = ((longest + k - 1) / k + kv_tile - 1) / kv_tile * kv_tile;
      if (cand < min_chunk) break;
      int64_t n = 0;
      for (size_t b = 0; b < tiles.size();) {
        size_t e = b;
        int32_t hi_max = 0;
        while (e < tiles.size() && tiles[e].entry == tiles[b].entry) hi_max = std::max(hi_max, tiles[e++].kv_hi);
        n += (int64_t)(e - b) * ((hi_max + cand - 1) / cand);
        b = e;
      }
      const double rounds = (double)((n + wave_slots - 1) / wave_slots);
      const double cost = rounds * (work / (double)n + fixed);
      if (best_chunk == 0 || cost < best * 0.999) {
        best = cost;
        best_chunk = cand;
      }
    }
    if (best_chunk) chunk = best_chunk;
  }

  keyed.clear();
  // tiles of one entry are consecutive in `tiles`
  for (size_t b = 0; b < tiles.size();) {
    size_t e = b;
    int32_t hi_max = 0;
    while (e < tiles.size() && tiles[e].entry == tiles[b].entry) hi_max = std::max(hi_max, tiles[e++].kv_hi);
    int32_t nsplit = (int32_t)((hi_max + chunk - 1) / chunk);
    // avoid a last split that is only a sliver
    if (nsplit > 1 && hi_max - (int64_t)(nsplit - 1) * chunk < chunk / 4) --nsplit;
    const int64_t each = ((hi_max + nsplit - 1) / nsplit + kv_tile - 1) / kv_tile * kv_tile;
    const size_t first = keyed.size();
    for (size_t k = b; k < e; ++k) {
      const RowTile& t = tiles[k];
      int32_t ns = (int32_t)((t.kv_hi + each - 1) / each);
      if (ns > 1 && t.kv_hi - (int64_t)(ns - 1) * each < each / 4) --ns;  // the previous chunk takes the sliver
      int32_t part0 = -1;
      if (ns > 1) {
        part0 = (int32_t)*part_rows;
        *part_rows += (int64_t)ns * t.nrows;
        merges->push_back({t.entry, t.row0, t.nrows, part0, ns, {0, 0, 0}});
      }
      for (int32_t sp = 0; sp < ns; ++sp) {
        DkItem it{};
        it.entry = t.entry;
        it.row0 = t.row0;
        it.nrows = t.nrows;
        it.kv_lo = (int32_t)(sp * each);
        it.kv_hi = sp + 1 == ns ? t.kv_hi : (int32_t)((sp + 1) * each);
        it.part_row0 = ns > 1 ? part0 + sp * t.nrows : -1;
        keyed.push_back({it, 0, sp});
      }
    }
    // cost of each (entry, chunk) group
    cost.assign((size_t)nsplit + 1, 0);
    for (size_t k = first; k < keyed.size(); ++k)
      cost[keyed[k].split] += (int64_t)(keyed[k].it.kv_hi - keyed[k].it.kv_lo) * keyed[k].it.nrows;
    for (size_t k = first; k < keyed.size(); ++k) keyed[k].group_cost = cost[keyed[k].split];
    b = e;
  }
  // longest first, so the tail of the launch is made of the cheapest items
  if (group) {
    std::stable_sort(keyed.begin(), keyed.end(), [](const Keyed& a, const Keyed& b) {
      if (a.group_cost != b.group_cost) return a.group_cost > b.group_cost;
      if (a.it.entry != b.it.entry) return a.it.entry < b.it.entry;
      if (a.split != b.split) return a.split < b.split;
      return a.it.row0 > b.it.row0;
    });
  } else {
    std::stable_sort(keyed.begin(), keyed.end(), [](const Keyed& a, const Keyed& b) {
      return (int64_t)(a.it.kv_hi - a.it.kv_lo) * a.it.nrows > (int64_t)(b.it.kv_hi - b.it.kv_lo) * b.it.nrows;
    });
  }
  for (const Keyed& k : keyed) items->push_back(k.it);
}

// The streaming kernel runs one workgroup per compute unit, and a workgroup walks a chain of units
// (item, KV head).  Its workgroups share no K/V rows, so a unit may run on any XCD.  The units arrive
// longest first and each joins the chain that is free first (longest-processing-time rule on machines of
// unequal speed: workgroup w runs on XCD w % 8, and the XCDs do not stream from HBM equally fast; among
// idle chains the faster ones are served first, so they get the longest units), so that all compute
// units finish together whatever the mix of context lengths.  With very many small units, runs of
// consecutive units are handed out as one block to keep the planning time down.
void chain_units(const std::vector<DkItem>& items, const PlanConfig& cfg, std::vector<std::pair<double, int32_t>>& heap,
                 std::vector<int32_t>& tail, std::vector<int32_t>* links, int32_t* n_chains) {
  const int64_t n_units = (int64_t)items.size() * cfg.n_kv_heads;
  const int32_t chains = (int32_t)std::min<int64_t>(n_units, std::max(cfg.stream_chains, 1));
  *n_chains = chains;
  links->assign((size_t)(chains + n_units), -1);
  int32_t* head = links->data();
  int32_t* next = links->data() + chains;
  if (n_units == chains) {  // one unit each: nothing to balance
    for (int32_t c = 0; c < chains; ++c) head[c] = c;
    return;
  }
  double inv_speed[8];
  for (int x = 0; x < 8; ++x) inv_speed[x] = 1.0 / (cfg.xcd_speed[x] > 0.f ? cfg.xcd_speed[x] : 1.f);
  typedef std::pair<double, int32_t> Free;  // (time at which the chain is free, chain)
  heap.resize((size_t)chains);
  for (int32_t c = 0; c < chains; ++c) heap[c] = {1e-6 * inv_speed[c & 7], c};
  const auto later = [](const Free& a, const Free& b) { return a > b; };
  std::make_heap(heap.begin(), heap.end(), later);
  tail.assign((size_t)chains, -1);
  const int64_t per_block = (n_units + 8 * (int64_t)chains - 1) / (8 * (int64_t)chains);
  for (int64_t u0 = 0; u0 < n_units; u0 += per_block) {
    const int64_t u1 = std::min(n_units, u0 + per_block);
    std::pop_heap(heap.begin(), heap.end(), later);
    Free& f = heap.back();
    const int32_t c = f.second;
    int64_t cost = 0;
    for (int64_t u = u0; u < u1; ++u) {
      const DkItem& it = items[(size_t)(u / cfg.n_kv_heads)];
      cost += (int64_t)(it.kv_hi - it.kv_lo) + cfg.stream_item_cost;
      if (tail[c] < 0) head[c] = (int32_t)u; else next[tail[c]] = (int32_t)u;
      tail[c] = (int32_t)u;
    }
    f.first += (double)cost * inv_speed[c & 7];
    std::push_heap(heap.begin(), heap.end(), later);
  }
}
// The tile kernel runs `slots` workgroups per KV head, each walking a chain of items.  The items arrive in launch
// order (grouped by (entry, key chunk), costliest group first) and each joins the chain that is free first, which is
// what a hardware dispatcher would do with one workgroup per item -- so the row tiles of a group still run at the
// same time and share their K/V tiles through L2 -- but without a workgroup start per item.
void chain_tile_items(const std::vector<DkItem>& items, int32_t kv_tile, int32_t slots, int32_t item_cost,
                      std::vector<std::pair<double, int32_t>>& heap, std::vector<int32_t>& tail,
                      std::vector<int32_t>* links, int32_t* n_chains) {
  const int32_t n = (int32_t)items.size();
  const int32_t chains = std::min(n, std::max(slots, 1));
  *n_chains = chains;
  links->assign((size_t)chains + (size_t)n, -1);
  if (n == 0) return;
  int32_t* head = links->data();
  int32_t* next = links->data() + chains;
  typedef std::pair<double, int32_t> Free;  // (time at which the chain is free, chain)
  heap.resize((size_t)chains);
  for (int32_t c = 0; c < chains; ++c) heap[c] = {0.0, c};
  const auto later = [](const Free& a, const Free& b) { return a > b; };
  std::make_heap(heap.begin(), heap.end(), later);
  tail.assign((size_t)chains, -1);
  for (int32_t i = 0; i < n; ++i) {
    std::pop_heap(heap.begin(), heap.end(), later);
    Free& f = heap.back();
    const int32_t c = f.second;
    if (tail[c] < 0) head[c] = i; else next[tail[c]] = i;
    tail[c] = i;
    f.first += (double)((items[i].kv_hi - items[i].kv_lo + kv_tile - 1) / kv_tile + item_cost);
    std::push_heap(heap.begin(), heap.end(), later);
  }
}
}  // namespace

int32_t build_plan(Pool& pool, const PlanConfig& cfg, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                   bool staged, AttendPlan* p) {
  int32_t rc = pool.check_batch(n_seqs, slots, cu_delta);
  if (rc != OK) return rc;
  p->entries.clear();
  p->segs.clear();
  p->tile_items.clear();
  p->stream_items.clear();
  p->merges.clear();
  p->stream_links.clear();
  p->stream_chains = 0;
  p->tile_links.clear();
  p->tile_chains = 0;
  p->part_rows = 0;
  p->total_tokens = n_seqs ? cu_delta[n_seqs] : 0;
  const int32_t group = cfg.n_q_heads / cfg.n_kv_heads;
  std::vector<Extent>& ext = p->ext;
  std::vector<RowTile>& tile_tiles = p->tile_tiles;
  std::vector<RowTile>& stream_tiles = p->stream_tiles;
  tile_tiles.clear();
  stream_tiles.clear();
  for (int32_t b = 0; b < n_seqs; ++b) {
    const int32_t delta = cu_delta[b + 1] - cu_delta[b];
    int64_t len = 0;
    rc = pool.extents_locked(slots[b], &ext, &len);
    if (rc != OK) return rc;
    if (!staged && delta > len) return ERR_INVALID;
    if (len + delta > INT32_MAX / 2) return ERR_UNSUPPORTED;
    DkEntry e{};
    e.seg_begin = (int32_t)p->segs.size();
    e.n = (int32_t)(staged ? len : len - delta);
    e.delta = delta;
    e.tok0 = cu_delta[b];
    if (delta > 0) {
      for (const Extent& x : ext) p->segs.push_back({x.cell, (int32_t)x.pos, (int32_t)x.len, 0, 0});
      if (staged) p->segs.push_back({(int64_t)cu_delta[b], e.n, delta, 1, 0});
    }
    e.seg_end = (int32_t)p->segs.size();
    p->entries.push_back(e);
    if (delta == 0 || !cfg.use_mfma) continue;
    const int32_t rows = group * delta;
    const int32_t ei = (int32_t)p->entries.size() - 1;
    if (rows <= cfg.stream_rows) {
      stream_tiles.push_back({ei, 0, rows, e.n + delta});
    } else {
      for (int32_t r0 = 0; r0 < rows; r0 += cfg.tile_rows) {
        const int32_t nr = std::min(cfg.tile_rows, rows - r0);
        const int32_t last_tok = (r0 + nr - 1) / group;
        tile_tiles.push_back({ei, r0, nr, e.n + last_tok + 1});
      }
    }
  }
  cut_items(tile_tiles, cfg.kv_tile, cfg.tile_target, cfg.tile_min_chunk, true, cfg.tile_wave_slots, cfg.tile_item_cost, p->keyed, p->cost,
            &p->tile_items, &p->merges, &p->part_rows);
  cut_items(stream_tiles, cfg.kv_tile, cfg.stream_target, cfg.stream_min_chunk, false, 0, 0, p->keyed, p->cost,
            &p->stream_items, &p->merges, &p->part_rows);
  chain_tile_items(p->tile_items, cfg.kv_tile, cfg.tile_wave_slots, cfg.tile_item_cost, p->heap, p->tail,
                   &p->tile_links, &p->tile_chains);
  chain_units(p->stream_items, cfg, p->heap, p->tail, &p->stream_links, &p->stream_chains);

  size_t off = 0;
  p->off_entries = off;
  off = align_up(off + p->entries.size() * sizeof(DkEntry), 256);
  p->off_segs = off;
  off = align_up(off + p->segs.size() * sizeof(DkSeg), 256);
  p->off_tile = off;
  off = align_up(off + p->tile_items.size() * sizeof(DkItem), 256);
  p->off_tile_links = off;
  off = align_up(off + p->tile_links.size() * sizeof(int32_t), 256);
  p->off_stream = off;
  off = align_up(off + p->stream_items.size() * sizeof(DkItem), 256);
  p->off_links = off;
  off = align_up(off + p->stream_links.size() * sizeof(int32_t), 256);
  p->off_merges = off;
  off = align_up(off + p->merges.size() * sizeof(DkMerge), 256);
  p->blob_bytes = off;
  p->off_parts = off;
  off += (size_t)p->part_rows * cfg.n_kv_heads * (cfg.head_dim + 2) * sizeof(float);
  p->total_bytes = align_up(off, 256) + 256;
  return OK;
}

}  // namespace dk
