#include "plan.hpp"

#include <algorithm>
#include <functional>
#include <queue>

namespace dk {

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

namespace {
typedef PlanRowTile RowTile;

// Work items of the streaming kernel: each entry's visible key range [0, kv_hi) is cut into nearly equal chunks
// (multiples of kv_tile) so that there are about `target` items per KV head and none is shorter than min_chunk;
// longest first.  Entries whose range is cut get partial rows and a merge record.
void cut_stream_items(const std::vector<RowTile>& tiles, int32_t kv_tile, int32_t target, int32_t min_chunk,
                      std::vector<DkItem>* items, std::vector<DkMerge>* merges, int64_t* part_rows) {
  if (tiles.empty()) return;
  int64_t total = 0;
  for (const RowTile& t : tiles) total += t.kv_hi;
  int64_t chunk = std::max<int64_t>(min_chunk, (total + target - 1) / target);
  chunk = (chunk + kv_tile - 1) / kv_tile * kv_tile;
  const size_t first = items->size();
  for (const RowTile& t : tiles) {
    int32_t ns = (int32_t)((t.kv_hi + chunk - 1) / chunk);
    if (ns > 1 && t.kv_hi - (int64_t)(ns - 1) * chunk < chunk / 4) --ns;  // no sliver at the end
    const int64_t each = ((t.kv_hi + ns - 1) / ns + kv_tile - 1) / kv_tile * kv_tile;
    ns = (int32_t)((t.kv_hi + each - 1) / each);
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
      items->push_back(it);
    }
  }
  std::stable_sort(items->begin() + (std::ptrdiff_t)first, items->end(), [](const DkItem& a, const DkItem& b) {
    return (int64_t)(a.kv_hi - a.kv_lo) * a.nrows > (int64_t)(b.kv_hi - b.kv_lo) * b.nrows;
  });
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
// Work items of the tile kernel.  `slots` workgroups per KV head each walk a chain of items; an item is a row
// tile against a piece of its visible key range.  Costs are counted in key tiles: an item of n tiles takes
// n + item_cost (pipeline ramp, output store).
//   1. Pieces: with at least as many row tiles as workgroups nothing is cut; with fewer, every entry's key range
//      is cut into floor(slots / row tiles) equal chunks, the same boundaries for all row tiles of the entry --
//      the workgroups walking one chunk read the same K/V tiles at the same time and share them through L2.
//   2. Longest piece first, each to the chain that is free first (pieces of one (entry, chunk) group are equally
//      long, so they stay neighbours and start together).
//   3. Levelling: while the busiest chain is more than a few tiles above the idlest, the tail of one of its
//      pieces is cut off and handed to the idlest chain, sized so that the two end together.  This is what makes
//      the chains finish together whatever the mix of lengths; it costs one more item and the partial rows of
//      the row tile that was cut.
// Row tiles that end up in several pieces get partial rows and a merge record.  Items are emitted chain by chain.
void cut_tile_items(AttendPlan* p, const PlanConfig& cfg) {
  const std::vector<RowTile>& tiles = p->tile_tiles;
  p->tile_chains = 0;
  if (tiles.empty()) return;
  const int32_t kt = cfg.kv_tile;
  const int32_t slots = std::max(cfg.tile_wave_slots, 1);
  const int32_t fixed = std::max(cfg.tile_item_cost, 0);
  const int32_t min_piece = std::max<int32_t>(std::max<int32_t>(1, cfg.tile_min_chunk / kt), fixed);  // tiles
  const int32_t n_tiles = (int32_t)tiles.size();
  const auto len_of = [&](const PlanPiece& q) { return (q.hi - q.lo + kt - 1) / kt; };

  std::vector<PlanPiece>& pieces = p->pieces;
  pieces.clear();
  const int32_t k0 = n_tiles < slots ? slots / n_tiles : 1;
  for (int32_t b = 0; b < n_tiles;) {  // tiles of one entry are consecutive
    int32_t e = b, hi_max = 0;
    while (e < n_tiles && tiles[e].entry == tiles[b].entry) hi_max = std::max(hi_max, tiles[e++].kv_hi);
    const int32_t longest = (hi_max + kt - 1) / kt;
    const int32_t k = std::max(1, std::min(k0, longest / min_piece));
    const int32_t each = (longest + k - 1) / k * kt;  // keys per chunk
    for (int32_t t = b; t < e; ++t)
      for (int32_t lo = 0; lo < tiles[t].kv_hi;) {
        int32_t hi = std::min(tiles[t].kv_hi, lo + each);
        if (tiles[t].kv_hi - hi < each / 4) hi = tiles[t].kv_hi;  // no sliver at the end
        pieces.push_back({t, lo, hi, -1});
        lo = hi;
      }
    b = e;
  }

  std::vector<int32_t>& order = p->order;
  order.resize(pieces.size());
  for (size_t i = 0; i < order.size(); ++i) order[i] = (int32_t)i;
  std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) {
    const PlanPiece &a = pieces[x], &b = pieces[y];
    const int32_t la = len_of(a), lb = len_of(b);
    if (la != lb) return la > lb;
    if (tiles[a.tile].entry != tiles[b.tile].entry) return tiles[a.tile].entry < tiles[b.tile].entry;
    if (a.lo != b.lo) return a.lo < b.lo;
    return tiles[a.tile].row0 > tiles[b.tile].row0;
  });

  std::vector<int32_t>&head = p->chain_head, &tail = p->chain_tail;
  std::vector<int64_t>& load = p->chain_load;
  head.assign((size_t)slots, -1);
  tail.assign((size_t)slots, -1);
  load.assign((size_t)slots, 0);
  const auto append = [&](int32_t c, int32_t i) {
    if (tail[c] < 0) head[c] = i; else pieces[tail[c]].next = i;
    tail[c] = i;
    pieces[i].next = -1;
    load[c] += len_of(pieces[i]) + fixed;
  };
  {
    typedef std::pair<double, int32_t> Free;  // (time at which the chain is free, chain)
    std::vector<Free>& heap = p->heap;
    heap.resize((size_t)slots);
    for (int32_t c = 0; c < slots; ++c) heap[c] = {0.0, c};
    const auto later = [](const Free& a, const Free& b) { return a > b; };
    std::make_heap(heap.begin(), heap.end(), later);
    for (int32_t i : order) {
      std::pop_heap(heap.begin(), heap.end(), later);
      Free& f = heap.back();
      append(f.second, i);
      f.first = (double)load[f.second];
      std::push_heap(heap.begin(), heap.end(), later);
    }
  }

  for (int32_t round = 0; round < 4 * slots; ++round) {
    int32_t busy = 0, idle = 0;
    for (int32_t c = 1; c < slots; ++c) {
      if (load[c] > load[busy]) busy = c;
      if (load[c] < load[idle]) idle = c;
    }
    // tiles to hand over so that both chains end together (the new item pays its fixed cost on the idle chain)
    const int64_t give = (load[busy] - load[idle] - fixed) / 2;
    if (give < min_piece) break;
    int32_t donor = -1;  // the last piece of the busy chain that stays a piece after giving
    for (int32_t i = head[busy]; i >= 0; i = pieces[i].next)
      if (len_of(pieces[i]) >= give + min_piece) donor = i;
    if (donor < 0) break;
    const int32_t cut = pieces[donor].lo + (len_of(pieces[donor]) - (int32_t)give) * kt;
    pieces.push_back({pieces[donor].tile, cut, pieces[donor].hi, -1});
    pieces[donor].hi = cut;
    load[busy] -= give;
    append(idle, (int32_t)pieces.size() - 1);
  }

  // partial rows and merge records of the row tiles that were cut
  std::vector<int32_t>&count = p->tile_pieces, &part0 = p->tile_part0;
  count.assign((size_t)n_tiles, 0);
  part0.assign((size_t)n_tiles, -1);
  for (const PlanPiece& q : pieces) ++count[q.tile];
  for (int32_t t = 0; t < n_tiles; ++t)
    if (count[t] > 1) {
      part0[t] = (int32_t)p->part_rows;
      p->part_rows += (int64_t)count[t] * tiles[t].nrows;
      p->merges.push_back({tiles[t].entry, tiles[t].row0, tiles[t].nrows, part0[t], count[t], {0, 0, 0}});
      count[t] = 0;  // from here on: pieces of the tile emitted so far
    } else {
      count[t] = -1;
    }

  std::vector<int32_t>& links = p->tile_links;
  int32_t chains = 0;
  for (int32_t c = 0; c < slots; ++c) chains += head[c] >= 0;
  p->tile_chains = chains;
  links.assign((size_t)chains + pieces.size(), -1);
  int32_t cc = 0;
  for (int32_t c = 0; c < slots; ++c) {
    if (head[c] < 0) continue;
    links[cc++] = (int32_t)p->tile_items.size();
    for (int32_t i = head[c]; i >= 0; i = pieces[i].next) {
      const PlanPiece& q = pieces[i];
      const RowTile& t = tiles[q.tile];
      DkItem it{};
      it.entry = t.entry;
      it.row0 = t.row0;
      it.nrows = t.nrows;
      it.kv_lo = q.lo;
      it.kv_hi = q.hi;
      it.part_row0 = count[q.tile] < 0 ? -1 : part0[q.tile] + count[q.tile]++ * t.nrows;
      const int32_t idx = (int32_t)p->tile_items.size();
      p->tile_items.push_back(it);
      if (pieces[i].next >= 0) links[(size_t)chains + idx] = idx + 1;
    }
  }
}
}  // namespace

int32_t build_plan(Pool& pool, const PlanConfig& cfg, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                   bool staged, AttendPlan* p, bool with_cells) {
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
  cut_tile_items(p, cfg);
  cut_stream_items(stream_tiles, cfg.kv_tile, cfg.stream_target, cfg.stream_min_chunk, &p->stream_items, &p->merges,
                   &p->part_rows);
  // Streaming units: with at least four units per workgroup they form a queue that the workgroups draw from at
  // run time (measured: +3-5 % on 700 decode slots, +1.5 % on 2048, because the compute units do not stream equally
  // fast; with two units per workgroup, as in a 64-slot verification batch, the queue has nothing to balance with
  // and the chains planned here are 1-2 % faster).  Not for a launch whose descriptors travel in the kernel
  // arguments (the queue's counter needs device memory) -- decided on a lower bound of the blob's size, and abi.hip
  // uploads every blob of a queued plan.
  p->stream_units = (int64_t)p->stream_items.size() * cfg.n_kv_heads;
  const size_t floor_bytes = p->entries.size() * sizeof(DkEntry) + p->segs.size() * sizeof(DkSeg) +
                             (p->tile_items.size() + p->stream_items.size()) * sizeof(DkItem);
  const int64_t per_wg = cfg.stream_queue == 2 ? 1 : 4;  // (2: queue whenever some workgroup gets a second unit)
  p->stream_queued = cfg.stream_queue != 0 && p->stream_units >= per_wg * (int64_t)std::max(cfg.stream_chains, 1) &&
                     p->stream_units > std::max(cfg.stream_chains, 1) && floor_bytes > (size_t)cfg.inline_blob_bytes;
  if (p->stream_queued) {
    p->stream_links.clear();
    p->stream_chains = (int32_t)std::min<int64_t>(p->stream_units, std::max(cfg.stream_chains, 1));
  } else {
    chain_units(p->stream_items, cfg, p->heap, p->tail, &p->stream_links, &p->stream_chains);
  }

  size_t off = 0;
  p->off_entries = off;
  off = align_up(off + p->entries.size() * sizeof(DkEntry), 16);
  p->off_segs = off;
  off = align_up(off + p->segs.size() * sizeof(DkSeg), 16);
  p->off_tile = off;
  off = align_up(off + p->tile_items.size() * sizeof(DkItem), 16);
  p->off_tile_links = off;
  off = align_up(off + p->tile_links.size() * sizeof(int32_t), 16);
  p->off_stream = off;
  off = align_up(off + p->stream_items.size() * sizeof(DkItem), 16);
  p->off_links = off;
  off = align_up(off + p->stream_links.size() * sizeof(int32_t), 16);
  p->off_merges = off;
  off = align_up(off + p->merges.size() * sizeof(DkMerge), 16);
  p->off_queue = off;
  if (p->stream_queued) off += 16;
  p->off_cells = off;
  if (with_cells) off = align_up(off + (size_t)p->total_tokens * sizeof(int32_t), 16);
  p->blob_bytes = off;  // descriptors: small blobs travel in the kernel arguments, larger ones are uploaded
  off = align_up(off, 256);
  p->off_parts = off;
  off += (size_t)p->part_rows * cfg.n_kv_heads * (cfg.head_dim + 2) * sizeof(float);
  p->total_bytes = align_up(off, 256) + 256;
  return OK;
}

}  // namespace dk
