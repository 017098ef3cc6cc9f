// Host-side planning of one dk_delta_attend call: resolves every slot's logical view into
// segments, cuts the work into workgroup-sized items (with the key range split when there are
// too few query rows to fill the chip) and lays the descriptors out for upload.
#pragma once
#include <cstddef>
#include <cstdint>
#include <utility>
#include <vector>

#include "device_types.h"
#include "pool.hpp"

namespace dk {

struct PlanConfig {
  int32_t n_q_heads, n_kv_heads, head_dim;
  bool use_mfma;          // bf16, D == 128, power-of-two group: the tiled kernels apply
  int32_t tile_rows;      // packed query rows per workgroup of the tile kernel
  int32_t stream_rows;    // max packed rows handled by the streaming (small-Delta) kernel
  int32_t kv_tile;        // keys per inner step; split boundaries are multiples of it
  int32_t tile_wave_slots;  // tile-kernel workgroups of one KV head that run at a time (its share of the CUs)
  int32_t stream_target;  // same, streaming kernel
  int32_t tile_min_chunk, stream_min_chunk;  // smallest key range worth its own item
  int32_t tile_item_cost;    // fixed cost of a tile item inside a chain, in key tiles (store phase, pipeline ramp)
  int32_t stream_chains;     // workgroups of the streaming kernel: one per compute unit
  int32_t stream_item_cost;  // fixed cost of an item in the chain balance, in keys
  float xcd_speed[8];        // relative K/V streaming rate of the XCD that workgroup w lands on (w % 8)
  int32_t stream_queue;      // 1: streaming units are drawn from a queue at run time when the blob is uploaded
  int32_t inline_blob_bytes; // a descriptor blob up to this size travels in the kernel arguments
};

// One packed row tile of an entry before its key range is cut: rows [row0, row0 + nrows) see keys [0, kv_hi).
struct PlanRowTile {
  int32_t entry, row0, nrows, kv_hi;
};
// A piece of a row tile's key range on its way to becoming a work item of the tile kernel.
struct PlanPiece {
  int32_t tile;    // index of its row tile
  int32_t lo, hi;  // key positions
  int32_t next;    // next piece of the same chain, -1 at the end
};

// A plan object may be reused from call to call: build_plan() clears it but keeps the capacity of its
// vectors, so that planning a batch like the previous one allocates nothing.
struct AttendPlan {
  // working storage of build_plan
  std::vector<Extent> ext;
  std::vector<PlanRowTile> tile_tiles, stream_tiles;
  std::vector<std::pair<double, int32_t>> heap;
  std::vector<int32_t> tail;
  std::vector<PlanPiece> pieces;
  std::vector<int32_t> order, chain_head, chain_tail, tile_pieces, tile_part0;
  std::vector<int64_t> chain_load;

  std::vector<DkEntry> entries;
  std::vector<DkSeg> segs;
  std::vector<DkItem> tile_items, stream_items;
  std::vector<DkMerge> merges;
  int64_t total_tokens = 0;
  int64_t part_rows = 0;
  // Streaming kernel: unit u = item u / n_kv_heads for KV head u % n_kv_heads.  Workgroup w walks the
  // chain stream_links[w], stream_links[n_chains + that unit], ... until a link is negative.
  std::vector<int32_t> stream_links;
  int32_t stream_chains = 0;
  // ... or, when stream_queued, starts with unit w and draws every further unit from a counter (off_queue, one
  // int32 that is uploaded holding stream_chains): the units are in longest-first order, no links are built.
  bool stream_queued = false;
  int64_t stream_units = 0;
  size_t off_queue = 0;
  // Tile kernel: tile_wave_slots workgroups per KV head, workgroup c of a head walks the items
  // tile_links[c], tile_links[tile_chains + that item], ...; the chains are the same for every KV head.
  std::vector<int32_t> tile_links;
  int32_t tile_chains = 0;
  size_t off_entries = 0, off_segs = 0, off_tile = 0, off_tile_links = 0, off_stream = 0, off_links = 0, off_merges = 0;
  size_t off_cells = 0;    // destination cell of every new token (int32), only when the plan was built with_cells
  size_t blob_bytes = 0;   // descriptors
  size_t off_parts = 0;    // fp32 partial rows, each (head_dim + 2) floats per KV head
  size_t total_bytes = 0;  // whole workspace
};

// Caller holds pool.mutex().  with_cells reserves, inside the descriptor blob, one int32 per new token for the
// cell it is to be written to (the call that appends and attends in one launch fills them in).
int32_t build_plan(Pool& pool, const PlanConfig& cfg, int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta,
                   bool staged, AttendPlan* plan, bool with_cells = false);

}  // namespace dk
