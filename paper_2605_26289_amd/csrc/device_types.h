// Plain structs shared by the host-side planner and the kernels (device memory layout of a call's
// descriptors).  Positions are logical token positions inside one sequence.
#pragma once
#include <stdint.h>

// A run of consecutive K/V rows holding logical positions [pos, pos + len).
// src 0: arena cells  (row r of KV head g at ((g * arena_cells) + start + r) * D)
// src 1: staged new tokens (row r of KV head g at ((start + r) * n_kv_heads + g) * D)
struct DkSeg {
  int64_t start;
  int32_t pos;
  int32_t len;
  int32_t src;
  int32_t pad;
};

// One batch entry: a slot with n cached tokens and delta new ones (paper Sec. 2.2: n_t, Delta_t).
struct DkEntry {
  int32_t seg_begin, seg_end;  // its segments, positions ascending, covering [0, n + delta)
  int32_t n;
  int32_t delta;
  int32_t tok0;  // first packed token row of the entry (cu_delta[b])
  int32_t pad[3];
};

// One workgroup's job: packed query rows [row0, row0 + nrows) of an entry (row r = token r / G,
// head r % G inside the KV group) against keys at positions [kv_lo, kv_hi).
struct DkItem {
  int32_t entry;
  int32_t row0;
  int32_t nrows;
  int32_t kv_lo, kv_hi;
  int32_t part_row0;  // >= 0: write fp32 partial rows here; < 0: write the final output
  int32_t pad[2];
};

// Rows whose key range was split over several items and must be merged.
struct DkMerge {
  int32_t entry;
  int32_t row0;
  int32_t nrows;
  int32_t part_row0;  // split s lives at part_row0 + s * nrows
  int32_t nsplit;
  int32_t pad[3];
};
