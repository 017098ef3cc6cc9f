// Launchers implemented in the .hip translation units.  All are asynchronous on `stream`.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_types.h"

namespace dk {

struct ArenaView {
  const void* k_arena;
  const void* v_arena;
  int64_t arena_cells;
  int32_t n_q_heads, n_kv_heads, head_dim;
  int32_t dtype;  // 0 f32, 1 bf16
};

// dst[cell_of[t]] <- src[t] (append) or dst[t] <- src[cell_of[t]] (gather) for K and V; cell < 0 skips.
hipError_t launch_kv_scatter(const ArenaView& a, void* k_arena, void* v_arena, const int32_t* cell_of_dev,
                             int64_t tok_base, int32_t n_tok, const void* k_new, const void* v_new,
                             hipStream_t stream);
hipError_t launch_kv_gather(const ArenaView& a, const int32_t* cell_of_dev, int64_t tok_base, int32_t n_tok,
                            void* k_out, void* v_out, hipStream_t stream);

// Appends of at most this many tokens carry their destination cells in the kernel arguments (host table,
// nothing is uploaded first).
constexpr int32_t KV_INLINE_MAX_TOKENS = 896;
hipError_t launch_kv_scatter_inline(const ArenaView& a, void* k_arena, void* v_arena, const int64_t* cell_of_host,
                                    int32_t n_tok, const void* k_new, const void* v_new, hipStream_t stream);

// Descriptors of at most this many bytes are passed to the kernels inside their arguments instead of being
// uploaded first: a short turn then costs no host-to-device copy (and no staging buffer).
constexpr int32_t INLINE_BLOB_BYTES = 3072;
struct InlineBlob {
  uint32_t w[INLINE_BLOB_BYTES / 4];
};

struct AttendArgs {
  // Host copy of the call's descriptor blob if it travels in the kernel arguments (then `entries`, `segs` and
  // every descriptor pointer handed to a launcher are byte offsets into the blob), else nullptr (then they are
  // device pointers).
  const InlineBlob* inline_blob = nullptr;
  ArenaView arena;
  const DkEntry* entries;
  int32_t n_entries;
  const DkSeg* segs;
  const void* q;
  const void* k_new;
  const void* v_new;
  void* out;
  float* lse;
  float* parts;     // split partials: [partial row][KV head][head_dim] fp32 sums
  float* parts_ml;  // [partial row][KV head][2]: running maximum (log2 units), weight sum
  float scale;
  int32_t total_tokens;
  // Small append-and-attend calls: destination arena cell of every new token (a section of the inline descriptor
  // blob); the MFMA kernel launched with `scatter` set also writes the rows of k_new / v_new into those cells.
  const int32_t* cells = nullptr;
  bool scatter = false;
};

// Scalar reference kernel: one wavefront per (token, query head).  Any supported shape and dtype.
hipError_t launch_attend_ref(const AttendArgs& a, hipStream_t stream);
// bf16 MFMA kernels (head_dim 128).
// One workgroup per (chain, KV head): chain c is items links[c], links[n_chains + that item], ... until a link
// is negative; every chain holds at least one item.
hipError_t launch_attend_tile(const AttendArgs& a, const DkItem* items, const int32_t* links, int32_t n_chains,
                              hipStream_t stream);
// Unit u = item u / n_kv_heads for KV head u % n_kv_heads; n_chains workgroups.
// queue == nullptr: workgroup w walks the chain links[w], links[n_chains + that unit], ... until a link is negative.
// queue != nullptr (DEVICE int32, holding n_chains when the kernel starts; not with an inline blob): workgroup w
// starts with unit w and draws every further unit from the counter (atomic add) until it reaches n_units; the
// units are expected longest first.  `links` is not read then.
// max_rows: the largest DkItem::nrows among the items (at most 64).
hipError_t launch_attend_stream(const AttendArgs& a, const DkItem* items, const int32_t* links, int32_t n_chains,
                                int32_t max_rows, int32_t* queue, int32_t n_units, hipStream_t stream);
// max_rows: the largest DkMerge::nrows among them (sizes the grid).
hipError_t launch_attend_merge(const AttendArgs& a, const DkMerge* merges, int32_t n_merges, int32_t max_rows,
                               hipStream_t stream);

// Greedy verification (argmax per logits row, accepted-draft count and next token per slot).
int64_t verify_workspace_bytes(int32_t total_rows, int64_t vocab, int32_t dtype);
hipError_t launch_verify_greedy(int32_t n_seqs, int32_t total_rows, const int32_t* cu_delta_dev, const void* logits,
                                int32_t dtype, int64_t vocab, int64_t row_stride, const int32_t* batch_tokens,
                                int32_t* argmax_out, int32_t* n_keep_out, int32_t* next_token_out, void* workspace,
                                hipStream_t stream);

}  // namespace dk
