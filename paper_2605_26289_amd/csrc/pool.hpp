// Host-side metadata of the sequence pool: slot table, free lists, cell allocator and
// the chains that realise constant-time prefix aliasing.  No device code, no HIP calls.
//
// Paper Sec. 3.1 (fixed pool of named sequences in one unified cache, transient and
// session regions, mutex-guarded free list, blocking acquire with timeout) and
// Sec. 3.3 / Alg. 1 (SeqAlias is metadata only and constant time in the prefix length).
#pragma once

#include <chrono>
#include <condition_variable>
#include <cstdint>
#include <deque>
#include <map>
#include <memory>
#include <mutex>
#include <set>
#include <vector>

namespace dk {

// A run of physically consecutive cells that holds logical positions [pos, pos + len).
struct Extent {
  int64_t cell;
  int64_t pos;
  int64_t len;
};

// Hands out granules (fixed-size runs of consecutive cells).  Keeps the free granules as
// maximal runs so that a growing sequence can usually extend in place, and places new
// sequences away from the growth frontier of existing ones so their extents stay long.
class GranuleAllocator {
 public:
  GranuleAllocator(int64_t n_granules);
  int64_t free_count() const { return free_; }
  int64_t total() const { return total_; }
  // Takes granule g if it is free.
  bool take(int64_t g);
  // Takes a granule that starts a fresh extent; -1 if none is free.
  int64_t take_fresh();
  void give_back(int64_t g);
  void mark_tail(int64_t g) { tails_.insert(g); }
  void unmark_tail(int64_t g) { tails_.erase(g); }

 private:
  void remove_from_run(std::map<int64_t, int64_t>::iterator it, int64_t g);
  std::map<int64_t, int64_t> runs_;  // start -> length, maximal and disjoint
  std::set<int64_t> tails_;          // last granule of each live node (places where a sequence may grow)
  int64_t free_;
  int64_t total_;
};

// A node owns the cells of one privately written stretch of a sequence.  Its logical
// range is [base, base + len); everything below `base` is read through `parent`,
// truncated at `base`.  A sequence that aliases another one gets a fresh, empty node
// whose parent is the donor's node: nothing is copied and nothing per cell is touched.
struct Node {
  Node(GranuleAllocator* a, int64_t granule_cells, std::shared_ptr<Node> p, int64_t b)
      : alloc(a), gr(granule_cells), parent(std::move(p)), base(b) {}
  ~Node();
  Node(const Node&) = delete;
  Node& operator=(const Node&) = delete;

  int64_t end() const { return base + len; }
  int64_t granules_needed(int64_t extra) const;  // granules an append of `extra` tokens must add
  void grow(int64_t extra);                      // caller has checked the allocator holds enough
  void shrink_to(int64_t new_len);               // own length, frees whole unused granules
  int64_t cell_of(int64_t own_offset) const {
    if (own_offset < borrow_cap) return borrow_cell + own_offset;
    const int64_t o = own_offset - borrow_cap;
    return granules[o / gr] * gr + o % gr;
  }

  GranuleAllocator* alloc;
  int64_t gr;
  std::shared_ptr<Node> parent;
  int64_t base;
  int64_t len = 0;
  int64_t frozen = 0;  // absolute position; own cells below it are visible to a child and never rewritten
  std::vector<int64_t> granules;
  // A node that continues exactly where its parent ends, after the parent's own sequence has gone, writes its
  // first cells into the unused rest of the parent's last granule: a turn that extends a cached conversation
  // then stays physically contiguous with it and wastes no granule.  The room is [borrow_cell, + borrow_cap);
  // the granule itself stays the parent's (the child keeps the parent alive).
  int64_t borrow_cell = -1;
  int64_t borrow_cap = 0;
  bool tail_lent = false;  // the unused rest of this node's last granule is some child's borrow room
  int32_t owners = 0;      // sequences whose newest node this is: they may still append to it
};

struct Slot {
  bool in_use = false;
  std::shared_ptr<Node> head;
  int64_t len = 0;
};

enum Status : int32_t {
  OK = 0, ERR_INVALID = -1, ERR_TIMEOUT = -2, ERR_NO_CELLS = -3, ERR_NO_SLOT = -4,
  ERR_DUP_SLOT = -5, ERR_UNSUPPORTED = -6, ERR_WORKSPACE = -7, ERR_HIP = -8
};

class Pool {
 public:
  Pool(int32_t n_slots, int32_t n_session, int64_t arena_cells, int32_t granule_cells);

  int32_t acquire(int32_t region, int64_t timeout_ms, int32_t* slot_out);
  int32_t release(int32_t slot);
  int32_t length(int32_t slot, int64_t* out);
  int32_t alias(int32_t donor, int32_t dst, int64_t p0, int64_t p1);
  int32_t trim(int32_t slot, int64_t new_len);
  // Several trims at once, all or nothing (slots distinct).
  int32_t trim_batch(int32_t n, const int32_t* slots, const int64_t* new_len);
  int32_t cells(int32_t slot, int64_t* out, int64_t cap);
  int32_t stats(int64_t* held, int64_t* free_cells);
  // runs of consecutive cells the slot's logical view consists of, and nodes on its chain
  int32_t seq_stats(int32_t slot, int64_t* segments, int64_t* chain_nodes);

  // Batched append bookkeeping: checks every slot, reserves the cells, advances the lengths and
  // reports the destination cell of every appended token (dst[t] = -1 for tokens not appended) and,
  // if asked, every slot's length before the call.  All or nothing.
  int32_t append(int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta, const int32_t* n_accept,
                 std::vector<int64_t>* dst_cell, std::vector<int64_t>* old_len = nullptr);

  // Logical view of a slot as merged extents, positions ascending.
  int32_t extents(int32_t slot, std::vector<Extent>* out, int64_t* len_out);
  int32_t check_batch(int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta);

  int64_t granule_cells() const { return gr_; }
  int64_t arena_cells() const { return alloc_.total() * gr_; }
  std::mutex& mutex() { return mu_; }

  // unlocked variants for callers that hold mutex()
  int32_t extents_locked(int32_t slot, std::vector<Extent>* out, int64_t* len_out);

 private:
  bool valid(int32_t slot) const { return slot >= 0 && slot < (int32_t)slots_.size() && slots_[slot].in_use; }
  int32_t trim_locked(int32_t slot, int64_t new_len);
  void set_head(Slot& s, std::shared_ptr<Node> n);
  static void resolve(const std::shared_ptr<Node>& head, int64_t len, std::vector<Extent>* out);

  std::mutex mu_;
  std::condition_variable cv_;
  int64_t gr_;
  GranuleAllocator alloc_;
  std::vector<Slot> slots_;
  std::deque<int32_t> free_[2];
  int32_t n_transient_;
};

}  // namespace dk
