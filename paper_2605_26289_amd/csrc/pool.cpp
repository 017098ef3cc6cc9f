// Host-side pool metadata (see pool.hpp).  Paper Sec. 3.1 and Sec. 3.3 / Alg. 1, Alg. 2.
#include "pool.hpp"

#include <algorithm>

namespace dk {

// ---------------------------------------------------------------- GranuleAllocator
GranuleAllocator::GranuleAllocator(int64_t n) : free_(n), total_(n) {
  if (n > 0) runs_[0] = n;
}

void GranuleAllocator::remove_from_run(std::map<int64_t, int64_t>::iterator it, int64_t g) {
  const int64_t s = it->first, l = it->second;
  runs_.erase(it);
  if (g > s) runs_[s] = g - s;
  if (g + 1 < s + l) runs_[g + 1] = s + l - (g + 1);
  --free_;
}

bool GranuleAllocator::take(int64_t g) {
  if (g < 0 || g >= total_) return false;
  auto it = runs_.upper_bound(g);
  if (it == runs_.begin()) return false;
  --it;
  if (g >= it->first + it->second) return false;
  remove_from_run(it, g);
  return true;
}

int64_t GranuleAllocator::take_fresh() {
  if (runs_.empty()) return -1;
  auto best = runs_.begin();
  for (auto it = runs_.begin(); it != runs_.end(); ++it)
    if (it->second > best->second) best = it;
  int64_t g = best->first;
  // If the run directly follows a cell range some sequence may still grow into, start in
  // the middle of the run so that both can keep extending contiguously.
  if (g > 0 && tails_.count(g - 1) && best->second >= 2) g += best->second / 2;
  remove_from_run(best, g);
  return g;
}

void GranuleAllocator::give_back(int64_t g) {
  int64_t s = g, l = 1;
  auto next = runs_.find(g + 1);
  if (next != runs_.end()) {
    l += next->second;
    runs_.erase(next);
  }
  auto it = runs_.lower_bound(g);
  if (it != runs_.begin()) {
    --it;
    if (it->first + it->second == g) {
      s = it->first;
      l += it->second;
      runs_.erase(it);
    }
  }
  runs_[s] = l;
  ++free_;
}

// ---------------------------------------------------------------- Node
Node::~Node() {
  if (borrow_cap > 0 && parent) parent->tail_lent = false;  // nothing refers to the borrowed cells any more
  if (!granules.empty()) alloc->unmark_tail(granules.back());
  for (int64_t g : granules) alloc->give_back(g);
}

int64_t Node::granules_needed(int64_t extra) const {
  const int64_t want = (std::max<int64_t>(0, len + extra - borrow_cap) + gr - 1) / gr;
  return std::max<int64_t>(0, want - (int64_t)granules.size());
}

void Node::grow(int64_t extra) {
  const int64_t add = granules_needed(extra);
  for (int64_t i = 0; i < add; ++i) {
    int64_t g = -1;
    if (!granules.empty()) {
      alloc->unmark_tail(granules.back());
      if (alloc->take(granules.back() + 1)) g = granules.back() + 1;
    } else if (borrow_cap > 0) {  // continue right behind the granule the first cells were borrowed from
      const int64_t after = (borrow_cell + borrow_cap) / gr;
      if (alloc->take(after)) g = after;
    }
    if (g < 0) g = alloc->take_fresh();
    granules.push_back(g);
    alloc->mark_tail(g);
  }
  len += extra;
}

void Node::shrink_to(int64_t new_len) {
  const int64_t keep = (std::max<int64_t>(0, new_len - borrow_cap) + gr - 1) / gr;
  if ((int64_t)granules.size() > keep) {
    alloc->unmark_tail(granules.back());
    while ((int64_t)granules.size() > keep) {
      alloc->give_back(granules.back());
      granules.pop_back();
    }
    if (!granules.empty()) alloc->mark_tail(granules.back());
  }
  len = new_len;
}

// ---------------------------------------------------------------- Pool
Pool::Pool(int32_t n_slots, int32_t n_session, int64_t arena_cells, int32_t granule_cells)
    : gr_(granule_cells), alloc_(arena_cells / granule_cells), slots_(n_slots), n_transient_(n_slots - n_session) {
  for (int32_t s = 0; s < n_transient_; ++s) free_[0].push_back(s);
  for (int32_t s = n_transient_; s < n_slots; ++s) free_[1].push_back(s);
}

void Pool::set_head(Slot& s, std::shared_ptr<Node> n) {
  if (s.head) --s.head->owners;
  s.head = std::move(n);
  if (s.head) ++s.head->owners;
}

int32_t Pool::acquire(int32_t region, int64_t timeout_ms, int32_t* slot_out) {
  if ((region != 0 && region != 1) || !slot_out) return ERR_INVALID;
  std::unique_lock<std::mutex> lk(mu_);
  auto ready = [&] { return !free_[region].empty(); };
  if (!ready()) {
    if (timeout_ms == 0) return ERR_TIMEOUT;
    if (timeout_ms < 0) {
      cv_.wait(lk, ready);
    } else if (!cv_.wait_for(lk, std::chrono::milliseconds(timeout_ms), ready)) {
      return ERR_TIMEOUT;
    }
  }
  const int32_t s = free_[region].front();
  free_[region].pop_front();
  slots_[s].in_use = true;
  set_head(slots_[s], nullptr);
  slots_[s].len = 0;
  *slot_out = s;
  return OK;
}

int32_t Pool::release(int32_t slot) {
  {
    std::lock_guard<std::mutex> lk(mu_);
    if (!valid(slot)) return ERR_NO_SLOT;
    set_head(slots_[slot], nullptr);  // cells live on while an alias chain still references the node
    slots_[slot].len = 0;
    slots_[slot].in_use = false;
    free_[slot >= n_transient_ ? 1 : 0].push_back(slot);
  }
  cv_.notify_all();
  return OK;
}

int32_t Pool::length(int32_t slot, int64_t* out) {
  std::lock_guard<std::mutex> lk(mu_);
  if (!valid(slot)) return ERR_NO_SLOT;
  if (!out) return ERR_INVALID;
  *out = slots_[slot].len;
  return OK;
}

int32_t Pool::alias(int32_t donor, int32_t dst, int64_t p0, int64_t p1) {
  std::lock_guard<std::mutex> lk(mu_);
  if (!valid(donor) || !valid(dst)) return ERR_NO_SLOT;
  if (p0 != 0) return ERR_UNSUPPORTED;
  if (donor == dst || p1 < 0 || p1 > slots_[donor].len || slots_[dst].len != 0) return ERR_INVALID;
  if (p1 == 0) return OK;
  // The node that holds position p1-1.  The walk is over alias generations, not over tokens.
  std::shared_ptr<Node> a = slots_[donor].head;
  while (a->base >= p1) a = a->parent;
  a->frozen = std::max(a->frozen, p1);
  std::shared_ptr<Node> fresh = std::make_shared<Node>(&alloc_, gr_, a, p1);
  // Continuing exactly at the end of a node nobody appends to any more: take over the unused rest of the
  // granule its last cell lies in (its own last granule, or what is left of the room it borrowed itself).
  if (p1 == a->end() && a->len > 0 && a->owners == 0 && !a->tail_lent) {
    int64_t room_cell = -1, room = 0;
    if (a->granules.empty()) {
      room_cell = a->borrow_cell + a->len;
      room = a->borrow_cap - a->len;
    } else if ((a->len - a->borrow_cap) % gr_ != 0) {
      const int64_t used = (a->len - a->borrow_cap) % gr_;
      room_cell = a->granules.back() * gr_ + used;
      room = gr_ - used;
    }
    if (room > 0) {
      fresh->borrow_cell = room_cell;
      fresh->borrow_cap = room;
      a->tail_lent = true;
    }
  }
  set_head(slots_[dst], std::move(fresh));
  slots_[dst].len = p1;
  return OK;
}

int32_t Pool::trim(int32_t slot, int64_t new_len) {
  std::lock_guard<std::mutex> lk(mu_);
  return trim_locked(slot, new_len);
}

int32_t Pool::trim_batch(int32_t n, const int32_t* slots, const int64_t* new_len) {
  if (n < 0 || (n > 0 && (!slots || !new_len))) return ERR_INVALID;
  std::lock_guard<std::mutex> lk(mu_);
  std::vector<char> seen(slots_.size(), 0);
  for (int32_t b = 0; b < n; ++b) {
    if (!valid(slots[b])) return ERR_NO_SLOT;
    if (seen[slots[b]]) return ERR_DUP_SLOT;
    seen[slots[b]] = 1;
    if (new_len[b] < 0 || new_len[b] > slots_[slots[b]].len) return ERR_INVALID;
  }
  for (int32_t b = 0; b < n; ++b) (void)trim_locked(slots[b], new_len[b]);
  return OK;
}

int32_t Pool::trim_locked(int32_t slot, int64_t new_len) {
  if (!valid(slot)) return ERR_NO_SLOT;
  Slot& s = slots_[slot];
  if (new_len < 0 || new_len > s.len) return ERR_INVALID;
  if (new_len == s.len) return OK;
  if (new_len == 0) {
    set_head(s, nullptr);
    s.len = 0;
    return OK;
  }
  std::shared_ptr<Node> h = s.head;
  if (h.use_count() == 2) h->frozen = 0;  // only `h` and the slot hold it: no child can see its cells
  if (new_len >= h->base && new_len >= h->frozen) {
    h->shrink_to(new_len - h->base);
  } else {
    // Cells at and beyond new_len may still be visible through an alias: leave them alone and
    // continue in a fresh node, so later appends cannot overwrite them.
    std::shared_ptr<Node> a = h;
    while (a->base >= new_len) a = a->parent;
    a->frozen = std::max(a->frozen, new_len);
    set_head(s, std::make_shared<Node>(&alloc_, gr_, a, new_len));
  }
  s.len = new_len;
  return OK;
}

void Pool::resolve(const std::shared_ptr<Node>& head, int64_t len, std::vector<Extent>* out) {
  out->clear();
  std::vector<std::pair<const Node*, int64_t>> parts;  // node, exclusive upper position it contributes
  int64_t limit = len;
  for (const Node* n = head.get(); n && limit > 0; n = n->parent.get()) {
    const int64_t hi = std::min(limit, n->end());
    if (hi > n->base) parts.emplace_back(n, hi);
    limit = std::min(limit, n->base);
  }
  for (auto it = parts.rbegin(); it != parts.rend(); ++it) {
    const Node* n = it->first;
    int64_t own = it->second - n->base;  // tokens of this node that are visible
    const auto add = [&](int64_t cell, int64_t pos, int64_t take) {
      if (!out->empty() && out->back().cell + out->back().len == cell && out->back().pos + out->back().len == pos) {
        out->back().len += take;
      } else {
        out->push_back({cell, pos, take});
      }
    };
    if (n->borrow_cap > 0 && own > 0) {  // first cells in the rest of the parent's last granule
      const int64_t take = std::min(own, n->borrow_cap);
      add(n->borrow_cell, n->base, take);
      own -= take;
    }
    for (size_t gi = 0; own > 0; ++gi) {
      const int64_t take = std::min(own, n->gr);
      add(n->granules[gi] * n->gr, n->base + n->borrow_cap + (int64_t)gi * n->gr, take);
      own -= take;
    }
  }
}

int32_t Pool::extents_locked(int32_t slot, std::vector<Extent>* out, int64_t* len_out) {
  if (!valid(slot)) return ERR_NO_SLOT;
  resolve(slots_[slot].head, slots_[slot].len, out);
  if (len_out) *len_out = slots_[slot].len;
  return OK;
}

int32_t Pool::extents(int32_t slot, std::vector<Extent>* out, int64_t* len_out) {
  std::lock_guard<std::mutex> lk(mu_);
  return extents_locked(slot, out, len_out);
}

int32_t Pool::cells(int32_t slot, int64_t* out, int64_t cap) {
  std::vector<Extent> ext;
  int64_t len = 0;
  int32_t rc = extents(slot, &ext, &len);
  if (rc != OK) return rc;
  if (!out && cap > 0) return ERR_INVALID;
  for (const Extent& e : ext)
    for (int64_t i = 0; i < e.len && e.pos + i < cap; ++i) out[e.pos + i] = e.cell + i;
  return OK;
}

int32_t Pool::stats(int64_t* held, int64_t* free_cells) {
  std::lock_guard<std::mutex> lk(mu_);
  if (held) *held = (alloc_.total() - alloc_.free_count()) * gr_;
  if (free_cells) *free_cells = alloc_.free_count() * gr_;
  return OK;
}

int32_t Pool::seq_stats(int32_t slot, int64_t* segments, int64_t* chain_nodes) {
  std::lock_guard<std::mutex> lk(mu_);
  if (!valid(slot)) return ERR_NO_SLOT;
  std::vector<Extent> ext;
  resolve(slots_[slot].head, slots_[slot].len, &ext);
  if (segments) *segments = (int64_t)ext.size();
  int64_t depth = 0;
  for (const Node* n = slots_[slot].head.get(); n; n = n->parent.get()) ++depth;
  if (chain_nodes) *chain_nodes = depth;
  return OK;
}

int32_t Pool::check_batch(int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta) {
  if (n_seqs < 0 || (n_seqs > 0 && (!slots || !cu_delta))) return ERR_INVALID;
  if (n_seqs == 0) return OK;
  if (cu_delta[0] != 0) return ERR_INVALID;
  std::vector<char> seen(slots_.size(), 0);
  for (int32_t b = 0; b < n_seqs; ++b) {
    if (!valid(slots[b])) return ERR_NO_SLOT;
    if (seen[slots[b]]) return ERR_DUP_SLOT;
    seen[slots[b]] = 1;
    if (cu_delta[b + 1] < cu_delta[b]) return ERR_INVALID;
  }
  return OK;
}

int32_t Pool::append(int32_t n_seqs, const int32_t* slots, const int32_t* cu_delta, const int32_t* n_accept,
                     std::vector<int64_t>* dst_cell, std::vector<int64_t>* old_len) {
  std::lock_guard<std::mutex> lk(mu_);
  int32_t rc = check_batch(n_seqs, slots, cu_delta);
  if (rc != OK) return rc;
  const int64_t total = n_seqs ? cu_delta[n_seqs] : 0;
  int64_t need = 0;
  for (int32_t b = 0; b < n_seqs; ++b) {
    const int64_t delta = cu_delta[b + 1] - cu_delta[b];
    const int64_t cnt = n_accept ? n_accept[b] : delta;
    if (cnt < 0 || cnt > delta) return ERR_INVALID;
    const Slot& s = slots_[slots[b]];
    need += s.head ? s.head->granules_needed(cnt) : (cnt + gr_ - 1) / gr_;
  }
  if (need > alloc_.free_count()) return ERR_NO_CELLS;
  dst_cell->assign(total, -1);
  if (old_len) {
    old_len->resize((size_t)n_seqs);
    for (int32_t b = 0; b < n_seqs; ++b) (*old_len)[b] = slots_[slots[b]].len;
  }
  for (int32_t b = 0; b < n_seqs; ++b) {
    const int64_t delta = cu_delta[b + 1] - cu_delta[b];
    const int64_t cnt = n_accept ? n_accept[b] : delta;
    if (cnt == 0) continue;
    Slot& s = slots_[slots[b]];
    if (!s.head) set_head(s, std::make_shared<Node>(&alloc_, gr_, nullptr, 0));
    Node& h = *s.head;
    const int64_t old = h.len;
    h.grow(cnt);
    for (int64_t j = 0; j < cnt; ++j) (*dst_cell)[cu_delta[b] + j] = h.cell_of(old + j);
    s.len += cnt;
  }
  return OK;
}

}  // namespace dk
