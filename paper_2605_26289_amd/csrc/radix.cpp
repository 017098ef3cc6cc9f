#include "radix.hpp"

#include <algorithm>

namespace dk {

Radix::Radix(Pool* pool, int64_t cell_budget, int32_t keep_last)
    : pool_(pool), budget_(cell_budget), keep_last_(keep_last) {}

Radix::~Radix() {
  // the donors go back to the pool; their cells are freed once no other sequence aliases them
  for (const auto& kv : donor_refs_) (void)pool_->release(kv.first);
}

Radix::Walk Radix::walk(const int32_t* tokens, int64_t n) {
  Node* node = &root_;
  int64_t pos = 0;
  while (pos < n) {
    auto it = node->children.find(tokens[pos]);
    if (it == node->children.end()) break;
    Node* child = it->second.get();
    const int64_t seg = (int64_t)child->tokens.size();
    int64_t j = 0;
    while (j < seg && pos + j < n && child->tokens[j] == tokens[pos + j]) ++j;
    child->touch = clock_;
    if (j < seg) return {child, j, pos + j};
    node = child;
    pos += j;
  }
  return {node, (int64_t)node->tokens.size(), pos};
}

int32_t Radix::begin_turn(int32_t slot, const int32_t* tokens, int64_t n, int64_t* n_past_out) {
  if (n < 0 || (n > 0 && !tokens) || !n_past_out) return ERR_INVALID;
  *n_past_out = 0;
  ++clock_;
  const Walk w = walk(tokens, n);
  const int64_t m = std::min<int64_t>(w.total, std::max<int64_t>(0, n - keep_last_));
  if (m <= 0) return OK;
  const int32_t rc = pool_->alias(w.node->donor, slot, 0, m);  // constant time, metadata only
  if (rc != OK) return rc;
  *n_past_out = m;
  return OK;
}

void Radix::collect_leaves(Node* n, std::vector<Node*>* out) {
  if (n->children.empty()) {
    if (n != &root_) out->push_back(n);
    return;
  }
  for (auto& kv : n->children) collect_leaves(kv.second.get(), out);
}

std::vector<int32_t> Radix::path_tokens(const Node* n) const {
  std::vector<const Node*> chain;
  for (; n && n != &root_; n = n->parent) chain.push_back(n);
  std::vector<int32_t> out;
  for (auto it = chain.rbegin(); it != chain.rend(); ++it) out.insert(out.end(), (*it)->tokens.begin(), (*it)->tokens.end());
  return out;
}

bool Radix::evict_oldest_leaf(const std::vector<const Node*>& protect) {
  std::vector<Node*> leaves;
  collect_leaves(&root_, &leaves);
  Node* victim = nullptr;
  std::vector<int32_t> victim_path;
  for (Node* leaf : leaves) {
    if (std::find(protect.begin(), protect.end(), leaf) != protect.end()) continue;
    if (victim && leaf->touch > victim->touch) continue;
    std::vector<int32_t> p = path_tokens(leaf);
    // oldest touch first; equal touches are ordered by token path so that the choice is fully defined
    if (!victim || leaf->touch < victim->touch || p < victim_path) {
      victim = leaf;
      victim_path = std::move(p);
    }
  }
  if (!victim) return false;
  evicted_.push_back(victim_path);
  cells_ -= (int64_t)victim->tokens.size();
  const int32_t donor = victim->donor;
  const int64_t start = victim->start;
  victim->parent->children.erase(victim->tokens[0]);  // destroys the node
  --n_nodes_;
  if (--donor_refs_[donor] == 0) {
    donor_refs_.erase(donor);
    (void)pool_->release(donor);
  } else {
    (void)pool_->trim(donor, start);  // the upper half of a split still names this donor
  }
  return true;
}

int32_t Radix::save(int32_t slot, const int32_t* tokens, int64_t n, int32_t* saved_out) {
  if (n < 0 || (n > 0 && !tokens)) return ERR_INVALID;
  if (saved_out) *saved_out = 0;
  int64_t have = 0;
  int32_t rc = pool_->length(slot, &have);
  if (rc != OK) return rc;
  if (have < n) return ERR_INVALID;  // the slot must hold the whole prompt
  ++clock_;
  Walk w = walk(tokens, n);
  if (w.total == n) {
    if (saved_out) *saved_out = 1;
    return OK;
  }
  const int64_t need = n - w.total;
  std::vector<const Node*> protect;
  for (const Node* p = w.node; p; p = p->parent) protect.push_back(p);
  while (cells_ + need > budget_)
    if (!evict_oldest_leaf(protect)) return OK;  // cannot make room: the turn goes unsaved
  int32_t donor = -1;
  while ((rc = pool_->acquire(1, 0, &donor)) != OK) {
    if (rc != ERR_TIMEOUT) return rc;
    if (!evict_oldest_leaf(protect)) return OK;
  }
  Node* node = w.node;
  if (w.in_node < (int64_t)node->tokens.size()) {  // diverged inside `node`: split it there
    std::unique_ptr<Node> lower(new Node());
    lower->tokens.assign(node->tokens.begin() + w.in_node, node->tokens.end());
    lower->start = node->start + w.in_node;
    lower->donor = node->donor;
    lower->touch = node->touch;
    lower->children = std::move(node->children);
    for (auto& kv : lower->children) kv.second->parent = lower.get();
    lower->parent = node;
    node->tokens.resize(w.in_node);
    node->children.clear();
    const int32_t first = lower->tokens[0];
    node->children[first] = std::move(lower);
    ++donor_refs_[node->donor];
    ++n_nodes_;
  }
  rc = pool_->alias(slot, donor, 0, n);
  if (rc != OK) {
    (void)pool_->release(donor);
    return rc;
  }
  std::unique_ptr<Node> fresh(new Node());
  fresh->tokens.assign(tokens + w.total, tokens + n);
  fresh->start = w.total;
  fresh->donor = donor;
  fresh->touch = clock_;
  fresh->parent = node;
  const int32_t first = fresh->tokens[0];
  node->children[first] = std::move(fresh);
  donor_refs_[donor] = 1;
  ++n_nodes_;
  cells_ += need;
  if (saved_out) *saved_out = 1;
  return OK;
}

void Radix::stats(int64_t* nodes, int64_t* cells, int64_t* donors, int64_t* evictions) const {
  if (nodes) *nodes = n_nodes_;
  if (cells) *cells = cells_;
  if (donors) *donors = (int64_t)donor_refs_.size();
  if (evictions) *evictions = (int64_t)evicted_.size();
}

int64_t Radix::evicted_path(int64_t i, int32_t* out, int64_t cap) const {
  if (i < 0 || i >= (int64_t)evicted_.size()) return -1;
  const std::vector<int32_t>& p = evicted_[i];
  for (int64_t k = 0; k < std::min<int64_t>(cap, (int64_t)p.size()); ++k) out[k] = p[k];
  return (int64_t)p.size();
}

}  // namespace dk
