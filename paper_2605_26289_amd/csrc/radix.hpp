// Radix prefix cache over the sequence pool (paper Sec. 3.3, Alg. 1): host metadata only.
#pragma once
#include <cstdint>
#include <map>
#include <memory>
#include <unordered_map>
#include <vector>

#include "pool.hpp"

namespace dk {

class Radix {
 public:
  Radix(Pool* pool, int64_t cell_budget, int32_t keep_last);
  ~Radix();

  // Alg. 1 lines 1-5: aliases the longest cached prefix of `tokens` into the (empty) slot.
  int32_t begin_turn(int32_t slot, const int32_t* tokens, int64_t n, int64_t* n_past_out);
  // Alg. 1 last line: the slot now holds all n tokens; commit the part the trie does not have yet.
  int32_t save(int32_t slot, const int32_t* tokens, int64_t n, int32_t* saved_out);
  void stats(int64_t* nodes, int64_t* cells, int64_t* donors, int64_t* evictions) const;
  // token path of the i-th shed leaf (oldest first); returns its length, copies at most cap tokens
  int64_t evicted_path(int64_t i, int32_t* out, int64_t cap) const;

 private:
  struct Node {
    std::vector<int32_t> tokens;
    int64_t start = 0;
    int32_t donor = -1;
    int64_t touch = 0;
    std::map<int32_t, std::unique_ptr<Node>> children;
    Node* parent = nullptr;
    int64_t end() const { return start + (int64_t)tokens.size(); }
  };
  struct Walk {
    Node* node;
    int64_t in_node;  // matched tokens of `node`
    int64_t total;    // matched tokens of the prompt
  };
  Walk walk(const int32_t* tokens, int64_t n);
  bool evict_oldest_leaf(const std::vector<const Node*>& protect);
  void collect_leaves(Node* n, std::vector<Node*>* out);
  std::vector<int32_t> path_tokens(const Node* n) const;

  Pool* pool_;
  int64_t budget_;
  int32_t keep_last_;
  Node root_;
  int64_t clock_ = 0;
  int64_t cells_ = 0;
  int64_t n_nodes_ = 0;
  std::unordered_map<int32_t, int32_t> donor_refs_;
  std::vector<std::vector<int32_t>> evicted_;
};

}  // namespace dk
