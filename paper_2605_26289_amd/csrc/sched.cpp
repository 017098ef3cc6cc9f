// Host-side helpers of the batching scheduler (paper Sec. 3.2): the workload-adaptive prefill chunk and
// the grouping of slots whose prompts continue identically beyond their radix match point.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <unordered_map>
#include <vector>

#include "../../include/deltakv.h"

namespace {

constexpr uint32_t kFnvOffset32 = 2166136261u;
constexpr uint32_t kFnvPrime32 = 16777619u;

uint32_t fnv1a32(const unsigned char* p, int64_t n) {
  uint32_t h = kFnvOffset32;
  for (int64_t i = 0; i < n; ++i) {
    h ^= p[i];
    h *= kFnvPrime32;
  }
  return h;
}

}  // namespace

extern "C" {

int32_t dk_fnv1a32(const void* bytes, int64_t n_bytes, uint32_t* hash_out) {
  if (n_bytes < 0 || (n_bytes > 0 && !bytes) || !hash_out) return DK_ERR_INVALID;
  *hash_out = fnv1a32((const unsigned char*)bytes, n_bytes);
  return DK_OK;
}

int32_t dk_prefill_chunk(int64_t n_batch, int32_t n_prefilling, int32_t latency_sensitive, int64_t* chunk_out) {
  if (n_batch <= 0 || n_prefilling <= 0 || !chunk_out) return DK_ERR_INVALID;
  const int64_t ceiling = (latency_sensitive && n_prefilling > 1) ? 1024 : 4096;
  *chunk_out = std::min<int64_t>(std::max<int64_t>(n_batch / n_prefilling, 128), ceiling);
  return DK_OK;
}

int32_t dk_prefill_groups(int32_t n_slots, const int32_t* const* tokens, const int64_t* n_tokens,
                          const int64_t* n_past, const int32_t* prefix_id, int32_t window, int32_t* leader_out,
                          int64_t* shared_out) {
  if (n_slots < 0 || window <= 0 || (n_slots > 0 && (!tokens || !n_tokens || !n_past || !prefix_id || !leader_out || !shared_out)))
    return DK_ERR_INVALID;
  struct Key {
    uint32_t hash;
    int32_t prefix;
    int64_t past;
    bool operator==(const Key& o) const { return hash == o.hash && prefix == o.prefix && past == o.past; }
  };
  struct KeyHash {
    size_t operator()(const Key& k) const { return (size_t)k.hash * 1000003u ^ (size_t)k.prefix * 7919u ^ (size_t)k.past; }
  };
  std::unordered_map<Key, std::vector<int32_t>, KeyHash> leaders;  // candidate leaders per key (collisions keep several)
  for (int32_t i = 0; i < n_slots; ++i) {
    if (n_past[i] < 0 || n_past[i] > n_tokens[i] || (n_tokens[i] > 0 && !tokens[i])) return DK_ERR_INVALID;
    leader_out[i] = i;
    shared_out[i] = n_past[i];
    if (n_tokens[i] - n_past[i] < window) continue;  // too little left to be worth a group
    const int32_t* next = tokens[i] + n_past[i];
    Key key{fnv1a32((const unsigned char*)next, (int64_t)window * 4), prefix_id[i], n_past[i]};
    std::vector<int32_t>& cands = leaders[key];
    bool joined = false;
    for (int32_t l : cands) {
      if (std::memcmp(tokens[l] + n_past[l], next, (size_t)window * 4) != 0) continue;  // hash collision
      // the follower takes over everything the two prompts have in common
      int64_t c = n_past[i] + window;
      const int64_t lim = std::min(n_tokens[l], n_tokens[i]);
      while (c < lim && tokens[l][c] == tokens[i][c]) ++c;
      leader_out[i] = l;
      shared_out[i] = c;
      joined = true;
      break;
    }
    if (!joined) cands.push_back(i);
  }
  return DK_OK;
}

}  // extern "C"
