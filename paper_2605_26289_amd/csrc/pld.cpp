// Prompt-lookup drafting on the host (paper Sec. 3.6, Alg. 2 line 1 and "Acceptance gating").
// The matcher works on raw token ids in CPU memory; nothing here touches the GPU.
#include <cstdint>

#include "../../include/deltakv.h"

extern "C" {

// For every earlier position `end` whose token equals the buffer's last one, extend the match
// backwards; keep the longest (capped at max_match), the latest among equals.  O(size * max_match).
int32_t dk_pld_lookup(const int32_t* recent, int64_t n_recent, int32_t min_match, int32_t max_match,
                      int32_t max_draft, int32_t* draft_out, int32_t* n_draft_out, int32_t* match_len_out) {
  if (n_recent < 0 || (n_recent > 0 && !recent) || min_match < 1 || max_match < min_match || max_draft < 0)
    return DK_ERR_INVALID;
  if (!n_draft_out || (max_draft > 0 && !draft_out)) return DK_ERR_INVALID;
  *n_draft_out = 0;
  if (match_len_out) *match_len_out = 0;
  if (n_recent < 2) return DK_OK;
  const int64_t last = n_recent - 1;
  int64_t best_len = 0, best_end = -1;
  for (int64_t end = last - 1; end >= 0; --end) {
    if (recent[end] != recent[last]) continue;
    int64_t n = 1;
    while (n < max_match && end - n >= 0 && recent[end - n] == recent[last - n]) ++n;
    if (n > best_len) {  // scanning from the latest position back: ties keep the later one
      best_len = n;
      best_end = end;
      if (n == max_match) break;  // nothing longer can be found, and nothing later remains
    }
  }
  if (best_len < min_match) return DK_OK;
  int64_t avail = last - best_end;  // tokens after the occurrence, up to the end of the buffer
  if (avail > max_draft) avail = max_draft;
  for (int64_t i = 0; i < avail; ++i) draft_out[i] = recent[best_end + 1 + i];
  *n_draft_out = (int32_t)avail;
  if (match_len_out) *match_len_out = (int32_t)best_len;
  return DK_OK;
}

int32_t dk_pld_gate(float* ema_inout, int32_t proposed, int32_t accepted, float beta, float threshold,
                    int32_t floor_len, int32_t max_len, int32_t* next_len_out) {
  if (!ema_inout || !next_len_out || proposed < 0 || accepted < 0 || accepted > proposed) return DK_ERR_INVALID;
  if (!(beta >= 0.f && beta <= 1.f) || floor_len < 0 || max_len < floor_len) return DK_ERR_INVALID;
  double ema = *ema_inout;
  if (proposed > 0) ema = (1.0 - (double)beta) * ema + (double)beta * ((double)accepted / (double)proposed);
  *ema_inout = (float)ema;
  *next_len_out = *ema_inout >= threshold ? max_len : floor_len;
  return DK_OK;
}

}  // extern "C"
