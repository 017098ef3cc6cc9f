"""Prompt-lookup drafting on the host (test oracle).

What is computed (paper Sec. 3.6 / Alg. 2, first line, and the paragraph "Acceptance gating"):
LookupNgram(R, G_tail, l, N) scans the slot's recent token buffer R -- the prompt followed by the
slot's own output so far -- for the longest suffix-anchored n-gram: the largest n >= l such that the
last n tokens of the buffer also occur earlier in it, and proposes the tokens that followed that
earlier occurrence, at most N of them.  The per-step proposal length is gated by a slot-local
exponential moving average of the acceptance rate: below a confidence threshold it drops to a floor.

Readings taken where the paper is silent:
  * n is capped by `max_match` (the paper gives no cap: pass len(R) for "no cap");
  * among several earlier occurrences of the same length the most recent one wins;
  * an occurrence must end before the buffer's last token (it may overlap the suffix itself, as in a
    periodic sequence), and its continuation may run into the suffix;
  * the moving average is ema <- (1 - beta) ema + beta (accepted / proposed), updated only on steps
    that proposed something; proposal length = max_len if ema >= threshold else floor_len.
The constants (l, N, beta, threshold, floor) are not given in the paper and are arguments here.

Written as the plain search: every length from the longest down, every position from the latest back.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def lookup_ngram(recent: Sequence[int], min_match: int, max_match: int, max_draft: int) -> Tuple[List[int], int]:
    """Returns (predicted tokens, matched n-gram length); ([], 0) when nothing of length >= min_match recurs."""
    r = [int(t) for t in recent]
    size = len(r)
    if min_match < 1 or max_match < min_match or max_draft < 0:
        raise ValueError("need 1 <= min_match <= max_match and max_draft >= 0")
    for n in range(min(max_match, size - 1), min_match - 1, -1):
        suffix = r[size - n:]
        for end in range(size - 2, n - 2, -1):  # occurrence = r[end-n+1 .. end]
            if r[end - n + 1:end + 1] == suffix:
                return r[end + 1:end + 1 + max_draft], n
    return [], 0


def gate(ema: float, proposed: int, accepted: int, beta: float, threshold: float, floor_len: int,
         max_len: int) -> Tuple[float, int]:
    """One update of the acceptance average and the proposal length it allows for the next step."""
    if proposed < 0 or accepted < 0 or accepted > proposed:
        raise ValueError("0 <= accepted <= proposed")
    if proposed > 0:
        ema = (1.0 - beta) * ema + beta * (accepted / proposed)
    return ema, (max_len if ema >= threshold else floor_len)
