"""Greedy verification of a speculative batch (test oracle).

What is computed (paper Sec. 3.6 / Alg. 2 and Sec. 3.8): the verify batch of one slot is
[G_last, predicted[0], ..., predicted[k-1]]; one forward pass returns logits[0..k], row s being the
model's distribution for the token that FOLLOWS batch position s.  Every generated token is the argmax
of its logits row (temperature 0).  Drafts are accepted from the front while
argmax(logits[s]) == predicted[s]; the first mismatch rejects the rest.  With `a` accepted drafts the
cache keeps 1 + a of the k + 1 batch positions (G_last and the accepted drafts); the token to emit
next is argmax(logits[a]) -- the model's own choice at the first position whose draft was wrong, or
after the last draft when all were right.

Readings taken where the paper is silent:
  * ties in the argmax go to the lowest token id;
  * a NaN logit counts as +infinity (so the first NaN-or-+inf entry of a row wins);
  * k = 0 (a batch of one token) is the plain decode step: nothing to accept, next = argmax(logits[0]).

No vectorised trickery: the accept loop is the algorithm's loop.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def greedy_argmax(logits) -> np.ndarray:
    """Lowest index of the largest entry of every row of a [rows, vocab] array (NaN counts as +inf)."""
    x = np.asarray(logits, dtype=np.float64)
    if x.ndim != 2:
        raise ValueError("logits must be [rows, vocab]")
    if x.shape[1] == 0:
        raise ValueError("empty vocabulary")
    x = np.where(np.isnan(x), np.inf, x)
    return np.argmax(x, axis=1).astype(np.int64)


def verify_accept(logits, batch_tokens: Sequence[int]) -> Tuple[int, int, np.ndarray]:
    """One slot.  logits [k+1, vocab], batch_tokens = [G_last, predicted[0..k-1]].

    Returns (n_keep, next_token, argmax_per_row) with n_keep = 1 + accepted drafts."""
    am = greedy_argmax(logits)
    k = len(batch_tokens) - 1
    if am.shape[0] != k + 1 or k < 0:
        raise ValueError("one logits row per batch token")
    accepted = 0
    for s in range(k):
        actual = int(am[s])
        if actual != int(batch_tokens[1 + s]):
            break
        accepted += 1
    return 1 + accepted, int(am[accepted]), am


def verify_batch(logits, batch_tokens, cu_delta) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Varlen batch: rows cu_delta[b]..cu_delta[b+1] belong to slot b.  Slots with no rows give (0, -1)."""
    logits = np.asarray(logits)
    n = len(cu_delta) - 1
    keep = np.zeros(n, np.int64)
    nxt = np.full(n, -1, np.int64)
    am_all = np.zeros(logits.shape[0], np.int64)
    for b in range(n):
        lo, hi = int(cu_delta[b]), int(cu_delta[b + 1])
        if hi == lo:
            continue
        keep[b], nxt[b], am_all[lo:hi] = verify_accept(logits[lo:hi], list(batch_tokens[lo:hi]))
    return keep, nxt, am_all


def sequential_greedy(model, prefix: List[int], steps: int) -> List[int]:
    """Plain decoding: one forward pass per token.  `model(tokens)` returns the logits row after `tokens`."""
    toks = list(prefix)
    out = []
    for _ in range(steps):
        t = int(greedy_argmax(np.asarray(model(toks))[None, :])[0])
        out.append(t)
        toks.append(t)
    return out
