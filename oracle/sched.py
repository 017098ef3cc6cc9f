"""Scheduler arithmetic of the paper's Sec. 3.2 (test oracle): chunk sizing, the FNV-1a hash, prefix grouping."""
from __future__ import annotations

from typing import List, Sequence, Tuple


def prefill_chunk(n_batch: int, n_prefilling: int, latency_sensitive: bool = False) -> int:
    """chunk = clamp(n_batch / N, 128, 4096); a fair 1024 ceiling when a small-max_tokens request is
    co-resident under contention (taken here as: more than one slot is prefilling)."""
    ceiling = 1024 if (latency_sensitive and n_prefilling > 1) else 4096
    return min(max(n_batch // n_prefilling, 128), ceiling)


def fnv1a32(data: bytes) -> int:
    """32-bit FNV-1a: offset basis 2166136261, prime 16777619 (Eq. 7 reduces it mod 2^32)."""
    h = 2166136261
    for b in data:
        h = ((h ^ b) * 16777619) % (1 << 32)
    return h


def prefill_groups(prompts: Sequence[Sequence[int]], n_past: Sequence[int], prefix_id: Sequence[int],
                   window: int = 8) -> Tuple[List[int], List[int]]:
    """Leader index and tokens shared with the leader, per slot.  No hashing here: the grouping condition
    itself (same cached prefix, same match point, identical next `window` tokens), first come first lead."""
    leader = list(range(len(prompts)))
    shared = [int(p) for p in n_past]
    for i, t in enumerate(prompts):
        if len(t) - n_past[i] < window:
            continue
        for l in range(i):
            if leader[l] != l or len(prompts[l]) - n_past[l] < window:
                continue
            if prefix_id[l] != prefix_id[i] or n_past[l] != n_past[i]:
                continue
            if list(prompts[l][n_past[l]:n_past[l] + window]) != list(t[n_past[i]:n_past[i] + window]):
                continue
            c = n_past[i] + window
            while c < min(len(t), len(prompts[l])) and t[c] == prompts[l][c]:
                c += 1
            leader[i], shared[i] = l, c
            break
    return leader, shared
