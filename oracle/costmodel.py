"""The paper's printed cost arithmetic, as plain functions (test oracle).

Sec. 1 / Sec. 4.1: a conversation starts from a system prompt and grows by a
fixed number of tokens per turn.  Sec. 2.2 (speedup of a later turn), Sec. 3.6
(forward passes with prompt-lookup speculation) and Sec. 3.10's worked KV-size
example (the line defining the formula is lost in the source; it is rebuilt
from the worked numbers as 2 * layers * width * tokens * bytes).
"""
from __future__ import annotations

from typing import List, Tuple


def prompt_lengths(system_tokens: int, per_turn: int, turns: int) -> List[Tuple[int, int]]:
    """[(n_past, n_total)] per turn: cells already cached and prompt length after the turn."""
    out = []
    n = system_tokens
    for _ in range(turns):
        out.append((n, n + per_turn))
        n += per_turn
    return out


def turn_speedup(n_t: int, delta_t: int) -> float:
    """Sec. 2.2: full re-prefill costs O(n_t), the delta path O(Delta_t)."""
    return n_t / delta_t


def pld_forward_passes(m: int, k: int) -> int:
    """Sec. 3.6: ceil(m / (k + 1)) batched decodes for m tokens with k accepted drafts each."""
    return -(-m // (k + 1))


def kv_entry_bytes(layers: int, width: int, tokens: int, bytes_per_elem: int) -> int:
    """K and V for every layer, `width` elements per token per layer."""
    return 2 * layers * width * tokens * bytes_per_elem


def kv_cell_bytes(n_kv_heads: int, head_dim: int, bytes_per_elem: int) -> int:
    """One cell = one token's K and V over all KV heads of one layer."""
    return 2 * n_kv_heads * head_dim * bytes_per_elem
