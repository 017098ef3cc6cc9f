"""Logical model of the sequence pool and its unified KV cache (test oracle).

Follows the paper's Sec. 3.1 (a fixed pool of named sequences inside one
unified cache, split into a transient and a session region, recycled through a
free list), Sec. 3.3 / Alg. 1 (SeqAlias(donor, dst, 0, m): the destination's
first m positions become the donor's cells, nothing is copied) and Alg. 2
(trimming the cache back to the last accepted position).

A sequence is a Python list of cell objects; a cell holds one token's K and V
for all KV heads.  Aliasing shares the *same cell objects*, so object identity
stands in for "same physical cells".  There is no arithmetic here at all.
"""
from __future__ import annotations

from typing import List, Optional

import numpy as np


class OracleError(Exception):
    """Raised with the name of the status the library must return for the same call."""

    def __init__(self, status: str):
        super().__init__(status)
        self.status = status


class _Cell:
    __slots__ = ("k", "v")

    def __init__(self, k, v):
        self.k = k  # [Hkv, D]
        self.v = v


class OraclePool:
    def __init__(self, n_slots: int, n_session_slots: int, arena_cells: Optional[int] = None):
        if n_slots <= 0 or not (0 <= n_session_slots <= n_slots):
            raise OracleError("INVALID")
        self.n_slots = n_slots
        self.n_session = n_session_slots
        # ids [0, n_slots - n_session) are the transient region, the rest the session region
        self.free = {0: list(range(0, n_slots - n_session_slots)),
                     1: list(range(n_slots - n_session_slots, n_slots))}
        self.in_use = [False] * n_slots
        self.seqs: List[List[_Cell]] = [[] for _ in range(n_slots)]
        self.arena_cells = arena_cells

    # -- slot lifecycle ---------------------------------------------------
    def acquire(self, region: int) -> int:
        if region not in (0, 1):
            raise OracleError("INVALID")
        if not self.free[region]:
            raise OracleError("TIMEOUT")  # a real pool blocks until its timeout
        s = self.free[region].pop(0)
        self.in_use[s] = True
        return s

    def release(self, slot: int) -> None:
        self._check(slot)
        self.seqs[slot] = []  # cells survive for as long as an alias still lists them
        self.in_use[slot] = False
        self.free[1 if slot >= self.n_slots - self.n_session else 0].append(slot)

    def _check(self, slot: int) -> None:
        if not (0 <= slot < self.n_slots) or not self.in_use[slot]:
            raise OracleError("NO_SLOT")

    # -- cache operations -------------------------------------------------
    def length(self, slot: int) -> int:
        self._check(slot)
        return len(self.seqs[slot])

    def append(self, slot: int, k_rows, v_rows) -> None:
        """k_rows, v_rows: [count, Hkv, D]; extends the sequence by count cells."""
        self._check(slot)
        k_rows, v_rows = np.asarray(k_rows), np.asarray(v_rows)
        assert k_rows.shape == v_rows.shape
        for t in range(k_rows.shape[0]):
            self.seqs[slot].append(_Cell(k_rows[t].copy(), v_rows[t].copy()))

    def alias(self, donor: int, dst: int, p0: int, p1: int) -> None:
        self._check(donor)
        self._check(dst)
        if p0 != 0:
            raise OracleError("UNSUPPORTED")
        if donor == dst or p1 < 0 or p1 > len(self.seqs[donor]) or len(self.seqs[dst]) != 0:
            raise OracleError("INVALID")
        self.seqs[dst] = list(self.seqs[donor][:p1])  # same cell objects, new list

    def trim(self, slot: int, new_len: int) -> None:
        self._check(slot)
        if new_len < 0 or new_len > len(self.seqs[slot]):
            raise OracleError("INVALID")
        del self.seqs[slot][new_len:]

    # -- views --------------------------------------------------------------
    def gather(self, slot: int):
        """Logical contents [len, Hkv, D] of K and of V (empty arrays keep the trailing dims unknown)."""
        self._check(slot)
        cells = self.seqs[slot]
        if not cells:
            return None, None
        return np.stack([c.k for c in cells]), np.stack([c.v for c in cells])

    def cell_ids(self, slot: int):
        self._check(slot)
        return [id(c) for c in self.seqs[slot]]

    def live_cells(self) -> int:
        """Distinct cells reachable from any sequence."""
        return len({id(c) for s in self.seqs for c in s})
