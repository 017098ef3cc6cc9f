"""Prefix cache of paper Sec. 3.3 / Alg. 1 as a flat ledger of saves (test oracle, no trie).

TEST INFRASTRUCTURE ONLY.  A second, structure-free statement of what the radix prefix cache
computes, written so that it shares no control flow with a trie: there are no nodes, no child maps,
no walk and no split routine.  The library's trie (and the trie-shaped oracle in radix.py) are
checked against it.

State.  Every successful save leaves one *record*: the full prompt that was saved (`path`) and the
half-open range of positions [lo, hi) whose cells that save added to the cache -- the cells the cache
did not hold yet (Sec. 3.3, "incremental save": one new piece per turn holding only the delta).  The
ranges of different records never cover the same (prompt prefix, position) twice, so
    cells held = sum of (hi - lo) = number of distinct prompt prefixes the records cover.
A record also carries the clock of its most recent touch and the donor sequence that keeps its
cells alive.

Definitions, all by comparison of token strings:
  lcp(a, b)          length of the longest common prefix.
  cached(T)          max over records of lcp(T, path) -- what is cached of a prompt T
                     (capped at |T| - keep_last for a turn: the last tokens always go through the model).
  a lookup or save of T *touches* record R when lcp(T, R.path) > R.lo: the prompt runs into the
                     cells R added.
  piece boundaries   when a new save diverges from R.path at a position p strictly inside (R.lo, R.hi),
                     R is cut at p into [lo, p) and [p, hi): from then on the two pieces age and are
                     shed separately (the upper one is now shared with the new prompt), both kept
                     alive by R's donor.
  leaf               a record whose path no other record's path properly extends.
  eviction           when a save needs more cells than the budget leaves (or no donor sequence is
                     free), the leaf with the oldest touch is shed -- ties by token path -- and its
                     cells are given back: its donor is trimmed to R.lo if another piece still uses
                     it, released otherwise.  Records touched by the save in progress are never shed
                     for it.  If nothing can be shed the save is skipped.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple


def lcp(a: Sequence[int], b: Sequence[int]) -> int:
    n = 0
    for x, y in zip(a, b):
        if x != y:
            break
        n += 1
    return n


class _Record:
    __slots__ = ("path", "lo", "hi", "touch", "donor")

    def __init__(self, path: Tuple[int, ...], lo: int, hi: int, touch: int, donor: int):
        self.path, self.lo, self.hi, self.touch, self.donor = path, lo, hi, touch, donor

    def key(self) -> Tuple[int, ...]:
        """The prompt prefix this piece ends at."""
        return self.path[: self.hi]


class FlatPrefixCache:
    """Same interface as the trie oracle: begin_turn / save over a pool with acquire, release, alias, trim."""

    def __init__(self, pool, cell_budget: int, keep_last: int = 1):
        self.pool = pool
        self.budget = int(cell_budget)
        self.keep_last = int(keep_last)
        self.records: List[_Record] = []
        self.clock = 0
        self.evicted: List[Tuple[int, ...]] = []

    # -- views ------------------------------------------------------------------------------------
    @property
    def cells(self) -> int:
        return sum(r.hi - r.lo for r in self.records)

    def distinct_positions(self) -> int:
        """Cells held, counted the slow way: distinct (prefix ending at a covered position)."""
        return len({r.path[:p + 1] for r in self.records for p in range(r.lo, r.hi)})

    def piece_count(self) -> int:
        return len(self.records)

    def donors(self) -> int:
        return len({r.donor for r in self.records})

    def cached(self, tokens: Sequence[int]) -> int:
        return max((lcp(tokens, r.key()) for r in self.records), default=0)

    # -- Alg. 1 -------------------------------------------------------------------------------------
    def _touch(self, tokens: Sequence[int]) -> List[_Record]:
        hit = [r for r in self.records if lcp(tokens, r.key()) > r.lo]
        for r in hit:
            r.touch = self.clock
        return hit

    def begin_turn(self, slot: int, tokens: Sequence[int]) -> int:
        """Lines 1-5 of Alg. 1: alias what is cached of the prompt into the empty slot; returns n_past."""
        self.clock += 1
        tokens = tuple(int(t) for t in tokens)
        hit = self._touch(tokens)
        m = min(self.cached(tokens), max(0, len(tokens) - self.keep_last))
        if m > 0:
            # any donor whose prompt covers the first m positions will do; take the deepest piece touched
            deepest = max(hit, key=lambda r: r.lo)
            self.pool.alias(deepest.donor, slot, 0, m)
        return m

    def save(self, slot: int, tokens: Sequence[int]) -> bool:
        """Last line of Alg. 1: the slot holds all of `tokens`; keep the part that is not cached yet."""
        self.clock += 1
        tokens = tuple(int(t) for t in tokens)
        mine = self._touch(tokens)
        have = self.cached(tokens)
        if have == len(tokens):
            return True
        need = len(tokens) - have
        while self.cells + need > self.budget:
            if not self._shed_stalest_leaf(mine):
                return False
        donor = self._donor(mine)
        if donor is None:
            return False
        # a piece that the prompt leaves half-way is cut there
        for r in list(self.records):
            if r.lo < have < r.hi and lcp(tokens, r.key()) == have:
                self.records.append(_Record(r.path, have, r.hi, r.touch, r.donor))
                r.hi = have
        self.pool.alias(slot, donor, 0, len(tokens))
        self.records.append(_Record(tokens, have, len(tokens), self.clock, donor))
        return True

    # -- eviction -----------------------------------------------------------------------------------
    def _donor(self, keep: List[_Record]) -> Optional[int]:
        while True:
            try:
                return self.pool.acquire(1)
            except Exception:
                if not self._shed_stalest_leaf(keep):
                    return None

    def _is_leaf(self, r: _Record) -> bool:
        k = r.key()
        return not any(o is not r and len(o.key()) > len(k) and o.key()[: len(k)] == k for o in self.records)

    def _shed_stalest_leaf(self, keep: List[_Record]) -> bool:
        cands = [r for r in self.records if self._is_leaf(r) and not any(r is k for k in keep)]
        if not cands:
            return False
        victim = min(cands, key=lambda r: (r.touch, r.key()))
        self.evicted.append(victim.key())
        self.records = [r for r in self.records if r is not victim]
        if any(r.donor == victim.donor for r in self.records):
            self.pool.trim(victim.donor, victim.lo)  # the piece above it still needs this donor
        else:
            self.pool.release(victim.donor)
        return True
