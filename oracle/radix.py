"""Radix prefix cache and the per-turn procedure around it (test oracle).

What is computed (paper Sec. 3.3, Alg. 1): shared prompt prefixes are kept in a radix trie keyed by
token sequences; a node owns a token segment and names a donor sequence whose KV state still holds
the cells of the whole path down to the node.  A turn (i) walks the trie for the longest cached
prefix of its prompt, (ii) aliases that prefix from the donor into its own fresh sequence -- metadata
only --, (iii) runs only the remaining delta tokens through the model, and (iv) saves incrementally:
the branch is walked to its tip and ONE new node is appended that holds only the delta cells.  When a
save would exceed the cell budget, the leaf whose most recent touch is oldest is shed, until it fits.

Readings taken where the paper is silent:
  * a match may end inside a node's segment; the alias then covers the partial node too (the donor
    holds the whole path), and a save that diverges inside a segment splits the node there, both
    halves naming the same donor (a donor sequence is released when its last node goes; when only
    the lower half of a split goes, the donor is trimmed back to the upper half's end);
  * `keep_last` tokens (default 1) always go through the model even if the whole prompt is cached,
    because the turn needs logits for its last position;
  * a node's donor is a sequence of the pool's session region that aliases the saving sequence, so
    that the saver itself can be released when its request ends;
  * the budget counts the cells the trie holds: the sum of its nodes' segment lengths; nodes on the
    path of the save in progress are never shed for that save; if nothing can be shed, or no session
    sequence can be had, the save is skipped (the turn itself is unaffected);
  * "touch" is a logical clock that ticks once per lookup or save.

The pool is anything with acquire(region) / release(slot) / alias(donor, dst, 0, m) / trim(slot, n):
the oracle pool model in the tests.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple


class _Node:
    __slots__ = ("tokens", "start", "donor", "touch", "children", "parent")

    def __init__(self, tokens, start, donor, parent):
        self.tokens: List[int] = tokens
        self.start: int = start  # position of tokens[0] in the prompt
        self.donor: Optional[int] = donor
        self.touch: int = 0
        self.children: Dict[int, "_Node"] = {}
        self.parent: Optional["_Node"] = parent

    @property
    def end(self) -> int:
        return self.start + len(self.tokens)


class OracleRadix:
    def __init__(self, pool, cell_budget: int, keep_last: int = 1):
        self.pool = pool
        self.budget = int(cell_budget)
        self.keep_last = int(keep_last)
        self.root = _Node([], 0, None, None)
        self.clock = 0
        self.cells = 0
        self.donor_refs: Dict[int, int] = {}
        self.evicted: List[Tuple[int, ...]] = []  # token paths of the shed leaves, in order

    # -- walking ----------------------------------------------------------------
    def _walk(self, tokens: Sequence[int]):
        """Deepest point of the trie along `tokens`: (node, matched tokens of that node, total matched)."""
        node, pos = self.root, 0
        while pos < len(tokens):
            child = node.children.get(int(tokens[pos]))
            if child is None:
                break
            j = 0
            while j < len(child.tokens) and pos + j < len(tokens) and child.tokens[j] == int(tokens[pos + j]):
                j += 1
            child.touch = self.clock
            if j < len(child.tokens):
                return child, j, pos + j
            node, pos = child, pos + j
        return node, len(node.tokens), pos

    def longest_prefix(self, tokens: Sequence[int]) -> Tuple[int, Optional[int]]:
        self.clock += 1
        node, _, m = self._walk(tokens)
        m = min(m, max(0, len(tokens) - self.keep_last))
        return (m, node.donor) if m > 0 else (0, None)

    # -- Alg. 1 ---------------------------------------------------------------
    def begin_turn(self, slot: int, tokens: Sequence[int]) -> int:
        """Lines 1-5 of Alg. 1: alias the longest cached prefix into the (empty) slot; returns n_past."""
        m, donor = self.longest_prefix(tokens)
        if m > 0:
            self.pool.alias(donor, slot, 0, m)
        return m

    def save(self, slot: int, tokens: Sequence[int]) -> bool:
        """Last line of Alg. 1, after the slot has been extended to hold all of `tokens`."""
        self.clock += 1
        tokens = [int(t) for t in tokens]
        node, j, pos = self._walk(tokens)
        if pos == len(tokens):
            return True  # nothing new beyond what the branch already holds
        need = len(tokens) - pos
        path = set()
        n = node
        while n is not None:
            path.add(id(n))
            n = n.parent
        while self.cells + need > self.budget:
            if not self._evict_oldest_leaf(path):
                return False
        donor = self._acquire_donor(path)
        if donor is None:
            return False
        if j < len(node.tokens):  # diverged inside `node`: split it at j
            lower = _Node(node.tokens[j:], node.start + j, node.donor, node)
            lower.touch = node.touch
            lower.children = node.children
            for c in lower.children.values():
                c.parent = lower
            node.tokens = node.tokens[:j]
            node.children = {lower.tokens[0]: lower}
            self.donor_refs[node.donor] += 1
        self.pool.alias(slot, donor, 0, len(tokens))
        fresh = _Node(tokens[pos:], pos, donor, node)
        fresh.touch = self.clock
        node.children[fresh.tokens[0]] = fresh
        self.donor_refs[donor] = 1
        self.cells += need
        return True

    # -- eviction ---------------------------------------------------------------
    def _acquire_donor(self, protected) -> Optional[int]:
        while True:
            try:
                return self.pool.acquire(1)
            except Exception:
                if not self._evict_oldest_leaf(protected):
                    return None

    def _leaves(self):
        out, stack = [], [self.root]
        while stack:
            n = stack.pop()
            if not n.children and n is not self.root:
                out.append(n)
            stack.extend(n.children.values())
        return out

    def _path_tokens(self, n) -> Tuple[int, ...]:
        parts = []
        while n is not None and n is not self.root:
            parts.append(n.tokens)
            n = n.parent
        return tuple(t for seg in reversed(parts) for t in seg)

    def _evict_oldest_leaf(self, protected) -> bool:
        cands = [n for n in self._leaves() if id(n) not in protected]
        if not cands:
            return False
        # oldest touch first; ties broken by the token path so that the order is fully defined
        victim = min(cands, key=lambda n: (n.touch, self._path_tokens(n)))
        self.evicted.append(self._path_tokens(victim))
        del victim.parent.children[victim.tokens[0]]
        self.cells -= len(victim.tokens)
        self.donor_refs[victim.donor] -= 1
        if self.donor_refs[victim.donor] == 0:
            del self.donor_refs[victim.donor]
            self.pool.release(victim.donor)
        else:
            self.pool.trim(victim.donor, victim.start)
        return True

    # -- views ------------------------------------------------------------------
    def node_count(self) -> int:
        count, stack = 0, [self.root]
        while stack:
            n = stack.pop()
            count += n is not self.root
            stack.extend(n.children.values())
        return count
