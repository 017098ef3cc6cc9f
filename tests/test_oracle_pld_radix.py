"""Pins of the host-side oracles: prompt-lookup drafting (Sec. 3.6) and the radix prefix cache (Sec. 3.3, Alg. 1)."""
import numpy as np
import pytest

import oracle
from oracle import FlatPrefixCache, OraclePool, OracleRadix

# the prefix cache is stated twice (flat ledger of saves, trie); every pin below holds for both
CACHES = [FlatPrefixCache, OracleRadix]


def _pieces(c):
    return c.piece_count() if isinstance(c, FlatPrefixCache) else c.node_count()


# ---- prompt lookup ---------------------------------------------------------------------------------

def _lookup_by_definition(r, lo, hi, n_draft):
    """Second formulation: collect every (length, end) whose n-gram equals the suffix, then pick."""
    best = None
    size = len(r)
    for end in range(0, size - 1):
        n = 0
        while n < hi and end - n >= 0 and r[end - n] == r[size - 1 - n]:
            n += 1
        # n = common length of the strings ending at `end` and at size-1 (capped at hi)
        if n >= lo and (best is None or (n, end) > best):
            best = (n, end)
    if best is None:
        return [], 0
    n, end = best
    return list(r[end + 1:end + 1 + n_draft]), n


def test_lookup_hand_cases():
    # a JSON-like tool call that recurs: the continuation of the earlier occurrence is proposed
    buf = [9, 1, 2, 3, 4, 5, 6, 7, 8, 1, 2, 3]
    assert oracle.lookup_ngram(buf, 2, 8, 4) == ([4, 5, 6, 7], 3)
    assert oracle.lookup_ngram(buf, 2, 8, 2) == ([4, 5], 3)
    assert oracle.lookup_ngram(buf, 4, 8, 4) == ([], 0)          # only 3 tokens recur
    assert oracle.lookup_ngram([1, 2, 3, 4], 1, 8, 4) == ([], 0)  # nothing recurs
    # the longest match wins over a more recent shorter one; among equals the most recent wins
    buf = [5, 6, 7, 1, 0, 0, 7, 2, 0, 0, 5, 6, 7]
    assert oracle.lookup_ngram(buf, 1, 8, 2) == ([1, 0], 3)
    buf = [7, 1, 3, 7, 2, 4, 7]
    assert oracle.lookup_ngram(buf, 1, 8, 1) == ([2], 1)
    assert oracle.lookup_ngram([7, 1, 0, 7, 2, 0, 7], 1, 8, 1) == ([2], 2)
    # periodic output: the occurrence overlaps the suffix and the draft runs into it
    assert oracle.lookup_ngram([1, 2, 1, 2, 1, 2], 2, 8, 4) == ([1, 2], 4)
    assert oracle.lookup_ngram([4, 4, 4, 4], 1, 2, 8) == ([4], 2)
    assert oracle.lookup_ngram([], 1, 4, 4) == ([], 0) and oracle.lookup_ngram([3], 1, 4, 4) == ([], 0)


@pytest.mark.parametrize("seed", range(6))
def test_lookup_matches_its_definition_on_repetitive_streams(seed):
    rng = np.random.default_rng(seed)
    for _ in range(60):
        size = int(rng.integers(0, 60))
        r = rng.integers(0, 4, size=size).tolist()  # tiny alphabet: plenty of repeats
        lo = int(rng.integers(1, 4))
        hi = lo + int(rng.integers(0, 6))
        nd = int(rng.integers(0, 7))
        assert oracle.lookup_ngram(r, lo, hi, nd) == tuple(_lookup_by_definition(r, lo, hi, nd))


def test_draft_of_a_recurring_prefix_is_fully_accepted():
    """The paper's example: a k = 11-token JSON prefix recurs, so one pass verifies 12 tokens (Eq. 8)."""
    call = list(range(100, 111))  # 11 tokens
    history = [1, 2, 3, 50, 51] + call + [7, 8, 9, 50, 51]
    draft, n = oracle.lookup_ngram(history, 2, 16, 11)
    assert draft == call and n == 2
    assert oracle.pld_forward_passes(20, len(draft)) == 2


def test_acceptance_gate():
    ema, length = 1.0, 8
    # structured region: everything accepted, the window stays open
    for _ in range(5):
        ema, length = oracle.pld_gate(ema, 8, 8, 0.5, 0.4, 1, 8)
    assert ema == 1.0 and length == 8
    # prose: nothing accepted, the average decays 1 -> .5 -> .25 and the window drops to the floor
    ema, length = oracle.pld_gate(ema, 8, 0, 0.5, 0.4, 1, 8)
    assert (ema, length) == (0.5, 8)
    ema, length = oracle.pld_gate(ema, 8, 0, 0.5, 0.4, 1, 8)
    assert (ema, length) == (0.25, 1)
    # a step that proposed nothing leaves the average alone
    assert oracle.pld_gate(0.25, 0, 0, 0.5, 0.4, 1, 8) == (0.25, 1)
    # recovery
    ema, length = oracle.pld_gate(0.25, 1, 1, 0.5, 0.4, 1, 8)
    assert (ema, length) == (0.625, 8)
    with pytest.raises(ValueError):
        oracle.pld_gate(0.5, 2, 3, 0.5, 0.4, 1, 8)


# ---- radix prefix cache --------------------------------------------------------------------------------

def _rows(tokens, upto=None):
    """K/V rows of a prompt: position p depends on tokens[0..p] only, as in a causal model."""
    out, h = [], 17
    for t in tokens[:upto]:
        h = (h * 1000003 + int(t) + 1) % (2 ** 31 - 1)
        out.append(h)
    return np.asarray(out, dtype=np.int64).reshape(-1, 1, 1)


def _turn(pool, radix, tokens):
    """Alg. 1 with a fresh transient sequence; returns n_past.  The sequence is released afterwards."""
    slot = pool.acquire(0)
    n_past = radix.begin_turn(slot, tokens)
    assert pool.length(slot) == n_past
    rows = _rows(tokens)
    pool.append(slot, rows[n_past:], -rows[n_past:])       # only the delta goes through the model
    k, v = pool.gather(slot)
    assert np.array_equal(k, rows) and np.array_equal(v, -rows)  # aliased prefix reads like a private copy
    radix.save(slot, tokens)
    pool.release(slot)
    return n_past


@pytest.mark.parametrize("Cache", CACHES)
def test_five_turn_conversation_returns_the_papers_cached_counts(Cache):
    """Sec. 1 / Sec. 4.1: a 200-token system prompt, +150 tokens per turn, 950 tokens on turn 5, 800 of them cached."""
    gold = {}
    for line in open(__file__.replace("test_oracle_pld_radix.py", "golden/paper_arithmetic.txt")):
        if line.strip() and not line.startswith("#"):
            key, val = line.split("=")[0].strip(), line.split("=")[1].split("#")[0].strip()
            gold[key] = val
    rng = np.random.default_rng(0)
    stream = rng.integers(0, 50000, size=950).tolist()
    pool = OraclePool(8, 6)
    radix = Cache(pool, cell_budget=4096)
    got = [_turn(pool, radix, stream[: 200 + 150 * t]) for t in range(6)]
    assert got == [0, 200, 350, 500, 650, 800]
    assert got[-1] == int(gold["final_turn_cached_tokens"]) and 200 + 150 * 5 == int(gold["final_prompt_tokens"])
    assert _pieces(radix) == 6 and radix.cells == 950 == pool.live_cells()  # one node per turn, delta cells only


@pytest.mark.parametrize("Cache", CACHES)
@pytest.mark.parametrize("seed", range(5))
def test_n_past_is_the_longest_common_prefix_with_anything_saved(seed, Cache):
    rng = np.random.default_rng(seed)
    pool = OraclePool(40, 36)
    radix = Cache(pool, cell_budget=10 ** 6)
    saved = []
    for _ in range(30):
        if saved and rng.random() < 0.7:   # extend or fork an earlier prompt
            base = saved[int(rng.integers(len(saved)))]
            cut = int(rng.integers(1, len(base) + 1))
            t = base[:cut] + rng.integers(0, 3, size=int(rng.integers(1, 12))).tolist()
        else:
            t = rng.integers(0, 3, size=int(rng.integers(1, 20))).tolist()
        want = 0
        for s in saved:
            c = 0
            while c < min(len(s), len(t)) and s[c] == t[c]:
                c += 1
            want = max(want, c)
        want = min(want, len(t) - 1)  # the last token always goes through the model
        assert _turn(pool, radix, t) == want
        saved.append(t)
        assert radix.cells == pool.live_cells()  # the trie holds exactly the distinct cells, no copies


@pytest.mark.parametrize("Cache", CACHES)
def test_leaf_oldest_eviction_keeps_the_shared_branch_and_sheds_stale_tails(Cache):
    system = list(range(1000, 1100))                 # shared preamble, 100 tokens
    tails = [[10 + i] * 40 for i in range(4)]        # four conversations, 40 private tokens each
    pool = OraclePool(12, 8)
    radix = Cache(pool, cell_budget=100 + 3 * 40)
    assert _turn(pool, radix, system) == 0
    for i in range(3):
        assert _turn(pool, radix, system + tails[i]) == 100
    assert radix.cells == 220
    assert _turn(pool, radix, system + tails[1]) == 139          # touch conversation 1 (all but the last token cached)
    assert _turn(pool, radix, system + tails[3]) == 100          # needs 40 cells: the oldest tail (0) goes
    assert radix.evicted == [tuple(system + tails[0])]
    assert radix.cells == 220 and pool.live_cells() == 220
    assert _turn(pool, radix, system + tails[0]) == 100          # its tail is gone, the preamble is not
    assert radix.evicted[-1] == tuple(system + tails[2])         # 2 is now the stalest; 1 was touched later
    assert _turn(pool, radix, system[:60] + [7, 7]) == 60        # forks inside the preamble's node: split
    assert radix.cells <= radix.budget


@pytest.mark.parametrize("Cache", CACHES)
def test_budget_and_donor_slots_never_exceeded_under_random_traffic(Cache):
    rng = np.random.default_rng(3)
    pool = OraclePool(10, 6)
    radix = Cache(pool, cell_budget=150)
    prompts = [rng.integers(0, 4, size=30).tolist() for _ in range(4)]
    for step in range(200):
        base = prompts[int(rng.integers(len(prompts)))]
        t = base[: int(rng.integers(1, 31))] + rng.integers(0, 4, size=int(rng.integers(0, 25))).tolist()
        _turn(pool, radix, t)
        assert radix.cells <= 150 and radix.cells == pool.live_cells()
        assert sum(pool.in_use[4:]) == (radix.donors() if Cache is FlatPrefixCache else len(radix.donor_refs)) <= 6
    assert len(radix.evicted) > 10


# ---- the flat ledger on its own terms -------------------------------------------------------------

def test_flat_ledger_counts_every_held_position_once():
    """cells (sum of the saves' ranges) == a slow recount of the distinct prompt prefixes covered == the distinct
    cell objects alive in the pool, under traffic that forks, extends, cuts pieces and sheds leaves."""
    rng = np.random.default_rng(5)
    pool = OraclePool(12, 8)
    cache = FlatPrefixCache(pool, cell_budget=120)
    prompts = [rng.integers(0, 3, size=25).tolist() for _ in range(3)]
    for _ in range(120):
        base = prompts[int(rng.integers(len(prompts)))]
        t = base[: int(rng.integers(1, 26))] + rng.integers(0, 3, size=int(rng.integers(0, 20))).tolist()
        _turn(pool, cache, t)
        assert cache.cells == cache.distinct_positions() == pool.live_cells() <= 120
    assert len(cache.evicted) > 5


def test_flat_ledger_hand_case_cut_piece_ages_separately():
    """Save abcdef, then abcxy: the first save's piece is cut at 3; shedding takes def or xy (leaves), never abc
    while something hangs below it; what is cached of 'abcdz' drops from 5 to 3 once def is shed."""
    a, b, c, d, e, f, x, y, z = range(1, 10)
    pool = OraclePool(8, 6)
    cache = FlatPrefixCache(pool, cell_budget=8)
    _turn(pool, cache, [a, b, c, d, e, f])                 # 6 cells
    assert _turn(pool, cache, [a, b, c, x, y]) == 3       # + 2 cells, cuts the first piece at 3
    assert cache.piece_count() == 3 and cache.cells == 8
    assert cache.cached([a, b, c, d, z]) == 4
    assert _turn(pool, cache, [a, b, c, x, y, z]) == 5    # needs 1 cell: the stalest leaf is def
    assert cache.evicted == [(a, b, c, d, e, f)]
    assert cache.cached([a, b, c, d, z]) == 3 and cache.cells == 6
    assert pool.live_cells() == 6
