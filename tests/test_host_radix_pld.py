"""The library's host-side components against their oracles (no GPU): radix prefix cache driving the real
pool, prompt-lookup drafting, acceptance gate, scheduler helpers.  Everything is compared exactly."""
import numpy as np
import pytest

import oracle
from oracle import FlatPrefixCache, OraclePool, OracleRadix
from paper_2605_26289_amd import binding as dk


def _pool(n_slots, n_session, arena_cells=1 << 16, granule=16):
    desc = dk.PoolDesc(n_slots, n_session, arena_cells, granule, 8, 2, 64, dk.BF16, 256 * 10, 256 * 20, 256 * 30, 1 << 20)
    return dk.pool_create(desc)


def _rows(tokens):
    out, h = [], 17
    for t in tokens:
        h = (h * 1000003 + int(t) + 1) % (2 ** 31 - 1)
        out.append(h)
    return np.asarray(out, dtype=np.int64)


class Both:
    """The library's trie on the library's pool, next to the flat ledger-of-saves model of the prefix cache (no trie:
    cached length, leaves, shed order and cells held are all defined by comparing token strings) on an oracle pool.
    The trie-shaped oracle runs alongside as a third statement of the same procedure."""

    def __init__(self, n_slots, n_session, budget):
        self.pool = _pool(n_slots, n_session)
        self.radix = dk.radix_create(self.pool, budget, 1)
        self.arena = np.zeros(1 << 16, dtype=np.int64)  # plays the K arena: one number per cell
        self.opool = OraclePool(n_slots, n_session)
        self.flat = FlatPrefixCache(self.opool, budget)
        self.tpool = OraclePool(n_slots, n_session)
        self.trie = OracleRadix(self.tpool, budget)

    def close(self):
        dk.radix_destroy(self.radix)
        assert dk.pool_stats(self.pool)[0] == 0  # destroying the trie released every donor: nothing leaks
        dk.pool_destroy(self.pool)

    def turn(self, tokens):
        slot = dk.seq_acquire(self.pool, 0)
        oslot, tslot = self.opool.acquire(0), self.tpool.acquire(0)
        n_past = dk.radix_begin_turn(self.radix, slot, tokens)
        assert n_past == self.flat.begin_turn(oslot, tokens) == self.trie.begin_turn(tslot, tokens)
        assert dk.seq_len(self.pool, slot) == n_past
        rows = _rows(tokens)
        delta = len(tokens) - n_past
        cells = dk.kv_reserve(self.pool, [slot], [0, delta])      # only the delta is written
        self.arena[cells] = rows[n_past:]
        for pool, sl in ((self.opool, oslot), (self.tpool, tslot)):
            pool.append(sl, rows[n_past:].reshape(-1, 1, 1), rows[n_past:].reshape(-1, 1, 1))
        got = self.arena[dk.seq_cells(self.pool, slot)]
        assert np.array_equal(got, rows)                          # aliased prefix + delta read as the whole prompt
        assert np.array_equal(self.opool.gather(oslot)[0].ravel(), rows)
        assert dk.radix_save(self.radix, slot, tokens) == self.flat.save(oslot, tokens) == self.trie.save(tslot, tokens)
        dk.seq_release(self.pool, slot)
        self.opool.release(oslot)
        self.tpool.release(tslot)
        nodes, cells_held, donors, shed = dk.radix_stats(self.radix)
        assert (nodes, cells_held, donors, shed) == (self.flat.piece_count(), self.flat.cells, self.flat.donors(),
                                                     len(self.flat.evicted))
        assert cells_held == self.flat.distinct_positions() == self.opool.live_cells()
        assert (nodes, cells_held, shed) == (self.trie.node_count(), self.trie.cells, len(self.trie.evicted))
        held, _free = dk.pool_stats(self.pool)
        assert held >= cells_held  # cells are handed out in granules, so the pool may hold a little more
        return n_past


def test_five_turn_conversation_skips_the_papers_cell_counts():
    b = Both(8, 6, 4096)
    stream = np.random.default_rng(0).integers(0, 50000, size=950).tolist()
    assert [b.turn(stream[: 200 + 150 * t]) for t in range(6)] == [0, 200, 350, 500, 650, 800]
    assert dk.radix_stats(b.radix)[:2] == (6, 950)
    b.close()


@pytest.mark.parametrize("seed", range(4))
def test_random_traffic_with_eviction_matches_the_oracle_step_by_step(seed):
    rng = np.random.default_rng(seed)
    b = Both(10, 6, 150)
    prompts = [rng.integers(0, 4, size=30).tolist() for _ in range(4)]
    for _ in range(150):
        base = prompts[int(rng.integers(len(prompts)))]
        t = base[: int(rng.integers(1, 31))] + rng.integers(0, 4, size=int(rng.integers(0, 25))).tolist()
        b.turn(t)
    shed = dk.radix_stats(b.radix)[3]
    assert shed > 10
    for i in range(shed):
        assert tuple(dk.radix_evicted_path(b.radix, i)) == b.flat.evicted[i] == b.trie.evicted[i]
    b.close()


def test_shared_preamble_survives_and_forks_split_nodes():
    b = Both(12, 8, 100 + 3 * 40)
    system = list(range(1000, 1100))
    tails = [[10 + i] * 40 for i in range(4)]
    assert b.turn(system) == 0
    assert [b.turn(system + tails[i]) for i in range(3)] == [100, 100, 100]
    assert b.turn(system + tails[1]) == 139
    assert b.turn(system + tails[3]) == 100
    assert dk.radix_evicted_path(b.radix, 0) == system + tails[0]
    assert b.turn(system[:60] + [7, 7]) == 60
    b.close()


def test_35_turn_workflow_stays_contiguous_and_wastes_no_granules():
    """The per-turn procedure of Alg. 1 on the 35-turn coding workflow (Delta ~ U{200..1200}, context growing to
    about 24k tokens): every turn is a fresh sequence that aliases the cached conversation and appends its delta.
    The delta's first cells go into the unused rest of the previous turn's last granule, so the conversation stays
    one run of consecutive cells (no ragged key tile per turn for the kernels), the arena holds no more than one
    granule beyond the logical cells, and the alias walk is as deep as there are turns, not tokens."""
    from paper_2605_26289_amd import workloads as wl
    w = wl.config3()
    gran = 256
    total = w.turns[-1].n_past[0] + w.turns[-1].delta[0]
    desc = dk.PoolDesc(40, 36, total + 64 * gran, gran, 32, 8, 128, dk.BF16, 256 * 10, 256 * 20, 256 * 30, 1 << 20)
    pool = dk.pool_create(desc)
    radix = dk.radix_create(pool, total + 1000, 1)
    tokens = np.random.default_rng(3).integers(0, 50000, size=total).tolist()
    worst_segments = 0
    for t, turn in enumerate(w.turns):
        n = turn.n_past[0] + turn.delta[0]
        slot = dk.seq_acquire(pool, 0)
        n_past = dk.radix_begin_turn(radix, slot, tokens[:n])
        assert n_past == turn.n_past[0]
        dk.kv_reserve(pool, [slot], [0, n - n_past])
        segments, depth = dk.seq_stats(pool, slot)
        worst_segments = max(worst_segments, segments)
        assert depth == t + 1                      # one alias generation per turn
        assert dk.radix_save(radix, slot, tokens[:n])
        dk.seq_release(pool, slot)
        held, _free = dk.pool_stats(pool)
        assert n <= held < n + gran                # internal fragmentation: less than one granule in all
    assert worst_segments == 1                     # the whole conversation is one run of consecutive cells
    cells = dk.seq_cells(pool, dk.seq_acquire(pool, 0))  # (an empty slot: just exercises the probe)
    assert cells.size == 0
    dk.radix_destroy(radix)
    assert dk.pool_stats(pool)[0] == 0
    dk.pool_destroy(pool)


def test_borrowed_tail_room_is_never_shared_between_two_continuations():
    """Two sequences continue the same released conversation at its end: only one may write into the unused rest of
    its last granule, and a continuation of a conversation whose own sequence is still alive never does."""
    gran = 16
    desc = dk.PoolDesc(6, 2, 4096, gran, 8, 2, 64, dk.BF16, 256 * 10, 256 * 20, 256 * 30, 1 << 20)
    pool = dk.pool_create(desc)
    a = dk.seq_acquire(pool, 0)
    dk.kv_reserve(pool, [a], [0, 40])              # 40 cells: two and a half granules
    keep = dk.seq_acquire(pool, 1)
    dk.seq_alias(pool, a, keep, 0, 40)             # a session sequence keeps the cells alive
    b = dk.seq_acquire(pool, 0)
    dk.seq_alias(pool, a, b, 0, 40)                # a is still alive and may append: b must not borrow
    cb = dk.kv_reserve(pool, [b], [0, 5])
    ca = dk.kv_reserve(pool, [a], [0, 5])
    assert set(cb.tolist()).isdisjoint(ca.tolist())
    base = dk.seq_cells(pool, a)
    assert ca.tolist() == list(range(base[39] + 1, base[39] + 6))    # a itself continues in place
    dk.seq_release(pool, a)
    dk.seq_release(pool, b)
    # now nobody appends to the 40-cell node any more... but a's five extra cells follow it in the same granule,
    # so continuations of the first 40 positions get fresh cells
    c, d = dk.seq_acquire(pool, 0), dk.seq_acquire(pool, 0)
    dk.seq_alias(pool, keep, c, 0, 40)
    dk.seq_alias(pool, keep, d, 0, 40)
    cc = dk.kv_reserve(pool, [c], [0, 12])
    cd = dk.kv_reserve(pool, [d], [0, 12])
    shared = set(dk.seq_cells(pool, keep).tolist())
    assert set(cc.tolist()).isdisjoint(cd.tolist())
    assert shared.isdisjoint(cc.tolist()) and shared.isdisjoint(cd.tolist())
    assert dk.seq_cells(pool, c)[:40].tolist() == dk.seq_cells(pool, keep).tolist()
    dk.pool_destroy(pool)


def test_radix_errors():
    pool = _pool(4, 2)
    radix = dk.radix_create(pool, 100)
    slot = dk.seq_acquire(pool, 0)
    with pytest.raises(dk.DeltaKVError) as e:
        dk.radix_save(radix, slot, [1, 2, 3])  # the slot does not hold the prompt yet
    assert e.value.name == "INVALID"
    with pytest.raises(dk.DeltaKVError) as e:
        dk.radix_begin_turn(radix, 3, [1, 2, 3]) if False else dk.radix_save(radix, 3, [1])  # slot not acquired
    assert e.value.name == "NO_SLOT"
    with pytest.raises(dk.DeltaKVError):
        dk.radix_create(pool, 0)
    dk.radix_destroy(radix)
    dk.pool_destroy(pool)


# ---- prompt lookup, gate, scheduler helpers -------------------------------------------------------

@pytest.mark.parametrize("seed", range(6))
def test_pld_lookup_matches_the_oracle(seed):
    rng = np.random.default_rng(seed)
    for _ in range(200):
        r = rng.integers(0, 4, size=int(rng.integers(0, 80))).tolist()
        lo = int(rng.integers(1, 4))
        hi = lo + int(rng.integers(0, 8))
        nd = int(rng.integers(0, 9))
        assert dk.pld_lookup(r, lo, hi, nd) == oracle.lookup_ngram(r, lo, hi, nd)
    with pytest.raises(dk.DeltaKVError):
        dk.pld_lookup([1, 2], 0, 4, 4)


def test_pld_gate_matches_the_oracle():
    rng = np.random.default_rng(1)
    ema_l = ema_o = 1.0
    for _ in range(300):
        proposed = int(rng.integers(0, 9))
        accepted = int(rng.integers(0, proposed + 1))
        ema_l, len_l = dk.pld_gate(ema_l, proposed, accepted, 0.25, 0.4, 1, 8)
        ema_o, len_o = oracle.pld_gate(ema_o, proposed, accepted, 0.25, 0.4, 1, 8)
        assert abs(ema_l - ema_o) < 1e-5
        if abs(ema_o - 0.4) > 1e-4:  # away from the threshold the float32 state cannot flip the decision
            assert len_l == len_o
        ema_o = ema_l  # keep the two on the same float32 state
    with pytest.raises(dk.DeltaKVError):
        dk.pld_gate(0.5, 2, 3, 0.5, 0.4, 1, 8)


def test_fnv1a_published_vectors_and_oracle():
    # test vectors published with the FNV reference code
    assert dk.fnv1a32(b"") == 0x811C9DC5 == oracle.fnv1a32(b"")
    assert dk.fnv1a32(b"a") == 0xE40C292C == oracle.fnv1a32(b"a")
    assert dk.fnv1a32(b"foobar") == 0xBF9CF968 == oracle.fnv1a32(b"foobar")
    rng = np.random.default_rng(2)
    for _ in range(50):
        data = rng.integers(0, 256, size=int(rng.integers(0, 100)), dtype=np.uint8).tobytes()
        assert dk.fnv1a32(data) == oracle.fnv1a32(data)


def test_prefill_chunk_follows_the_papers_clamp():
    assert dk.prefill_chunk(4096, 1) == 4096           # one active prefill fills the batch
    assert dk.prefill_chunk(8192, 1) == 4096
    assert dk.prefill_chunk(4096, 8) == 512
    assert dk.prefill_chunk(4096, 64) == 128           # never below 128
    assert dk.prefill_chunk(8192, 2, True) == 1024     # fair ceiling next to a latency-sensitive request
    assert dk.prefill_chunk(8192, 1, True) == 4096     # no contention, no narrowing
    for nb in (1, 100, 2048, 4096, 16384, 100000):
        for n in (1, 2, 3, 7, 32, 500):
            for ls in (False, True):
                assert dk.prefill_chunk(nb, n, ls) == oracle.prefill_chunk(nb, n, ls)


def test_prefill_groups_burst_of_agents_sharing_a_schema_preamble():
    rng = np.random.default_rng(4)
    schema = rng.integers(0, 1000, size=300).tolist()
    other = rng.integers(0, 1000, size=300).tolist()
    prompts = [schema + rng.integers(0, 1000, size=int(rng.integers(5, 40))).tolist() for _ in range(6)]
    prompts += [other + [1, 2, 3], other + [4, 5], schema[:5], schema + [9]]
    n_past = [0] * len(prompts)
    pid = [0] * len(prompts)
    leader, shared = dk.prefill_groups(prompts, n_past, pid, 8)
    assert (leader, shared) == oracle.prefill_groups(prompts, n_past, pid, 8)
    assert leader[:6] == [0] * 6 and all(s >= 300 for s in shared[1:6])
    assert leader[6:8] == [6, 6] and shared[7] == 300
    assert leader[8] == 8 and shared[8] == 0           # fewer than K tokens left: not grouped
    assert leader[9] == 0 and shared[9] == 300
    # different match points or cached prefixes never group
    leader, shared = dk.prefill_groups(prompts[:3], [0, 8, 0], [0, 0, 1], 8)
    assert leader == [0, 1, 2]
    for seed in range(20):
        r = np.random.default_rng(100 + seed)
        ps = [r.integers(0, 2, size=int(r.integers(0, 30))).tolist() for _ in range(8)]
        past = [int(r.integers(0, len(p) + 1)) if r.random() < 0.3 else 0 for p in ps]
        ids = r.integers(0, 2, size=8).tolist()
        assert dk.prefill_groups(ps, past, ids, 3) == oracle.prefill_groups(ps, past, ids, 3)
