"""Host-side bookkeeping of the library against the logical pool model (no GPU).

The C ABI's metadata calls need no device: arena pointers are opaque here.  A NumPy array plays
the arena; tokens are written at the cells dk_kv_reserve hands out and read back through
dk_seq_cells, and the result must equal the oracle pool's logical contents bit for bit.
"""
import ctypes as C
import os
import re
import threading
import time

import numpy as np
import pytest

from oracle import OracleError, OraclePool
from paper_2605_26289_amd import binding as dk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _pool(n_slots=4, n_session=0, arena_cells=1024, granule=16, hq=8, hkv=2, d=64, dtype=dk.BF16):
    desc = dk.PoolDesc(n_slots, n_session, arena_cells, granule, hq, hkv, d, dtype, 256 * 10, 256 * 20, 256 * 30, 1 << 20)
    return dk.pool_create(desc)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "deltakv.h")).read()
    declared = set(re.findall(r"\b(dk_[a-z_0-9]+)\s*\(", header))
    assert declared and "dk_delta_attend" in declared and "dk_kv_append" in declared
    lib = dk.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(dk.SIGNATURES)


def test_every_status_code_has_its_own_message():
    codes = [0] + list(range(-1, -11, -1))
    texts = [dk.strerror(c) for c in codes]
    assert all(t and "unknown" not in t.lower() for t in texts) and len(set(texts)) == len(texts)
    assert "unknown" in dk.strerror(-99).lower() or dk.strerror(-99) not in texts


def test_create_rejects_bad_descriptions():
    def rc(**kw):
        base = dict(n_slots=2, n_session_slots=0, arena_cells=512, granule_cells=16, n_q_heads=8, n_kv_heads=2,
                    head_dim=64, dtype=dk.BF16, k_arena=256, v_arena=512, dev_meta=768, dev_meta_bytes=1 << 20,
                    host_staging=None, host_staging_bytes=0, staging_depth=0)
        base.update(kw)
        d = dk.PoolDesc(*[base[f[0]] for f in dk.PoolDesc._fields_])
        out = C.c_void_p()
        r = dk.lib().dk_pool_create(C.byref(d), C.byref(out))
        if r == 0:
            dk.pool_destroy(out)
        return dk.STATUS_NAMES[r]
    assert rc() == "OK"
    assert rc(n_slots=0) == "INVALID"
    assert rc(n_session_slots=3) == "INVALID"
    assert rc(head_dim=96) == "UNSUPPORTED"
    assert rc(n_q_heads=7) == "UNSUPPORTED"
    assert rc(dtype=5) == "UNSUPPORTED"
    assert rc(k_arena=0) == "INVALID"
    assert rc(k_arena=257) == "INVALID"
    assert rc(dev_meta_bytes=16) == "INVALID"
    assert rc(arena_cells=8) == "INVALID"
    assert rc(host_staging_bytes=1 << 20) == "INVALID"          # bytes without memory
    assert rc(host_staging=4096) == "INVALID"                   # memory without bytes
    assert rc(host_staging=4097, host_staging_bytes=8 << 20) == "INVALID"   # misaligned
    assert rc(host_staging=4096, host_staging_bytes=8 << 10) == "INVALID"   # buffers below 64 KiB
    assert rc(staging_depth=65) == "INVALID"


def test_tuning_names_and_ranges_and_no_environment_channel(monkeypatch):
    monkeypatch.setenv("DELTAKV_STREAM_CHAINS", "3")  # the library reads no environment variable
    p = _pool()
    dk.set_tuning(p, "stream_chains", 128)
    dk.set_tuning(p, "xcd_speed3", 0.93)
    dk.set_tuning(p, "stream_rows", 32)
    dk.set_tuning(p, "stream_rows", 96)
    for name, value, err in (("stream_chains", 0, "INVALID"), ("stream_rows", 97, "INVALID"), ("stream_rows", 31, "INVALID"), ("stream_chains", 1.5, "INVALID"),
                             ("xcd_speed8", 1.0, "UNSUPPORTED"), ("xcd_speed0", 0.0, "INVALID"),
                             ("no_such_knob", 1, "UNSUPPORTED"), ("tile_min_chunk", 8, "INVALID")):
        with pytest.raises(dk.DeltaKVError) as e:
            dk.set_tuning(p, name, value)
        assert e.value.name == err, (name, value)
    dk.pool_destroy(p)


def test_launching_calls_without_staging_memory_report_workspace():
    """A pool created for host-only use (no staging memory): an append too long for the in-argument cell table
    fails before it touches any state."""
    p = _pool(arena_cells=1 << 14)
    s = dk.seq_acquire(p, 0)
    with pytest.raises(dk.DeltaKVError) as e:
        dk._check(dk.lib().dk_kv_append(p, 1, (C.c_int32 * 1)(s), (C.c_int32 * 2)(0, 2000), None, 256, 256, None),
                  "kv_append")
    assert e.value.name == "WORKSPACE"
    assert dk.seq_len(p, s) == 0 and dk.pool_stats(p)[0] == 0
    with pytest.raises(dk.DeltaKVError, match="WORKSPACE"):  # nothing to wait for either
        dk.staging_wait(p)
    assert dk.lib().dk_staging_wait(None) == -1
    dk.pool_destroy(p)


def test_regions_timeout_and_blocking_acquire():
    p = _pool(n_slots=3, n_session=1)
    a, b = dk.seq_acquire(p, 0), dk.seq_acquire(p, 0)
    s = dk.seq_acquire(p, 1)
    assert sorted([a, b]) == [0, 1] and s == 2
    for region in (0, 1):
        with pytest.raises(dk.DeltaKVError, match="TIMEOUT"):
            dk.seq_acquire(p, region, 0)
    t0 = time.perf_counter()
    with pytest.raises(dk.DeltaKVError, match="TIMEOUT"):
        dk.seq_acquire(p, 0, 50)
    assert time.perf_counter() - t0 >= 0.045
    got = []
    th = threading.Thread(target=lambda: got.append(dk.seq_acquire(p, 0, 5000)))
    th.start()
    time.sleep(0.05)
    dk.seq_release(p, a)
    th.join(2)
    assert got == [a]
    with pytest.raises(dk.DeltaKVError, match="INVALID"):
        dk.seq_acquire(p, 2, 0)
    with pytest.raises(dk.DeltaKVError, match="NO_SLOT"):
        dk.seq_release(p, 7)
    dk.seq_release(p, b)
    with pytest.raises(dk.DeltaKVError, match="NO_SLOT"):
        dk.seq_release(p, b)
    dk.pool_destroy(p)


def test_error_rules_match_the_oracle_model():
    p = _pool(n_slots=2, n_session=1)
    o = OraclePool(2, 1)
    a, b = dk.seq_acquire(p, 0), dk.seq_acquire(p, 1)
    assert (a, b) == (o.acquire(0), o.acquire(1))
    dk.kv_reserve(p, [a], [0, 4])
    o.append(a, np.zeros((4, 1, 1)), np.zeros((4, 1, 1)))
    cases = [(a, b, 1, 3), (a, a, 0, 2), (a, b, 0, 5), (a, b, 0, -1), (a, b, 0, 0), (a, b, 0, 2), (a, b, 0, 1), (a, 5, 0, 1)]
    for args in cases:
        want = "OK"
        try:
            o.alias(*args)
        except OracleError as e:
            want = e.status
        got = dk.STATUS_NAMES[dk.lib().dk_seq_alias(p, *args)]
        assert got == want, (args, got, want)
    for slot, new_len in [(b, 3), (b, -1), (b, 1), (a, 4), (a, 0)]:
        want = "OK"
        try:
            o.trim(slot, new_len)
        except OracleError as e:
            want = e.status
        assert dk.STATUS_NAMES[dk.lib().dk_seq_trim(p, slot, new_len)] == want
        assert dk.seq_len(p, slot) == o.length(slot)
    dk.pool_destroy(p)


def test_batch_argument_errors_and_all_or_nothing_append():
    p = _pool(n_slots=3, arena_cells=64, granule=16)  # 4 granules
    s = [dk.seq_acquire(p, 0) for _ in range(3)]
    with pytest.raises(dk.DeltaKVError, match="DUP_SLOT"):
        dk.kv_reserve(p, [s[0], s[0]], [0, 1, 2])
    with pytest.raises(dk.DeltaKVError, match="INVALID"):
        dk.kv_reserve(p, [s[0]], [1, 2])
    with pytest.raises(dk.DeltaKVError, match="INVALID"):
        dk.kv_reserve(p, [s[0], s[1]], [0, 3, 2])
    with pytest.raises(dk.DeltaKVError, match="INVALID"):
        dk.kv_reserve(p, [s[0]], [0, 3], n_accept=[4])
    with pytest.raises(dk.DeltaKVError, match="NO_SLOT"):
        dk.kv_reserve(p, [9], [0, 3])
    dk.kv_reserve(p, [s[0], s[1]], [0, 17, 20])  # 2 + 1 granules
    assert dk.pool_stats(p) == (48, 16)
    with pytest.raises(dk.DeltaKVError, match="NO_CELLS"):
        dk.kv_reserve(p, [s[1], s[2]], [0, 13, 30])  # s1 fits in its granule, s2 needs 2: only 1 free
    assert [dk.seq_len(p, x) for x in s] == [17, 3, 0] and dk.pool_stats(p) == (48, 16)
    cells = dk.kv_reserve(p, [s[2]], [0, 9], n_accept=[4])
    assert (cells[:4] >= 0).all() and (cells[4:] == -1).all() and dk.seq_len(p, s[2]) == 4
    dk.seq_release(p, s[0])
    assert dk.pool_stats(p) == (32, 32)
    dk.pool_destroy(p)


def test_alias_is_metadata_only_and_shares_cells():
    p = _pool(n_slots=4, arena_cells=4096, granule=16)
    a, b, c = (dk.seq_acquire(p, 0) for _ in range(3))
    dk.kv_reserve(p, [a], [0, 100])
    held = dk.pool_stats(p)[0]
    dk.seq_alias(p, a, b, 0, 70)
    assert dk.pool_stats(p)[0] == held  # no cell was allocated by the alias
    ca, cb = dk.seq_cells(p, a), dk.seq_cells(p, b)
    assert len(cb) == 70 and np.array_equal(cb, ca[:70])
    # both grow privately; the donor keeps writing behind position 70 of its own cells
    ga = dk.kv_reserve(p, [a], [0, 10])
    gb = dk.kv_reserve(p, [b], [0, 10])
    assert set(ga).isdisjoint(gb) and set(gb).isdisjoint(ca)
    assert np.array_equal(dk.seq_cells(p, b)[:70], ca[:70])
    # alias of an alias, shorter than the first alias point: still the donor's cells
    dk.seq_alias(p, b, c, 0, 75)
    cc = dk.seq_cells(p, c)
    assert np.array_equal(cc[:70], ca[:70]) and np.array_equal(cc[70:], gb[:5])
    # releasing the donor keeps the shared cells allocated and unchanged
    dk.seq_release(p, a)
    assert np.array_equal(dk.seq_cells(p, b)[:70], ca[:70])
    d = dk.seq_acquire(p, 0)
    fresh = dk.kv_reserve(p, [d], [0, 200])
    assert set(fresh).isdisjoint(set(dk.seq_cells(p, b))) and set(fresh).isdisjoint(set(dk.seq_cells(p, c)))
    dk.pool_destroy(p)


def test_trim_below_alias_point_never_overwrites_shared_cells():
    p = _pool(n_slots=2, arena_cells=1024, granule=16)
    a, b = dk.seq_acquire(p, 0), dk.seq_acquire(p, 0)
    dk.kv_reserve(p, [a], [0, 40])
    dk.seq_alias(p, a, b, 0, 30)
    shared = dk.seq_cells(p, b).copy()
    dk.seq_trim(p, a, 20)
    new = dk.kv_reserve(p, [a], [0, 25])
    assert set(new).isdisjoint(shared)
    assert np.array_equal(dk.seq_cells(p, b), shared)
    assert np.array_equal(dk.seq_cells(p, a)[:20], shared[:20])
    # trimming back above everything shared reuses the slot's own cells
    dk.seq_trim(p, a, 30)
    again = dk.kv_reserve(p, [a], [0, 5])
    assert np.array_equal(again, new[10:15])
    dk.pool_destroy(p)


def test_alias_cost_does_not_grow_with_prefix_length():
    p = _pool(n_slots=3, arena_cells=1 << 22, granule=256)
    a, b = dk.seq_acquire(p, 0), dk.seq_acquire(p, 0)
    dk.kv_reserve(p, [a], [0, 2_000_000])

    def timed(m, reps=300):
        best = 1e9
        for _ in range(5):
            t0 = time.perf_counter()
            for _ in range(reps):
                dk.seq_alias(p, a, b, 0, m)
                dk.seq_trim(p, b, 0)
            best = min(best, (time.perf_counter() - t0) / reps)
        return best
    small, large = timed(256), timed(2_000_000)
    assert large < 3 * small + 5e-6, (small, large)
    dk.pool_destroy(p)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_random_walk_matches_oracle_pool_bit_for_bit(seed):
    rng = np.random.default_rng(seed)
    n_slots, hkv, d, gran = 6, 2, 4, 8
    arena_cells = 2048
    p = _pool(n_slots=n_slots, n_session=2, arena_cells=arena_cells, granule=gran, hq=4, hkv=hkv, d=64)
    o = OraclePool(n_slots, 2)
    arena_k = np.zeros((arena_cells, hkv, d), dtype=np.float32)
    arena_v = np.zeros_like(arena_k)
    live = {}
    for step in range(400):
        op = rng.choice(["acquire", "append", "alias", "trim", "release", "verify"], p=[0.1, 0.4, 0.15, 0.15, 0.08, 0.12])
        if op == "acquire":
            region = int(rng.integers(0, 2))
            try:
                want = o.acquire(region)
            except OracleError:
                with pytest.raises(dk.DeltaKVError, match="TIMEOUT"):
                    dk.seq_acquire(p, region, 0)
                continue
            assert dk.seq_acquire(p, region, 0) == want
            live[want] = True
        elif not live:
            continue
        elif op == "append":
            chosen = [int(s) for s in rng.permutation(list(live))[: int(rng.integers(1, len(live) + 1))]]
            deltas = [int(rng.integers(0, 30)) for _ in chosen]
            cu = np.concatenate([[0], np.cumsum(deltas)]).astype(np.int32)
            k = rng.standard_normal((cu[-1], hkv, d)).astype(np.float32)
            v = rng.standard_normal((cu[-1], hkv, d)).astype(np.float32)
            acc = [int(rng.integers(0, dl + 1)) for dl in deltas] if rng.random() < 0.3 else None
            cells = dk.kv_reserve(p, chosen, cu, acc)
            for b, s in enumerate(chosen):
                cnt = deltas[b] if acc is None else acc[b]
                lo = cu[b]
                assert (cells[lo:lo + cnt] >= 0).all() and (cells[lo + cnt:cu[b + 1]] == -1).all()
                arena_k[cells[lo:lo + cnt]] = k[lo:lo + cnt]
                arena_v[cells[lo:lo + cnt]] = v[lo:lo + cnt]
                o.append(s, k[lo:lo + cnt], v[lo:lo + cnt])
        elif op == "alias" and len(live) >= 2:
            donor, dst = [int(x) for x in rng.permutation(list(live))[:2]]
            m = int(rng.integers(0, o.length(donor) + 1))
            want = "OK"
            try:
                o.alias(donor, dst, 0, m)
            except OracleError as e:
                want = e.status
            assert dk.STATUS_NAMES[dk.lib().dk_seq_alias(p, donor, dst, 0, m)] == want
        elif op == "trim":
            s = int(rng.choice(list(live)))
            new_len = int(rng.integers(0, o.length(s) + 1))
            o.trim(s, new_len)
            dk.seq_trim(p, s, new_len)
        elif op == "release":
            s = int(rng.choice(list(live)))
            o.release(s)
            dk.seq_release(p, s)
            del live[s]
        # every live slot: same length, same logical bytes, alias sharing mirrored exactly
        if op == "verify" or step % 25 == 0:
            ids = {}
            for s in live:
                assert dk.seq_len(p, s) == o.length(s)
                cells = dk.seq_cells(p, s)
                ko, vo = o.gather(s)
                if ko is not None:
                    assert np.array_equal(arena_k[cells], ko) and np.array_equal(arena_v[cells], vo)
                for c, oid in zip(cells, o.cell_ids(s)):
                    assert ids.setdefault(int(c), oid) == oid  # same cell <=> same oracle cell object
            assert len(set(ids.values())) == len(ids)
            held, free = dk.pool_stats(p)
            assert held + free == arena_cells and held >= len(ids)
    dk.pool_destroy(p)


def test_long_extents_under_interleaved_growth():
    # many slots growing in lockstep should still end up with long contiguous runs
    p = _pool(n_slots=16, arena_cells=16 * 4096, granule=64)
    s = [dk.seq_acquire(p, 0) for _ in range(16)]
    for _ in range(30):
        dk.kv_reserve(p, s, np.arange(17) * 100)
    runs = []
    for x in s:
        c = dk.seq_cells(p, x)
        runs.append(1 + int((np.diff(c) != 1).sum()))
    assert max(runs) <= 8, runs
    dk.pool_destroy(p)


def test_trim_batch_is_all_or_nothing():
    p = _pool(n_slots=4, arena_cells=4096)
    a, b, c = (dk.seq_acquire(p, 0) for _ in range(3))
    dk.kv_reserve(p, [a, b, c], [0, 50, 90, 100])
    dk.seq_trim_batch(p, [a, c], [20, 0])
    assert [dk.seq_len(p, s) for s in (a, b, c)] == [20, 40, 0]
    for slots, lens, err in (([a, b], [10, 41], "INVALID"), ([a, a], [1, 2], "DUP_SLOT"), ([a, 3], [1, 0], "NO_SLOT")):
        with pytest.raises(dk.DeltaKVError) as e:
            dk.seq_trim_batch(p, slots, lens)
        assert e.value.name == err
        assert [dk.seq_len(p, s) for s in (a, b, c)] == [20, 40, 0]   # nothing moved
    dk.seq_trim_batch(p, [], [])
    dk.pool_destroy(p)
