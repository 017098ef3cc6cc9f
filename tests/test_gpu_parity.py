"""GPU parity: the HIP library against the fp64 oracle on the same seeded inputs (needs an MI355X).

Tolerances (bf16 inputs, fp32 accumulation): max abs error <= 1e-2 and max error relative to
max(|oracle|, rms of the oracle row) <= 2e-2; fp32 pools: max abs <= 1e-4.  Bookkeeping (append
placement, aliasing, trim) is compared bit for bit.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26289_amd import binding as dk
from paper_2605_26289_amd import workloads as wl
from gpu_util import Mirror, check_close, to_dev

pytestmark = pytest.mark.gpu

SMALL = wl.Shape(8, 2, 128, "bf16")


def _run_turns(w: wl.Workload, granule=0, variant=0, check_every=1):
    """Plays a workload turn by turn (append then attend, or staged attend then append) against the oracle."""
    sh = w.shape
    m = Mirror(sh, w.n_slots, w.cells_needed() + (granule or 256) * (w.n_slots + 2), granule, seed=w.seed)
    dk.set_attend_variant(m.pool.handle, variant)
    slots = [m.acquire() for _ in range(w.n_slots)]
    if w.alias_prefix:
        m.append([slots[0]], [w.alias_prefix])
        for s in slots[1:]:
            m.alias(slots[0], s, w.alias_prefix)
    for s, h in zip(slots, w.history):
        if h:
            m.append([s], [h])
    worst = (0.0, 0.0)
    for ti, t in enumerate(w.turns):
        for s, n in zip(t.slots, t.n_past):
            assert m.pool.length(s) == n
        total = sum(t.delta)
        q = m.draw(total, sh.n_q_heads)
        if not t.staged:
            m.append(t.slots, t.delta)
            out, lse, cu = m.attend_appended(t.slots, t.delta, q, lse=True)
            if ti % check_every == 0 or ti == len(w.turns) - 1:
                ref, ref_lse = m.oracle_appended(t.slots, t.delta, q)
                a, r = check_close(out, ref, sh.dtype, f"{w.name} turn {ti}")
                worst = (max(worst[0], a), max(worst[1], r))
                assert np.abs(lse.cpu().numpy() - ref_lse).max() < 2e-3
        else:
            kn, vn = m.draw(total, sh.n_kv_heads), m.draw(total, sh.n_kv_heads)
            cu = np.concatenate([[0], np.cumsum(t.delta)]).astype(np.int32)
            knd, vnd = to_dev(kn, sh.dtype), to_dev(vn, sh.dtype)
            out = m.pool.attend(t.slots, cu, to_dev(q, sh.dtype), sh.scale, knd, vnd)
            caches = [m.cache(s) for s in t.slots]
            ref, _ = oracle.delta_attend_batch(q, caches, kn, vn, cu, sh.scale)
            a, r = check_close(out, ref, sh.dtype, f"{w.name} staged turn {ti}")
            worst = (max(worst[0], a), max(worst[1], r))
            m.append(t.slots, t.delta, kn, vn, n_accept=t.n_accept)
            for s in t.slots[:4]:
                m.check_gather(s)
    m.pool.close()
    return worst


def test_kv_append_gather_bit_exact_with_alias_and_trim():
    m = Mirror(SMALL, 4, 4096, granule=16, seed=1)
    a, b, c, d = (m.acquire() for _ in range(4))
    m.append([a], [100])
    m.alias(a, b, 70)
    m.append([a, b, c], [13, 40, 5])
    m.alias(b, d, 90)
    m.append([d, a], [33, 1], n_accept=[20, 0])
    m.trim(a, 50)
    m.append([a], [29])
    for s in (a, b, c, d):
        m.check_gather(s)
    assert np.array_equal(m.pool.cells(b)[:70], m.pool.cells(d)[:70])
    m.pool.close()


@pytest.mark.parametrize("variant", [0, 1])
def test_config1_fp32_single_session(variant):
    a, r = _run_turns(wl.config1(), variant=variant)
    assert a <= 1e-4


@pytest.mark.parametrize("variant", [0, 1])
def test_config2_five_turn_agent(variant):
    _run_turns(wl.config2(), variant=variant)


@pytest.mark.parametrize("variant", [0, 1])
def test_config3_scaled_coding_workflow(variant):
    # same 35-turn structure at 1/8 of the lengths: the oracle finishes in seconds
    _run_turns(wl.scaled(wl.config3(), 0.125), variant=variant, check_every=6)


@pytest.mark.parametrize("variant", [0, 1])
def test_config4_scaled_multi_agent_alias(variant):
    _run_turns(wl.scaled(wl.config4(), 0.125), granule=64, variant=variant)


def test_scaled_configs_keep_the_production_head_shape():
    """Configs 3-5 are checked on every row at 1/8 of their lengths but with the production heads (32 query heads on
    8 KV heads), so the tile kernel's "workgroup id mod 8 = KV head" mapping, the levelled chains and the merge are
    covered row by row, not on a sample."""
    for w in (wl.scaled(wl.config3(), 0.125), wl.scaled(wl.config4(), 0.125), wl.scaled(wl.config5(n_slots=16), 0.125)):
        assert (w.shape.n_q_heads, w.shape.n_kv_heads, w.shape.head_dim) == (32, 8, 128)


@pytest.mark.parametrize("variant", [0, 1])
def test_config5_scaled_spec_verify(variant):
    _run_turns(wl.scaled(wl.config5(n_slots=16), 0.125), variant=variant)


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("n,delta", [(0, 1), (0, 5), (1, 1), (63, 1), (64, 2), (65, 16), (200, 17), (3, 70), (0, 300),
                                     (129, 64), (1000, 9), (257, 130), (0, 20), (31, 21), (200, 24), (1000, 22)])
def test_edge_shapes_appended_and_staged_agree_with_oracle(n, delta, variant):
    sh = SMALL
    m = Mirror(sh, 2, 4096, granule=16, seed=n * 1000 + delta)
    dk.set_attend_variant(m.pool.handle, variant)
    s, t = m.acquire(), m.acquire()
    if n:
        k0, v0, _ = m.append([s], [n])
        m.append([t], [n], k0, v0)
    q = m.draw(delta, sh.n_q_heads)
    kn, vn = m.draw(delta, sh.n_kv_heads), m.draw(delta, sh.n_kv_heads)
    # staged on slot s
    out_s = m.pool.attend([s], [0, delta], to_dev(q, sh.dtype), sh.scale, to_dev(kn, sh.dtype), to_dev(vn, sh.dtype))
    ref, _ = oracle.delta_attend(q, *m.cache(s), kn, vn, sh.scale)
    check_close(out_s, ref, sh.dtype, "staged", row_scaled=True)
    # appended on slot t
    m.append([t], [delta], kn, vn)
    out_a, _, _ = m.attend_appended([t], [delta], q)
    check_close(out_a, ref, sh.dtype, "appended", row_scaled=True)
    m.pool.close()


@pytest.mark.parametrize("variant", [0, 1])
def test_varlen_batch_with_empty_entries_and_mixed_delta(variant):
    sh = SMALL
    m = Mirror(sh, 6, 8192, granule=32, seed=7)
    dk.set_attend_variant(m.pool.handle, variant)
    slots = [m.acquire() for _ in range(6)]
    hist = [0, 300, 77, 1200, 5, 640]
    for s, h in zip(slots, hist):
        if h:
            m.append([s], [h])
    deltas = [3, 0, 129, 1, 0, 40]
    order = [3, 1, 5, 0, 4, 2]
    sl = [slots[i] for i in order]
    dl = [deltas[i] for i in order]
    q = m.draw(sum(dl), sh.n_q_heads)
    m.append(sl, dl)
    out, lse, cu = m.attend_appended(sl, dl, q, lse=True)
    ref, ref_lse = m.oracle_appended(sl, dl, q)
    check_close(out, ref, sh.dtype, "varlen", row_scaled=True)
    assert np.abs(lse.cpu().numpy() - ref_lse).max() < 2e-3
    m.pool.close()


@pytest.mark.parametrize("variant", [0, 1])
def test_rows_sum_to_one_and_dominant_key(variant):
    sh = SMALL
    m = Mirror(sh, 1, 8192, seed=3)
    dk.set_attend_variant(m.pool.handle, variant)
    s = m.acquire()
    n, delta = 3000, 33
    k = m.draw(n + delta, sh.n_kv_heads)
    v = np.ones_like(k)
    m.append([s], [n + delta], k, v)
    q = m.draw(delta, sh.n_q_heads)
    out, _, _ = m.attend_appended([s], [delta], q)
    assert np.abs(out.float().cpu().numpy() - 1.0).max() <= 2 ** -7  # softmax weights sum to 1
    m.pool.close()


def test_aliased_prefix_reads_equal_private_copy():
    sh = SMALL
    m = Mirror(sh, 3, 8192, granule=64, seed=11)
    a, b, c = (m.acquire() for _ in range(3))
    k0, v0, _ = m.append([a], [700])
    m.alias(a, b, 650)
    m.append([c], [650], k0[:650], v0[:650])  # private copy of the same rows
    delta = 20
    kn, vn = m.draw(delta, sh.n_kv_heads), m.draw(delta, sh.n_kv_heads)
    m.append([b, c], [delta, delta], np.concatenate([kn, kn]), np.concatenate([vn, vn]))
    q = m.draw(delta, sh.n_q_heads)
    out, _, _ = m.attend_appended([b, c], [delta, delta], np.concatenate([q, q]))
    # same logical rows through different physical extents: tile boundaries differ, so the two
    # results may differ by summation order only
    ref, _ = m.oracle_appended([b, c], [delta, delta], np.concatenate([q, q]))
    check_close(out, ref, sh.dtype, "alias vs private")
    assert np.array_equal(ref[:delta], ref[delta:])
    # The two evaluations round their weights against different reference maxima and sum in a different order, so
    # before the bf16 store they differ by a few 2^-9-relative terms; after it they are the same bf16 value or
    # neighbouring ones.  With 650+ keys every |o| here is below 0.5, where neighbouring bf16 values are at most
    # 2^-9 = 1.95e-3 apart: the bound is "one bf16 step at the outputs' magnitude".
    assert np.abs(ref).max() < 0.5
    assert (out[:delta].float() - out[delta:].float()).abs().max().item() <= 2.0 ** -9
    m.pool.close()


def test_chunked_delta_equals_one_call_within_tolerance():
    sh = SMALL
    m = Mirror(sh, 2, 8192, seed=13)
    s, t = m.acquire(), m.acquire()
    k0, v0, _ = m.append([s], [500])
    m.append([t], [500], k0, v0)
    delta = 96
    q = m.draw(delta, sh.n_q_heads)
    kn, vn = m.draw(delta, sh.n_kv_heads), m.draw(delta, sh.n_kv_heads)
    m.append([s], [delta], kn, vn)
    whole, _, _ = m.attend_appended([s], [delta], q)
    parts = []
    for i in range(0, delta, 32):
        m.append([t], [32], kn[i:i + 32], vn[i:i + 32])
        o, _, _ = m.attend_appended([t], [32], q[i:i + 32])
        parts.append(o)
    ref, _ = m.oracle_appended([s], [delta], q)
    check_close(whole, ref, sh.dtype, "whole")
    check_close(torch.cat(parts), ref, sh.dtype, "chunked")
    m.pool.close()


def test_errors_from_gpu_entry_points():
    sh = SMALL
    m = Mirror(sh, 2, 1024, granule=16, seed=17)
    s = m.acquire()
    m.append([s], [10])
    q = to_dev(m.draw(20, sh.n_q_heads), sh.dtype)
    out = torch.empty_like(q)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(dk.DeltaKVError, match="INVALID"):  # appended mode with delta > len
        dk.delta_attend(m.pool.handle, [s], [0, 20], q, out, sh.scale, workspace=ws)
    with pytest.raises(dk.DeltaKVError, match="WORKSPACE"):
        dk.delta_attend(m.pool.handle, [s], [0, 5], q, out, sh.scale, workspace=None)
    with pytest.raises(dk.DeltaKVError, match="DUP_SLOT"):
        dk.delta_attend(m.pool.handle, [s, s], [0, 2, 4], q, out, sh.scale, workspace=ws)
    with pytest.raises(dk.DeltaKVError, match="NO_CELLS"):
        big = to_dev(m.draw(2000, sh.n_kv_heads), sh.dtype)
        dk.kv_append(m.pool.handle, [s], [0, 2000], big, big)
    assert m.pool.length(s) == 10
    m.check_gather(s)
    m.pool.close()


@pytest.mark.parametrize("delta", [4, 9, 22, 300])
def test_growing_scores_exercise_the_lazy_rescale(delta):
    """Keys whose scores keep outgrowing the reference maximum (by far more than the rescale slack, several
    times along the prefix, and again inside the new block): the deferred O rescale of the tile kernel and the
    conditional rescale of the stream kernel (one, two and three row blocks) must both land on the oracle's
    result."""
    sh = SMALL
    m = Mirror(sh, 1, 8192, seed=23)
    s = m.acquire()
    n = 1500
    rng = np.random.default_rng(23)
    k = m.draw(n + delta, sh.n_kv_heads)
    v = m.draw(n + delta, sh.n_kv_heads)
    q = m.draw(delta, sh.n_q_heads)
    # a common direction u: keys carry a staircase of it (steps every ~190 positions, plus a final step among the
    # new tokens), queries a positive multiple, so the row maxima climb by ~15 log2 units per step
    u = wl.round_to_bf16(rng.standard_normal(sh.head_dim).astype(np.float32))
    u /= np.linalg.norm(u)
    step = (np.arange(n + delta) // 190).astype(np.float32)
    k = wl.round_to_bf16(k + (step * 3.0)[:, None, None] * u[None, None, :])
    q = wl.round_to_bf16(q + 40.0 * u[None, None, :])
    m.append([s], [n + delta], k, v)
    out, lse, _ = m.attend_appended([s], [delta], q, lse=True)
    ref, ref_lse = m.oracle_appended([s], [delta], q)
    check_close(out, ref, sh.dtype, "growing scores", row_scaled=True)
    assert np.abs(lse.cpu().numpy() - ref_lse).max() < 5e-3 * max(1.0, np.abs(ref_lse).max() / 10)
    m.pool.close()


def test_split_chunks_with_rows_that_see_nothing_of_a_chunk():
    """A long prefix forces the planner to split the keys; with a diagonal inside the last chunk some rows of a
    row tile see none of that chunk's keys (their partial is empty) and the merge must ignore it."""
    sh = SMALL
    m = Mirror(sh, 1, 1 << 15, seed=29)
    s = m.acquire()
    n, delta = 9000, 200
    m.append([s], [n])
    kn, vn = m.draw(delta, sh.n_kv_heads), m.draw(delta, sh.n_kv_heads)
    q = m.draw(delta, sh.n_q_heads)
    out_s = m.pool.attend([s], [0, delta], to_dev(q, sh.dtype), sh.scale, to_dev(kn, sh.dtype), to_dev(vn, sh.dtype))
    ref, _ = oracle.delta_attend(q, *m.cache(s), kn, vn, sh.scale)
    check_close(out_s, ref, sh.dtype, "split, staged")
    m.pool.close()


@pytest.mark.parametrize("hq,hkv", [(4, 4), (4, 2), (16, 2), (16, 1), (6, 2)])
@pytest.mark.parametrize("n,delta", [(300, 3), (500, 6), (700, 100), (40, 260)])
def test_group_sizes_from_mha_to_sixteen_heads_per_kv_head(hq, hkv, n, delta):
    """G = Hq/Hkv of 1, 2, 8, 16 (MFMA kernels, rows packed G per token) and 3 (not a power of two: reference kernel)."""
    sh = wl.Shape(hq, hkv, 128, "bf16")
    m = Mirror(sh, 2, 4096, granule=32, seed=hq * 100 + hkv * 10 + delta)
    s = m.acquire()
    m.append([s], [n])
    kn, vn = m.draw(delta, hkv), m.draw(delta, hkv)
    q = m.draw(delta, hq)
    out = m.pool.attend([s], [0, delta], to_dev(q, "bf16"), sh.scale, to_dev(kn, "bf16"), to_dev(vn, "bf16"))
    ref, _ = oracle.delta_attend(q, *m.cache(s), kn, vn, sh.scale)
    check_close(out, ref, "bf16", f"G={hq // hkv}", row_scaled=True)
    m.pool.close()


@pytest.mark.parametrize("n,delta", [(1000, 9), (900, 21), (777, 200), (130, 70)])
def test_cells_outside_the_slot_never_reach_the_result(n, delta):
    """Arena canary: every cell the slots do not own holds NaN.  Ragged tiles, clamped rows, the dummy loads past
    the end of a key range and aliased prefixes must only ever touch owned cells, or the output turns NaN."""
    sh = SMALL
    m = Mirror(sh, 3, 8192, granule=16, seed=31)
    m.pool.k_arena.fill_(float("nan"))
    m.pool.v_arena.fill_(float("nan"))
    a, b = m.acquire(), m.acquire()
    m.append([a], [n])
    m.alias(a, b, n - 37)            # b reads a's cells up to an unaligned boundary, then its own
    m.append([b], [61])
    kn, vn = m.draw(2 * delta, sh.n_kv_heads), m.draw(2 * delta, sh.n_kv_heads)
    q = m.draw(2 * delta, sh.n_q_heads)
    out = m.pool.attend([a, b], [0, delta, 2 * delta], to_dev(q, sh.dtype), sh.scale, to_dev(kn, sh.dtype), to_dev(vn, sh.dtype))
    assert torch.isfinite(out.float()).all()
    ref_a, _ = oracle.delta_attend(q[:delta], *m.cache(a), kn[:delta], vn[:delta], sh.scale)
    ref_b, _ = oracle.delta_attend(q[delta:], *m.cache(b), kn[delta:], vn[delta:], sh.scale)
    check_close(out, np.concatenate([ref_a, ref_b]), sh.dtype, "canary", row_scaled=True)
    m.append([a, b], [delta, delta], kn, vn)   # appended mode reads the same cells back
    out2, _, _ = m.attend_appended([a, b], [delta, delta], q)
    check_close(out2, np.concatenate([ref_a, ref_b]), sh.dtype, "canary appended", row_scaled=True)
    m.pool.close()


def test_sequence_guard_returns_the_slot_on_every_exit_path():
    m = Mirror(SMALL, 1, 1024, granule=16, seed=37)
    with m.pool.sequence() as s:
        m.pool.append([s], [0, 5], to_dev(m.draw(5, SMALL.n_kv_heads), "bf16"), to_dev(m.draw(5, SMALL.n_kv_heads), "bf16"))
        with pytest.raises(dk.DeltaKVError, match="TIMEOUT"):
            m.pool.acquire()                       # the only slot is taken
    with pytest.raises(RuntimeError, match="boom"):
        with m.pool.sequence() as s2:
            assert s2 == s and m.pool.length(s2) == 0  # released and recycled empty
            raise RuntimeError("boom")
    assert m.pool.acquire() == s                   # the exception path released it too
    m.pool.close()


def test_attend_timing_ring_keeps_the_last_calls_in_order():
    """The per-call kernel timer: n recorded calls give n positive durations, oldest first, and the
    ring keeps only the most recent ones; a larger batch takes longer than a tiny one."""
    m = Mirror(SMALL, 2, 16384, seed=41)
    a, b = m.acquire(), m.acquire()
    m.append([a, b], [6000, 40])
    h = m.pool.handle
    with pytest.raises(dk.DeltaKVError):
        dk.last_attend_ms(h)  # recording is off: nothing to report
    dk.set_attend_timing(h, 3)
    q_big, q_small = m.draw(512, SMALL.n_q_heads), m.draw(1, SMALL.n_q_heads)
    m.attend_appended([b], [1], q_small)  # warm-up, will be pushed out of the ring
    for slots, deltas, q in (([a], [512], q_big), ([b], [1], q_small), ([a], [512], q_big)):
        m.attend_appended(slots, deltas, q)
    ms = dk.attend_times(h)
    assert ms.shape == (3,) and (ms > 0).all()
    assert ms[0] > ms[1] and ms[2] > ms[1]
    assert dk.last_attend_ms(h) == pytest.approx(float(ms[2]))
    assert dk.attend_times(h, cap=2).tolist() == pytest.approx(ms[1:].tolist())
    dk.set_attend_timing(h, 0)
    assert dk.attend_times(h).size == 0
    m.pool.close()


@pytest.mark.parametrize("n_slots,n_hi", [(300, 400), (1400, 90)])
def test_many_small_slots_walk_chains_of_units(n_slots, n_hi):
    """More (slot, KV head) units than compute units: each streaming workgroup walks a chain of them (600
    units: two or three each; 2800 units: handed out in blocks).  Every slot's rows must still come out right."""
    rng = np.random.default_rng(n_slots)
    m = Mirror(SMALL, n_slots, n_slots * (n_hi + 8) + 4096, granule=16, seed=n_slots)
    slots = [m.acquire() for _ in range(n_slots)]
    hist = rng.integers(0, n_hi + 1, size=n_slots).tolist()
    live = [s for s, h in zip(slots, hist) if h]
    m.append(live, [h for h in hist if h])
    deltas = rng.integers(0, 4, size=n_slots).tolist()  # decode, short verify steps and idle slots mixed
    deltas[0], deltas[-1] = 3, 1
    q = m.draw(sum(deltas), SMALL.n_q_heads)
    m.append(slots, deltas)
    out, lse, _ = m.attend_appended(slots, deltas, q, lse=True)
    ref, ref_lse = m.oracle_appended(slots, deltas, q)
    check_close(out, ref, SMALL.dtype, f"{n_slots} slots")
    assert np.abs(lse.cpu().numpy() - ref_lse).max() < 2e-3
    m.pool.close()


APPEND_ATTEND_CASES = {
    # name: (shape, histories, deltas of two turns)
    "tile": (wl.PRODUCTION, [900, 0, 3000], [[300, 70, 129], [64, 17, 700]]),
    "stream": (wl.PRODUCTION, [5, 0, 2100, 333, 64], [[9, 1, 16, 0, 3], [1, 1, 9, 2, 0]]),
    "mixed": (SMALL, [1200, 40, 0, 700], [[400, 1, 3, 16], [2, 260, 9, 0]]),
    "fp32 reference path": (wl.Shape(4, 2, 64, "f32"), [200, 0, 31], [[150, 3, 1], [1, 40, 0]]),
    "long single turn": (wl.PRODUCTION, [0], [[1500], [1100]]),
    # small calls: the copy is folded into the tile kernel, the stream kernel, and the first of both
    "small tile turn": (wl.PRODUCTION, [800], [[150], [150]]),
    "small stream step": (wl.PRODUCTION, [700, 0, 64], [[9, 1, 4], [1, 9, 16]]),
    "small tile and stream": (SMALL, [300, 20], [[40, 2], [3, 70]]),
    "small stream step, three row blocks": (wl.PRODUCTION, [700, 0, 2000], [[24, 1, 17], [9, 21, 20]]),
}


@pytest.mark.parametrize("case", sorted(APPEND_ATTEND_CASES))
def test_append_attend_is_append_then_attend(case):
    """dk_append_attend against dk_kv_append + dk_delta_attend on a twin pool fed the same rows: results against the
    oracle, then lengths, cell numbers and the gathered arena contents of every slot bit for bit."""
    sh, hist, turns = APPEND_ATTEND_CASES[case]
    cells = sum(hist) + sum(sum(t) for t in turns) + len(hist) * 600 + 1024
    fused, plain = Mirror(sh, len(hist), cells, granule=64, seed=5), Mirror(sh, len(hist), cells, granule=64, seed=5)
    slots = [fused.acquire() for _ in hist]
    assert slots == [plain.acquire() for _ in hist]
    for m in (fused, plain):
        m.append([s for s, h in zip(slots, hist) if h], [h for h in hist if h])
    for turn, deltas in enumerate(turns):
        q = fused.draw(sum(deltas), sh.n_q_heads)
        plain.draw(sum(deltas), sh.n_q_heads)  # keep the twin's generator in step
        out_f, lse_f, _ = fused.append_attend(slots, deltas, q, lse=True)
        plain.append(slots, deltas)
        out_p, lse_p, _ = plain.attend_appended(slots, deltas, q, lse=True)
        ref, ref_lse = fused.oracle_appended(slots, deltas, q)
        check_close(out_f, ref, sh.dtype, f"{case} turn {turn} fused", row_scaled=True)
        check_close(out_p, ref, sh.dtype, f"{case} turn {turn} plain", row_scaled=True)
        assert np.abs(lse_f.cpu().numpy() - ref_lse).max() < 2e-3
        for s in slots:
            assert fused.pool.length(s) == plain.pool.length(s)
            assert np.array_equal(dk.seq_cells(fused.pool.handle, s), dk.seq_cells(plain.pool.handle, s))
            fused.check_gather(s)
            kf, vf = fused.pool.gather(s)
            kp, vp = plain.pool.gather(s)
            assert torch.equal(kf, kp) and torch.equal(vf, vp)
    fused.pool.close()
    plain.pool.close()


def test_append_attend_that_does_not_fit_changes_nothing():
    sh = SMALL
    m = Mirror(sh, 2, 512, granule=64, seed=1)
    a, b = m.acquire(), m.acquire()
    m.append([a, b], [100, 50])
    deltas = [300, 200]  # 500 more cells than the arena has left
    cu = np.concatenate([[0], np.cumsum(deltas)]).astype(np.int32)
    q = to_dev(m.draw(sum(deltas), sh.n_q_heads), sh.dtype)
    k = to_dev(m.draw(sum(deltas), sh.n_kv_heads), sh.dtype)
    with pytest.raises(dk.DeltaKVError, match="NO_CELLS"):
        m.pool.append_attend([a, b], cu, q, k, k, sh.scale)
    assert (m.pool.length(a), m.pool.length(b)) == (100, 50)
    m.check_gather(a)
    m.check_gather(b)
    with pytest.raises(dk.DeltaKVError, match="INVALID"):  # the new rows are required
        dk.append_attend(m.pool.handle, [a], [0, 4], q, None, None, torch.empty_like(q), sh.scale, None,
                         m.pool.ensure_workspace([a], [0, 4], 2))
    m.pool.close()


def test_busy_staging_ring_and_the_matching_wait():
    """Two staging buffers and calls whose descriptors need an upload: a launching call that finds both buffers in
    flight reports BUSY and enqueues nothing; after dk_staging_wait the same call goes through, and the results of
    all calls are right.  (Whether BUSY shows up depends on how far the host gets ahead of the device, so it is
    provoked with a long queue, but only its consequences are asserted.)"""
    from paper_2605_26289_amd import DevicePool
    sh = wl.PRODUCTION
    n_slots, n = 96, 3000
    pool = DevicePool(n_slots, n_slots * (n + 512), sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype, staging_depth=2)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    slots = [pool.acquire() for _ in range(n_slots)]
    kv = torch.randn((n, sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    for s_ in slots:
        pool.append([s_], [0, n], kv, kv)
    cu = np.arange(n_slots + 1, dtype=np.int32) * 3
    q = torch.randn((int(cu[-1]), sh.n_q_heads, sh.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    kn = torch.randn((int(cu[-1]), sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
    ws = pool.ensure_workspace(slots, cu, True)
    outs = [torch.empty_like(q) for _ in range(24)]
    s_arr, s_p = dk._i32(slots)
    c_arr, c_p = dk._i32(cu)
    busy = 0
    torch.cuda.synchronize()
    for out in outs:
        call = lambda: dk.lib().dk_delta_attend(pool.handle, n_slots, s_p, c_p, q.data_ptr(), kn.data_ptr(), kn.data_ptr(),  # noqa: E731
                                                float(sh.scale), out.data_ptr(), None, ws.data_ptr(), ws.numel(), None)
        rc = call()
        if rc == dk.BUSY:
            busy += 1
            dk.staging_wait(pool.handle)
            rc = call()  # the buffer this call takes is free now, whatever else is still queued
        assert rc == 0, rc
    torch.cuda.synchronize()
    for out in outs[1:]:
        assert torch.equal(out, outs[0])
    print(f"[busy] {busy} of {len(outs)} calls found the ring full")
    pool.close()


def test_queued_and_planned_units_give_identical_bits():
    """Which workgroup computes a streaming unit -- drawn from the run-time queue, or walked in a chain planned on the
    host -- has no influence on the unit's result: the same batch under both settings, bit for bit."""
    sh = wl.PRODUCTION
    rng = np.random.default_rng(31)
    n_slots = 200  # 1600 units: queued by default
    m = Mirror(sh, n_slots, n_slots * 700 + 4096, granule=64, seed=3)
    slots = [m.acquire() for _ in range(n_slots)]
    hist = rng.integers(1, 600, size=n_slots).tolist()
    m.append(slots, hist)
    deltas = rng.integers(1, 10, size=n_slots).tolist()
    q = m.draw(sum(deltas), sh.n_q_heads)
    m.append(slots, deltas)
    out_q, _, _ = m.attend_appended(slots, deltas, q)
    dk.set_tuning(m.pool.handle, "stream_queue", 0)
    out_c, _, _ = m.attend_appended(slots, deltas, q)
    dk.set_tuning(m.pool.handle, "stream_queue", 1)
    out_q2, _, _ = m.attend_appended(slots, deltas, q)
    assert torch.equal(out_q, out_c) and torch.equal(out_q, out_q2)
    ref, _ = m.oracle_appended(slots, deltas, q)
    check_close(out_q, ref, sh.dtype, "queued units", row_scaled=True)
    m.pool.close()


def test_rows_between_the_kernels_limits_agree_with_the_oracle_in_both_kernels():
    """Sequences of 65 to 96 packed rows go to the streaming kernel by default and to the tile kernel when the
    limit is tuned down: both must land on the oracle's result (and within twice the tolerance of each other)."""
    sh = wl.PRODUCTION
    group = sh.n_q_heads // sh.n_kv_heads
    rng = np.random.default_rng(47)
    n_slots = 24
    m = Mirror(sh, n_slots, n_slots * 2300 + 4096, granule=64, seed=47)
    slots = [m.acquire() for _ in range(n_slots)]
    hist = rng.integers(1, 2200, size=n_slots).tolist()
    m.append(slots, hist)
    deltas = rng.integers(64 // group + 1, 96 // group + 1, size=n_slots).tolist()
    q = m.draw(sum(deltas), sh.n_q_heads)
    m.append(slots, deltas)
    out_s, lse_s, _ = m.attend_appended(slots, deltas, q, lse=True)
    dk.set_tuning(m.pool.handle, "stream_rows", 64)
    out_t, lse_t, _ = m.attend_appended(slots, deltas, q, lse=True)
    dk.set_tuning(m.pool.handle, "stream_rows", 96)
    ref, ref_lse = m.oracle_appended(slots, deltas, q)
    check_close(out_s, ref, sh.dtype, "streaming kernel, three row blocks", row_scaled=True)
    check_close(out_t, ref, sh.dtype, "tile kernel, fewer than 97 rows", row_scaled=True)
    assert np.abs(lse_s.cpu().numpy() - ref_lse).max() < 2e-3 and np.abs(lse_t.cpu().numpy() - ref_lse).max() < 2e-3
    m.pool.close()


@pytest.mark.parametrize("seed", range(6))
def test_chains_of_streaming_units_with_one_two_and_three_row_blocks(seed):
    """Hundreds of slots with Delta from 0 up to the streaming kernel's limit (96 packed rows: its three-block form,
    with narrower units beside the widest), then up to 64 and up to 32 rows (the two-block and one-block forms),
    short and long histories: every workgroup changes units many times, each change overlapping the next unit's
    first requests with the merge of the finished one."""
    rng = np.random.default_rng(77000 + seed)
    sh = (SMALL, wl.PRODUCTION, wl.Shape(16, 4, 128, "bf16"))[seed % 3]
    group = sh.n_q_heads // sh.n_kv_heads
    n_slots = min(int(rng.integers(40, 700)), 250 if sh is wl.PRODUCTION else 700)
    n_hi = int(rng.choice([30, 90, 400, 1500]))
    m = Mirror(sh, n_slots, n_slots * (n_hi + 60 + 2 * 64) + 4096, granule=int(rng.choice([16, 64])), seed=seed)
    slots = [m.acquire() for _ in range(n_slots)]
    hist = rng.integers(0, n_hi + 1, size=n_slots).tolist()
    m.append([s for s, h in zip(slots, hist) if h], [h for h in hist if h])
    for turn in range(3):
        deltas = rng.integers(0, (96, 64, 32)[turn] // group + 1, size=n_slots).tolist()
        q = m.draw(sum(deltas), sh.n_q_heads)
        m.append(slots, deltas)
        out, lse, _ = m.attend_appended(slots, deltas, q, lse=True)
        ref, ref_lse = m.oracle_appended(slots, deltas, q)
        check_close(out, ref, sh.dtype, f"seed {seed} turn {turn}", row_scaled=True)
        assert np.abs(lse.cpu().numpy() - ref_lse).max() < 2e-3
    m.pool.close()


@pytest.mark.parametrize("seed", range(10))
def test_random_batches_match_the_oracle(seed):
    """Seeded random batch structures: slot count, histories (some grown over several appends and trimmed back,
    some behind an aliased prefix), per-slot Delta from decode to several row tiles, idle slots, granule size,
    staged or appended mode, two consecutive turns.  Whatever the planner makes of them -- row tiles, key chunks,
    merge records, chains of streaming units -- every output row must match the oracle."""
    rng = np.random.default_rng(9000 + seed)
    sh = (wl.Shape(16, 4, 128, "bf16"), SMALL, wl.PRODUCTION)[seed % 3]
    n_slots = int(rng.integers(1, 13))
    granule = int(rng.choice([16, 64, 256]))
    hist = [int(rng.choice([0, rng.integers(1, 200), rng.integers(200, 3000), rng.integers(3000, 9000)])) for _ in range(n_slots)]
    prefix = int(rng.integers(1, 700)) if n_slots > 1 and rng.random() < 0.6 else 0
    m = Mirror(sh, n_slots, sum(hist) + prefix + n_slots * (2 * granule + 2100) + 4096, granule=granule, seed=seed)
    slots = [m.acquire() for _ in range(n_slots)]
    if prefix:
        m.append([slots[0]], [prefix])
        for s in slots[1:]:
            if rng.random() < 0.7:
                m.alias(slots[0], s, int(rng.integers(1, prefix + 1)))
    for s, h in zip(slots, hist):
        for part in np.diff(np.concatenate([[0], np.sort(rng.integers(0, h + 1, size=2)), [h]])).tolist():
            if part:
                m.append([s], [int(part)])
        if h > 10 and rng.random() < 0.3:
            m.trim(s, m.pool.length(s) - int(rng.integers(1, 10)))
    choices = [0, 1, 1, 2, 5, 9, 16, 17, 21, 24, 25, 40, 64, 65, 130, 300, 700, 1030]
    for turn in range(2):
        order = rng.permutation(n_slots).tolist()
        sl = [slots[i] for i in order]
        dl = [int(rng.choice(choices)) for _ in sl]
        if sum(dl) == 0:
            dl[0] = 3
        total = sum(dl)
        q = m.draw(total, sh.n_q_heads)
        kn, vn = m.draw(total, sh.n_kv_heads), m.draw(total, sh.n_kv_heads)
        cu = np.concatenate([[0], np.cumsum(dl)]).astype(np.int32)
        if rng.random() < 0.5:  # staged: attend first, then append what was accepted
            out = m.pool.attend(sl, cu, to_dev(q, sh.dtype), sh.scale, to_dev(kn, sh.dtype), to_dev(vn, sh.dtype))
            ref, _ = oracle.delta_attend_batch(q, [m.cache(s) for s in sl], kn, vn, cu, sh.scale)
            check_close(out, ref, sh.dtype, f"seed {seed} turn {turn} staged", row_scaled=True)
            m.append(sl, dl, kn, vn, n_accept=[int(rng.integers(0, d + 1)) for d in dl])
        elif (seed + turn) % 2:  # both at once: dk_append_attend
            lse = torch.empty((total, sh.n_q_heads), dtype=torch.float32, device="cuda")
            out = m.pool.append_attend(sl, cu, to_dev(q, sh.dtype), to_dev(kn, sh.dtype), to_dev(vn, sh.dtype),
                                       sh.scale, lse=lse)
            for b, s in enumerate(sl):
                m.model.append(s, kn[cu[b]:cu[b + 1]], vn[cu[b]:cu[b + 1]])
            ref, ref_lse = m.oracle_appended(sl, dl, q)
            check_close(out, ref, sh.dtype, f"seed {seed} turn {turn} append_attend", row_scaled=True)
            assert np.abs(lse.cpu().numpy() - ref_lse).max() < 2e-3
        else:
            m.append(sl, dl, kn, vn)
            out, lse, _ = m.attend_appended(sl, dl, q, lse=True)
            ref, ref_lse = m.oracle_appended(sl, dl, q)
            check_close(out, ref, sh.dtype, f"seed {seed} turn {turn} appended", row_scaled=True)
            assert np.abs(lse.cpu().numpy() - ref_lse).max() < 2e-3
    for s in slots[:3]:
        m.check_gather(s)
    m.pool.close()
