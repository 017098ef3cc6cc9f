"""Parity at the full sizes of the workload configs, in the launch configuration bench.py times.

The whole batch runs on the GPU exactly as one bench step does (same Scenario object); the oracle then
recomputes a sample of output rows one by one: for a handful of slots (first, last, shortest and longest
prefix among those whose K/V history was mirrored to the host) a spread of new-token rows over all query
heads.  Inputs are the seeded device-side draws of the bench, copied to the host as inputs only.
"""
from __future__ import annotations

import numpy as np
import pytest

import oracle
from gpu_util import ABS_TOL, REL_TOL

pytestmark = pytest.mark.gpu


def _sampled_parity(name: str, keep: int, rows_per_slot: int):
    import torch
    import bench

    w, turn = bench.make_workload(name)
    sc = bench.Scenario(w, turn, keep_host_slots=min(keep, w.n_slots))
    sc.step()
    torch.cuda.synchronize()
    t, sh = sc.turn, sc.sh
    gpu = sc.out.float().cpu().numpy()
    assert np.isfinite(gpu).all()
    q = sc.q.float().cpu().numpy()
    kn = sc.k_new.float().cpu().numpy()
    vn = sc.v_new.float().cpu().numpy()
    kept = [b for b, s in enumerate(t.slots) if s in sc.keep and t.delta[b] > 0]
    assert kept
    by_len = sorted(kept, key=lambda b: t.n_past[b])
    chosen = sorted({kept[0], kept[-1], by_len[0], by_len[-1]})
    worst_abs = worst_rel = 0.0
    checked = 0
    for b in chosen:
        lo, hi = int(sc.cu[b]), int(sc.cu[b + 1])
        kc, vc = sc.host_cache(t.slots[b])
        kc, vc = kc[: t.n_past[b]], vc[: t.n_past[b]]
        assert kc.shape[0] == t.n_past[b]
        rows = sorted(set(np.linspace(0, hi - lo - 1, min(rows_per_slot, hi - lo)).astype(int).tolist()))
        ref, _ = oracle.delta_attend(q[lo:hi], kc, vc, kn[lo:hi], vn[lo:hi], sh.scale, rows)
        diff = np.abs(gpu[lo:hi][rows] - ref[rows])
        rms = np.sqrt((ref[rows] ** 2).mean(axis=-1, keepdims=True))
        worst_abs = max(worst_abs, float(diff.max()))
        worst_rel = max(worst_rel, float((diff / np.maximum(np.abs(ref[rows]), rms)).max()))
        checked += len(rows)
    assert worst_abs <= ABS_TOL and worst_rel <= REL_TOL, (name, worst_abs, worst_rel, checked)
    # the step left the pool as it found it (append + trim, or accept + trim)
    for s, n in zip(t.slots, t.n_past):
        assert sc.pool.length(s) == n


def test_config5_full_size_spec_verify_sampled_rows():
    _sampled_parity("c5", keep=12, rows_per_slot=9)


def test_config4_full_size_multi_agent_sampled_rows():
    _sampled_parity("c4", keep=16, rows_per_slot=12)


def test_config4_full_size_delta512_sampled_rows():
    _sampled_parity("c4_512", keep=6, rows_per_slot=12)


def test_config3_full_size_final_turn_sampled_rows():
    _sampled_parity("c3", keep=1, rows_per_slot=16)


def test_context_cap_chunk_ceiling_and_decode_sampled_rows():
    """The largest shapes the paper's deployment allows (Sec. 4.1: 32 768-token context; Sec. 3.2: prefill chunks
    of at most 4096 tokens): one slot takes a 4096-token chunk that fills its context to the cap, another decodes
    its last token at the cap, in one call.  Sampled rows against the oracle."""
    from gpu_util import Mirror
    from paper_2605_26289_amd import workloads as wl

    cap, chunk = 32768, 4096
    m = Mirror(wl.PRODUCTION, 2, 2 * cap + 1024, seed=77)
    a, b = m.acquire(), m.acquire()
    m.append([a], [cap - chunk])
    m.append([b], [cap - 1])
    deltas = [chunk, 1]
    q = m.draw(chunk + 1, wl.PRODUCTION.n_q_heads)
    m.append([a, b], deltas)
    assert m.pool.length(a) == cap and m.pool.length(b) == cap
    out, lse, _ = m.attend_appended([a, b], deltas, q, lse=True)
    rows = [sorted({0, 1, 63, 64, 255, 256, 1000, 2047, 2048, 4031, 4094, 4095}), [0]]
    ref, ref_lse = m.oracle_appended([a, b], deltas, q, rows_per_seq=rows)
    pick = np.array(rows[0] + [chunk])
    gpu = out.float().cpu().numpy()[pick]
    assert np.isfinite(out.float().cpu().numpy()).all()
    diff = np.abs(gpu - ref[pick])
    rms = np.sqrt((ref[pick] ** 2).mean(axis=-1, keepdims=True))
    assert diff.max() <= ABS_TOL and (diff / np.maximum(np.abs(ref[pick]), rms)).max() <= REL_TOL
    assert np.abs(lse.cpu().numpy()[pick] - ref_lse[pick]).max() < 2e-3
    m.pool.close()
