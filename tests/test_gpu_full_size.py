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
