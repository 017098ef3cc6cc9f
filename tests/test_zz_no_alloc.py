"""The entry point that allocates nothing (dk_delta_attend_noalloc) against dk_delta_attend, through the C ABI.

Two calls in a row on one GPU, the second with a smaller batch: both share the library's built-in scratch array,
which keeps the first call's contents.  Each result must equal dk_delta_attend's for the same call bit for bit
(same plan, same kernels, only the workspace differs) and match the oracle within the parity bounds.  Covers both
kernels and the split-and-merge path (partials in the scratch array), staged and appended mode, and the size limit.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26289_amd import binding as dk
from paper_2605_26289_amd import workloads as wl
from gpu_util import Mirror, check_close, to_dev

pytestmark = pytest.mark.gpu


def _both_ways(m, slots, deltas, q, kn=None, vn=None):
    """Runs the call through both entry points; returns (noalloc output, workspace output, lse pair)."""
    sh = m.shape
    cu = np.concatenate([[0], np.cumsum(deltas)]).astype(np.int32)
    qd = to_dev(q, sh.dtype)
    knd = None if kn is None else to_dev(kn, sh.dtype)
    vnd = None if vn is None else to_dev(vn, sh.dtype)
    total = int(cu[-1])
    lse_a = torch.full((total, sh.n_q_heads), float("nan"), dtype=torch.float32, device="cuda")
    lse_b = torch.full_like(lse_a, float("nan"))
    out_a = torch.full_like(qd, float("nan"))
    dk.delta_attend_noalloc(m.pool.handle, slots, cu, qd, out_a, sh.scale, knd, vnd, lse_a)
    out_b = torch.full_like(qd, float("nan"))
    ws = m.pool.ensure_workspace(slots, cu, kn is not None)
    dk.delta_attend(m.pool.handle, slots, cu, qd, out_b, sh.scale, knd, vnd, lse_b, ws)
    torch.cuda.synchronize()
    return out_a, out_b, lse_a, lse_b, cu


def test_no_alloc_entry_point_equals_delta_attend_on_two_calls_in_a_row():
    sh = wl.Shape(8, 2, 128, "bf16")
    m = Mirror(sh, 4, 1 << 15, granule=64, seed=101)
    a, b, c, d = (m.acquire() for _ in range(4))
    m.append([a], [9000])          # long prefix: the tile kernel splits its keys, partials go through the scratch
    m.alias(a, b, 2500)
    m.append([b, c, d], [300, 1200, 40])

    # call 1: large mixed batch, appended mode (tile kernel with split + merge, stream kernel for the short rows)
    deltas = [200, 130, 9, 3]
    slots = [a, b, c, d]
    m.append(slots, deltas)
    q = m.draw(sum(deltas), sh.n_q_heads)
    need = dk.attend_workspace_bytes(m.pool.handle, slots, np.concatenate([[0], np.cumsum(deltas)]).astype(np.int32), False)
    assert 0 < need <= dk.STATIC_SCRATCH_BYTES
    out_a, out_b, lse_a, lse_b, _ = _both_ways(m, slots, deltas, q)
    assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b)
    ref, ref_lse = m.oracle_appended(slots, deltas, q)
    check_close(out_a, ref, sh.dtype, "no-alloc call 1")
    assert np.abs(lse_a.cpu().numpy() - ref_lse).max() < 2e-3

    # call 2, straight after: a smaller batch, staged mode, other slots first
    deltas2 = [5, 70]
    slots2 = [d, b]
    q2 = m.draw(sum(deltas2), sh.n_q_heads)
    kn, vn = m.draw(sum(deltas2), sh.n_kv_heads), m.draw(sum(deltas2), sh.n_kv_heads)
    out_a2, out_b2, lse_a2, lse_b2, cu2 = _both_ways(m, slots2, deltas2, q2, kn, vn)
    assert torch.equal(out_a2, out_b2) and torch.equal(lse_a2, lse_b2)
    ref2, _ = oracle.delta_attend_batch(q2, [m.cache(s) for s in slots2], kn, vn, cu2, sh.scale)
    check_close(out_a2, ref2, sh.dtype, "no-alloc call 2")
    m.pool.close()


def test_no_alloc_entry_point_with_units_drawn_from_the_queue():
    """A decode batch with enough streaming units for the run-time queue: its counter lives in the built-in array
    too, is set by every call's descriptor upload, and two calls in a row give dk_delta_attend's bits."""
    sh = wl.PRODUCTION
    n_slots = 160  # 1280 units
    rng = np.random.default_rng(7)
    m = Mirror(sh, n_slots, n_slots * 600 + 4096, granule=64, seed=105)
    slots = [m.acquire() for _ in range(n_slots)]
    m.append(slots, rng.integers(1, 400, size=n_slots).tolist())
    for turn in range(2):
        deltas = rng.integers(1, 5, size=n_slots).tolist()
        m.append(slots, deltas)
        q = m.draw(sum(deltas), sh.n_q_heads)
        out_a, out_b, lse_a, lse_b, _ = _both_ways(m, slots, deltas, q)
        assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b)
        ref, _ = m.oracle_appended(slots, deltas, q)
        check_close(out_a, ref, sh.dtype, f"no-alloc queued call {turn}", row_scaled=True)
    m.pool.close()


def test_no_alloc_entry_point_turns_down_what_its_scratch_cannot_hold():
    """A single long session whose key range is split many ways needs more partial rows than the built-in array
    holds: the call reports WORKSPACE, launches nothing and leaves the output untouched."""
    sh = wl.PRODUCTION
    n, delta = 20000, 1200
    m = Mirror(sh, 1, n + delta + 1024, seed=103)
    s = m.acquire()
    kv = to_dev(m.draw(4000, sh.n_kv_heads), sh.dtype)
    for _ in range(n // 4000):
        m.pool.append([s], [0, 4000], kv, kv)   # contents do not matter here
    m.pool.append([s], [0, delta], kv[:delta], kv[:delta])
    cu = np.asarray([0, delta], dtype=np.int32)
    need = dk.attend_workspace_bytes(m.pool.handle, [s], cu, False)
    assert need > dk.STATIC_SCRATCH_BYTES
    q = to_dev(m.draw(delta, sh.n_q_heads), sh.dtype)
    out = torch.full_like(q, 7.0)
    with pytest.raises(dk.DeltaKVError, match="WORKSPACE"):
        dk.delta_attend_noalloc(m.pool.handle, [s], cu, q, out, sh.scale)
    torch.cuda.synchronize()
    assert (out == 7.0).all()
    m.pool.close()
