"""Pins for the logical pool model and the paper's printed arithmetic (no GPU)."""
import os

import numpy as np
import pytest

import oracle
from oracle import OracleError, OraclePool
from paper_2605_26289_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_arithmetic.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        line = line.split("#")[0].strip()
        if line:
            k, v = [t.strip() for t in line.split("=")]
            out[k] = float(v)
    return out


def test_paper_conversation_arithmetic():
    g = _gold()
    lens = oracle.prompt_lengths(int(g["system_prompt_tokens"]), int(g["tokens_per_turn"]), int(g["turns"]))
    assert [p for p, _ in lens] == [200, 350, 500, 650, 800]
    assert lens[-1] == (int(g["final_turn_cached_tokens"]), int(g["final_prompt_tokens"]))
    assert lens[-1][1] - lens[-1][0] == g["final_turn_new_tokens"]
    sp = oracle.turn_speedup(lens[-1][1], lens[-1][1] - lens[-1][0])
    assert abs(sp - 950 / 150) < 1e-12
    ratio = g["tokens_per_turn"] / g["final_prompt_tokens"]
    assert g["delta_ratio_lo"] <= ratio <= g["delta_ratio_hi"] + 0.01
    # the workload generator reproduces the same per-turn cached lengths
    w = wl.config2()
    assert [t.n_past[0] for t in w.turns] == [p for p, _ in lens]
    assert w.cells_needed() == int(g["final_prompt_tokens"])


def test_paper_pld_and_memory_arithmetic():
    g = _gold()
    assert oracle.pld_forward_passes(int(g["pld_m"]), int(g["pld_k"])) == g["pld_batched_decodes"]
    assert oracle.pld_forward_passes(20, 0) == 20
    assert oracle.pld_forward_passes(24, 11) == 2 and oracle.pld_forward_passes(25, 11) == 3
    b = oracle.kv_entry_bytes(int(g["kv_layers"]), int(g["kv_width"]), int(g["kv_tokens"]), int(g["kv_bytes_per_elem"]))
    assert b == 524_288_000 and round(b / 1e6) == g["kv_entry_megabytes"]
    assert oracle.kv_cell_bytes(8, 128, 2) == 4096


def _rows(r, count, hkv=2, d=4):
    return r.standard_normal((count, hkv, d)), r.standard_normal((count, hkv, d))


def test_alias_shares_cells_and_reads_like_a_private_copy():
    r = np.random.default_rng(0)
    p = OraclePool(4, 2)
    a = p.acquire(0)
    b = p.acquire(1)
    c = p.acquire(1)
    k, v = _rows(r, 10)
    p.append(a, k, v)
    p.alias(a, b, 0, 6)
    assert p.length(b) == 6 and p.cell_ids(b) == p.cell_ids(a)[:6]
    p.append(c, k[:6], v[:6])  # private copy of the same rows
    kb, vb = p.gather(b)
    kc, vc = p.gather(c)
    np.testing.assert_array_equal(kb, kc)
    np.testing.assert_array_equal(vb, vc)
    assert set(p.cell_ids(c)).isdisjoint(p.cell_ids(a))
    # attention through the alias equals attention through the private copy
    q = r.standard_normal((2, 4, 4))
    kn, vn = _rows(r, 2)
    o1, _ = oracle.delta_attend(q, kb, vb, kn, vn, 0.5)
    o2, _ = oracle.delta_attend(q, kc, vc, kn, vn, 0.5)
    np.testing.assert_array_equal(o1, o2)
    assert p.live_cells() == 16


def test_donor_and_alias_grow_independently_and_release_keeps_cells():
    r = np.random.default_rng(1)
    p = OraclePool(4, 0)
    a, b = p.acquire(0), p.acquire(0)
    k, v = _rows(r, 8)
    p.append(a, k, v)
    p.alias(a, b, 0, 5)
    k2, v2 = _rows(r, 3)
    k3, v3 = _rows(r, 2)
    p.append(a, k2, v2)
    p.append(b, k3, v3)
    ka, _ = p.gather(a)
    kb, _ = p.gather(b)
    np.testing.assert_array_equal(ka, np.concatenate([k, k2]))
    np.testing.assert_array_equal(kb, np.concatenate([k[:5], k3]))
    p.release(a)
    kb2, _ = p.gather(b)
    np.testing.assert_array_equal(kb2, kb)
    a2 = p.acquire(0)
    assert p.length(a2) == 0
    # trimming a donor below the alias point must not disturb the alias
    p.append(a2, k, v)
    c = p.acquire(0)
    p.alias(a2, c, 0, 6)
    p.trim(a2, 2)
    p.append(a2, k2, v2)
    np.testing.assert_array_equal(p.gather(c)[0], k[:6])
    np.testing.assert_array_equal(p.gather(a2)[0], np.concatenate([k[:2], k2]))


def test_trim_and_verify_accept_paths_agree():
    # Alg. 2: append all k+1 then trim to the last accepted == append only the accepted
    r = np.random.default_rng(2)
    k0, v0 = _rows(r, 7)
    kd, vd = _rows(r, 9)
    for accepted in (0, 3, 8):
        p, q = OraclePool(1, 0), OraclePool(1, 0)
        s, t = p.acquire(0), q.acquire(0)
        p.append(s, k0, v0)
        q.append(t, k0, v0)
        p.append(s, kd, vd)
        p.trim(s, 7 + 1 + accepted)
        q.append(t, kd[: 1 + accepted], vd[: 1 + accepted])
        np.testing.assert_array_equal(p.gather(s)[0], q.gather(t)[0])
        np.testing.assert_array_equal(p.gather(s)[1], q.gather(t)[1])
        assert p.length(s) == 8 + accepted


def test_error_rules():
    p = OraclePool(2, 1)
    a = p.acquire(0)
    b = p.acquire(1)
    with pytest.raises(OracleError, match="TIMEOUT"):
        p.acquire(0)
    r = np.random.default_rng(3)
    p.append(a, *_rows(r, 4))
    for args, status in [((a, b, 1, 3), "UNSUPPORTED"), ((a, a, 0, 2), "INVALID"), ((a, b, 0, 5), "INVALID"),
                         ((a, b, 0, -1), "INVALID")]:
        with pytest.raises(OracleError, match=status):
            p.alias(*args)
    p.alias(a, b, 0, 0)  # m = 0 is a no-op
    assert p.length(b) == 0
    p.alias(a, b, 0, 2)
    with pytest.raises(OracleError, match="INVALID"):
        p.alias(a, b, 0, 1)  # destination not empty
    with pytest.raises(OracleError, match="INVALID"):
        p.trim(b, 3)
    p.release(b)
    with pytest.raises(OracleError, match="NO_SLOT"):
        p.length(b)
    with pytest.raises(OracleError, match="NO_SLOT"):
        p.release(b)


def test_workload_generators_are_seeded_and_in_range():
    w3 = wl.config3()
    assert len(w3.turns) == 35 and all(200 <= t.delta[0] <= 1200 for t in w3.turns)
    assert w3.turns[0].n_past == [0]
    assert [t.n_past[0] for t in w3.turns[1:]] == list(np.cumsum([t.delta[0] for t in w3.turns])[:-1])
    assert wl.config3().turns[7].delta == w3.turns[7].delta
    w4 = wl.config4()
    t = w4.turns[0]
    assert sorted(t.slots) == list(range(16)) and w4.alias_prefix == 2048
    assert all(64 <= d <= 512 for d in t.delta) and all(2048 + 1024 <= n <= 2048 + 8192 for n in t.n_past)
    w5 = wl.config5()
    t = w5.turns[0]
    assert len(t.slots) == 64 and set(t.delta) == {9} and t.staged
    assert all(4096 <= n <= 16384 for n in t.n_past) and all(1 <= a <= 9 for a in t.n_accept)
    x = wl.normal(np.random.default_rng(5), (1000,), "bf16")
    assert np.array_equal(wl.bits_to_f32(wl.bf16_bits(x)), x)  # exactly representable
    import torch
    y = np.random.default_rng(6).standard_normal(4096, dtype=np.float32)
    np.testing.assert_array_equal(wl.round_to_bf16(y), torch.from_numpy(y).to(torch.bfloat16).float().numpy())
