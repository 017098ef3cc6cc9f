"""Pins for the fp64 attention oracle (no GPU).

Each test fixes the oracle to something other than itself: a closed form, a
brute-force loop, a separately written full recompute, a library routine, or
an invariance the definition implies.  A dropped term, a wrong sign or index,
or a transposed operand in oracle/attention.py fails at least one of them.
"""
import math

import numpy as np
import pytest
import torch

import oracle


def _rand(seed, n, delta, hq, hkv, d):
    r = np.random.default_rng(seed)
    return (r.standard_normal((delta, hq, d)), r.standard_normal((n, hkv, d)), r.standard_normal((n, hkv, d)),
            r.standard_normal((delta, hkv, d)), r.standard_normal((delta, hkv, d)))


@pytest.mark.parametrize("n,delta,hq,hkv,d", [(0, 1, 2, 1, 2), (3, 3, 2, 1, 2), (2, 3, 4, 2, 3), (5, 1, 6, 3, 4)])
def test_brute_force_tiny(n, delta, hq, hkv, d):
    q, kc, vc, kn, vn = _rand(1, n, delta, hq, hkv, d)
    o, l = oracle.delta_attend(q, kc, vc, kn, vn, 0.7)
    ob, lb = oracle.brute_force_delta_attend(q, kc, vc, kn, vn, 0.7)
    np.testing.assert_allclose(o, ob, rtol=0, atol=1e-13)
    np.testing.assert_allclose(l, lb, rtol=0, atol=1e-13)


def test_empty_cache_single_token_returns_its_own_value():
    q, kc, vc, kn, vn = _rand(2, 0, 1, 4, 2, 8)
    o, l = oracle.delta_attend(q, kc, vc, kn, vn, 0.35)
    for h in range(4):
        np.testing.assert_allclose(o[0, h], vn[0, h // 2], atol=1e-15)
        # a single visible key: LSE is its scaled score
        assert abs(l[0, h] - 0.35 * float(q[0, h] @ kn[0, h // 2])) < 1e-13


def test_hand_computed_two_keys():
    # one head, D=1: scores 0 and ln(3) -> weights 1/4, 3/4
    q = np.array([[[1.0]]])
    kc = np.array([[[0.0]]])
    vc = np.array([[[8.0]]])
    kn = np.array([[[math.log(3.0)]]])
    vn = np.array([[[4.0]]])
    o, l = oracle.delta_attend(q, kc, vc, kn, vn, 1.0)
    assert abs(o[0, 0, 0] - (0.25 * 8.0 + 0.75 * 4.0)) < 1e-14
    assert abs(l[0, 0] - math.log(4.0)) < 1e-14


def test_delta_rows_equal_tail_of_full_recompute():
    n, delta, hq, hkv, d = 37, 23, 8, 2, 16
    r = np.random.default_rng(3)
    q_all = r.standard_normal((n + delta, hq, d))
    k_all = r.standard_normal((n + delta, hkv, d))
    v_all = r.standard_normal((n + delta, hkv, d))
    full = oracle.full_recompute(q_all, k_all, v_all, 0.25)
    o, _ = oracle.delta_attend(q_all[n:], k_all[:n], v_all[:n], k_all[n:], v_all[n:], 0.25)
    np.testing.assert_allclose(o, full[n:], rtol=0, atol=1e-13)
    # and the n = 0 special case is the whole full recompute
    o0, _ = oracle.delta_attend(q_all, k_all[:0], v_all[:0], k_all, v_all, 0.25)
    np.testing.assert_allclose(o0, full, rtol=0, atol=1e-13)


def test_delta_one_is_single_token_decode():
    q, kc, vc, kn, vn = _rand(4, 50, 1, 8, 4, 16)
    o, _ = oracle.delta_attend(q, kc, vc, kn, vn, 0.25)
    ref = oracle.decode_one(q[0], np.concatenate([kc, kn]), np.concatenate([vc, vn]), 0.25)
    np.testing.assert_allclose(o[0], ref, rtol=0, atol=1e-14)


def test_verify_batch_equals_sequential_decodes():
    # Alg. 2: one k+1 batch must equal k+1 successive single-token steps
    q, kc, vc, kn, vn = _rand(5, 40, 9, 8, 2, 16)
    o, _ = oracle.delta_attend(q, kc, vc, kn, vn, 0.25)
    for i in range(9):
        k_seen = np.concatenate([kc, kn[: i + 1]])
        v_seen = np.concatenate([vc, vn[: i + 1]])
        np.testing.assert_allclose(o[i], oracle.decode_one(q[i], k_seen, v_seen, 0.25), rtol=0, atol=1e-14)


def test_library_sdpa_float64_with_bottom_right_mask():
    n, delta, hq, hkv, d = 29, 13, 8, 2, 32
    q, kc, vc, kn, vn = _rand(6, n, delta, hq, hkv, d)
    o, _ = oracle.delta_attend(q, kc, vc, kn, vn, 0.2)
    g = hq // hkv
    k_all = torch.from_numpy(np.concatenate([kc, kn])).repeat_interleave(g, dim=1).permute(1, 0, 2)
    v_all = torch.from_numpy(np.concatenate([vc, vn])).repeat_interleave(g, dim=1).permute(1, 0, 2)
    qt = torch.from_numpy(q).permute(1, 0, 2)
    i = torch.arange(delta)[:, None]
    j = torch.arange(n + delta)[None, :]
    mask = j <= (n + i)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, k_all, v_all, attn_mask=mask, scale=0.2)
    np.testing.assert_allclose(o, ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-13)


def test_zero_keys_give_running_prefix_mean():
    n, delta, hq, hkv, d = 11, 6, 4, 2, 8
    q, kc, vc, kn, vn = _rand(7, n, delta, hq, hkv, d)
    o, l = oracle.delta_attend(q, np.zeros_like(kc), vc, np.zeros_like(kn), vn, 0.3)
    v_all = np.concatenate([vc, vn])
    for i in range(delta):
        for h in range(hq):
            np.testing.assert_allclose(o[i, h], v_all[: n + i + 1, h // 2].mean(axis=0), atol=1e-14)
            assert abs(l[i, h] - math.log(n + i + 1)) < 1e-13
    o2, _ = oracle.delta_attend(np.zeros_like(q), kc, vc, kn, vn, 0.3)
    np.testing.assert_allclose(o2, o, atol=1e-14)


def test_dominant_key_selects_its_value():
    n, delta, hq, hkv, d = 20, 4, 2, 1, 8
    q, kc, vc, kn, vn = _rand(8, n, delta, hq, hkv, d)
    q[:] = 0.0
    q[:, :, 0] = 1.0
    kc[:, :, 0] = 0.0
    kn[:, :, 0] = 0.0
    kc[7, 0, 0] = 60.0  # +60 margin over every other key
    o, _ = oracle.delta_attend(q, kc, vc, kn, vn, 1.0)
    np.testing.assert_allclose(o, np.broadcast_to(vc[7, 0], o.shape), atol=1e-20 + 1e3 * math.exp(-60.0))


def test_causality_future_new_tokens_do_not_matter():
    q, kc, vc, kn, vn = _rand(9, 10, 8, 4, 2, 8)
    o, _ = oracle.delta_attend(q, kc, vc, kn, vn, 0.3)
    kn2, vn2 = kn.copy(), vn.copy()
    kn2[5:] += 100.0
    vn2[5:] -= 50.0
    o2, _ = oracle.delta_attend(q, kc, vc, kn2, vn2, 0.3)
    np.testing.assert_array_equal(o[:5], o2[:5])
    assert np.abs(o[5:] - o2[5:]).max() > 1.0


def test_softmax_rows_sum_to_one_via_constant_values():
    q, kc, vc, kn, vn = _rand(10, 33, 7, 4, 2, 8)
    o, _ = oracle.delta_attend(q, kc, np.ones_like(vc), kn, np.ones_like(vn), 0.3)
    np.testing.assert_allclose(o, 1.0, atol=1e-14)


def test_invariances():
    n, delta, hq, hkv, d = 31, 9, 8, 2, 16
    q, kc, vc, kn, vn = _rand(11, n, delta, hq, hkv, d)
    o, l = oracle.delta_attend(q, kc, vc, kn, vn, 0.25)
    # (i) a constant added to every key shifts every score of a row equally
    c = np.random.default_rng(0).standard_normal((1, hkv, d)) * 3
    o1, l1 = oracle.delta_attend(q, kc + c, vc, kn + c, vn, 0.25)
    np.testing.assert_allclose(o1, o, atol=1e-12)
    g = hq // hkv
    shift = 0.25 * np.einsum("ihd,hd->ih", q, np.repeat(c[0], g, axis=0))
    np.testing.assert_allclose(l1, l + shift, atol=1e-12)
    # (ii) permuting cached tokens (K and V together) changes nothing: no positions inside
    perm = np.random.default_rng(1).permutation(n)
    o2, _ = oracle.delta_attend(q, kc[perm], vc[perm], kn, vn, 0.25)
    np.testing.assert_allclose(o2, o, atol=1e-13)
    # (iii) Q * a with scale / a
    o3, _ = oracle.delta_attend(q * 4.0, kc, vc, kn, vn, 0.25 / 4.0)
    np.testing.assert_allclose(o3, o, atol=1e-13)
    # (iv) the scale really multiplies the scores
    o4, _ = oracle.delta_attend(q, kc, vc, kn, vn, 0.5)
    assert np.abs(o4 - o).max() > 1e-3


def test_gqa_head_mapping_consecutive_query_heads_share():
    n, delta, hq, hkv, d = 12, 3, 6, 3, 4
    q, kc, vc, kn, vn = _rand(12, n, delta, hq, hkv, d)
    o, _ = oracle.delta_attend(q, kc, vc, kn, vn, 0.5)
    for h in range(hq):
        g = h // 2
        o_h, _ = oracle.delta_attend(q[:, h:h + 1], kc[:, g:g + 1], vc[:, g:g + 1], kn[:, g:g + 1], vn[:, g:g + 1], 0.5)
        np.testing.assert_allclose(o[:, h], o_h[:, 0], atol=1e-14)


def test_chunked_delta_equals_unchunked():
    # Alg. 1 feeds the delta in steps of b tokens; the result must not depend on b
    n, delta, hq, hkv, d = 17, 12, 4, 2, 8
    q, kc, vc, kn, vn = _rand(13, n, delta, hq, hkv, d)
    o, l = oracle.delta_attend(q, kc, vc, kn, vn, 0.3)
    for b in (1, 5, 12):
        kcur, vcur = kc, vc
        parts, lparts = [], []
        for i in range(0, delta, b):
            oi, li = oracle.delta_attend(q[i:i + b], kcur, vcur, kn[i:i + b], vn[i:i + b], 0.3)
            parts.append(oi)
            lparts.append(li)
            kcur = np.concatenate([kcur, kn[i:i + b]])
            vcur = np.concatenate([vcur, vn[i:i + b]])
        np.testing.assert_allclose(np.concatenate(parts), o, atol=1e-14)
        np.testing.assert_allclose(np.concatenate(lparts), l, atol=1e-14)


def test_rows_subset_matches_full():
    q, kc, vc, kn, vn = _rand(14, 25, 10, 4, 2, 8)
    o, l = oracle.delta_attend(q, kc, vc, kn, vn, 0.3)
    o_s, l_s = oracle.delta_attend(q, kc, vc, kn, vn, 0.3, rows=[0, 4, 9])
    for i in (0, 4, 9):
        np.testing.assert_array_equal(o_s[i], o[i])
        np.testing.assert_array_equal(l_s[i], l[i])
    assert not o_s[1].any()


def test_batch_is_independent_per_entry_and_order_free():
    hq, hkv, d = 4, 2, 8
    r = np.random.default_rng(15)
    ns, ds = [5, 0, 9], [3, 4, 0]
    caches = [(r.standard_normal((n, hkv, d)), r.standard_normal((n, hkv, d))) for n in ns]
    cu = np.concatenate([[0], np.cumsum(ds)])
    q = r.standard_normal((cu[-1], hq, d))
    kn = r.standard_normal((cu[-1], hkv, d))
    vn = r.standard_normal((cu[-1], hkv, d))
    o, l = oracle.delta_attend_batch(q, caches, kn, vn, cu, 0.4)
    for b in range(3):
        lo, hi = cu[b], cu[b + 1]
        if hi > lo:
            ob, lb = oracle.delta_attend(q[lo:hi], *caches[b], kn[lo:hi], vn[lo:hi], 0.4)
            np.testing.assert_array_equal(o[lo:hi], ob)
            np.testing.assert_array_equal(l[lo:hi], lb)
    # reversed batch order: every entry's rows are unchanged
    order = [1, 0]
    cu2 = np.array([0, ds[1], ds[1] + ds[0]])
    pick = np.concatenate([np.arange(cu[1], cu[2]), np.arange(cu[0], cu[1])])
    o2, _ = oracle.delta_attend_batch(q[pick], [caches[b] for b in order], kn[pick], vn[pick], cu2, 0.4)
    np.testing.assert_array_equal(o2, o[pick])
