"""The pieces composed the way the paper's two procedures use them, on the GPU, against the oracle.

Alg. 1 (radix-cached per-turn processing): longest cached prefix -> metadata-only alias -> only the delta goes
through kv_append / delta_attend -> incremental save.  Sec. 3.2 grouped prefill: one leader forward pass, the
followers alias its state.  Alg. 2 (speculative step): prompt-lookup draft -> Delta = k+1 verify attention ->
on-device argmax + accept -> append of the accepted tokens.

There is no model here: a token's K/V/Q rows are seeded draws that depend on the token prefix up to and
including it (as they would in a causal transformer), and logits are synthetic.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26289_amd import DevicePool
from paper_2605_26289_amd import binding as dk
from paper_2605_26289_amd import workloads as wl
from gpu_util import check_close, to_dev

pytestmark = pytest.mark.gpu

SH = wl.Shape(8, 2, 128, "bf16")


def _activations(tokens):
    """q [n, Hq, D], k, v [n, Hkv, D]: row p is a function of tokens[0..p] only."""
    q = np.zeros((len(tokens), SH.n_q_heads, SH.head_dim), np.float32)
    k = np.zeros((len(tokens), SH.n_kv_heads, SH.head_dim), np.float32)
    v = np.zeros_like(k)
    h = 17
    for p, t in enumerate(tokens):
        h = (h * 1000003 + int(t) + 1) % (2 ** 31 - 1)
        rng = np.random.default_rng(h)
        q[p] = wl.normal(rng, q.shape[1:], "bf16")
        k[p] = wl.normal(rng, k.shape[1:], "bf16")
        v[p] = wl.normal(rng, v.shape[1:], "bf16")
    return q, k, v


def _decode_delta(pool, slot, tokens, n_past):
    """Decode(sigma, batch) of Alg. 1 for tokens[n_past:]: append the delta's K/V, attend, return the rows."""
    q, k, v = _activations(tokens)
    delta = len(tokens) - n_past
    cu = [0, delta]
    pool.append([slot], cu, to_dev(k[n_past:], "bf16"), to_dev(v[n_past:], "bf16"))
    out = pool.attend([slot], cu, to_dev(q[n_past:], "bf16"), SH.scale)
    ref, _ = oracle.delta_attend(q[n_past:], k[:n_past], v[:n_past], k[n_past:], v[n_past:], SH.scale)
    check_close(out, ref, "bf16", f"delta rows of a {len(tokens)}-token prompt with {n_past} cached")
    return out


def test_alg1_turns_with_shared_preamble_process_only_the_delta():
    rng = np.random.default_rng(7)
    pool = DevicePool(12, 8192, SH.n_q_heads, SH.n_kv_heads, SH.head_dim, "bf16", n_session_slots=8)
    radix = dk.radix_create(pool.handle, 4096)
    preamble = rng.integers(0, 30000, size=300).tolist()
    convs = [preamble + rng.integers(0, 30000, size=int(rng.integers(40, 90))).tolist() for _ in range(3)]
    expected_past = [0, 300, 300]
    for turn in range(2):
        for a in range(3):
            if turn == 1:
                convs[a] = convs[a] + rng.integers(0, 30000, size=int(rng.integers(30, 70))).tolist()
            slot = pool.acquire(0)
            n_past = dk.radix_begin_turn(radix, slot, convs[a])
            if turn == 0:
                assert n_past == expected_past[a]
            else:
                assert n_past == prev_len[a]      # everything of the previous turn is cached
            _decode_delta(pool, slot, convs[a], n_past)
            assert dk.radix_save(radix, slot, convs[a])
            pool.release(slot)
        prev_len = [len(c) for c in convs]
    nodes, cells, donors, shed = dk.radix_stats(radix)
    assert shed == 0 and cells == 300 + sum(len(c) - 300 for c in convs)  # the preamble is held once
    torch.cuda.synchronize()
    dk.radix_destroy(radix)
    pool.close()


def test_grouped_prefill_followers_alias_the_leaders_state():
    rng = np.random.default_rng(8)
    pool = DevicePool(8, 8192, SH.n_q_heads, SH.n_kv_heads, SH.head_dim, "bf16")
    schema = rng.integers(0, 30000, size=260).tolist()
    prompts = [schema + rng.integers(0, 30000, size=int(rng.integers(20, 60))).tolist() for _ in range(4)]
    prompts.append(rng.integers(0, 30000, size=120).tolist())  # an unrelated request in the same burst
    leader, shared = dk.prefill_groups(prompts, [0] * 5, [0] * 5, 8)
    assert leader == [0, 0, 0, 0, 4] and shared[1:4] == [260, 260, 260]
    slots = [pool.acquire(0) for _ in prompts]
    for i in (0, 4):                                            # leaders: one forward pass each
        _decode_delta(pool, slots[i], prompts[i], 0)
    for i in (1, 2, 3):                                         # followers: alias, then only their own tail
        pool.alias(slots[leader[i]], slots[i], shared[i])
        _decode_delta(pool, slots[i], prompts[i], shared[i])
        assert pool.cells(slots[i])[:260].tolist() == pool.cells(slots[0])[:260].tolist()
    torch.cuda.synchronize()
    pool.close()


def test_alg2_speculative_step_lookup_verify_accept_append():
    rng = np.random.default_rng(9)
    vocab, n_slots, k_max = 4096, 6, 8
    pool = DevicePool(n_slots, 1 << 14, SH.n_q_heads, SH.n_kv_heads, SH.head_dim, "bf16")
    slots, histories, batches = [], [], []
    for s in range(n_slots):
        call = rng.integers(0, vocab, size=12).tolist()                   # a recurring tool-call pattern
        hist = rng.integers(0, vocab, size=200).tolist() + call + rng.integers(0, vocab, size=30).tolist() + call[:3]
        draft, n = dk.pld_lookup(hist, 2, 16, k_max)
        assert (draft, n) == oracle.lookup_ngram(hist, 2, 16, k_max) and draft == call[3:11]
        slot = pool.acquire(0)
        _q, k, v = _activations(hist[:-1])                                # G_last is not in the cache yet
        pool.append([slot], [0, len(hist) - 1], to_dev(k, "bf16"), to_dev(v, "bf16"))
        slots.append(slot)
        histories.append(hist)
        batches.append([hist[-1]] + draft)                                # [G_last, predicted...]
    deltas = [len(b) for b in batches]
    cu = np.concatenate([[0], np.cumsum(deltas)]).astype(np.int32)
    rows = int(cu[-1])
    # verify attention from staged K/V (the cache is not modified)
    acts = [_activations(h[:-1] + b) for h, b in zip(histories, batches)]
    q = np.concatenate([a[0][-d:] for a, d in zip(acts, deltas)])
    kn = np.concatenate([a[1][-d:] for a, d in zip(acts, deltas)])
    vn = np.concatenate([a[2][-d:] for a, d in zip(acts, deltas)])
    kn_d, vn_d = to_dev(kn, "bf16"), to_dev(vn, "bf16")
    out = pool.attend(slots, cu, to_dev(q, "bf16"), SH.scale, kn_d, vn_d)
    caches = [(a[1][:-d], a[2][:-d]) for a, d in zip(acts, deltas)]
    ref, _ = oracle.delta_attend_batch(q, caches, kn, vn, cu.astype(np.int64), SH.scale)
    check_close(out, ref, "bf16", "verify batch")
    # synthetic logits: the "model" agrees with the first a_s drafts of slot s
    agree = [8, 0, 3, 8, 1, 5]
    logits = wl.normal(rng, (rows, vocab), "bf16")
    toks = np.concatenate(batches).astype(np.int32)
    for s in range(n_slots):
        for j in range(deltas[s] - 1):
            want = batches[s][1 + j] if j < agree[s] else (batches[s][1 + j] + 1) % vocab
            logits[cu[s] + j, want] = 50.0
    keep_ref, next_ref, _ = oracle.verify_batch(logits, toks, cu)
    assert keep_ref.tolist() == [1 + a for a in agree]
    keep_d = torch.empty(n_slots, dtype=torch.int32, device="cuda")
    next_d = torch.empty(n_slots, dtype=torch.int32, device="cuda")
    ws = torch.empty(dk.verify_workspace_bytes(rows, vocab, dk.BF16), dtype=torch.uint8, device="cuda")
    dk.verify_greedy(n_slots, rows, torch.from_numpy(cu).cuda(), to_dev(logits, "bf16"), dk.BF16, vocab, vocab,
                     torch.from_numpy(toks).cuda(), keep_d, next_d, ws)
    keep = keep_d.cpu().numpy()                                            # the only thing the host reads back
    assert np.array_equal(keep, keep_ref) and np.array_equal(next_d.cpu().numpy(), next_ref)
    before = [pool.length(s) for s in slots]
    pool.append(slots, cu, kn_d, vn_d, n_accept=keep.tolist())             # append only the accepted tokens
    for s in range(n_slots):
        assert pool.length(slots[s]) == before[s] + keep[s]
        kg, _vg = pool.gather(slots[s])
        want = np.concatenate([acts[s][1][:-deltas[s]], kn[cu[s]:cu[s] + keep[s]]])
        assert np.array_equal(kg.float().cpu().numpy(), want)              # same contents as append-all-then-trim
    pool.close()


def test_mixed_prefill_and_decode_batch_sized_by_the_chunking_rule():
    """One scheduler iteration of Sec. 3.2: four slots prefill at once, so the chunking rule cuts the token batch
    into equal chunks, and those chunks share ONE delta_attend call with decode (Delta = 1) and draft-verification
    (Delta = 1 + k) rows of other slots -- the tile kernel and the streaming kernel both run inside the call.  At 1/8
    of the lengths so that the oracle covers every row; production head shape."""
    from gpu_util import Mirror
    sh = wl.PRODUCTION
    chunk = dk.prefill_chunk(4096 // 8, 4)                       # 512-token batch over 4 prefilling slots: 128 each
    assert chunk == 128
    w = wl.mixed_prefill_decode(chunk, n_prefill=4, n_decode=20, prefill_n=1024, n_lo=512, n_hi=2048)
    t = w.turns[0]
    assert sorted(set(t.delta)) == [1, 9, 128]                   # decode, verify and prefill rows in one batch
    m = Mirror(sh, w.n_slots, w.cells_needed() + 256 * (w.n_slots + 2), seed=w.seed)
    slots = [m.acquire() for _ in range(w.n_slots)]
    for s, h in zip(slots, w.history):
        m.append([s], [h])
    q = m.draw(sum(t.delta), sh.n_q_heads)
    m.append(t.slots, t.delta)
    out, lse, _ = m.attend_appended(t.slots, t.delta, q, lse=True)
    ref, ref_lse = m.oracle_appended(t.slots, t.delta, q)
    check_close(out, ref, "bf16", "mixed prefill + decode batch")
    assert np.abs(lse.cpu().numpy() - ref_lse).max() < 2e-3
    m.pool.close()


def test_alg2_step_with_nothing_read_back_between_its_stages():
    """Alg. 2 as the benchmark times it: append all k+1 tokens, verify attention in appended mode, on-device argmax
    and accept, asynchronous copy of the kept counts, and only then -- the deferred part -- one batched trim.  The
    cache must end up exactly as after appending only the accepted tokens."""
    from gpu_util import Mirror
    sh = SH
    rng = np.random.default_rng(10)
    vocab, n_slots, k = 2048, 5, 8
    m = Mirror(sh, n_slots, 1 << 14, seed=10)
    slots = [m.acquire() for _ in range(n_slots)]
    hist = [300, 1000, 37, 640, 2000]
    for s, h in zip(slots, hist):
        m.append([s], [h])
    deltas = [1 + k] * n_slots
    cu = np.concatenate([[0], np.cumsum(deltas)]).astype(np.int32)
    rows = int(cu[-1])
    q = m.draw(rows, sh.n_q_heads)
    kn, vn = m.draw(rows, sh.n_kv_heads), m.draw(rows, sh.n_kv_heads)
    logits = wl.normal(rng, (rows, vocab), "bf16")
    toks = rng.integers(0, vocab, size=rows).astype(np.int32)
    agree = [8, 0, 3, 5, 1]
    for s in range(n_slots):
        for j in range(k):
            want = int(toks[cu[s] + 1 + j]) if j < agree[s] else (int(toks[cu[s] + 1 + j]) + 1) % vocab
            logits[cu[s] + j, want] = 60.0
    keep_ref, _next_ref, _ = oracle.verify_batch(logits, toks, cu)
    assert keep_ref.tolist() == [1 + a for a in agree]
    # device side, one stream, no readback until the end
    knd, vnd = to_dev(kn, "bf16"), to_dev(vn, "bf16")
    m.pool.append(slots, cu, knd, vnd)
    out = m.pool.attend(slots, cu, to_dev(q, "bf16"), sh.scale)
    keep_d = torch.empty(n_slots, dtype=torch.int32, device="cuda")
    next_d = torch.empty(n_slots, dtype=torch.int32, device="cuda")
    ws = torch.empty(dk.verify_workspace_bytes(rows, vocab, dk.BF16), dtype=torch.uint8, device="cuda")
    dk.verify_greedy(n_slots, rows, torch.from_numpy(cu).cuda(), to_dev(logits, "bf16"), dk.BF16, vocab, vocab,
                     torch.from_numpy(toks).cuda(), keep_d, next_d, ws)
    keep_h = torch.empty(n_slots, dtype=torch.int32, pin_memory=True)
    keep_h.copy_(keep_d, non_blocking=True)
    done = torch.cuda.Event()
    done.record()
    done.synchronize()                                            # the deferred part starts here
    keep = keep_h.numpy()
    assert np.array_equal(keep, keep_ref)
    m.pool.trim_batch(slots, [h + int(c) for h, c in zip(hist, keep)])
    # the oracle pool appends only the accepted tokens
    for b, s in enumerate(slots):
        m.model.append(s, kn[cu[b]:cu[b] + keep[b]], vn[cu[b]:cu[b] + keep[b]])
        m.check_gather(s)
    caches = [(m.cache(s)[0][:h], m.cache(s)[1][:h]) for s, h in zip(slots, hist)]
    ref, _ = oracle.delta_attend_batch(q, caches, kn, vn, cu.astype(np.int64), sh.scale)
    check_close(out, ref, "bf16", "verify attention over appended drafts")
    m.pool.close()
