"""Pins of the greedy-verification oracle (paper Sec. 3.6 / Alg. 2, Sec. 3.8) -- CPU only."""
import numpy as np
import pytest

import oracle


def test_argmax_brute_force_with_ties_and_infinities():
    rng = np.random.default_rng(1)
    for _ in range(50):
        rows, vocab = int(rng.integers(1, 6)), int(rng.integers(1, 40))
        x = rng.integers(-3, 4, size=(rows, vocab)).astype(np.float64)  # many ties
        if rng.random() < 0.3:
            x[rng.integers(rows), rng.integers(vocab)] = np.inf
        if rng.random() < 0.3:
            x[rng.integers(rows), :] = -np.inf
        got = oracle.greedy_argmax(x)
        for r in range(rows):
            best, where = None, None
            for i in range(vocab):  # first strictly larger entry wins
                if best is None or x[r, i] > best:
                    best, where = x[r, i], i
            assert got[r] == where


def test_argmax_special_values():
    assert oracle.greedy_argmax([[0.0, -0.0, 0.0]])[0] == 0       # signed zeros tie: lowest id
    assert oracle.greedy_argmax([[-0.0, 0.0]])[0] == 0
    assert oracle.greedy_argmax([[1.0, np.nan, np.inf]])[0] == 1   # NaN counts as +inf, first one wins
    assert oracle.greedy_argmax([[1.0, np.inf, np.nan]])[0] == 1
    assert oracle.greedy_argmax([[-np.inf, -np.inf]])[0] == 0


def _one_hot_rows(winners, vocab):
    x = np.zeros((len(winners), vocab))
    for r, w in enumerate(winners):
        x[r, w] = 1.0
    return x


@pytest.mark.parametrize("k,first_wrong", [(8, 0), (8, 1), (8, 5), (8, 8), (1, 0), (1, 1), (0, 0), (11, 11)])
def test_accept_count_hand_cases(k, first_wrong):
    """Drafts 0..first_wrong-1 are what the model would say, draft first_wrong (if any) is not."""
    vocab = 50
    model_says = [(7 * s + 3) % vocab for s in range(k + 1)]  # argmax of logits row s
    drafts = [model_says[s] if s < first_wrong else (model_says[s] + 1) % vocab for s in range(k)]
    keep, nxt, am = oracle.verify_accept(_one_hot_rows(model_says, vocab), [42] + drafts)
    assert keep == 1 + min(first_wrong, k)
    assert nxt == model_says[min(first_wrong, k)]
    assert list(am) == model_says


def test_a_later_match_after_a_mismatch_is_not_accepted():
    vocab = 10
    model_says = [1, 2, 3, 4]
    drafts = [1, 9, 3]  # draft 1 wrong, draft 2 would match its row but must be rejected
    keep, nxt, _ = oracle.verify_accept(_one_hot_rows(model_says, vocab), [0] + drafts)
    assert (keep, nxt) == (2, 2)


def _toy_model(seed, vocab):
    """Deterministic stand-in for a language model: the logits depend on the whole token prefix."""
    def model(tokens):
        h = seed
        for t in tokens:
            h = (h * 1000003 + int(t) + 12345) % (2 ** 61 - 1)
        return np.random.default_rng(h).standard_normal(vocab)
    return model


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4])
def test_speculative_decoding_emits_exactly_the_sequential_tokens(seed):
    """Sec. 3.6 'correctness-preserving': whatever the drafts, verify + accept reproduces plain decoding."""
    vocab, steps = 17, 40
    model = _toy_model(seed, vocab)
    prefix = [3, 1, 4, 1, 5]
    want = oracle.sequential_greedy(model, prefix, steps)
    rng = np.random.default_rng(100 + seed)
    toks = list(prefix)
    # the first token has to come from a plain decode step (k = 0)
    keep, nxt, _ = oracle.verify_accept(np.asarray(model(toks))[None, :], [toks[-1]])
    assert keep == 1
    emitted = [nxt]
    passes = 1
    while len(emitted) < steps:
        g_last = emitted[-1]
        k = int(rng.integers(0, 6))
        truth = want[len(emitted):len(emitted) + k]
        drafts = [t if rng.random() < 0.7 else int(rng.integers(vocab)) for t in truth]
        drafts += [int(rng.integers(vocab)) for _ in range(k - len(drafts))]
        batch = [g_last] + drafts
        base = toks + emitted[:-1]
        logits = np.stack([model(base + batch[: s + 1]) for s in range(len(batch))])
        keep, nxt, _ = oracle.verify_accept(logits, batch)
        emitted += drafts[: keep - 1] + [nxt]
        passes += 1
    assert emitted[:steps] == want
    assert passes <= steps


def test_all_drafts_right_needs_the_papers_number_of_passes():
    """Eq. 8 with the worked numbers: m = 20 tokens, k = 11 right drafts per pass -> ceil(20/12) = 2 passes."""
    vocab, m, k = 31, 20, 11
    model = _toy_model(9, vocab)
    prefix = [2, 7]
    want = oracle.sequential_greedy(model, prefix, m + 1)
    emitted = [want[0]]  # token 0 comes from the prompt's own forward pass
    passes = 0
    while len(emitted) < m + 1:
        drafts = want[len(emitted):len(emitted) + k]
        batch = [emitted[-1]] + drafts
        base = prefix + emitted[:-1]
        logits = np.stack([model(base + batch[: s + 1]) for s in range(len(batch))])
        keep, nxt, _ = oracle.verify_accept(logits, batch)
        assert keep == len(batch)
        emitted += drafts + [nxt]
        passes += 1
    assert passes == oracle.pld_forward_passes(m, k) == 2


def test_batch_form_matches_per_slot_calls_and_skips_empty_slots():
    rng = np.random.default_rng(5)
    vocab = 23
    deltas = [3, 0, 1, 9, 4]
    cu = np.concatenate([[0], np.cumsum(deltas)])
    logits = rng.standard_normal((cu[-1], vocab))
    toks = rng.integers(0, vocab, size=cu[-1])
    am = oracle.greedy_argmax(logits)
    # make some drafts right so that accept counts vary
    for b, d in enumerate(deltas):
        for s in range(max(0, d - 1)):
            if rng.random() < 0.6:
                toks[cu[b] + 1 + s] = am[cu[b] + s]
    keep, nxt, am_all = oracle.verify_batch(logits, toks, cu)
    assert np.array_equal(am_all, am)
    for b, d in enumerate(deltas):
        if d == 0:
            assert (keep[b], nxt[b]) == (0, -1)
            continue
        k1, n1, _ = oracle.verify_accept(logits[cu[b]:cu[b + 1]], toks[cu[b]:cu[b + 1]])
        assert (keep[b], nxt[b]) == (k1, n1)
        assert 1 <= keep[b] <= d
