"""Plain fp64 definition of delta-prefill attention (test oracle).

What is computed (paper Sec. 2.2 and Sec. 3.3 / Alg. 1, Sec. 3.6 / Alg. 2):
a turn ingests only its Delta new tokens.  Each new token attends over
everything before it in the conversation, i.e. the n cached tokens of the
sequence plus the new tokens up to and including itself, and the result must be
the same as if the whole n+Delta prompt had been processed from scratch.  The
speculative-verify batch of Alg. 2 (current token plus k drafts) is the same
computation with Delta = k+1.

Readings taken where the paper is silent:
  * grouped-query attention: query head h reads KV head h // (Hq // Hkv);
  * bottom-right causal alignment: new row i sees absolute positions 0..n+i;
  * the softmax scale is an argument; positions are already encoded in Q and K.

Everything is float64 and there is no tiling, fusion or reordering.
"""
from __future__ import annotations

import math
from typing import Iterable, Optional, Sequence, Tuple

import numpy as np


def _as64(x) -> np.ndarray:
    return np.asarray(x, dtype=np.float64)


def delta_attend(
    q,
    k_cache,
    v_cache,
    k_new,
    v_new,
    scale: float,
    rows: Optional[Iterable[int]] = None,
) -> Tuple[np.ndarray, np.ndarray]:
    """Attention of Delta new tokens over a cached prefix plus their own causal block.

    q        [Delta, Hq,  D]   queries of the new tokens
    k_cache  [n,     Hkv, D]   cached keys, logical positions 0..n-1 (n may be 0)
    v_cache  [n,     Hkv, D]
    k_new    [Delta, Hkv, D]   keys / values of the new tokens (positions n..n+Delta-1)
    v_new    [Delta, Hkv, D]
    rows     optional subset of new-token indices to evaluate (others are left 0)

    Returns (O [Delta, Hq, D], LSE [Delta, Hq]) in float64, where LSE is the
    natural-log sum of exp of the scaled scores of the visible keys.
    """
    q = _as64(q)
    k_cache, v_cache = _as64(k_cache), _as64(v_cache)
    k_new, v_new = _as64(k_new), _as64(v_new)
    delta, hq, d = q.shape
    n, hkv, _ = k_cache.shape
    assert hq % hkv == 0
    group = hq // hkv
    assert k_new.shape == (delta, hkv, d) and v_new.shape == (delta, hkv, d)
    assert v_cache.shape == (n, hkv, d)

    k_all = np.concatenate([k_cache, k_new], axis=0)  # positions 0 .. n+Delta-1
    v_all = np.concatenate([v_cache, v_new], axis=0)

    out = np.zeros((delta, hq, d), dtype=np.float64)
    lse = np.zeros((delta, hq), dtype=np.float64)
    which = range(delta) if rows is None else [int(r) for r in rows]
    for g in range(hkv):
        k_g = np.ascontiguousarray(k_all[:, g, :])  # [n+Delta, D]
        v_g = np.ascontiguousarray(v_all[:, g, :])
        heads = slice(g * group, (g + 1) * group)  # the query heads that share KV head g
        for i in which:
            visible = n + i + 1  # absolute positions 0 .. n+i
            s = scale * (q[i, heads, :] @ k_g[:visible].T)  # [group, visible]
            m = s.max(axis=1, keepdims=True)
            p = np.exp(s - m)
            z = p.sum(axis=1, keepdims=True)
            out[i, heads, :] = (p / z) @ v_g[:visible]
            lse[i, heads] = (m + np.log(z))[:, 0]
    return out, lse


def delta_attend_batch(
    q,
    caches: Sequence[Tuple[np.ndarray, np.ndarray]],
    k_new,
    v_new,
    cu_delta: Sequence[int],
    scale: float,
    rows_per_seq: Optional[Sequence[Optional[Iterable[int]]]] = None,
) -> Tuple[np.ndarray, np.ndarray]:
    """A batch is the single-sequence definition applied independently per entry.

    Rows of q / k_new / v_new / O are packed in batch order: entry b owns rows
    cu_delta[b] .. cu_delta[b+1]-1.  caches[b] = (K_cache_b, V_cache_b) is the
    logical content of entry b's sequence (already resolved through any alias).
    """
    q = _as64(q)
    k_new, v_new = _as64(k_new), _as64(v_new)
    total, hq, d = q.shape
    assert cu_delta[0] == 0 and cu_delta[-1] == total
    out = np.zeros((total, hq, d), dtype=np.float64)
    lse = np.zeros((total, hq), dtype=np.float64)
    for b, (kc, vc) in enumerate(caches):
        lo, hi = int(cu_delta[b]), int(cu_delta[b + 1])
        if hi == lo:
            continue
        rows = None if rows_per_seq is None else rows_per_seq[b]
        o_b, l_b = delta_attend(q[lo:hi], kc, vc, k_new[lo:hi], v_new[lo:hi], scale, rows)
        out[lo:hi] = o_b
        lse[lo:hi] = l_b
    return out, lse


def full_recompute(q_all, k_all, v_all, scale: float) -> np.ndarray:
    """From-scratch causal attention with every one of the N tokens as a query.

    Written separately from delta_attend (matrix form, explicit lower-triangular
    mask) so that the two can check each other: the last Delta rows of this
    result are what a delta-prefill turn must produce (paper Sec. 3.3: the
    delta path is an optimisation of a full re-prefill, not an approximation).

    q_all [N, Hq, D], k_all / v_all [N, Hkv, D]  ->  O [N, Hq, D]
    """
    q_all, k_all, v_all = _as64(q_all), _as64(k_all), _as64(v_all)
    n_tok, hq, d = q_all.shape
    hkv = k_all.shape[1]
    group = hq // hkv
    tri = np.tril(np.ones((n_tok, n_tok), dtype=bool))  # query t sees keys <= t
    out = np.empty_like(q_all)
    for h in range(hq):
        g = h // group
        scores = scale * (q_all[:, h, :] @ k_all[:, g, :].T)
        scores = np.where(tri, scores, -np.inf)
        scores = scores - scores.max(axis=1, keepdims=True)
        w = np.exp(scores)
        w = w / w.sum(axis=1, keepdims=True)
        out[:, h, :] = w @ v_all[:, g, :]
    return out


def decode_one(q1, k_all, v_all, scale: float) -> np.ndarray:
    """Single-token decode: one query over all keys, no mask.  q1 [Hq, D]."""
    q1, k_all, v_all = _as64(q1), _as64(k_all), _as64(v_all)
    hq, d = q1.shape
    group = hq // k_all.shape[1]
    out = np.empty((hq, d), dtype=np.float64)
    for h in range(hq):
        g = h // group
        s = scale * (k_all[:, g, :] @ q1[h])
        w = np.exp(s - s.max())
        out[h] = (w / w.sum()) @ v_all[:, g, :]
    return out


def brute_force_delta_attend(q, k_cache, v_cache, k_new, v_new, scale: float):
    """Pure-Python scalar loops, for tiny shapes only.  Same contract as delta_attend."""
    q = _as64(q).tolist()
    kc, vc = _as64(k_cache).tolist(), _as64(v_cache).tolist()
    kn, vn = _as64(k_new).tolist(), _as64(v_new).tolist()
    delta, hq, d = len(q), len(q[0]), len(q[0][0])
    n = len(kc)
    hkv = len(kn[0])
    group = hq // hkv
    keys = kc + kn
    vals = vc + vn
    out = [[[0.0] * d for _ in range(hq)] for _ in range(delta)]
    lse = [[0.0] * hq for _ in range(delta)]
    for i in range(delta):
        for h in range(hq):
            g = h // group
            scores = []
            for j in range(n + i + 1):
                acc = 0.0
                for c in range(d):
                    acc += q[i][h][c] * keys[j][g][c]
                scores.append(scale * acc)
            top = max(scores)
            weights = [math.exp(s - top) for s in scores]
            z = math.fsum(weights)
            for c in range(d):
                out[i][h][c] = math.fsum(w * vals[j][g][c] for j, w in enumerate(weights)) / z
            lse[i][h] = top + math.log(z)
    return np.array(out), np.array(lse)
