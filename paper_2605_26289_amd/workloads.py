"""Seeded synthetic inputs shaped like the paper's agentic traces.

This module only draws shapes and random tensors.  It contains none of the
method's arithmetic and is the one module that both the library's tests and
the CPU oracle's tests may use, so that both sides consume identical inputs.

The paper's own traces (prompts, tool schemas, model activations) are not
available; the generators below keep their structure: a system prompt followed
by fixed-size turns (Sec. 1, Sec. 4.1), a 35-turn deepening conversation
(Sec. 4.2, Sec. 5.2), many agents sharing a schema preamble through aliasing
(Sec. 3.2, Sec. 5.3) and k+1-token speculative verification batches (Sec. 3.6).
Activations are replaced by N(0,1) draws.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

BASE_SEED = 26289


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even); returns float32 holding bf16 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    rounded = (bits + (np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x_bf16_as_f32: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already exactly representable in bf16."""
    x = np.ascontiguousarray(x_bf16_as_f32, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(bits_u16: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits_u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal(rng: np.random.Generator, shape, dtype: str) -> np.ndarray:
    """N(0,1) float32 draws; for dtype 'bf16' rounded once to bf16 (still stored as float32)."""
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if dtype == "bf16":
        x = round_to_bf16(x)
    elif dtype != "f32":
        raise ValueError(dtype)
    return x


@dataclass
class Shape:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str  # "f32" | "bf16"

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))


PRODUCTION = Shape(32, 8, 128, "bf16")


@dataclass
class Turn:
    """One call: for every listed slot, `delta` new tokens on top of `n_past` cached ones."""
    slots: List[int]
    n_past: List[int]
    delta: List[int]
    staged: bool = False  # True: attend first from staged K/V, append (accepted) afterwards
    n_accept: List[int] = field(default_factory=list)


@dataclass
class Workload:
    name: str
    shape: Shape
    n_slots: int
    seed: int
    alias_prefix: int = 0  # slots 1.. alias this many tokens of slot 0
    history: List[int] = field(default_factory=list)  # private tokens per slot ingested before the timed turns
    turns: List[Turn] = field(default_factory=list)

    def cells_needed(self) -> int:
        total = self.alias_prefix + sum(self.history)
        grow = {}
        for t in self.turns:
            for s, d in zip(t.slots, t.delta):
                grow[s] = grow.get(s, 0) + d
        return total + sum(grow.values())


def config1(seed: int = BASE_SEED + 1) -> Workload:
    """Single session, 4 query heads on 1 KV head, D=64, fp32, n=200, Delta=150."""
    return Workload("c1_fp32_single", Shape(4, 1, 64, "f32"), 1, seed, history=[200],
                    turns=[Turn([0], [200], [150])])


def config2(seed: int = BASE_SEED + 2) -> Workload:
    """5-turn agent conversation: 200-token system prompt then 150 tokens per turn (Sec. 1)."""
    turns = [Turn([0], [200 + 150 * t], [150]) for t in range(5)]
    return Workload("c2_agent_5turn", PRODUCTION, 1, seed, history=[200], turns=turns)


def config3(seed: int = BASE_SEED + 3, n_turns: int = 35, lo: int = 200, hi: int = 1200) -> Workload:
    """35-turn coding workflow: per-turn Delta ~ U{lo..hi}; the prefix grows to about 24k tokens."""
    rng = np.random.default_rng(seed)
    deltas = rng.integers(lo, hi + 1, size=n_turns).tolist()
    turns, n = [], 0
    for d in deltas:
        turns.append(Turn([0], [n], [int(d)]))
        n += int(d)
    return Workload("c3_coding_35turn", PRODUCTION, 1, seed, history=[0], turns=turns)


def config4(seed: int = BASE_SEED + 4, n_slots: int = 16, prefix: int = 2048,
            hist_lo: int = 1024, hist_hi: int = 8192, d_lo: int = 64, d_hi: int = 512,
            fixed_delta: int = 0) -> Workload:
    """Interleaved multi-agent traffic: every slot aliases one shared prefix and holds a private history."""
    rng = np.random.default_rng(seed)
    hist = rng.integers(hist_lo, hist_hi + 1, size=n_slots).tolist()
    delta = rng.integers(d_lo, d_hi + 1, size=n_slots).tolist()
    if fixed_delta:
        delta = [fixed_delta] * n_slots
    order = rng.permutation(n_slots).tolist()
    turn = Turn([int(s) for s in order], [prefix + int(hist[s]) for s in order], [int(delta[s]) for s in order])
    return Workload("c4_multi_agent", PRODUCTION, n_slots, seed, alias_prefix=prefix,
                    history=[int(h) for h in hist], turns=[turn])


def config5(seed: int = BASE_SEED + 5, n_slots: int = 64, n_lo: int = 4096, n_hi: int = 16384,
            k_draft: int = 8) -> Workload:
    """Speculative verification: Delta = 1 + k_draft per slot over long prefixes, then append the accepted."""
    rng = np.random.default_rng(seed)
    n = rng.integers(n_lo, n_hi + 1, size=n_slots).tolist()
    # acceptance is bimodal (Sec. 3.6): all drafts in structured regions, almost none in prose
    full = rng.random(n_slots) < 0.6
    few = rng.integers(0, 3, size=n_slots)
    accepted = np.where(full, k_draft, np.minimum(few, k_draft))
    turn = Turn(list(range(n_slots)), [int(x) for x in n], [1 + k_draft] * n_slots, staged=True,
                n_accept=[1 + int(a) for a in accepted])
    return Workload("c5_spec_verify", PRODUCTION, n_slots, seed, history=[int(x) for x in n], turns=[turn])


def mixed_prefill_decode(chunk: int, seed: int = BASE_SEED + 6, n_prefill: int = 4, n_decode: int = 60,
                         prefill_n: int = 8192, n_lo: int = 4096, n_hi: int = 16384, k_draft: int = 8) -> Workload:
    """Heterogeneous PREFILL+DECODE batch of one scheduler iteration (Sec. 3.2): n_prefill slots each take one prefill
    chunk of `chunk` tokens (the caller sizes it with the chunking rule) on top of about prefill_n cached tokens, while
    n_decode slots decode one token or verify a k_draft-token draft (Delta 1 or 1 + k_draft), all in one call, in a
    seeded order.  Appended mode: the step appends every slot's new tokens, then attends."""
    rng = np.random.default_rng(seed)
    n_slots = n_prefill + n_decode
    n_past = [int(prefill_n + rng.integers(0, 512)) for _ in range(n_prefill)]
    n_past += rng.integers(n_lo, n_hi + 1, size=n_decode).tolist()
    delta = [int(chunk)] * n_prefill + [int(1 + k_draft * int(rng.random() < 0.5)) for _ in range(n_decode)]
    order = rng.permutation(n_slots).tolist()
    turn = Turn([int(s) for s in order], [int(n_past[s]) for s in order], [int(delta[s]) for s in order])
    return Workload("mixed_prefill_decode", PRODUCTION, n_slots, seed, history=[int(x) for x in n_past], turns=[turn])


def token_stream(w: Workload, vocab: int = 50000) -> List[int]:
    """Token ids of a single-conversation workload (configs 2 and 3), for the radix-cached per-turn procedure: the
    prompt of turn t is the first n_past + delta ids."""
    rng = np.random.default_rng(w.seed + 500)
    total = (w.history[0] if w.history else 0) + sum(t.delta[0] for t in w.turns)
    return rng.integers(0, vocab, size=total).tolist()


def scaled(w: Workload, factor: float, min_tokens: int = 1) -> Workload:
    """Same structure with every length multiplied by `factor` (for cases the oracle finishes in seconds)."""
    f = lambda x: max(min_tokens, int(round(x * factor)))  # noqa: E731
    hist = [f(h) if h else 0 for h in w.history]
    prefix = f(w.alias_prefix) if w.alias_prefix else 0
    turns = []
    grown = {s: prefix + hist[s] for s in range(w.n_slots)}
    for t in w.turns:
        nt = Turn(list(t.slots), [], [], t.staged, list(t.n_accept))
        for s, d in zip(t.slots, t.delta):
            dd = d if t.staged else f(d)
            nt.n_past.append(grown[s])
            nt.delta.append(dd)
            if not t.staged:
                grown[s] += dd
        turns.append(nt)
    return Workload(w.name + f"_x{factor:g}", w.shape, w.n_slots, w.seed, prefix, hist, turns)
