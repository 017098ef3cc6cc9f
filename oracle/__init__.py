"""CPU oracle for delta-prefill attention over a pooled, prefix-aliased KV cache.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain, obviously-correct
definition that the HIP library is checked against.  It shares no code with the
GPU path and must never be imported by the product package; only the tests, the
smoke check and the benchmark's CPU-baseline leg may use it.

Parity status: every function here is pinned by the CPU test-suite (closed
forms, brute force, a second independently written full recompute, a library
attention routine, the paper's printed arithmetic; the verify step by a
brute-force loop, hand cases and the equivalence with token-by-token
decoding that the paper calls correctness-preserving; the prefix cache -- stated twice, as a
flat ledger of saves (prefix_cache.py) and as a trie (radix.py) -- by brute-force longest common
prefixes, a slow recount of the distinct positions held, budget invariants, a hand-checked shed
order and the paper's cached-token counts; the prompt-lookup search by a second formulation).  Parity unpinned: the
absolute output values of the five benchmark workloads are printed nowhere in the
paper, so those are pinned only through these invariants.
"""
from .attention import (  # noqa: F401
    delta_attend,
    delta_attend_batch,
    full_recompute,
    brute_force_delta_attend,
    decode_one,
)
from .pool import OraclePool, OracleError  # noqa: F401
from .verify import greedy_argmax, verify_accept, verify_batch, sequential_greedy  # noqa: F401
from .pld import lookup_ngram, gate as pld_gate  # noqa: F401
from .radix import OracleRadix  # noqa: F401
from .prefix_cache import FlatPrefixCache  # noqa: F401
from .sched import prefill_chunk, fnv1a32, prefill_groups  # noqa: F401
from .costmodel import (  # noqa: F401
    prompt_lengths,
    turn_speedup,
    pld_forward_passes,
    kv_entry_bytes,
    kv_cell_bytes,
)
