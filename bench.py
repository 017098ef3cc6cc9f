#!/usr/bin/env python3
"""Benchmark of the delta-prefill hot path on one MI355X.

A step is one pass of the whole path over one synthetic batch: kv_append + delta_attend (appended
mode) or delta_attend from staged K/V + kv_append of the accepted tokens (speculative verify),
followed by the metadata-only trim that rewinds the slots so that every step sees the same state.
Inputs are resident in HBM before the clock starts.  Prints one JSON line.

Workloads (synthetic stand-ins for the paper's agentic traces, see paper_2605_26289_amd/workloads.py):
  c5       speculative verification, 64 slots, prefixes U[4k,16k], Delta = 9 (HBM-bound)   [default]
  c4       16 slots aliasing a 2048-token prefix, histories U[1k,8k], Delta U[64,512]      (MFMA)
  c4_512   the same with Delta = 512 for every slot                                        (MFMA)
  c3       35-turn coding workflow, Delta U[200,1200]; reports the final turn               (MFMA)
  c2       5-turn agent conversation, Delta = 150 (launch-latency bound)
  mixed    one scheduler iteration: 4 prefill chunks sized by the chunking rule + 60 decode / verify slots
  c2_alg1, c3_alg1   the same conversations through the radix-cached per-turn procedure (Alg. 1): every turn
           acquires a sequence, aliases the cached prefix, appends and attends only the delta, saves, releases
  alg2     the speculative step (Alg. 2) on c5's batch with nothing read back between its stages: append the
           k+1 tokens, verify attention, on-device argmax + accept, asynchronous copy of the kept counts, trim
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c5",
                    choices=["c5", "c4", "c4_512", "c3", "c2", "mixed", "c2_alg1", "c3_alg1", "alg2", "verify"])
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE",
                    help="planner tuning passed to dk_set_tuning on every pool (repeatable)")
    ap.add_argument("--step", default="fused", choices=["fused", "separate"],
                    help="fused: dk_append_attend (one launch appends and attends) then the trims; separate: "
                         "dk_kv_append and dk_delta_attend as two calls, in the order the workload's mode states")
    ap.add_argument("--host-profile", action="store_true",
                    help="instead of the benchmark, print where the host time of a step goes (plan, upload, launches)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the oracle timing leg")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the secondary measurements (MFMA regime, verify, the other configs)")
    ap.add_argument("--drafts", type=int, default=8,
                    help="c5 only: drafts per slot (Delta = 1 + drafts; 0 is plain decode, 15 fills the stream kernel)")
    ap.add_argument("--vocab", type=int, default=128256, help="vocabulary size of the greedy-verification leg")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="instead of the benchmark, run a plain device copy of this many MiB five times "
                         "(reference reading for the HBM traffic counters)")
    return ap.parse_args()


def attend_flops(n, delta, hq, d):
    return 4 * hq * d * (delta * n + delta * (delta + 1) // 2)


def attend_bytes(n, delta, hq, hkv, d, e):
    return 2 * hkv * (n + delta) * d * e + 2 * delta * hq * d * e


class Scenario:
    """A pool filled with its history, plus the device inputs of one repeated step."""

    def __init__(self, w, turn_index=-1, keep_host_slots=0, pre_turns=True):
        import torch
        from paper_2605_26289_amd import DevicePool
        self.torch = torch
        self.w = w
        sh = w.shape
        self.sh = sh
        gen = torch.Generator(device="cuda")
        gen.manual_seed(w.seed)
        self.gen = gen
        cells = w.cells_needed() + 512 * (w.n_slots + 2)
        self.pool = DevicePool(w.n_slots, cells, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype)
        for name, value in TUNING:
            from paper_2605_26289_amd import binding as _dk
            _dk.set_tuning(self.pool.handle, name, value)
        self.slots = [self.pool.acquire() for _ in range(w.n_slots)]
        self.host_kv = {}
        self.keep = set(self.slots[:keep_host_slots])
        if w.alias_prefix:
            self._ingest(self.slots[0], w.alias_prefix)
            for s in self.slots[1:]:
                self.pool.alias(self.slots[0], s, w.alias_prefix)
                if s in self.keep:
                    self.host_kv[s] = [self.host_kv[self.slots[0]][0]] if self.slots[0] in self.host_kv else []
        for s, h in zip(self.slots, w.history):
            if h:
                self._ingest(s, h)
        turns = w.turns
        self.turn = turns[turn_index]
        if pre_turns:  # play the earlier turns of a multi-turn conversation (appends only)
            for t in turns[: len(turns) + turn_index if turn_index < 0 else turn_index]:
                for s, d in zip(t.slots, t.delta):
                    self._ingest(s, d)
        t = self.turn
        t.slots = np.asarray(t.slots, dtype=np.int32)  # marshalled once, not per step
        t.n_past = np.asarray(t.n_past, dtype=np.int64)
        for s, n in zip(t.slots, t.n_past):
            assert self.pool.length(s) == n, (s, self.pool.length(s), n)
        total = sum(t.delta)
        self.total = total
        self.cu = np.concatenate([[0], np.cumsum(t.delta)]).astype(np.int32)
        dt = self.pool.torch_dtype
        self.q = torch.randn((total, sh.n_q_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(dt)
        self.k_new = torch.randn((total, sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(dt)
        self.v_new = torch.randn((total, sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(dt)
        self.out = torch.empty_like(self.q)
        self.n_accept = np.asarray(t.n_accept, dtype=np.int32) if t.staged and t.n_accept else None
        self.keep_len = None if self.n_accept is None else t.n_past + self.n_accept.astype(np.int64)
        # size the workspace once, in the state the attend call will see
        if FUSED_STEP:
            self.pool.ensure_workspace(t.slots, self.cu, 2)
        elif t.staged:
            self.pool.ensure_workspace(t.slots, self.cu, True)
        else:
            self.pool.append(t.slots, self.cu, self.k_new, self.v_new)
            self.pool.ensure_workspace(t.slots, self.cu, False)
            self._rewind()
        torch.cuda.synchronize()

    def _ingest(self, slot, count, chunk=65536):
        torch = self.torch
        sh = self.sh
        dt = self.pool.torch_dtype
        done = 0
        while done < count:
            c = min(chunk, count - done)
            k = torch.randn((c, sh.n_kv_heads, sh.head_dim), generator=self.gen, device="cuda", dtype=torch.float32).to(dt)
            v = torch.randn((c, sh.n_kv_heads, sh.head_dim), generator=self.gen, device="cuda", dtype=torch.float32).to(dt)
            self.pool.append([slot], [0, c], k, v)
            if slot in self.keep:
                self.host_kv.setdefault(slot, []).append((k.float().cpu().numpy(), v.float().cpu().numpy()))
            done += c

    def _rewind(self):
        self.pool.trim_batch(self.turn.slots, self.turn.n_past)

    def step(self):
        t = self.turn
        if FUSED_STEP:
            # Decode(sigma, batch): all new tokens appended and attended by one launch; a verification batch then
            # drops its rejected drafts (Alg. 2's trim), host metadata only
            self.pool.append_attend(t.slots, self.cu, self.q, self.k_new, self.v_new, self.sh.scale, out=self.out)
            if self.keep_len is not None:
                self.pool.trim_batch(t.slots, self.keep_len)
        elif t.staged:
            self.pool.attend(t.slots, self.cu, self.q, self.sh.scale, self.k_new, self.v_new, out=self.out)
            self.pool.append(t.slots, self.cu, self.k_new, self.v_new, self.n_accept)
        else:
            self.pool.append(t.slots, self.cu, self.k_new, self.v_new)
            self.pool.attend(t.slots, self.cu, self.q, self.sh.scale, out=self.out)
        self._rewind()

    def algorithmic(self):
        sh, t = self.sh, self.turn
        e = 2 if sh.dtype == "bf16" else 4
        fl = sum(attend_flops(n, d, sh.n_q_heads, sh.head_dim) for n, d in zip(t.n_past, t.delta))
        by = sum(attend_bytes(n, d, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, e) for n, d in zip(t.n_past, t.delta) if d)
        return fl, by

    def run(self, steps, warmup):
        from paper_2605_26289_amd import binding as dk
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        dk.set_attend_timing(self.pool.handle, min(256, max(1, steps)))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        kernel_ms = dk.attend_times(self.pool.handle)
        dk.set_attend_timing(self.pool.handle, 0)
        # the same steps once more without the event records (two per step, about 4 us of stream time each)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        self.ms_per_step_no_events = (time.perf_counter() - t0) / steps * 1e3
        return wall / steps, float(np.mean(kernel_ms)), float(np.median(kernel_ms))

    def host_cache(self, slot):
        parts = self.host_kv.get(slot, [])
        sh = self.sh
        if not parts:
            z = np.zeros((0, sh.n_kv_heads, sh.head_dim), np.float32)
            return z, z
        return np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts])


def make_workload(name, drafts=8):
    from paper_2605_26289_amd import workloads as wl
    if name == "c5":
        return wl.config5(k_draft=drafts), -1
    if name == "c4":
        return wl.config4(), -1
    if name == "c4_512":
        return wl.config4(fixed_delta=512), -1
    if name == "c3":
        return wl.config3(), -1
    if name == "c2":
        return wl.config2(), -1
    if name == "mixed":
        from paper_2605_26289_amd import binding as dk
        # 4 slots prefill at once: the chunking rule of Sec. 3.2 cuts the 4096-token batch into 1024-token chunks
        return wl.mixed_prefill_decode(chunk=dk.prefill_chunk(4096, 4)), -1
    raise ValueError(name)


TUNING = []  # (name, value) pairs applied to every pool (--tune)
FUSED_STEP = True  # --step: dk_append_attend per step; False: dk_kv_append and dk_delta_attend as separate calls
def _traffic_table():
    """Lines of profiles/hbm_traffic.txt: (commit the readings were taken at, {workload: bytes per launch})."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.txt")
    commit, table = None, {}
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "#" and f[1] == "commit":
                commit = f[2]
            elif len(f) == 4 and not line.startswith("#"):
                table[f[0]] = table.get(f[0], 0) + int(f[2]) + int(f[3])
    except OSError:
        pass
    return commit, table


TRAFFIC_COMMIT, _TRAFFIC = _traffic_table()
TRAFFIC_SOURCE = "quoted: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings of this command taken at commit " \
                 f"{TRAFFIC_COMMIT}, kept in profiles/hbm_traffic.txt (all kernels of the call; not re-measured in this run)"


def measured_traffic(name):
    """HBM bytes per launch of the workload's attention (or verification) kernels as read by rocprofv3 counters
    (None if never profiled).  The counters cannot be read from inside this process; the readings of the profiled
    runs of this same command are kept as text under profiles/ and quoted here."""
    return _TRAFFIC.get(name)


def roofline_for(name, flops, nbytes, kernel_ms):
    """kernel_ms: median duration of the call's attention work (all kernels of dk_delta_attend), from HIP events the
    library records on the launch stream."""
    sec = kernel_ms * 1e-3
    traffic = measured_traffic(name)
    hbm = nbytes / sec / 1e9
    mfma = flops / sec / 1e12
    if name in ("c5", "c2"):
        return {"bound": "hbm", "achieved": round(hbm, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(hbm / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": TRAFFIC_SOURCE}
    r = {"bound": "mfma", "achieved": round(mfma, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
         "frac": round(mfma / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic, "traffic_source": TRAFFIC_SOURCE}
    if name == "mixed":  # both kernels in one call: the streaming part is bound by HBM, the tile part by the MFMA pipe
        r["hbm_frac_of_whole_call"] = round(hbm / HBM_PEAK_GBS, 4)
    return r


def verify_leg(w, vocab, steps, warmup):
    """Greedy verification of the batch's k+1 rows per slot over synthetic bf16 logits (the step after the verify
    attention in the paper's Alg. 2).  Times dk_verify_greedy alone with HIP events on the launch stream.  The calls
    rotate over enough distinct logits buffers that consecutive calls cannot be served from the 256 MB Infinity
    Cache: every logit comes from HBM."""
    import torch
    from paper_2605_26289_amd import binding as dk
    t = w.turns[-1]
    cu = np.concatenate([[0], np.cumsum(t.delta)]).astype(np.int32)
    rows, n = int(cu[-1]), len(t.delta)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed + 1000)
    one = rows * vocab * 2
    n_buf = max(2, -(-(640 << 20) // one))  # at least 640 MB in rotation
    logits = [torch.randn((rows, vocab), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
              for _ in range(n_buf)]
    am = logits[0].float().argmax(dim=1).to(torch.int32)  # only used to plant drafts that will be accepted
    toks = torch.randint(0, vocab, (rows,), generator=gen, device="cuda", dtype=torch.int32)
    accept = torch.rand((rows,), generator=gen, device="cuda") < 0.8
    toks[1:] = torch.where(accept[1:], am[:-1], toks[1:])
    cu_d = torch.from_numpy(cu).cuda()
    keep = torch.empty(n, dtype=torch.int32, device="cuda")
    nxt = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = torch.empty(dk.verify_workspace_bytes(rows, vocab, dk.BF16), dtype=torch.uint8, device="cuda")
    run = lambda i: dk.verify_greedy(n, rows, cu_d, logits[i % n_buf], dk.BF16, vocab, vocab, toks, keep, nxt, ws)  # noqa: E731
    for i in range(max(warmup, n_buf)):
        run(i)
    run(0)
    torch.cuda.synchronize()
    kept = round(float(keep.float().mean().item()), 2)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for i, (a, b) in enumerate(ev):
        a.record()
        run(i + 1)
        b.record()
    torch.cuda.synchronize()
    ms = float(np.median([a.elapsed_time(b) for a, b in ev]))
    ach = one / (ms * 1e-3) / 1e9
    return {"workload": f"greedy verification of {n} slots x {rows // max(n, 1)} rows, vocab {vocab}, bf16 logits, "
                        f"{n_buf} logits buffers in rotation ({n_buf * one >> 20} MiB)",
            "rows": rows, "ms": round(ms, 4), "rows_per_s": round(rows / (ms * 1e-3), 1),
            "mean_kept_tokens": kept,
            "roofline": {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": measured_traffic("verify"),
                         "traffic_source": TRAFFIC_SOURCE}}


def alg1_leg(w, reps, warmup):
    """The radix-cached per-turn procedure of the paper's Alg. 1 over a whole conversation: per turn, acquire a
    transient sequence, alias the longest cached prefix (metadata only), append and attend only the delta, save the
    turn into the prefix cache, release the sequence.  Reports throughput over all turns and how the conversation lies
    in the arena at its last turn (runs of consecutive cells, alias generations, cells held against logical cells)."""
    import torch
    from paper_2605_26289_amd import DevicePool
    from paper_2605_26289_amd import binding as dk
    from paper_2605_26289_amd import workloads as wl
    sh = w.shape
    tokens = wl.token_stream(w)
    prompts = []
    if w.history and w.history[0]:
        prompts.append(w.history[0])  # the system prompt is ingested (and cached) first, as its own turn
    prompts += [t.n_past[0] + t.delta[0] for t in w.turns]
    n_turns, total = len(prompts), prompts[-1]
    pool = DevicePool(n_turns + 6, total + 4096, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype,
                      n_session_slots=n_turns + 2)
    for name, value in TUNING:
        dk.set_tuning(pool.handle, name, value)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed)
    dt = pool.torch_dtype
    biggest = max(b - a for a, b in zip([0] + prompts[:-1], prompts))
    q = torch.randn((biggest, sh.n_q_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(dt)
    k = torch.randn((biggest, sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(dt)
    v = torch.randn((biggest, sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(dt)
    out = torch.empty_like(q)
    toks = np.asarray(tokens, dtype=np.int32)
    layout = {}

    def conversation(record=False):
        radix = dk.radix_create(pool.handle, total + 1024, 1)
        past = []
        for t, n in enumerate(prompts):
            slot = pool.acquire(0)
            n_past = dk.radix_begin_turn(radix, slot, toks[:n])
            past.append(n_past)
            d = n - n_past
            cu = np.asarray([0, d], dtype=np.int32)
            if FUSED_STEP:
                pool.append_attend([slot], cu, q[:d], k[:d], v[:d], sh.scale, out=out[:d])
            else:
                pool.append([slot], cu, k[:d], v[:d])
                pool.attend([slot], cu, q[:d], sh.scale, out=out[:d])
            if record and t == n_turns - 1:
                seg, depth = dk.seq_stats(pool.handle, slot)
                layout.update(segments_last_turn=seg, alias_generations=depth)
            dk.radix_save(radix, slot, toks[:n])
            pool.release(slot)
        if record:
            held, _ = dk.pool_stats(pool.handle)
            layout.update(cells_held=held, cells_logical=total, n_past_per_turn=past)
        torch.cuda.synchronize()
        dk.radix_destroy(radix)

    for _ in range(warmup):
        conversation()
    conversation(record=True)
    dk.set_attend_timing(pool.handle, min(256, n_turns))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        conversation()
    wall = (time.perf_counter() - t0) / reps
    kern = dk.attend_times(pool.handle)  # the last conversation's turns, oldest first
    dk.set_attend_timing(pool.handle, 0)
    new_tokens = sum(n - p for n, p in zip(prompts, layout["n_past_per_turn"]))
    first, last = w.turns[0], w.turns[-1]
    res = {"workload": f"{w.name} through Alg. 1 (acquire, radix alias, append delta, attend, save, release)",
           "turns": n_turns, "new_tokens": int(new_tokens), "cached_tokens_skipped": int(sum(layout["n_past_per_turn"])),
           "tokens_per_s": round(new_tokens / wall, 1), "ms_per_conversation": round(wall * 1e3, 4),
           "ms_per_turn": round(wall * 1e3 / n_turns, 4),
           "last_turn": {"n_past": int(layout["n_past_per_turn"][-1]), "delta": int(prompts[-1] - layout["n_past_per_turn"][-1]),
                         "attend_kernel_ms": round(float(kern[-1]), 4) if len(kern) else None},
           "segments_last_turn": int(layout["segments_last_turn"]), "alias_generations": int(layout["alias_generations"]),
           "cells_held": int(layout["cells_held"]), "cells_logical": int(layout["cells_logical"]),
           "fragmentation": round(layout["cells_held"] / max(layout["cells_logical"], 1) - 1.0, 4)}
    if len(kern):
        fl = attend_flops(res["last_turn"]["n_past"], res["last_turn"]["delta"], sh.n_q_heads, sh.head_dim)
        res["last_turn"]["achieved_tflops"] = round(fl / (float(kern[-1]) * 1e-3) / 1e12, 1)
    pool.close()
    return res


def alg2_leg(w, vocab, steps, warmup):
    """One speculative step of the paper's Alg. 2 per timed step, on one stream, with nothing read back between its
    stages: kv_append of all k+1 tokens, verify attention over them (appended mode), greedy verification of the
    (synthetic) logits on the device, an asynchronous copy of the kept counts to pinned memory.  The trim that drops
    the rejected tokens is deferred to the start of the next step, when the host reads the counts it needs anyway to
    build the next batch; it then rewinds the slots so that every step sees the same state."""
    import torch
    from paper_2605_26289_amd import DevicePool
    from paper_2605_26289_amd import binding as dk
    sh = w.shape
    t = w.turns[-1]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed + 7)
    cells = w.cells_needed() + 512 * (w.n_slots + 2)
    pool = DevicePool(w.n_slots, cells, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.dtype)
    for name, value in TUNING:
        dk.set_tuning(pool.handle, name, value)
    dt = pool.torch_dtype
    slots = np.asarray([pool.acquire() for _ in range(w.n_slots)], dtype=np.int32)
    for s, h in zip(slots, w.history):
        done = 0
        while done < h:
            c = min(65536, h - done)
            kv = torch.randn((c, sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(dt)
            pool.append([s], [0, c], kv, kv)
            done += c
    cu = np.concatenate([[0], np.cumsum(t.delta)]).astype(np.int32)
    rows, n = int(cu[-1]), len(t.delta)
    n_past = np.asarray(t.n_past, dtype=np.int64)
    q = torch.randn((rows, sh.n_q_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(dt)
    kn = torch.randn((rows, sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(dt)
    vn = torch.randn((rows, sh.n_kv_heads, sh.head_dim), generator=gen, device="cuda", dtype=torch.float32).to(dt)
    out = torch.empty_like(q)
    logits = torch.randn((rows, vocab), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    am = logits.float().argmax(dim=1).to(torch.int32)
    toks = torch.randint(0, vocab, (rows,), generator=gen, device="cuda", dtype=torch.int32)
    accept = torch.rand((rows,), generator=gen, device="cuda") < 0.8
    toks[1:] = torch.where(accept[1:], am[:-1], toks[1:])
    cu_d = torch.from_numpy(cu).cuda()
    keep_d = torch.empty(n, dtype=torch.int32, device="cuda")
    next_d = torch.empty(n, dtype=torch.int32, device="cuda")
    keep_h = torch.empty(n, dtype=torch.int32, pin_memory=True)
    vws = torch.empty(dk.verify_workspace_bytes(rows, vocab, dk.BF16), dtype=torch.uint8, device="cuda")
    copied = torch.cuda.Event()
    slots_sorted = slots[np.asarray(t.slots)]
    pool.ensure_workspace(slots_sorted, cu, 2)
    pool.append(slots_sorted, cu, kn, vn)
    pool.ensure_workspace(slots_sorted, cu, False)
    pool.trim_batch(slots_sorted, n_past)
    pending = [False]

    def settle():
        """The deferred part of the previous step: read the kept counts, drop the rejected tokens."""
        if pending[0]:
            copied.synchronize()
            pool.trim_batch(slots_sorted, n_past + keep_h.numpy())
            pool.trim_batch(slots_sorted, n_past)  # benchmark only: every step starts from the same state
            pending[0] = False

    def step():
        settle()
        if FUSED_STEP:
            pool.append_attend(slots_sorted, cu, q, kn, vn, sh.scale, out=out)
        else:
            pool.append(slots_sorted, cu, kn, vn)
            pool.attend(slots_sorted, cu, q, sh.scale, out=out)
        dk.verify_greedy(n, rows, cu_d, logits, dk.BF16, vocab, vocab, toks, keep_d, next_d, vws)
        keep_h.copy_(keep_d, non_blocking=True)
        copied.record()
        pending[0] = True

    for _ in range(warmup):
        step()
    settle()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    settle()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    kept = float(keep_h.float().mean().item())
    res = {"workload": f"Alg. 2 step on {w.name}: kv_append(k+1) + verify attention + on-device argmax/accept + "
                       "async copy of kept counts + deferred trim",
           "slots": n, "rows": rows, "ms_per_step": round(wall * 1e3, 4), "verified_tokens_per_s": round(rows / wall, 1),
           "kept_tokens_per_s": round(kept * n / wall, 1), "mean_kept_tokens": round(kept, 2),
           "host_syncs_inside_step": 0}
    pool.close()
    return res


def other_configs(steps, warmup):
    """Throughput of the remaining workload configs, a few steps each, for the record (no roofline claim for the
    launch-bound ones).  c3 is reported for its median turn and its final turn."""
    from paper_2605_26289_amd import workloads as wl
    import torch
    out = {}
    c3 = wl.config3()
    median_turn = int(np.argsort([t.delta[0] * (t.n_past[0] + 1) for t in c3.turns])[len(c3.turns) // 2])
    mixed, _ = make_workload("mixed")
    for key, w, turn in (("c1_fp32_single", wl.config1(), -1), ("c2_agent_5turn_final", wl.config2(), -1),
                         ("c3_coding_median_turn", c3, median_turn), ("c3_coding_final_turn", c3, -1),
                         ("c4_multi_agent", wl.config4(), -1), ("mixed_prefill_decode", mixed, -1)):
        sc = Scenario(w, turn)
        step_s, _, kern_ms = sc.run(steps, warmup)  # median kernel time
        fl, by = sc.algorithmic()
        out[key] = {"new_tokens_per_step": int(sc.total), "cached_tokens": int(sum(sc.turn.n_past)),
                    "tokens_per_s": round(sc.total / step_s, 1), "ms_per_step": round(step_s * 1e3, 4),
                    "ms_per_step_no_events": round(sc.ms_per_step_no_events, 4),
                    "attend_kernel_ms": round(kern_ms, 4),
                    "achieved_tflops": round(fl / (kern_ms * 1e-3) / 1e12, 1),
                    "mfma_frac": round(fl / (kern_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                    "achieved_gbs": round(by / (kern_ms * 1e-3) / 1e9, 1),
                    "hbm_frac": round(by / (kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        del sc
        torch.cuda.empty_cache()
    return out


def cpu_baseline(sc, budget_s):
    """Times the fp64 oracle, as it stands, on a bounded sample of the same batch; also checks the GPU rows."""
    import oracle
    cores = len(os.sched_getaffinity(0))
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        blas_threads = cores
    t = sc.turn
    sh = sc.sh
    done_tokens, spent, worst_abs, worst_rel, used, checked = 0, 0.0, 0.0, 0.0, 0, 0
    gpu = sc.out.float().cpu().numpy()
    q = sc.q.float().cpu().numpy()
    kn = sc.k_new.float().cpu().numpy()
    vn = sc.v_new.float().cpu().numpy()
    passes = 0
    while spent < min(10.0, budget_s):  # about 10 s of oracle work: whole passes over the mirrored slots
        before = spent
        for b, s in enumerate(t.slots):
            if s not in sc.keep or t.delta[b] == 0:
                continue
            if spent > budget_s:
                break
            lo, hi = int(sc.cu[b]), int(sc.cu[b + 1])
            kc, vc = sc.host_cache(s)
            kc, vc = kc[: t.n_past[b]], vc[: t.n_past[b]]
            rows = None
            if hi - lo > 32:  # long deltas: a spread of rows is enough for the timing sample
                rows = sorted(set(np.linspace(0, hi - lo - 1, 16).astype(int).tolist()))
            t0 = time.perf_counter()
            ref, _ = oracle.delta_attend(q[lo:hi], kc, vc, kn[lo:hi], vn[lo:hi], sh.scale, rows)
            spent += time.perf_counter() - t0
            sel = list(range(hi - lo)) if rows is None else rows
            done_tokens += len(sel)
            if passes == 0:  # the GPU rows are checked once
                diff = np.abs(gpu[lo:hi][sel] - ref[sel])
                rms = np.sqrt((ref[sel] ** 2).mean(axis=-1, keepdims=True))
                worst_abs = max(worst_abs, float(diff.max()))
                worst_rel = max(worst_rel, float((diff / np.maximum(np.abs(ref[sel]), rms)).max()))
                used += 1
                checked = done_tokens
        passes += 1
        if spent == before:
            break
    if not done_tokens:
        return None, None
    one_thread = None
    if threadpool_limits is not None:  # per-core figure: the same oracle calls with the BLAS pinned to one thread
        spent1, tokens1 = 0.0, 0
        with threadpool_limits(limits=1):
            for b, s in enumerate(t.slots):
                if s not in sc.keep or t.delta[b] == 0 or spent1 > min(4.0, budget_s / 3):
                    continue
                lo, hi = int(sc.cu[b]), int(sc.cu[b + 1])
                kc, vc = sc.host_cache(s)
                kc, vc = kc[: t.n_past[b]], vc[: t.n_past[b]]
                rows = None if hi - lo <= 32 else sorted(set(np.linspace(0, hi - lo - 1, 16).astype(int).tolist()))
                t0 = time.perf_counter()
                oracle.delta_attend(q[lo:hi], kc, vc, kn[lo:hi], vn[lo:hi], sh.scale, rows)
                spent1 += time.perf_counter() - t0
                tokens1 += (hi - lo) if rows is None else len(rows)
        if tokens1:
            one_thread = round(tokens1 / spent1, 2)
    base = {"value": round(done_tokens / spent, 2), "unit": "new tokens/s", "cores": int(min(cores, blas_threads)),
            "host_cores_available": int(cores), "blas_threads": int(blas_threads), "one_thread_value": one_thread,
            "kind": "oracle",
            "sample": f"{checked} new-token rows of {used} slot(s) of the same batch, {passes} pass(es), "
                      f"fp64 NumPy, {spent:.1f} s"}
    return base, {"max_abs": worst_abs, "max_rel": worst_rel, "rows": checked}


def host_profile(args):
    """Where the host time of a step goes, for a workload whose step is shorter than its launch path (c2 by default):
    wall time per Python-level call, and inside the library per phase (dk_host_times)."""
    import torch
    from paper_2605_26289_amd import binding as dk
    name = args.workload if args.workload in ("c2", "c3", "c4", "c4_512", "c5", "mixed") else "c2"
    w, turn = make_workload(name, args.drafts)
    sc = Scenario(w, turn)
    t = sc.turn
    for _ in range(max(args.warmup, 20)):
        sc.step()
    torch.cuda.synchronize()
    n = max(args.steps, 200)
    dk.host_times(sc.pool.handle, reset=True)
    acc = {"append_attend": [], "kv_append": [], "delta_attend": [], "trim_batch": []}
    t_all = time.perf_counter()
    host_wall = 0.0
    t_chunk = time.perf_counter()
    for i in range(n):
        if i and i % 16 == 0:
            # the launch queue is finite and the runtime stalls for tens of milliseconds when it is full: drain it
            # every 16 steps, outside the host-time account
            host_wall += time.perf_counter() - t_chunk
            torch.cuda.synchronize()
            t_chunk = time.perf_counter()
        a = time.perf_counter()
        if FUSED_STEP:
            sc.pool.append_attend(t.slots, sc.cu, sc.q, sc.k_new, sc.v_new, sc.sh.scale, out=sc.out)
            c = time.perf_counter()
            acc["append_attend"].append(c - a)
            if sc.keep_len is not None:
                sc.pool.trim_batch(t.slots, sc.keep_len)
        elif t.staged:
            sc.pool.attend(t.slots, sc.cu, sc.q, sc.sh.scale, sc.k_new, sc.v_new, out=sc.out)
            b = time.perf_counter()
            sc.pool.append(t.slots, sc.cu, sc.k_new, sc.v_new, sc.n_accept)
            c = time.perf_counter()
            acc["delta_attend"].append(b - a)
            acc["kv_append"].append(c - b)
        else:
            sc.pool.append(t.slots, sc.cu, sc.k_new, sc.v_new)
            b = time.perf_counter()
            sc.pool.attend(t.slots, sc.cu, sc.q, sc.sh.scale, out=sc.out)
            c = time.perf_counter()
            acc["kv_append"].append(b - a)
            acc["delta_attend"].append(c - b)
        sc._rewind()
        acc["trim_batch"].append(time.perf_counter() - c)
    acc = {k: v for k, v in acc.items() if v}
    host_wall += time.perf_counter() - t_chunk
    torch.cuda.synchronize()
    total_wall = time.perf_counter() - t_all
    inside, calls = dk.host_times(sc.pool.handle)
    _, _, kern_ms = sc.run(50, 5)
    print(json.dumps({"workload": w.name, "steps": n, "host_us_per_step": round(host_wall / n * 1e6, 2),
                      "wall_us_per_step_with_gpu_drain": round(total_wall / n * 1e6, 2),
                      "attend_kernel_us": round(kern_ms * 1e3, 2),
                      "python_call_us_median": {k: round(float(np.median(v)) * 1e6, 2) for k, v in acc.items()},
                      "python_call_us_mean": {k: round(float(np.mean(v)) * 1e6, 2) for k, v in acc.items()},
                      "python_call_us_max": {k: round(float(np.max(v)) * 1e6, 2) for k, v in acc.items()},
                      "inside_library_us": {k: round(v / n, 2) for k, v in inside.items()},
                      "calls": {"delta_attend": calls[0], "kv_append": calls[1]}}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no multi-GPU part (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback)", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_per_launch": n, "launches": 5}))
        return
    global FUSED_STEP
    FUSED_STEP = args.step == "fused"
    for item in args.tune:
        name, _, value = item.partition("=")
        TUNING.append((name, float(value)))
    from paper_2605_26289_amd import workloads as wl
    if args.host_profile:
        host_profile(args)
        return
    if args.workload in ("c2_alg1", "c3_alg1"):
        w = wl.config2() if args.workload == "c2_alg1" else wl.config3()
        print(json.dumps(alg1_leg(w, max(3, args.steps // 2), 2)))
        return
    if args.workload == "alg2":
        print(json.dumps(alg2_leg(wl.config5(k_draft=args.drafts), args.vocab, args.steps, args.warmup)))
        return
    if args.workload == "verify":
        print(json.dumps(verify_leg(wl.config5(k_draft=args.drafts), args.vocab, args.steps, args.warmup)))
        return
    w, turn = make_workload(args.workload, args.drafts)
    keep = 0 if args.no_cpu_baseline else min(w.n_slots, 32)
    sc = Scenario(w, turn, keep_host_slots=keep)
    step_s, kern_mean_ms, kern_med_ms = sc.run(args.steps, args.warmup)
    flops, nbytes = sc.algorithmic()
    result = {
        "metric": "delta-prefill new tokens/sec", "value": round(sc.total / step_s, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(step_s * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": sc.sh.dtype, "data": "synthetic",
        "config": {"workload": w.name, "slots": w.n_slots, "new_tokens_per_step": int(sc.total),
                   "n_q_heads": sc.sh.n_q_heads, "n_kv_heads": sc.sh.n_kv_heads, "head_dim": sc.sh.head_dim,
                   "cached_tokens": int(sum(sc.turn.n_past)), "mode": "fused" if FUSED_STEP else ("staged" if sc.turn.staged else "appended"),
                   "step": ("append_attend + trim" if FUSED_STEP else
                            "delta_attend + kv_append + trim" if sc.turn.staged else "kv_append + delta_attend + trim")},
        "ms_per_step_no_events": round(sc.ms_per_step_no_events, 4),
        "attend_kernel_ms": round(kern_med_ms, 4), "attend_kernel_ms_mean": round(kern_mean_ms, 4),
        "attend_only_tokens_per_s": round(sc.total / (kern_med_ms * 1e-3), 1),
        "algorithmic": {"flops": int(flops), "bytes": int(nbytes)},
        "roofline": roofline_for(args.workload, flops, nbytes, kern_med_ms),
    }
    if not args.no_extra and args.workload == "c5":
        # The secondary legs run before the CPU leg on purpose: ten seconds of host-only work let the GPU drop
        # into a low-power state, and the first milliseconds after that are not representative.
        # second regime in the same run: Delta = 512 on every slot of the multi-agent batch (MFMA-bound)
        w2, t2 = make_workload("c4_512")
        sc2 = Scenario(w2, t2)
        s2, _, km2 = sc2.run(args.steps, max(args.warmup, 10))
        f2, b2 = sc2.algorithmic()
        result["extra"] = {"workload": w2.name + "_delta512", "new_tokens_per_step": int(sc2.total),
                           "tokens_per_s": round(sc2.total / s2, 1), "ms_per_step": round(s2 * 1e3, 4),
                           "ms_per_step_no_events": round(sc2.ms_per_step_no_events, 4),
                           "attend_kernel_ms": round(km2, 4), "roofline": roofline_for("c4_512", f2, b2, km2)}
        del sc2
        torch.cuda.empty_cache()
        result["verify"] = verify_leg(w, args.vocab, args.steps, args.warmup)
        result["alg2_step"] = alg2_leg(w, args.vocab, args.steps, args.warmup)
        result["other_configs"] = other_configs(max(5, args.steps // 2), 3)
        result["alg1"] = {"c2": alg1_leg(wl.config2(), 10, 2), "c3": alg1_leg(wl.config3(), 3, 1)}
    if not args.no_cpu_baseline:
        base, parity = cpu_baseline(sc, args.cpu_seconds)
        result["cpu_baseline"] = base
        result["parity_sample"] = parity
    else:
        result["cpu_baseline"] = None
    del sc
    print(json.dumps(result))


if __name__ == "__main__":
    main()
