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
    ap.add_argument("--workload", default="c5", choices=["c5", "c4", "c4_512", "c3", "c2"])
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
        # size the workspace once, in the state the attend call will see
        if t.staged:
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
        for s, n in zip(self.turn.slots, self.turn.n_past):
            self.pool.trim(s, n)

    def step(self):
        t = self.turn
        if t.staged:
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
    raise ValueError(name)


def measured_traffic(name):
    """HBM bytes per launch of the workload's dominant kernel as read by rocprofv3 counters (None if never profiled).

    The counters cannot be read from inside this process; the readings of the profiled runs of this same command
    are kept as text under profiles/ and quoted here."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 4 and f[0] == name:
                return int(f[2]) + int(f[3])
    except OSError:
        pass
    return None


def roofline_for(name, flops, nbytes, kernel_ms):
    sec = kernel_ms * 1e-3
    traffic = measured_traffic(name)
    if name in ("c5", "c2"):
        ach = nbytes / sec / 1e9
        return {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": traffic}
    ach = flops / sec / 1e12
    return {"bound": "mfma", "achieved": round(ach, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": traffic}


def verify_leg(w, vocab, steps, warmup):
    """Greedy verification of the batch's k+1 rows per slot over synthetic bf16 logits (the step after the verify
    attention in the paper's Alg. 2).  Times dk_verify_greedy alone with HIP events on the launch stream."""
    import torch
    from paper_2605_26289_amd import binding as dk
    t = w.turns[-1]
    cu = np.concatenate([[0], np.cumsum(t.delta)]).astype(np.int32)
    rows, n = int(cu[-1]), len(t.delta)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(w.seed + 1000)
    logits = torch.randn((rows, vocab), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    am = logits.float().argmax(dim=1).to(torch.int32)  # only used to plant drafts that will be accepted
    toks = torch.randint(0, vocab, (rows,), generator=gen, device="cuda", dtype=torch.int32)
    accept = torch.rand((rows,), generator=gen, device="cuda") < 0.8
    toks[1:] = torch.where(accept[1:], am[:-1], toks[1:])
    cu_d = torch.from_numpy(cu).cuda()
    keep = torch.empty(n, dtype=torch.int32, device="cuda")
    nxt = torch.empty(n, dtype=torch.int32, device="cuda")
    ws = torch.empty(dk.verify_workspace_bytes(rows, vocab, dk.BF16), dtype=torch.uint8, device="cuda")
    run = lambda: dk.verify_greedy(n, rows, cu_d, logits, dk.BF16, vocab, vocab, toks, keep, nxt, ws)  # noqa: E731
    for _ in range(warmup):
        run()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        run()
        b.record()
    torch.cuda.synchronize()
    ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    nbytes = rows * vocab * 2
    ach = nbytes / (ms * 1e-3) / 1e9
    return {"workload": f"greedy verification of {n} slots x {rows // max(n, 1)} rows, vocab {vocab}, bf16 logits",
            "rows": rows, "ms": round(ms, 4), "rows_per_s": round(rows / (ms * 1e-3), 1),
            "mean_kept_tokens": round(float(keep.float().mean().item()), 2),
            "roofline": {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": None}}


def other_configs(steps, warmup):
    """Throughput of the remaining workload configs, a few steps each, for the record (no roofline claim for the
    launch-bound ones).  c3 is reported for its median turn and its final turn."""
    from paper_2605_26289_amd import workloads as wl
    import torch
    out = {}
    c3 = wl.config3()
    median_turn = int(np.argsort([t.delta[0] * (t.n_past[0] + 1) for t in c3.turns])[len(c3.turns) // 2])
    for key, w, turn in (("c1_fp32_single", wl.config1(), -1), ("c2_agent_5turn_final", wl.config2(), -1),
                         ("c3_coding_median_turn", c3, median_turn), ("c3_coding_final_turn", c3, -1),
                         ("c4_multi_agent", wl.config4(), -1)):
        sc = Scenario(w, turn)
        step_s, kern_ms, _ = sc.run(steps, warmup)
        fl, by = sc.algorithmic()
        out[key] = {"new_tokens_per_step": int(sc.total), "cached_tokens": int(sum(sc.turn.n_past)),
                    "tokens_per_s": round(sc.total / step_s, 1), "ms_per_step": round(step_s * 1e3, 4),
                    "attend_kernel_ms": round(kern_ms, 4),
                    "achieved_tflops": round(fl / (kern_ms * 1e-3) / 1e12, 1),
                    "achieved_gbs": round(by / (kern_ms * 1e-3) / 1e9, 1)}
        del sc
        torch.cuda.empty_cache()
    return out


def cpu_baseline(sc, budget_s):
    """Times the fp64 oracle, as it stands, on a bounded sample of the same batch; also checks the GPU rows."""
    import oracle
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
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
    base = {"value": round(done_tokens / spent, 2), "unit": "new tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{checked} new-token rows of {used} slot(s) of the same batch, {passes} pass(es), "
                      f"fp64 NumPy, {spent:.1f} s"}
    return base, {"max_abs": worst_abs, "max_rel": worst_rel, "rows": checked}


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
                   "cached_tokens": int(sum(sc.turn.n_past)), "mode": "staged" if sc.turn.staged else "appended",
                   "step": "delta_attend + kv_append + trim"},
        "attend_kernel_ms": round(kern_mean_ms, 4), "attend_kernel_ms_median": round(kern_med_ms, 4),
        "attend_only_tokens_per_s": round(sc.total / (kern_mean_ms * 1e-3), 1),
        "algorithmic": {"flops": int(flops), "bytes": int(nbytes)},
        "roofline": roofline_for(args.workload, flops, nbytes, kern_mean_ms),
    }
    if not args.no_extra and args.workload == "c5":
        # The secondary legs run before the CPU leg on purpose: ten seconds of host-only work let the GPU drop
        # into a low-power state, and the first milliseconds after that are not representative.
        # second regime in the same run: Delta = 512 on every slot of the multi-agent batch (MFMA-bound)
        w2, t2 = make_workload("c4_512")
        sc2 = Scenario(w2, t2)
        s2, km2, _ = sc2.run(args.steps, max(args.warmup, 10))
        f2, b2 = sc2.algorithmic()
        result["extra"] = {"workload": w2.name + "_delta512", "new_tokens_per_step": int(sc2.total),
                           "tokens_per_s": round(sc2.total / s2, 1), "ms_per_step": round(s2 * 1e3, 4),
                           "attend_kernel_ms": round(km2, 4), "roofline": roofline_for("c4_512", f2, b2, km2)}
        del sc2
        torch.cuda.empty_cache()
        result["verify"] = verify_leg(w, args.vocab, args.steps, args.warmup)
        result["other_configs"] = other_configs(max(5, args.steps // 2), 3)
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
