"""ctypes binding of libdeltakv: argument marshalling only.

Function names mirror the C ABI (include/deltakv.h) without the dk_ prefix.  Device memory and
streams come from PyTorch; nothing is computed here.  If the shared library has not been built,
every call raises: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdeltakv.so")

F32, BF16 = 0, 1
OK = 0
STATUS_NAMES = {0: "OK", -1: "INVALID", -2: "TIMEOUT", -3: "NO_CELLS", -4: "NO_SLOT", -5: "DUP_SLOT",
                -6: "UNSUPPORTED", -7: "WORKSPACE", -8: "HIP", -9: "BUSY", -10: "NO_MEMORY"}
BUSY = -9


class DeltaKVError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        self.name = STATUS_NAMES.get(status, str(status))
        super().__init__(f"{where}: {self.name} ({detail})" if detail else f"{where}: {self.name}")


class PoolDesc(C.Structure):
    _fields_ = [("n_slots", C.c_int32), ("n_session_slots", C.c_int32), ("arena_cells", C.c_int64),
                ("granule_cells", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("dtype", C.c_int32), ("k_arena", C.c_void_p), ("v_arena", C.c_void_p),
                ("dev_meta", C.c_void_p), ("dev_meta_bytes", C.c_int64), ("host_staging", C.c_void_p),
                ("host_staging_bytes", C.c_int64), ("staging_depth", C.c_int32)]


_lib = None

_I32P = C.POINTER(C.c_int32)
_I64P = C.POINTER(C.c_int64)

SIGNATURES = {
    "dk_meta_bytes": (C.c_int32, [C.POINTER(PoolDesc), _I64P]),
    "dk_staging_bytes": (C.c_int32, [C.POINTER(PoolDesc), _I64P]),
    "dk_set_tuning": (C.c_int32, [C.c_void_p, C.c_char_p, C.c_double]),
    "dk_pool_create": (C.c_int32, [C.POINTER(PoolDesc), C.POINTER(C.c_void_p)]),
    "dk_pool_destroy": (C.c_int32, [C.c_void_p]),
    "dk_seq_acquire": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int64, _I32P]),
    "dk_seq_release": (C.c_int32, [C.c_void_p, C.c_int32]),
    "dk_seq_len": (C.c_int32, [C.c_void_p, C.c_int32, _I64P]),
    "dk_seq_alias": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_int64]),
    "dk_seq_trim": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int64]),
    "dk_seq_trim_batch": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, _I64P]),
    "dk_kv_append": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, _I32P, _I32P, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dk_kv_reserve": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, _I32P, _I32P, _I64P]),
    "dk_attend_workspace_bytes": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, _I32P, C.c_int32, _I64P]),
    "dk_delta_attend": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, _I32P, C.c_void_p, C.c_void_p, C.c_void_p,
                                    C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]),
    "dk_append_attend": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, _I32P, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]),
    "dk_delta_attend_noalloc": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, _I32P, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dk_staging_wait": (C.c_int32, [C.c_void_p]),
    "dk_seq_cells": (C.c_int32, [C.c_void_p, C.c_int32, _I64P, C.c_int64]),
    "dk_seq_gather": (C.c_int32, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "dk_seq_stats": (C.c_int32, [C.c_void_p, C.c_int32, _I64P, _I64P]),
    "dk_pool_stats": (C.c_int32, [C.c_void_p, _I64P, _I64P]),
    "dk_verify_workspace_bytes": (C.c_int32, [C.c_int32, C.c_int64, C.c_int32, _I64P]),
    "dk_verify_greedy": (C.c_int32, [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int64,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64,
                                     C.c_void_p]),
    "dk_radix_create": (C.c_int32, [C.c_void_p, C.c_int64, C.c_int32, C.POINTER(C.c_void_p)]),
    "dk_radix_destroy": (C.c_int32, [C.c_void_p]),
    "dk_radix_begin_turn": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, C.c_int64, _I64P]),
    "dk_radix_save": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, C.c_int64, _I32P]),
    "dk_radix_stats": (C.c_int32, [C.c_void_p, _I64P, _I64P, _I64P, _I64P]),
    "dk_radix_evicted_path": (C.c_int32, [C.c_void_p, C.c_int64, _I32P, C.c_int64, _I64P]),
    "dk_pld_lookup": (C.c_int32, [_I32P, C.c_int64, C.c_int32, C.c_int32, C.c_int32, _I32P, _I32P, _I32P]),
    "dk_pld_gate": (C.c_int32, [C.POINTER(C.c_float), C.c_int32, C.c_int32, C.c_float, C.c_float, C.c_int32,
                                C.c_int32, _I32P]),
    "dk_prefill_chunk": (C.c_int32, [C.c_int64, C.c_int32, C.c_int32, _I64P]),
    "dk_fnv1a32": (C.c_int32, [C.c_void_p, C.c_int64, C.POINTER(C.c_uint32)]),
    "dk_prefill_groups": (C.c_int32, [C.c_int32, C.POINTER(_I32P), _I64P, _I64P, _I32P, C.c_int32, _I32P, _I64P]),
    "dk_set_attend_variant": (C.c_int32, [C.c_void_p, C.c_int32]),
    "dk_set_attend_timing": (C.c_int32, [C.c_void_p, C.c_int32]),
    "dk_attend_times": (C.c_int32, [C.c_void_p, C.POINTER(C.c_float), C.c_int32, _I32P]),
    "dk_last_attend_ms": (C.c_int32, [C.c_void_p, C.POINTER(C.c_float)]),
    "dk_host_times": (C.c_int32, [C.c_void_p, C.c_int32, C.POINTER(C.c_double), _I64P]),
    "dk_strerror": (C.c_char_p, [C.c_int32]),
    "dk_last_hip_error": (C.c_int32, [C.c_void_p]),
}


def lib() -> C.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2605_26289_amd.build` "
                "(there is no CPU fallback)")
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _check(rc: int, where: str, pool=None):
    if rc != OK:
        detail = ""
        if rc == -8 and pool is not None:
            detail = f"hipError {lib().dk_last_hip_error(pool)}"
        raise DeltaKVError(rc, where, detail)


def _i32(values: Optional[Sequence[int]]):
    if values is None:
        return None, None
    arr = np.ascontiguousarray(values, dtype=np.int32)
    return arr, arr.ctypes.data_as(_I32P)


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    h = int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)
    return h or None


# --------------------------------------------------------------------------- pool
def meta_bytes(desc: PoolDesc) -> int:
    out = C.c_int64()
    _check(lib().dk_meta_bytes(C.byref(desc), C.byref(out)), "meta_bytes")
    return out.value


def staging_bytes(desc: PoolDesc) -> int:
    out = C.c_int64()
    _check(lib().dk_staging_bytes(C.byref(desc), C.byref(out)), "staging_bytes")
    return out.value


def set_tuning(pool, name: str, value: float) -> None:
    _check(lib().dk_set_tuning(pool, name.encode(), float(value)), f"set_tuning({name})")


def _launch(call, where: str, pool, stream):
    """Runs a launching call; when every staging buffer is still in flight (BUSY) waits for one to come free and repeats.
    The C ABI itself never waits: back-pressure is the caller's policy, and this is the binding's."""
    rc = call()
    while rc == BUSY:
        # wait for the oldest upload only: the work queued behind it keeps the device busy meanwhile
        _check(lib().dk_staging_wait(pool), "staging_wait", pool)
        rc = call()
    _check(rc, where, pool)


def staging_wait(pool) -> None:
    _check(lib().dk_staging_wait(pool), "staging_wait", pool)


def pool_create(desc: PoolDesc) -> C.c_void_p:
    out = C.c_void_p()
    _check(lib().dk_pool_create(C.byref(desc), C.byref(out)), "pool_create")
    return out


def pool_destroy(pool) -> None:
    _check(lib().dk_pool_destroy(pool), "pool_destroy")


def seq_acquire(pool, region: int = 0, timeout_ms: int = 0) -> int:
    out = C.c_int32()
    _check(lib().dk_seq_acquire(pool, region, timeout_ms, C.byref(out)), "seq_acquire")
    return out.value


def seq_release(pool, slot: int) -> None:
    _check(lib().dk_seq_release(pool, slot), "seq_release")


def seq_len(pool, slot: int) -> int:
    out = C.c_int64()
    _check(lib().dk_seq_len(pool, slot, C.byref(out)), "seq_len")
    return out.value


def seq_alias(pool, donor: int, dst: int, p0: int, p1: int) -> None:
    _check(lib().dk_seq_alias(pool, donor, dst, p0, p1), "seq_alias")


def seq_trim(pool, slot: int, new_len: int) -> None:
    _check(lib().dk_seq_trim(pool, slot, new_len), "seq_trim")


def seq_trim_batch(pool, slots, new_len) -> None:
    s_arr, s_p = _i32(slots)
    n_arr = np.ascontiguousarray(new_len, dtype=np.int64)
    _check(lib().dk_seq_trim_batch(pool, len(s_arr), s_p, n_arr.ctypes.data_as(_I64P)), "seq_trim_batch")


def seq_cells(pool, slot: int) -> np.ndarray:
    n = seq_len(pool, slot)
    out = np.full(n, -1, dtype=np.int64)
    _check(lib().dk_seq_cells(pool, slot, out.ctypes.data_as(_I64P), n), "seq_cells")
    return out


def seq_stats(pool, slot: int):
    """(runs of consecutive cells, alias generations) of a slot"""
    seg, depth = C.c_int64(), C.c_int64()
    _check(lib().dk_seq_stats(pool, slot, C.byref(seg), C.byref(depth)), "seq_stats")
    return seg.value, depth.value


def pool_stats(pool):
    held, free = C.c_int64(), C.c_int64()
    _check(lib().dk_pool_stats(pool, C.byref(held), C.byref(free)), "pool_stats")
    return held.value, free.value


# --------------------------------------------------------------------------- GPU calls
def kv_append(pool, slots, cu_delta, k_new, v_new, n_accept=None, stream=None) -> None:
    s_arr, s_p = _i32(slots)
    c_arr, c_p = _i32(cu_delta)
    a_arr, a_p = _i32(n_accept)
    st = _stream(stream)
    _launch(lambda: lib().dk_kv_append(pool, len(s_arr), s_p, c_p, a_p, _ptr(k_new), _ptr(v_new), st),
            "kv_append", pool, stream)


def kv_reserve(pool, slots, cu_delta, n_accept=None) -> np.ndarray:
    s_arr, s_p = _i32(slots)
    c_arr, c_p = _i32(cu_delta)
    a_arr, a_p = _i32(n_accept)
    out = np.full(int(c_arr[-1]) if len(c_arr) else 0, -2, dtype=np.int64)
    _check(lib().dk_kv_reserve(pool, len(s_arr), s_p, c_p, a_p, out.ctypes.data_as(_I64P)), "kv_reserve")
    return out


def attend_workspace_bytes(pool, slots, cu_delta, staged) -> int:
    """staged: False / 0 appended mode, True / 1 staged mode, 2 for append_attend."""
    s_arr, s_p = _i32(slots)
    c_arr, c_p = _i32(cu_delta)
    out = C.c_int64()
    _check(lib().dk_attend_workspace_bytes(pool, len(s_arr), s_p, c_p, int(staged), C.byref(out)),
           "attend_workspace_bytes", pool)
    return out.value


def delta_attend(pool, slots, cu_delta, q, out, scale: float, k_new=None, v_new=None, lse=None,
                 workspace=None, stream=None) -> None:
    s_arr, s_p = _i32(slots)
    c_arr, c_p = _i32(cu_delta)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = _stream(stream)
    _launch(lambda: lib().dk_delta_attend(pool, len(s_arr), s_p, c_p, _ptr(q), _ptr(k_new), _ptr(v_new),
                                          float(scale), _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes, st),
            "delta_attend", pool, stream)


def append_attend(pool, slots, cu_delta, q, k_new, v_new, out, scale: float, lse=None, workspace=None,
                  stream=None) -> None:
    s_arr, s_p = _i32(slots)
    c_arr, c_p = _i32(cu_delta)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = _stream(stream)
    _launch(lambda: lib().dk_append_attend(pool, len(s_arr), s_p, c_p, _ptr(q), _ptr(k_new), _ptr(v_new),
                                           float(scale), _ptr(out), _ptr(lse), _ptr(workspace), ws_bytes, st),
            "append_attend", pool, stream)


STATIC_SCRATCH_BYTES = 32 << 20


def delta_attend_noalloc(pool, slots, cu_delta, q, out, scale: float, k_new=None, v_new=None, lse=None,
                         stream=None) -> None:
    s_arr, s_p = _i32(slots)
    c_arr, c_p = _i32(cu_delta)
    st = _stream(stream)
    _launch(lambda: lib().dk_delta_attend_noalloc(pool, len(s_arr), s_p, c_p, _ptr(q), _ptr(k_new), _ptr(v_new),
                                                  float(scale), _ptr(out), _ptr(lse), st),
            "delta_attend_noalloc", pool, stream)


def verify_workspace_bytes(total_rows: int, vocab: int, dtype: int) -> int:
    out = C.c_int64()
    _check(lib().dk_verify_workspace_bytes(int(total_rows), int(vocab), int(dtype), C.byref(out)),
           "verify_workspace_bytes")
    return out.value


def verify_greedy(n_seqs: int, total_rows: int, cu_delta_dev, logits, dtype: int, vocab: int, row_stride: int,
                  batch_tokens, n_keep_out, next_token_out, workspace, argmax_out=None, stream=None) -> None:
    """All tensors are device tensors; nothing is synchronised."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().dk_verify_greedy(int(n_seqs), int(total_rows), _ptr(cu_delta_dev), _ptr(logits), int(dtype),
                                  int(vocab), int(row_stride), _ptr(batch_tokens), _ptr(argmax_out),
                                  _ptr(n_keep_out), _ptr(next_token_out), _ptr(workspace), ws_bytes,
                                  _stream(stream)), "verify_greedy")


# -- host-only: radix prefix cache, prompt lookup, scheduler helpers ---------------------------------------
def radix_create(pool, cell_budget: int, keep_last: int = 1) -> C.c_void_p:
    out = C.c_void_p()
    _check(lib().dk_radix_create(pool, int(cell_budget), int(keep_last), C.byref(out)), "radix_create")
    return out


def radix_destroy(radix) -> None:
    _check(lib().dk_radix_destroy(radix), "radix_destroy")


def radix_begin_turn(radix, slot: int, tokens) -> int:
    t_arr, t_p = _i32(tokens)
    out = C.c_int64()
    _check(lib().dk_radix_begin_turn(radix, slot, t_p, len(t_arr), C.byref(out)), "radix_begin_turn")
    return out.value


def radix_save(radix, slot: int, tokens) -> bool:
    t_arr, t_p = _i32(tokens)
    out = C.c_int32()
    _check(lib().dk_radix_save(radix, slot, t_p, len(t_arr), C.byref(out)), "radix_save")
    return bool(out.value)


def radix_stats(radix):
    """(nodes, cells held, donor slots held, leaves shed so far)"""
    v = [C.c_int64() for _ in range(4)]
    _check(lib().dk_radix_stats(radix, *[C.byref(x) for x in v]), "radix_stats")
    return tuple(x.value for x in v)


def radix_evicted_path(radix, index: int):
    n = C.c_int64()
    _check(lib().dk_radix_evicted_path(radix, index, None, 0, C.byref(n)), "radix_evicted_path")
    out = np.zeros(max(n.value, 1), dtype=np.int32)
    _check(lib().dk_radix_evicted_path(radix, index, out.ctypes.data_as(_I32P), n.value, C.byref(n)),
           "radix_evicted_path")
    return out[: n.value].tolist()


def pld_lookup(recent, min_match: int, max_match: int, max_draft: int):
    """(draft tokens, matched n-gram length)"""
    r_arr, r_p = _i32(recent)
    draft = np.zeros(max(max_draft, 1), dtype=np.int32)
    k, n = C.c_int32(), C.c_int32()
    _check(lib().dk_pld_lookup(r_p, len(r_arr), min_match, max_match, max_draft, draft.ctypes.data_as(_I32P),
                               C.byref(k), C.byref(n)), "pld_lookup")
    return draft[: k.value].tolist(), n.value


def pld_gate(ema: float, proposed: int, accepted: int, beta: float, threshold: float, floor_len: int, max_len: int):
    """(new average, proposal length for the next step)"""
    e, nxt = C.c_float(ema), C.c_int32()
    _check(lib().dk_pld_gate(C.byref(e), proposed, accepted, beta, threshold, floor_len, max_len, C.byref(nxt)),
           "pld_gate")
    return e.value, nxt.value


def prefill_chunk(n_batch: int, n_prefilling: int, latency_sensitive: bool = False) -> int:
    out = C.c_int64()
    _check(lib().dk_prefill_chunk(n_batch, n_prefilling, int(latency_sensitive), C.byref(out)), "prefill_chunk")
    return out.value


def fnv1a32(data: bytes) -> int:
    out = C.c_uint32()
    buf = C.create_string_buffer(data, len(data))
    _check(lib().dk_fnv1a32(buf, len(data), C.byref(out)), "fnv1a32")
    return out.value


def prefill_groups(prompts, n_past, prefix_id, window: int = 8):
    """(leader index per slot, tokens shared with the leader per slot)"""
    n = len(prompts)
    arrs = [np.ascontiguousarray(p, dtype=np.int32) for p in prompts]
    ptrs = (_I32P * max(n, 1))(*[a.ctypes.data_as(_I32P) for a in arrs])
    lens = np.asarray([len(a) for a in arrs], dtype=np.int64)
    past = np.ascontiguousarray(n_past, dtype=np.int64)
    pid = np.ascontiguousarray(prefix_id, dtype=np.int32)
    leader = np.zeros(max(n, 1), dtype=np.int32)
    shared = np.zeros(max(n, 1), dtype=np.int64)
    _check(lib().dk_prefill_groups(n, ptrs, lens.ctypes.data_as(_I64P), past.ctypes.data_as(_I64P),
                                   pid.ctypes.data_as(_I32P), window, leader.ctypes.data_as(_I32P),
                                   shared.ctypes.data_as(_I64P)), "prefill_groups")
    return leader[:n].tolist(), shared[:n].tolist()


def seq_gather(pool, slot: int, k_out, v_out, stream=None) -> None:
    st = _stream(stream)
    _launch(lambda: lib().dk_seq_gather(pool, slot, _ptr(k_out), _ptr(v_out), st), "seq_gather", pool, stream)


def set_attend_variant(pool, variant: int) -> None:
    _check(lib().dk_set_attend_variant(pool, variant), "set_attend_variant")


def set_attend_timing(pool, n_calls: int) -> None:
    _check(lib().dk_set_attend_timing(pool, int(n_calls)), "set_attend_timing", pool)


def attend_times(pool, cap: int = 256) -> np.ndarray:
    out = np.zeros(cap, dtype=np.float32)
    n = C.c_int32()
    _check(lib().dk_attend_times(pool, out.ctypes.data_as(C.POINTER(C.c_float)), cap, C.byref(n)), "attend_times", pool)
    return out[: n.value].copy()


def last_attend_ms(pool) -> float:
    out = C.c_float()
    _check(lib().dk_last_attend_ms(pool, C.byref(out)), "last_attend_ms", pool)
    return out.value


HOST_PHASES = ("plan", "stage", "upload", "launch", "append_bookkeeping", "append_launch")


def host_times(pool, reset: bool = False):
    """({phase: microseconds}, (delta_attend calls, kv_append calls)) since the last reset"""
    us = (C.c_double * len(HOST_PHASES))()
    calls = (C.c_int64 * 2)()
    _check(lib().dk_host_times(pool, int(reset), us, calls), "host_times")
    return dict(zip(HOST_PHASES, list(us))), (calls[0], calls[1])


def strerror(status: int) -> str:
    return lib().dk_strerror(status).decode()
