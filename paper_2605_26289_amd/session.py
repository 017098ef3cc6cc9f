"""Device-memory plumbing around one pool: the arena, the metadata scratch and a growable workspace.

PyTorch is used for allocation and streams only.
"""
from __future__ import annotations

import contextlib
from typing import Iterator, Optional, Sequence

import torch

from . import binding as dk


class DevicePool:
    """Owns the device buffers of one pool and forwards to the C ABI."""

    def __init__(self, n_slots: int, arena_cells: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                 dtype: str = "bf16", n_session_slots: int = 0, granule_cells: int = 0, device: str = "cuda:0",
                 staging_depth: int = 0):
        if not torch.cuda.is_available():
            raise RuntimeError("deltakv needs a GPU: no CPU fallback exists")
        self.device = torch.device(device)
        self.torch_dtype = {"bf16": torch.bfloat16, "f32": torch.float32}[dtype]
        self.n_q_heads, self.n_kv_heads, self.head_dim = n_q_heads, n_kv_heads, head_dim
        gran = granule_cells or 256
        arena_cells = (arena_cells + gran - 1) // gran * gran
        self.arena_cells = arena_cells
        self.k_arena = torch.empty((n_kv_heads, arena_cells, head_dim), dtype=self.torch_dtype, device=self.device)
        self.v_arena = torch.empty_like(self.k_arena)
        desc = dk.PoolDesc(n_slots, n_session_slots, arena_cells, granule_cells, n_q_heads, n_kv_heads, head_dim,
                           dk.BF16 if dtype == "bf16" else dk.F32, self.k_arena.data_ptr(), self.v_arena.data_ptr(),
                           None, 0, None, 0, staging_depth)
        nbytes = dk.meta_bytes(desc)
        self.dev_meta = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        desc.dev_meta = self.dev_meta.data_ptr()
        desc.dev_meta_bytes = nbytes
        # pinned staging memory for descriptor uploads: allocated here, once, never by a launching call
        self.host_staging = torch.empty(dk.staging_bytes(desc) + 256, dtype=torch.uint8, pin_memory=True)
        base = self.host_staging.data_ptr()
        desc.host_staging = (base + 255) // 256 * 256
        desc.host_staging_bytes = dk.staging_bytes(desc)
        self.handle = dk.pool_create(desc)
        self.workspace: Optional[torch.Tensor] = None

    def close(self) -> None:
        if self.handle is not None:
            torch.cuda.synchronize(self.device)
            dk.pool_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- host-only -------------------------------------------------------
    def acquire(self, region: int = 0, timeout_ms: int = 0) -> int:
        return dk.seq_acquire(self.handle, region, timeout_ms)

    def release(self, slot: int) -> None:
        dk.seq_release(self.handle, slot)

    @contextlib.contextmanager
    def sequence(self, region: int = 0, timeout_ms: int = 0) -> Iterator[int]:
        """Scope guard around acquire / release: the sequence goes back to the pool on every exit path."""
        slot = self.acquire(region, timeout_ms)
        try:
            yield slot
        finally:
            self.release(slot)

    def length(self, slot: int) -> int:
        return dk.seq_len(self.handle, slot)

    def alias(self, donor: int, dst: int, m: int) -> None:
        dk.seq_alias(self.handle, donor, dst, 0, m)

    def trim(self, slot: int, new_len: int) -> None:
        dk.seq_trim(self.handle, slot, new_len)

    def trim_batch(self, slots: Sequence[int], new_len: Sequence[int]) -> None:
        dk.seq_trim_batch(self.handle, slots, new_len)

    def cells(self, slot: int):
        return dk.seq_cells(self.handle, slot)

    # -- GPU ---------------------------------------------------------------
    def append(self, slots: Sequence[int], cu_delta: Sequence[int], k_new, v_new, n_accept=None) -> None:
        dk.kv_append(self.handle, slots, cu_delta, k_new, v_new, n_accept)

    def ensure_workspace(self, slots, cu_delta, staged) -> torch.Tensor:
        need = dk.attend_workspace_bytes(self.handle, slots, cu_delta, staged)
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = torch.empty(int(need * 1.25) + 4096, dtype=torch.uint8, device=self.device)
        return self.workspace

    def attend(self, slots, cu_delta, q, scale: float, k_new=None, v_new=None, out=None, lse=None):
        if out is None:
            out = torch.empty_like(q)
        if self.workspace is None:
            self.ensure_workspace(slots, cu_delta, k_new is not None)
        try:  # the library checks the size itself: only a call that outgrows the buffer pays for a size query
            dk.delta_attend(self.handle, slots, cu_delta, q, out, scale, k_new, v_new, lse, self.workspace)
        except dk.DeltaKVError as e:
            if e.name != "WORKSPACE":
                raise
            ws = self.ensure_workspace(slots, cu_delta, k_new is not None)
            dk.delta_attend(self.handle, slots, cu_delta, q, out, scale, k_new, v_new, lse, ws)
        return out

    def append_attend(self, slots, cu_delta, q, k_new, v_new, scale: float, out=None, lse=None):
        """Appends every entry's new tokens and attends them, in one call (no separate copy kernel)."""
        if out is None:
            out = torch.empty_like(q)
        if self.workspace is None:
            self.ensure_workspace(slots, cu_delta, 2)
        try:
            dk.append_attend(self.handle, slots, cu_delta, q, k_new, v_new, out, scale, lse, self.workspace)
        except dk.DeltaKVError as e:
            if e.name != "WORKSPACE":
                raise
            ws = self.ensure_workspace(slots, cu_delta, 2)
            dk.append_attend(self.handle, slots, cu_delta, q, k_new, v_new, out, scale, lse, ws)
        return out

    def gather(self, slot: int):
        n = self.length(slot)
        k = torch.empty((n, self.n_kv_heads, self.head_dim), dtype=self.torch_dtype, device=self.device)
        v = torch.empty_like(k)
        dk.seq_gather(self.handle, slot, k, v)
        return k, v
