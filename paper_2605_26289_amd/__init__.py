"""deltakv: delta-prefill attention over a pooled, prefix-aliased KV cache for MI355X (gfx950).

The work is done by libdeltakv.so (HIP kernels behind a C ABI, see include/deltakv.h); `binding`
marshals arguments, `session.DevicePool` owns the device buffers a pool needs.
"""
from . import binding  # noqa: F401
from .session import DevicePool  # noqa: F401
