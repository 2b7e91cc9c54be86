"""Fused decode-step attention over a segment KV cache for MI355X (gfx950).

`binding` marshals torch device tensors into the C-ABI library `libsegkv.so`
(HIP kernels under `csrc/`); `workloads` draws the seeded synthetic inputs.
The library is loaded on first use of an entry point, not at import.
"""
from . import binding, build, workloads  # noqa: F401
from .binding import (SegkvDims, SegkvError, append_kv, load_library, make_dims,  # noqa: F401
                      prepare_sdpa_decode, sdpa_decode, status_string, stream_read_probe, workspace_bytes)
