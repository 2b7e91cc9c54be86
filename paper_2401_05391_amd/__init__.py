"""Fused decode-step attention over a segment KV cache for MI355X (gfx950).

`binding` marshals torch device tensors into the C-ABI library `libsegkv.so`
(HIP kernels under `csrc/`); `workloads` draws the seeded synthetic inputs.
The library is loaded on first use of an entry point, not at import.
"""
from . import binding, build, workloads  # noqa: F401
from .binding import (SegkvDims, SegkvError, append_kv, cache_segment_bytes,  # noqa: F401
                      cache_standard_bytes, cache_token_bytes, grow_response, lineage_bytes,
                      lineage_update, load_library, sdpa_decode_lineage,
                      make_dims, prepare_sdpa_decode, response_capacity, rope_append, sdpa_decode, sdpa_decode_ragged,
                      sdpa_decode_seq_first_prompt, sdpa_decode_static_scratch, sdpa_prefill, probe_mfma_rate,
                      status_string, stream_read_probe, value_stagger_bytes, workspace_bytes)
