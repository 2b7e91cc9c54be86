"""Thin ctypes binding of libsegkv.so -- argument marshalling only.

Every step of the decode attention runs inside the library's HIP kernels; this
module just turns torch tensors into device pointers and sizes.  PyTorch is
used for device memory and streams, nothing else.  There is no CPU fallback:
if the library cannot be loaded the import of the entry points raises.

Names and arguments mirror include/segkv.h.
"""
from __future__ import annotations

import ctypes
from typing import Optional

from . import build as _build

SEGKV_OK = 0
SEGKV_INVALID_ARG = -1
SEGKV_UNSUPPORTED = -2
SEGKV_MISALIGNED = -3
SEGKV_WORKSPACE_TOO_SMALL = -4
SEGKV_HIP_ERROR = -5
SEGKV_STATIC_SCRATCH_EXCEEDED = -6
STATIC_SCRATCH_BYTES = 16 << 20

EXPORTS = ("segkv_append_kv", "segkv_sdpa_decode", "segkv_workspace_bytes",
           "segkv_status_string", "segkv_stream_read_probe", "segkv_cache_token_bytes",
           "segkv_cache_standard_bytes", "segkv_cache_segment_bytes", "segkv_response_capacity",
           "segkv_grow_response", "segkv_sdpa_prefill", "segkv_value_stagger_bytes",
           "segkv_rope_append", "segkv_sdpa_decode_ragged", "segkv_sdpa_decode_seq_first_prompt",
           "segkv_lineage_bytes", "segkv_lineage_update", "segkv_sdpa_decode_lineage",
           "segkv_sdpa_decode_static_scratch", "segkv_reload_tuning", "segkv_probe_mfma_rate")


class SegkvDims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "beam", "Hq", "Hkv", "D", "Lp", "T", "Tcap")]


class SegkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def load_library():
    """Load libsegkv.so, building it first only if no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not _build.is_built():
        _build.build_library()
    # PyTorch owns the device memory and streams that are handed to the library,
    # so both must talk to the same HIP runtime: import torch first, so that the
    # runtime it ships is the one libsegkv.so resolves its HIP symbols against.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_build.LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(SegkvDims)
    lib.segkv_append_kv.restype = ctypes.c_int
    lib.segkv_append_kv.argtypes = [vp, vp, vp, vp, i32, dp, vp]
    lib.segkv_sdpa_decode.restype = ctypes.c_int
    lib.segkv_sdpa_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz,
                                      ctypes.c_float, dp, vp]
    lib.segkv_sdpa_decode_static_scratch.restype = ctypes.c_int
    lib.segkv_sdpa_decode_static_scratch.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                                     ctypes.c_float, dp, vp]
    lib.segkv_reload_tuning.restype = None
    lib.segkv_reload_tuning.argtypes = []
    lib.segkv_probe_mfma_rate.restype = ctypes.c_int
    lib.segkv_probe_mfma_rate.argtypes = [vp, vp, vp, i32, i32, vp]
    lib.segkv_sdpa_decode_ragged.restype = ctypes.c_int
    lib.segkv_sdpa_decode_ragged.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz,
                                             ctypes.c_float, dp, vp]
    lib.segkv_sdpa_decode_seq_first_prompt.restype = ctypes.c_int
    lib.segkv_sdpa_decode_seq_first_prompt.argtypes = lib.segkv_sdpa_decode_ragged.argtypes
    lib.segkv_lineage_bytes.restype = sz
    lib.segkv_lineage_bytes.argtypes = [dp, i32]
    lib.segkv_lineage_update.restype = ctypes.c_int
    lib.segkv_lineage_update.argtypes = [vp, i32, vp, i32, dp, vp]
    lib.segkv_sdpa_decode_lineage.restype = ctypes.c_int
    lib.segkv_sdpa_decode_lineage.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, sz,
                                              ctypes.c_float, dp, vp]
    lib.segkv_workspace_bytes.restype = sz
    lib.segkv_workspace_bytes.argtypes = [dp]
    lib.segkv_value_stagger_bytes.restype = sz
    lib.segkv_value_stagger_bytes.argtypes = [dp]
    lib.segkv_status_string.restype = ctypes.c_char_p
    lib.segkv_status_string.argtypes = [ctypes.c_int]
    lib.segkv_stream_read_probe.restype = ctypes.c_int
    lib.segkv_stream_read_probe.argtypes = [vp, sz, vp, vp]
    u64 = ctypes.c_uint64
    lib.segkv_cache_token_bytes.restype = u64
    lib.segkv_cache_token_bytes.argtypes = [i32, i32, i32, i32]
    lib.segkv_cache_standard_bytes.restype = u64
    lib.segkv_cache_standard_bytes.argtypes = [i32, i32, i32, i32, u64]
    lib.segkv_cache_segment_bytes.restype = u64
    lib.segkv_cache_segment_bytes.argtypes = [i32, i32, i32, i32, u64]
    lib.segkv_response_capacity.restype = i32
    lib.segkv_response_capacity.argtypes = [i32]
    lib.segkv_sdpa_prefill.restype = ctypes.c_int
    lib.segkv_sdpa_prefill.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, dp, vp]
    lib.segkv_rope_append.restype = ctypes.c_int
    lib.segkv_rope_append.argtypes = [vp, vp, vp, vp, vp, vp, i32, ctypes.c_float, i32, i32, dp, vp]
    lib.segkv_grow_response.restype = ctypes.c_int
    lib.segkv_grow_response.argtypes = [vp, vp, vp, vp, i32, dp, vp]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().segkv_status_string(int(status)).decode()


def make_dims(B, beam, Hq, Hkv, D, Lp, T, Tcap) -> SegkvDims:
    return SegkvDims(B, beam, Hq, Hkv, D, Lp, T, Tcap)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("libsegkv takes contiguous device tensors")
    return t.data_ptr()


def _stream_handle(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def workspace_bytes(dims: SegkvDims) -> int:
    return int(load_library().segkv_workspace_bytes(ctypes.byref(dims)))


def value_stagger_bytes(dims: SegkvDims) -> int:
    return int(load_library().segkv_value_stagger_bytes(ctypes.byref(dims)))


def append_kv(resp_k, resp_v, k_new, v_new, t: int, dims: SegkvDims, stream=None) -> None:
    rc = load_library().segkv_append_kv(_ptr(resp_k), _ptr(resp_v), _ptr(k_new), _ptr(v_new),
                                        int(t), ctypes.byref(dims), _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_append_kv")


def rope_append(q, k_new, v_new, resp_k, resp_v, t: int, dims: SegkvDims, rope_base: float,
                rotary_dim: int, interleaved: bool = False, positions=None, stream=None) -> None:
    rc = load_library().segkv_rope_append(_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(resp_k),
                                          _ptr(resp_v), _ptr(positions), int(t), float(rope_base),
                                          int(rotary_dim), int(bool(interleaved)),
                                          ctypes.byref(dims), _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_rope_append")


def sdpa_decode(out, q, prompt_k, prompt_v, resp_k, resp_v, parent, dims: SegkvDims, scale: float,
                k_new=None, v_new=None, alibi_slopes=None, anc_out=None, workspace=None,
                stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load_library().segkv_sdpa_decode(
        _ptr(out), _ptr(q), _ptr(prompt_k), _ptr(prompt_v), _ptr(resp_k), _ptr(resp_v),
        _ptr(parent), _ptr(k_new), _ptr(v_new), _ptr(alibi_slopes), _ptr(anc_out),
        _ptr(workspace), ws_bytes, float(scale), ctypes.byref(dims), _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_sdpa_decode")


def sdpa_decode_static_scratch(out, q, prompt_k, prompt_v, resp_k, resp_v, parent, dims: SegkvDims,
                               scale: float, k_new=None, v_new=None, alibi_slopes=None,
                               anc_out=None, stream=None) -> None:
    """sdpa_decode without a workspace argument: partials go to the library's static buffer."""
    rc = load_library().segkv_sdpa_decode_static_scratch(
        _ptr(out), _ptr(q), _ptr(prompt_k), _ptr(prompt_v), _ptr(resp_k), _ptr(resp_v),
        _ptr(parent), _ptr(k_new), _ptr(v_new), _ptr(alibi_slopes), _ptr(anc_out),
        float(scale), ctypes.byref(dims), _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_sdpa_decode_static_scratch")


def sdpa_decode_ragged(out, q, prompt_k, prompt_v, resp_k, resp_v, parent, prompt_lens,
                       dims: SegkvDims, scale: float, k_new=None, v_new=None, alibi_slopes=None,
                       anc_out=None, workspace=None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load_library().segkv_sdpa_decode_ragged(
        _ptr(out), _ptr(q), _ptr(prompt_k), _ptr(prompt_v), _ptr(resp_k), _ptr(resp_v),
        _ptr(parent), _ptr(k_new), _ptr(v_new), _ptr(alibi_slopes), _ptr(prompt_lens),
        _ptr(anc_out), _ptr(workspace), ws_bytes, float(scale), ctypes.byref(dims),
        _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_sdpa_decode_ragged")


def sdpa_decode_seq_first_prompt(out, q, prompt_k, prompt_v, resp_k, resp_v, parent,
                                 dims: SegkvDims, scale: float, k_new=None, v_new=None,
                                 alibi_slopes=None, prompt_lens=None, anc_out=None, workspace=None,
                                 stream=None) -> None:
    """prompt_k / prompt_v are [Lp, B, Hkv, D]; otherwise sdpa_decode_ragged."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load_library().segkv_sdpa_decode_seq_first_prompt(
        _ptr(out), _ptr(q), _ptr(prompt_k), _ptr(prompt_v), _ptr(resp_k), _ptr(resp_v),
        _ptr(parent), _ptr(k_new), _ptr(v_new), _ptr(alibi_slopes), _ptr(prompt_lens),
        _ptr(anc_out), _ptr(workspace), ws_bytes, float(scale), ctypes.byref(dims),
        _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_sdpa_decode_seq_first_prompt")


def lineage_bytes(dims: SegkvDims, capacity: int) -> int:
    return int(load_library().segkv_lineage_bytes(ctypes.byref(dims), int(capacity)))


def lineage_update(lineage, capacity: int, parent_row, t: int, dims: SegkvDims, stream=None) -> None:
    """One generated token: parent_row is row t of the parent table (None for t == 0)."""
    rc = load_library().segkv_lineage_update(_ptr(lineage), int(capacity), _ptr(parent_row), int(t),
                                             ctypes.byref(dims), _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_lineage_update")


def sdpa_decode_lineage(out, q, prompt_k, prompt_v, resp_k, resp_v, lineage, capacity: int,
                        dims: SegkvDims, scale: float, k_new=None, v_new=None, alibi_slopes=None,
                        prompt_lens=None, workspace=None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load_library().segkv_sdpa_decode_lineage(
        _ptr(out), _ptr(q), _ptr(prompt_k), _ptr(prompt_v), _ptr(resp_k), _ptr(resp_v),
        _ptr(lineage), int(capacity), _ptr(k_new), _ptr(v_new), _ptr(alibi_slopes),
        _ptr(prompt_lens), _ptr(workspace), ws_bytes, float(scale), ctypes.byref(dims),
        _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_sdpa_decode_lineage")


def prepare_sdpa_decode(out, q, prompt_k, prompt_v, resp_k, resp_v, parent, dims: SegkvDims,
                        scale: float, k_new=None, v_new=None, alibi_slopes=None, anc_out=None,
                        workspace=None, stream=None, prompt_seq_first: bool = False,
                        lineage=None, lineage_capacity: int = 0):
    """Marshal the arguments once; returns a zero-argument callable that enqueues
    the same segkv_sdpa_decode call each time (for launch loops where per-call
    Python marshalling would rival the kernel time).  The tensors must stay alive.
    prompt_seq_first: the prompt tensors are [Lp, B, Hkv, D] and the call is
    segkv_sdpa_decode_seq_first_prompt.  lineage: the call is
    segkv_sdpa_decode_lineage with this list (`parent` is not used)."""
    lib = load_library()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    vp = ctypes.c_void_p
    head = [vp(_ptr(t)) for t in (out, q, prompt_k, prompt_v, resp_k, resp_v, parent, k_new,
                                  v_new, alibi_slopes)]
    tail = ([vp(_ptr(anc_out)), vp(_ptr(workspace)), ctypes.c_size_t(ws_bytes),
             ctypes.c_float(scale), ctypes.byref(dims), vp(_stream_handle(stream))])
    if lineage is not None:
        fn, name = lib.segkv_sdpa_decode_lineage, "segkv_sdpa_decode_lineage"
        args = (head[:6] + [vp(_ptr(lineage)), ctypes.c_int32(lineage_capacity)] + head[7:]
                + [vp(None)] + tail[1:])
    elif prompt_seq_first:
        fn, name, args = (lib.segkv_sdpa_decode_seq_first_prompt,
                          "segkv_sdpa_decode_seq_first_prompt", head + [vp(None)] + tail)
    else:
        fn, name, args = lib.segkv_sdpa_decode, "segkv_sdpa_decode", head + tail

    def call() -> None:
        rc = fn(*args)
        if rc != SEGKV_OK:
            raise SegkvError(rc, name)
    return call


def sdpa_prefill(out, q, k, v, dims: SegkvDims, scale: float, alibi_slopes=None, stream=None) -> None:
    rc = load_library().segkv_sdpa_prefill(_ptr(out), _ptr(q), _ptr(k), _ptr(v), _ptr(alibi_slopes),
                                           float(scale), ctypes.byref(dims), _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_sdpa_prefill")


def probe_mfma_rate(operands, out, clocks, n_groups: int, iters: int, stream=None) -> None:
    """Measurement only: a register-resident chain of the fp16 matrix instruction (see segkv.h)."""
    rc = load_library().segkv_probe_mfma_rate(_ptr(operands), _ptr(out), _ptr(clocks), int(n_groups),
                                              int(iters), _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_probe_mfma_rate")


def cache_token_bytes(L: int, H: int, D: int, elem_bytes: int = 2) -> int:
    return int(load_library().segkv_cache_token_bytes(L, H, D, elem_bytes))


def cache_standard_bytes(BS: int, BW: int, n_prompt: int, n_response: int, token_bytes: int) -> int:
    return int(load_library().segkv_cache_standard_bytes(BS, BW, n_prompt, n_response, token_bytes))


def cache_segment_bytes(BS: int, BW: int, n_prompt: int, n_response: int, token_bytes: int) -> int:
    return int(load_library().segkv_cache_segment_bytes(BS, BW, n_prompt, n_response, token_bytes))


def response_capacity(n_response: int) -> int:
    return int(load_library().segkv_response_capacity(n_response))


def grow_response(new_k, new_v, old_k, old_v, dims: SegkvDims, stream=None) -> None:
    """Copy the valid rows of the old response buffers into larger new ones."""
    rc = load_library().segkv_grow_response(_ptr(new_k), _ptr(new_v), _ptr(old_k), _ptr(old_v),
                                            int(new_k.shape[0]), ctypes.byref(dims),
                                            _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_grow_response")


def stream_read_probe(src, sink, stream=None) -> None:
    nbytes = (src.numel() * src.element_size()) // 16 * 16
    rc = load_library().segkv_stream_read_probe(_ptr(src), nbytes, _ptr(sink),
                                                _stream_handle(stream))
    if rc != SEGKV_OK:
        raise SegkvError(rc, "segkv_stream_read_probe")
