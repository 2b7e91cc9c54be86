"""ctypes front end of the fp64 CPU oracle (``segkv_oracle.c``).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only the tests, the smoke check and the
benchmark's cpu_baseline leg import this.  It never imports the GPU package.
Arguments are numpy arrays; fp16 tensors are handed to C as their raw 16-bit
patterns and decoded there exactly.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "segkv_oracle.c")
_LIB = os.path.join(_HERE, "libsegkv_oracle.so")


class _Dims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "beam", "Hq", "Hkv", "D", "Lp", "T", "Tcap")]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP, no vector intrinsics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.segkv_oracle_num_threads.restype = ctypes.c_int
        lib.segkv_oracle_append_kv.restype = ctypes.c_int
        lib.segkv_oracle_sdpa_decode.restype = ctypes.c_int
        lib.segkv_oracle_ancestors.restype = None
        lib.segkv_oracle_sdpa_prefill.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().segkv_oracle_num_threads())


def _u16(a: np.ndarray) -> np.ndarray:
    assert a.dtype == np.float16 and a.flags.c_contiguous, "need contiguous fp16"
    return a.view(np.uint16)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def ancestors(parent: np.ndarray, B: int, W: int) -> np.ndarray:
    """Resolved ancestor slots anc[T, B*W] from the raw parent table."""
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    T = parent.shape[0]
    assert parent.shape == (T, B * W)
    anc = np.empty((T, B * W), dtype=np.int32)
    _load().segkv_oracle_ancestors(_p(parent), ctypes.c_int32(B), ctypes.c_int32(W),
                                   ctypes.c_int32(T), _p(anc))
    return anc


def append_kv(resp_k: np.ndarray, resp_v: np.ndarray, k_new: np.ndarray,
              v_new: np.ndarray, t: int) -> None:
    """In place: row ``t`` of the response buffers := the step's K/V."""
    Tcap, N, Hkv, D = resp_k.shape
    d = _Dims(1, N, Hkv, Hkv, D, 0, 1, Tcap)  # only the row size and Tcap matter
    rc = _load().segkv_oracle_append_kv(_p(_u16(resp_k)), _p(_u16(resp_v)),
                                        _p(_u16(k_new)), _p(_u16(v_new)),
                                        ctypes.c_int32(t), ctypes.byref(d))
    if rc != 0:
        raise ValueError("append_kv: row out of range")


def sdpa_decode(q: np.ndarray, prompt_k: np.ndarray, prompt_v: np.ndarray,
                resp_k: np.ndarray, resp_v: np.ndarray, parent: np.ndarray,
                W: int, T: int, scale: float, slopes: Optional[np.ndarray] = None,
                pairs: Optional[np.ndarray] = None, want_probs: bool = False
                ) -> Tuple[np.ndarray, np.ndarray, Optional[np.ndarray]]:
    """fp64 attention context for every (beam row, query head), or for the rows
    listed in ``pairs`` [[n, hq], ...].

    ``resp_k/resp_v`` must already contain the current step's K/V in row T-1.
    Returns (out, anc, probs): out is [B*W, Hq, D] (or [len(pairs), D]) float64,
    anc is [T, B*W] int32, probs is [rows, Lp+T] float64 or None.
    """
    N, Hq, D = q.shape
    B, Lp, Hkv, D2 = prompt_k.shape
    Tcap = resp_k.shape[0]
    assert D2 == D and N == B * W and prompt_v.shape == prompt_k.shape
    assert resp_k.shape == (Tcap, N, Hkv, D) and resp_v.shape == resp_k.shape
    parent = np.ascontiguousarray(parent[:T], dtype=np.int32)
    assert parent.shape == (T, N)
    d = _Dims(B, W, Hq, Hkv, D, Lp, T, Tcap)
    if pairs is not None:
        pairs = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
        rows = pairs.shape[0]
        out = np.empty((rows, D), dtype=np.float64)
    else:
        rows = N * Hq
        out = np.empty((N, Hq, D), dtype=np.float64)
    probs = np.empty((rows, Lp + T), dtype=np.float64) if want_probs else None
    anc = np.empty((T, N), dtype=np.int32)
    sl = None if slopes is None else np.ascontiguousarray(slopes, dtype=np.float64)
    rc = _load().segkv_oracle_sdpa_decode(
        _p(out), _p(probs), _p(anc), _p(_u16(q)), _p(_u16(prompt_k)), _p(_u16(prompt_v)),
        _p(_u16(resp_k)), _p(_u16(resp_v)), _p(parent), _p(sl), ctypes.c_double(scale),
        ctypes.byref(d), _p(pairs), ctypes.c_int64(rows))
    if rc != 0:
        raise ValueError("sdpa_decode: invalid dimensions")
    return out, anc, probs


def sdpa_decode_ragged(q: np.ndarray, prompt_k: np.ndarray, prompt_v: np.ndarray,
                       resp_k: np.ndarray, resp_v: np.ndarray, parent: np.ndarray,
                       W: int, T: int, scale: float, prompt_lens: np.ndarray,
                       slopes: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Per-request prompt lengths (a padded static batch): request b owns prompt rows
    0..prompt_lens[b]-1 of prompt_k[b] / prompt_v[b]; the rows behind them are padding
    and take no part.  By definition this is the attention of each request taken on
    its own with Lp = prompt_lens[b] -- which is how it is computed here: one call
    of sdpa_decode per request on the sliced tensors (positions then follow from the
    request's own length: response step s sits at prompt_lens[b] + s).
    Returns (out [B*W, Hq, D] float64, anc [T, B*W] int32)."""
    N, Hq, D = q.shape
    B = N // W
    out = np.empty((N, Hq, D), dtype=np.float64)
    anc = np.empty((T, N), dtype=np.int32)
    for b in range(B):
        rows = slice(b * W, (b + 1) * W)
        lb = int(prompt_lens[b])
        o, a, _ = sdpa_decode(np.ascontiguousarray(q[rows]),
                              np.ascontiguousarray(prompt_k[b:b + 1, :lb]),
                              np.ascontiguousarray(prompt_v[b:b + 1, :lb]),
                              np.ascontiguousarray(resp_k[:, rows]),
                              np.ascontiguousarray(resp_v[:, rows]),
                              np.ascontiguousarray(parent[:T, rows]), W, T, scale, slopes=slopes)
        out[rows] = o
        anc[:, rows] = a
    return out, anc


def sdpa_prefill(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float,
                 slopes: Optional[np.ndarray] = None, rows: Optional[np.ndarray] = None) -> np.ndarray:
    """fp64 causal prefill attention.  q [B,N0,Hq,D], k/v [B,N0,Hkv,D] fp16.
    Returns [B,N0,Hq,D] float64, or [len(rows), D] for rows = [[b, i, hq], ...]."""
    B, N0, Hq, D = q.shape
    Hkv = k.shape[2]
    assert k.shape == (B, N0, Hkv, D) and v.shape == k.shape
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
        n = rows.shape[0]
        out = np.empty((n, D), dtype=np.float64)
    else:
        n = B * N0 * Hq
        out = np.empty((B, N0, Hq, D), dtype=np.float64)
    sl = None if slopes is None else np.ascontiguousarray(slopes, dtype=np.float64)
    rc = _load().segkv_oracle_sdpa_prefill(
        _p(out), _p(_u16(q)), _p(_u16(k)), _p(_u16(v)), _p(sl), ctypes.c_double(scale),
        ctypes.c_int32(B), ctypes.c_int32(N0), ctypes.c_int32(Hq), ctypes.c_int32(Hkv),
        ctypes.c_int32(D), _p(rows), ctypes.c_int64(n))
    if rc != 0:
        raise ValueError("sdpa_prefill: invalid dimensions")
    return out
