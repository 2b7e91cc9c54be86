"""Second, independent statement of the same result -- TEST INFRASTRUCTURE.

Replays the *standard* decoder graph that the paper's kernel replaces
(arxiv 2401.05391, Section 3.1, the flow before simplification): every beam
keeps its own contiguous K/V cache ``[B*W, length, Hkv, D]`` (Section 3.2, the
standard cache with the prompt duplicated W times); at every step the past
cache is re-ordered with ``index_select`` by that step's beam indices and the
step's own K/V are concatenated behind it; attention is then ordinary dense
softmax attention over that cache with KV heads repeated for grouped queries.

Nothing here resolves ancestors or touches the segment layout, which is what
makes it a pin for ``segkv_oracle.c``: the two only agree if the ancestor walk
has the right direction, base and offsets.  numpy only, small inputs only.
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def replay_standard_cache(prompt: np.ndarray, resp: np.ndarray, parent: np.ndarray,
                          W: int, T: int) -> np.ndarray:
    """Contiguous per-beam cache after T steps of reorder-then-append.

    prompt [B, Lp, Hkv, D]; resp [>=T, B*W, Hkv, D] where resp[s, n] is the row
    that beam slot n produced at step s; parent [T, B*W] request-local slots.
    Returns [B*W, Lp+T, Hkv, D] float64.
    """
    B = prompt.shape[0]
    N = B * W
    offs = (np.arange(N) // W) * W                      # first slot of each request
    cache = np.repeat(prompt.astype(np.float64), W, axis=0)   # prompt duplicated W times
    for s in range(T):
        src = offs + parent[s].astype(np.int64)         # global row each slot continues
        cache = cache[src]                              # index_select on the beam axis
        cache = np.concatenate([cache, resp[s].astype(np.float64)[:, None]], axis=1)  # cat
    return cache


def dense_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                    scale: float, slopes: Optional[np.ndarray] = None):
    """Plain softmax attention of one query per beam row over its own cache.

    q [N, Hq, D]; k_cache, v_cache [N, L, Hkv, D].  Returns (out [N,Hq,D],
    probs [N,Hq,L]) in float64.
    """
    N, Hq, D = q.shape
    Hkv = k_cache.shape[2]
    group = Hq // Hkv
    k = np.repeat(k_cache, group, axis=2)               # [N, L, Hq, D]
    v = np.repeat(v_cache, group, axis=2)
    qd = q.astype(np.float64)
    logits = scale * np.einsum("nhd,nlhd->nhl", qd, k)
    if slopes is not None:
        pos = np.arange(k.shape[1], dtype=np.float64)
        logits = logits + slopes.astype(np.float64)[None, :, None] * pos[None, None, :]
    logits = logits - logits.max(axis=-1, keepdims=True)
    w = np.exp(logits)
    w = w / w.sum(axis=-1, keepdims=True)
    out = np.einsum("nhl,nlhd->nhd", w, v)
    return out, w


def sdpa_decode_dense(q, prompt_k, prompt_v, resp_k, resp_v, parent, W, T, scale,
                      slopes=None):
    """The whole standard path: replay the caches, then dense attention."""
    kc = replay_standard_cache(prompt_k, resp_k, parent, W, T)
    vc = replay_standard_cache(prompt_v, resp_v, parent, W, T)
    return dense_attention(q, kc, vc, scale, slopes)
