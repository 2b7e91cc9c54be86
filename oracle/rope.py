"""fp64 CPU oracle of the producer step ahead of the decode attention: rotary
position embedding of the step's query and key, and the append of the step's
key/value to the response segment (arxiv 2401.05391, Section 3.1: RoPE follows
the QKV projection and is fused to a single kernel; the step's Key_t / Value_t
go into their row of the pre-allocated sequence-first buffers).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: imported only by tests.  numpy, float64.

The paper gives no formula for RoPE; the reading taken here is the published
one (RoFormer, as used by Llama2 and GPT-J, the paper's models):
  theta_i = base^(-2 i / R), i = 0 .. R/2 - 1, R = rotary dimension (<= D),
  a pair (a, b) of one head vector at position `pos` becomes
  (a cos(pos theta_i) - b sin(pos theta_i),  b cos(pos theta_i) + a sin(pos theta_i)),
  the pair being elements (i, i + R/2) ("half" convention, Llama2) or
  (2 i, 2 i + 1) ("interleaved" convention, GPT-J); elements >= R are kept.
The decode step t of a request with Lp prompt tokens sits at position Lp + t
(prompt token i at i), the same positions the ALiBi bias uses.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np


def pair_indices(rotary_dim: int, interleaved: bool) -> Tuple[np.ndarray, np.ndarray]:
    i = np.arange(rotary_dim // 2)
    if interleaved:
        return 2 * i, 2 * i + 1
    return i, i + rotary_dim // 2


def rotate(x: np.ndarray, pos: np.ndarray, base: float, rotary_dim: int,
           interleaved: bool) -> np.ndarray:
    """x [rows, H, D] (any float dtype) at integer positions pos [rows] -> float64."""
    x = np.asarray(x, dtype=np.float64)
    rows, _, D = x.shape
    assert rotary_dim % 2 == 0 and 0 <= rotary_dim <= D
    ia, ib = pair_indices(rotary_dim, interleaved)
    theta = np.power(float(base), -2.0 * np.arange(rotary_dim // 2) / rotary_dim)
    ang = np.asarray(pos, dtype=np.float64).reshape(rows, 1, 1) * theta.reshape(1, 1, -1)
    c, s = np.cos(ang), np.sin(ang)
    out = x.copy()
    a, b = x[..., ia], x[..., ib]
    out[..., ia] = a * c - b * s
    out[..., ib] = b * c + a * s
    return out


def rope_append(q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray, resp_k: np.ndarray,
                resp_v: np.ndarray, t: int, W: int, Lp: int, base: float, rotary_dim: int,
                interleaved: bool, positions: Optional[np.ndarray] = None) -> np.ndarray:
    """Returns the rotated query [B*W, Hq, D] in float64; writes row t of resp_k
    (rotated key rounded to fp16, round to nearest even) and of resp_v (copy).
    `positions` [B] overrides the per-request position Lp + t."""
    N = q.shape[0]
    B = N // W
    pos_b = np.full(B, Lp + t, dtype=np.int64) if positions is None else np.asarray(positions)
    pos = np.repeat(pos_b, W)
    q_rot = rotate(q, pos, base, rotary_dim, interleaved)
    k_rot = rotate(k_new, pos, base, rotary_dim, interleaved)
    resp_k[t] = k_rot.astype(np.float16)
    resp_v[t] = v_new
    return q_rot
