"""KV-cache memory model of arxiv 2401.05391, Section 3.2 -- TEST INFRASTRUCTURE.

The three closed forms exactly as the paper states them (Eq. 1-3), in plain
Python integers, and the growth rule of the response buffer (capacity rises in
steps of 16 rows).  Pinned by the numbers the paper prints for its GPT-J-6B
example (tests/golden/kv_cache_memory_worked_example.txt).
"""
from __future__ import annotations

import numpy as np

STEP = 16  # Section 3.2: N_step grows with step = 16


def cache_token(L: int, H: int, D: int, sizeof_datatype: int) -> int:
    """Eq. (1): the 2 is key and value."""
    return 2 * L * H * D * sizeof_datatype


def cache_standard(BS: int, BW: int, n_prompt: int, n_response: int, token: int) -> int:
    """Eq. (2): prompt and response concatenated per beam."""
    return BS * BW * (n_prompt + n_response) * token


def capacity(n_response: int, step: int = STEP) -> int:
    """Ceil(N_response / step) * step."""
    return -(-n_response // step) * step if n_response > 0 else 0


def cache_segment(BS: int, BW: int, n_prompt: int, n_response: int, token: int,
                  step: int = STEP) -> int:
    """Eq. (3): prompt once per request, response at its grown capacity."""
    return BS * (n_prompt + BW * capacity(n_response, step)) * token


def grow(old: np.ndarray, T: int, tcap_new: int, fill) -> np.ndarray:
    """New buffer of tcap_new rows: the first T rows are the old ones, the rest `fill`."""
    new = np.full((tcap_new,) + old.shape[1:], fill, dtype=old.dtype)
    new[:T] = old[:T]
    return new
