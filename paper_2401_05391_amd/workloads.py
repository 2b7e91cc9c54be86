"""Seeded synthetic workloads for the fused segment-KV decode attention.

This module only *draws inputs*: shapes, seeded random tensors, parent tables
and NaN poison.  It contains none of the method's arithmetic (no ancestor
resolution, no attention) so that the CPU oracle and the GPU library, which
must stay independent, can both be fed the same bytes from here.  numpy only.

Shapes follow the paper's problem statement for the decode-phase attention
kernel (arxiv 2401.05391, Section 3.3): query ``[B*W, Hq, D]``, prompt K/V
``[B, Lp, Hkv, D]`` (batch first, stored once per request, Section 3.2),
response K/V ``[Tcap, B*W, Hkv, D]`` (sequence first, pre-allocated and grown in
units of 16 rows, Section 3.2).  The paper's own kernel experiment (Section 4.1)
runs on synthetic tensors of model shapes; the recipes below do the same.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import numpy as np

RESPONSE_GROWTH_STEP = 16  # Section 3.2: response capacity grows in steps of 16 rows


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    B: int          # requests in the batch
    W: int          # beam width
    Hq: int         # query heads
    Hkv: int        # key/value heads (Hq % Hkv == 0)
    D: int          # head dimension
    Lp: int         # prompt length
    T: int          # valid response rows, including the current step's row
    alibi: bool = False
    parents: str = "uniform"   # "uniform" | "identity" | "zeros"
    seed: int = 0

    @property
    def Tcap(self) -> int:
        return max(1, math.ceil(self.T / RESPONSE_GROWTH_STEP)) * RESPONSE_GROWTH_STEP

    @property
    def N(self) -> int:
        return self.B * self.W

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


# The five benchmark configurations (index = position in the baseline list).
CONFIGS: Dict[str, Workload] = {
    "tiny": Workload("tiny", B=1, W=4, Hq=4, Hkv=4, D=64, Lp=32, T=8, seed=0),
    "gptj6b": Workload("gptj6b", B=16, W=4, Hq=16, Hkv=16, D=256, Lp=1024, T=128, seed=1),
    "llama2_7b_greedy": Workload("llama2_7b_greedy", B=128, W=1, Hq=32, Hkv=32, D=128,
                                 Lp=1024, T=128, parents="identity", seed=2),
    "llama2_70b_gqa": Workload("llama2_70b_gqa", B=32, W=4, Hq=64, Hkv=8, D=128,
                               Lp=2048, T=256, seed=3),
    "bloom176b_alibi": Workload("bloom176b_alibi", B=8, W=4, Hq=112, Hkv=112, D=128,
                                Lp=1024, T=128, alibi=True, seed=4),
}


# The paper's own kernel experiment (Section 4.1, Figure 6): the attention
# shape of Llama2-13B (40 heads of 128), beam width 4, 1024 prompt tokens, 128
# response steps, batch size swept from 1 to 64.
FIG6_BATCH_SIZES = (1, 2, 4, 8, 16, 32, 64)


def fig6_workload(batch_size: int) -> Workload:
    return Workload(f"llama2_13b_bs{batch_size}", B=batch_size, W=4, Hq=40, Hkv=40, D=128,
                    Lp=1024, T=128, seed=13)


# Section 3.2 sizes its memory example at N_prompt = N_response = 1024, beam
# width 4, batch 32: the point where the response segment is as long as the
# prompt.  Same two model shapes as Section 4's single-tile models.
RESPONSE_HEAVY: Dict[str, Workload] = {
    "gptj6b_1024_1024": Workload("gptj6b_1024_1024", B=32, W=4, Hq=16, Hkv=16, D=256,
                                 Lp=1024, T=1024, seed=21),
    "llama2_13b_1024_1024": Workload("llama2_13b_1024_1024", B=32, W=4, Hq=40, Hkv=40, D=128,
                                     Lp=1024, T=1024, seed=22),
}


def find_workload(name: str) -> Workload:
    """A workload by name: the benchmark configurations, the response-heavy
    points, or llama2_13b_bs<N> of the Figure 6 sweep."""
    if name in CONFIGS:
        return CONFIGS[name]
    if name in RESPONSE_HEAVY:
        return RESPONSE_HEAVY[name]
    if name.startswith("llama2_13b_bs"):
        return fig6_workload(int(name[len("llama2_13b_bs"):]))
    raise KeyError(name)


def alibi_slopes(Hq: int) -> np.ndarray:
    """Per-head slopes 2^(-8 h / Hq), h = 1..Hq (fp32).  The formula lives only
    here; both the oracle and the GPU library take the array as an input."""
    h = np.arange(1, Hq + 1, dtype=np.float64)
    return np.exp2(-8.0 * h / Hq).astype(np.float32)


def _normal_f16(rng: np.random.Generator, shape) -> np.ndarray:
    """fp16 rounding of N(0,1) draws, generated in slabs to bound peak memory."""
    out = np.empty(shape, dtype=np.float16)
    flat = out.reshape(-1)
    slab = 1 << 24
    for lo in range(0, flat.size, slab):
        hi = min(flat.size, lo + slab)
        flat[lo:hi] = rng.standard_normal(hi - lo, dtype=np.float32)
    return out


def make_parent(wl: Workload, rng: np.random.Generator) -> np.ndarray:
    """Parent table [T, B*W] int32 with request-local slots in [0, W)."""
    if wl.parents == "identity":
        return np.tile(np.arange(wl.W, dtype=np.int32), (wl.T, wl.B))
    if wl.parents == "zeros":
        return np.zeros((wl.T, wl.N), dtype=np.int32)
    if wl.parents == "uniform":
        return rng.integers(0, wl.W, size=(wl.T, wl.N), dtype=np.int32)
    raise ValueError(f"unknown parent recipe {wl.parents!r}")


def make_inputs(wl: Workload, poison: bool = True) -> Dict[str, Optional[np.ndarray]]:
    """Draw one decode step's operands.

    Returns numpy arrays:
      q                [B*W, Hq, D]        fp16
      prompt_k/v       [B, Lp, Hkv, D]     fp16
      resp_k/v         [Tcap, B*W, Hkv, D] fp16; rows 0..T-2 hold past steps,
                       row T-1 (the current step, not yet appended) and rows
                       >= T hold NaN when ``poison`` else zeros
      k_new/v_new      [B*W, Hkv, D]       fp16, the current step's K/V
      parent           [T, B*W]            int32
      slopes           [Hq] fp32 or None
    """
    rng = np.random.default_rng(wl.seed)
    N, Tcap = wl.N, wl.Tcap
    q = _normal_f16(rng, (N, wl.Hq, wl.D))
    prompt_k = _normal_f16(rng, (wl.B, wl.Lp, wl.Hkv, wl.D))
    prompt_v = _normal_f16(rng, (wl.B, wl.Lp, wl.Hkv, wl.D))
    fill = np.float16(np.nan) if poison else np.float16(0)
    resp_k = np.full((Tcap, N, wl.Hkv, wl.D), fill, dtype=np.float16)
    resp_v = np.full((Tcap, N, wl.Hkv, wl.D), fill, dtype=np.float16)
    if wl.T > 1:
        resp_k[: wl.T - 1] = _normal_f16(rng, (wl.T - 1, N, wl.Hkv, wl.D))
        resp_v[: wl.T - 1] = _normal_f16(rng, (wl.T - 1, N, wl.Hkv, wl.D))
    k_new = _normal_f16(rng, (N, wl.Hkv, wl.D))
    v_new = _normal_f16(rng, (N, wl.Hkv, wl.D))
    parent = make_parent(wl, rng)
    return {
        "q": q, "prompt_k": prompt_k, "prompt_v": prompt_v,
        "resp_k": resp_k, "resp_v": resp_v, "k_new": k_new, "v_new": v_new,
        "parent": parent, "slopes": alibi_slopes(wl.Hq) if wl.alibi else None,
    }
