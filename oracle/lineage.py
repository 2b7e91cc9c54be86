"""Reference for the per-request lineage list kept across decode steps.

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only the tests import this.  It never
imports the GPU package.  Plain Python on small integers.

Section 3.3 of arxiv 2401.05391 hands the attention kernel an index tensor that
says, for every beam and every past step, which row of the response K/V buffer
the beam reads (the same bookkeeping as FasterTransformer's beam-search cache
indirection), and that tensor is updated once per generated token, not per
layer.  The list here is that tensor with equal rows merged: one entry per
*distinct* (step, slot) row that some beam of the request still descends from,
with the set of beams that read it.

Two functions, written independently of each other so that each pins the other:

  entries_from_ancestors   the definition, from a resolved ancestor table
  update                   the per-step rule that needs only the newest parent row

Entry encoding (also the device format): (step << 16) | (slot << 8) | mask,
mask bit j = beam j of the request reads this row.  Order: by step, and by slot
within a step.
"""
from __future__ import annotations

from typing import List, Sequence


def encode(step: int, slot: int, mask: int) -> int:
    return (step << 16) | (slot << 8) | mask


def decode(entry: int):
    return entry >> 16, (entry >> 8) & 0xFF, entry & 0xFF


def entries_from_ancestors(anc, b: int, W: int) -> List[int]:
    """The definition.  anc[s][b*W + j] is the slot whose response row beam j of
    request b reads at step s (Section 3.3's index tensor, transposed); an entry
    exists for every slot that occurs at a step, with the beams it occurs for."""
    out = []
    for s in range(len(anc)):
        row = [int(anc[s][b * W + j]) for j in range(W)]
        for slot in sorted(set(row)):
            mask = sum(1 << j for j in range(W) if row[j] == slot)
            out.append(encode(s, slot, mask))
    return out


def update(entries: Sequence[int], parent_row: Sequence[int], t: int, W: int) -> List[int]:
    """One generated token.  parent_row[j] is the slot, at step t-1, of the hypothesis
    that beam j extends at step t (ignored when t == 0: step 0 extends the shared
    prompt).  Beam j now reads, at every earlier step, what beam parent_row[j] read
    before: an old entry is kept for exactly the beams whose parent was among its
    readers, and disappears when no beam's was.  Step t itself adds one row per
    beam: beam j's own slot j."""
    out = []
    if t > 0:
        for e in entries:
            step, slot, mask = decode(e)
            new_mask = sum(1 << j for j in range(W) if (mask >> int(parent_row[j])) & 1)
            if new_mask:
                out.append(encode(step, slot, new_mask))
    for j in range(W):
        out.append(encode(t, j, 1 << j))
    return out
