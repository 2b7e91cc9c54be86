"""Pins for oracle/lineage.py: the per-step update rule against the definition
(built on the ancestor recursion that test_oracle_pins.py pins), against a
simulation that never resolves ancestors at all, against closed forms, and
against a case small enough to follow by hand."""
import numpy as np
import pytest

from oracle import lineage
from oracle import segkv_oracle as oracle


def _parents(rng, T, B, W, kind):
    if kind == "identity":
        return np.tile(np.arange(W, dtype=np.int32), (T, B))
    if kind == "zeros":
        return np.zeros((T, B * W), dtype=np.int32)
    return rng.integers(0, W, (T, B * W)).astype(np.int32)


def _run_updates(parent, b, W, upto):
    ent = []
    for t in range(upto):
        ent = lineage.update(ent, parent[t, b * W:(b + 1) * W], t, W)
    return ent


@pytest.mark.parametrize("W", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("kind", ["uniform", "identity", "zeros"])
def test_update_rule_reproduces_the_definition_at_every_step(W, kind):
    rng = np.random.default_rng(100 + W)
    T, B = 37, 3
    parent = _parents(rng, T, B, W, kind)
    for b in range(B):
        ent = []
        for t in range(T):
            ent = lineage.update(ent, parent[t, b * W:(b + 1) * W], t, W)
            anc = oracle.ancestors(np.ascontiguousarray(parent[:t + 1]), B, W)
            assert ent == lineage.entries_from_ancestors(anc, b, W), (b, t)


@pytest.mark.parametrize("W", [2, 4, 5])
def test_list_describes_the_caches_a_reordering_framework_would_hold(W):
    # The standard graph (Section 3.1): every beam owns a contiguous cache; each step
    # the caches are re-ordered by the parent row (index_select) and the step's own
    # row is appended.  Rows are tagged (step, slot at creation).  No ancestor table.
    rng = np.random.default_rng(7 + W)
    T = 25
    parent = rng.integers(0, W, (T, W)).astype(np.int32)
    caches = [[] for _ in range(W)]
    ent = []
    for t in range(T):
        if t > 0:
            caches = [list(caches[int(parent[t, j])]) for j in range(W)]
        for j in range(W):
            caches[j].append((t, j))
        ent = lineage.update(ent, parent[t], t, W)
        for j in range(W):
            seen = [(s, slot) for s, slot, mask in map(lineage.decode, ent) if (mask >> j) & 1]
            assert seen == caches[j], (t, j)


@pytest.mark.parametrize("W", [1, 3, 8])
def test_masks_partition_the_beams_and_entries_are_ordered(W):
    rng = np.random.default_rng(55 + W)
    T = 60
    parent = rng.integers(0, W, (T, W)).astype(np.int32)
    ent = _run_updates(parent, 0, W, T)
    assert ent == sorted(ent)                       # by step, then slot: the encoding's own order
    for s in range(T):
        masks = [m for st, _, m in map(lineage.decode, ent) if st == s]
        assert sum(masks) == (1 << W) - 1 and all(masks)
        for i, a in enumerate(masks):
            for c in masks[i + 1:]:
                assert a & c == 0


def test_entries_of_old_steps_only_ever_disappear():
    rng = np.random.default_rng(9)
    W, T = 4, 50
    parent = rng.integers(0, W, (T, W)).astype(np.int32)
    ent, before = [], {}
    for t in range(T):
        ent = lineage.update(ent, parent[t], t, W)
        now = {}
        for s, slot, _ in map(lineage.decode, ent):
            now.setdefault(s, set()).add(slot)
        for s, slots in before.items():
            assert now[s] <= slots
        before = now


def test_closed_forms():
    W, T = 4, 9
    ident = _run_updates(_parents(None, T, 1, W, "identity"), 0, W, T)
    assert ident == [lineage.encode(s, j, 1 << j) for s in range(T) for j in range(W)]
    zeros = _run_updates(_parents(None, T, 1, W, "zeros"), 0, W, T)
    want = [lineage.encode(s, 0, (1 << W) - 1) for s in range(T - 1)]
    want += [lineage.encode(T - 1, j, 1 << j) for j in range(W)]
    assert zeros == want


def test_two_beams_by_hand():
    # step 0: both beams start from the prompt, each writes its own row
    e = lineage.update([], [0, 0], 0, 2)
    assert e == [lineage.encode(0, 0, 0b01), lineage.encode(0, 1, 0b10)]
    # step 1: both beams extend hypothesis 1 -> row (0,1) is read by both, (0,0) by nobody
    e = lineage.update(e, [1, 1], 1, 2)
    assert e == [lineage.encode(0, 1, 0b11), lineage.encode(1, 0, 0b01), lineage.encode(1, 1, 0b10)]
    # step 2: beam 0 extends hypothesis 1, beam 1 extends hypothesis 0
    e = lineage.update(e, [1, 0], 2, 2)
    assert e == [lineage.encode(0, 1, 0b11),
                 lineage.encode(1, 0, 0b10), lineage.encode(1, 1, 0b01),
                 lineage.encode(2, 0, 0b01), lineage.encode(2, 1, 0b10)]
