"""Pins for the CPU oracle: everything here runs without a GPU.

The oracle (oracle/segkv_oracle.c) is checked against things that are not
itself: a replay of the standard reorder-and-concatenate cache with dense
attention (oracle/dense_gather.py), a library attention routine for beam=1,
closed forms, invariants, and the paper's worked index datum.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import dense_gather
from oracle import segkv_oracle as oracle
from paper_2401_05391_amd.workloads import CONFIGS, Workload, make_inputs


def _oracle_inputs(wl, poison=True):
    """Inputs with the current step appended (what the oracle's attention reads)."""
    x = make_inputs(wl, poison=poison)
    oracle.append_kv(x["resp_k"], x["resp_v"], x["k_new"], x["v_new"], wl.T - 1)
    return x


def _run_oracle(wl, x, **kw):
    return oracle.sdpa_decode(x["q"], x["prompt_k"], x["prompt_v"], x["resp_k"], x["resp_v"],
                              x["parent"], wl.W, wl.T, wl.scale, slopes=x["slopes"], **kw)


def _run_dense(wl, x):
    return dense_gather.sdpa_decode_dense(x["q"], x["prompt_k"], x["prompt_v"], x["resp_k"],
                                          x["resp_v"], x["parent"], wl.W, wl.T, wl.scale,
                                          slopes=x["slopes"])


SMALL = [
    CONFIGS["tiny"],
    Workload("gqa", B=2, W=4, Hq=8, Hkv=2, D=16, Lp=9, T=11, seed=11),
    Workload("alibi", B=2, W=3, Hq=6, Hkv=6, D=8, Lp=7, T=5, alibi=True, seed=12),
    Workload("gqa_alibi", B=1, W=2, Hq=4, Hkv=1, D=32, Lp=5, T=17, alibi=True, seed=13),
    Workload("no_prompt", B=2, W=4, Hq=2, Hkv=2, D=8, Lp=0, T=6, seed=14),
    Workload("first_step", B=3, W=4, Hq=2, Hkv=1, D=8, Lp=6, T=1, seed=15),
    Workload("wide_beam", B=1, W=8, Hq=2, Hkv=2, D=8, Lp=3, T=20, seed=16),
    Workload("greedy", B=3, W=1, Hq=4, Hkv=2, D=16, Lp=10, T=9, parents="identity", seed=17),
]


# ---------------------------------------------------------------- append ----
def test_append_writes_exactly_one_row():
    wl = CONFIGS["tiny"]
    x = make_inputs(wl, poison=False)
    before_k, before_v = x["resp_k"].copy(), x["resp_v"].copy()
    oracle.append_kv(x["resp_k"], x["resp_v"], x["k_new"], x["v_new"], wl.T - 1)
    assert np.array_equal(x["resp_k"][wl.T - 1], x["k_new"])
    assert np.array_equal(x["resp_v"][wl.T - 1], x["v_new"])
    keep = np.ones(wl.Tcap, dtype=bool)
    keep[wl.T - 1] = False
    assert np.array_equal(x["resp_k"][keep], before_k[keep])
    assert np.array_equal(x["resp_v"][keep], before_v[keep])
    with pytest.raises(ValueError):
        oracle.append_kv(x["resp_k"], x["resp_v"], x["k_new"], x["v_new"], wl.Tcap)


# ------------------------------------------------------------- ancestors ----
def test_ancestors_identity_parents():
    B, W, T = 3, 4, 9
    parent = np.tile(np.arange(W, dtype=np.int32), (T, B))
    anc = oracle.ancestors(parent, B, W)
    assert np.array_equal(anc, parent)


def test_ancestors_constant_parents():
    B, W, T, c = 2, 4, 7, 2
    parent = np.full((T, B * W), c, dtype=np.int32)
    anc = oracle.ancestors(parent, B, W)
    assert np.array_equal(anc[T - 1], np.tile(np.arange(W), B))
    assert np.all(anc[: T - 1] == c)


def test_ancestors_permutation_composition():
    # One request; every step applies a permutation.  Written out by hand:
    # the slot of beam j at step s is P_{s+1}[P_{s+2}[...P_{T-1}[j]]].
    W, T = 4, 5
    perms = [np.array(p, dtype=np.int32) for p in
             ([0, 1, 2, 3], [1, 2, 3, 0], [3, 2, 1, 0], [0, 2, 1, 3], [2, 0, 3, 1])]
    parent = np.stack(perms)
    anc = oracle.ancestors(parent, 1, W)
    for j in range(W):
        cur = j
        assert anc[T - 1, j] == j
        for s in range(T - 1, 0, -1):
            cur = perms[s][cur]
            assert anc[s - 1, j] == cur


def test_ancestors_ignore_row_zero_of_parent_table():
    rng = np.random.default_rng(5)
    B, W, T = 2, 4, 6
    parent = rng.integers(0, W, size=(T, B * W), dtype=np.int32)
    other = parent.copy()
    other[0] = rng.integers(0, W, size=B * W)
    assert np.array_equal(oracle.ancestors(parent, B, W), oracle.ancestors(other, B, W))


@pytest.mark.parametrize("B,W,T,seed", [(1, 4, 8, 0), (3, 4, 33, 1), (2, 8, 40, 2), (5, 2, 17, 3),
                                        (2, 1, 5, 4), (1, 3, 1, 5)])
def test_ancestors_match_replayed_standard_cache(B, W, T, seed):
    # Give every response row a unique code; replaying index_select + cat must
    # leave, at position s of beam n's cache, the code of row (s, anc[s][n]).
    rng = np.random.default_rng(seed)
    parent = rng.integers(0, W, size=(T, B * W), dtype=np.int32)
    N = B * W
    codes = (np.arange(T)[:, None] * N + np.arange(N)[None, :]).astype(np.float64)
    resp = codes[:, :, None, None]
    prompt = np.zeros((B, 0, 1, 1))
    cache = dense_gather.replay_standard_cache(prompt, resp, parent, W, T)[:, :, 0, 0]
    anc = oracle.ancestors(parent, B, W)
    offs = (np.arange(N) // W) * W
    for s in range(T):
        expect = s * N + offs + anc[s]
        assert np.array_equal(cache[:, s].astype(np.int64), expect)
    assert anc.min() >= 0 and anc.max() < W


def test_ancestors_exhaustive_tiny():
    # Every parent table for W=2, T=3 (row 0 fixed: it is ignored) against a
    # direct enumeration of "who did I come from".
    W, T = 2, 3
    for rows in itertools.product(itertools.product(range(W), repeat=W), repeat=T - 1):
        parent = np.array([(0, 0)] + list(rows), dtype=np.int32)
        anc = oracle.ancestors(parent, 1, W)
        for j in range(W):
            at2 = j
            at1 = parent[2][at2]
            at0 = parent[1][at1]
            assert (anc[2, j], anc[1, j], anc[0, j]) == (at2, at1, at0)


def test_paper_worked_index_datum(golden_dir):
    # Section 3.3: the value of the index tensor at (beam position, time step)
    # names the item of that time step in the key cache that the position uses.
    kv = {}
    with open(os.path.join(golden_dir, "index_select_worked_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = line.split("=")
                kv[k.strip()] = int(v)
    j = kv["beam_position"] - 1          # 0-based slot
    s = kv["time_step"] - 1              # 0-based step
    want = kv["selected_item"] - 1
    assert kv["index_value"] - 1 == want
    # Build a parent table whose resolved index at (s, j) is `want`, then read
    # back, through the attention value itself, which row was used.
    W, T, D, Lp = 4, s + 2, 8, 3
    parent = np.tile(np.arange(W, dtype=np.int32), (T, 1))
    parent[s + 1, j] = want              # slot j at step s+1 extends slot `want` of step s
    anc = oracle.ancestors(parent, 1, W)
    assert anc[s, j] == want
    q = np.zeros((W, 1, D), dtype=np.float16)
    q[:, 0, 0] = 8.0
    prompt_k = np.zeros((1, Lp, 1, D), dtype=np.float16)
    prompt_v = np.zeros((1, Lp, 1, D), dtype=np.float16)
    resp_k = np.zeros((16, W, 1, D), dtype=np.float16)
    resp_v = np.zeros((16, W, 1, D), dtype=np.float16)
    resp_k[s, :, 0, 0] = 60.0            # all rows of step s dominate the softmax
    resp_v[s, :, 0, 0] = np.arange(1, W + 1)   # value = 1-based item number
    out, _, _ = oracle.sdpa_decode(q, prompt_k, prompt_v, resp_k, resp_v, parent, W, T, 1.0)
    assert abs(out[j, 0, 0] - kv["selected_item"]) < 1e-9
    for other in range(W):
        if other != j:
            assert abs(out[other, 0, 0] - (other + 1)) < 1e-9


# ------------------------------------------------- attention vs dense path ----
@pytest.mark.parametrize("wl", SMALL, ids=lambda w: w.name)
def test_matches_dense_attention_over_replayed_cache(wl):
    x = _oracle_inputs(wl)
    out, anc, probs = _run_oracle(wl, x, want_probs=True)
    # the dense replay cannot digest NaN poison: blank rows >= T (never read by the oracle)
    xr = dict(x)
    xr["resp_k"] = np.nan_to_num(x["resp_k"], nan=0.0)
    xr["resp_v"] = np.nan_to_num(x["resp_v"], nan=0.0)
    ref, ref_p = _run_dense(wl, xr)
    assert np.all(np.isfinite(out))
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(probs.reshape(ref_p.shape), ref_p, rtol=0, atol=1e-13)


def test_brute_force_triple_loop_tiny():
    # Pure-Python loops over the explicitly gathered cache (prompt copied per
    # beam, KV heads copied per query head), nothing vectorised.
    wl = Workload("brute", B=1, W=3, Hq=4, Hkv=2, D=4, Lp=3, T=4, alibi=True, seed=21)
    x = _oracle_inputs(wl)
    out, _, _ = _run_oracle(wl, x)
    kc = dense_gather.replay_standard_cache(x["prompt_k"], np.nan_to_num(x["resp_k"]),
                                            x["parent"], wl.W, wl.T)
    vc = dense_gather.replay_standard_cache(x["prompt_v"], np.nan_to_num(x["resp_v"]),
                                            x["parent"], wl.W, wl.T)
    L = wl.Lp + wl.T
    group = wl.Hq // wl.Hkv
    for n in range(wl.N):
        for h in range(wl.Hq):
            z = []
            for i in range(L):
                dot = 0.0
                for e in range(wl.D):
                    dot += float(x["q"][n, h, e]) * float(kc[n, i, h // group, e])
                z.append(wl.scale * dot + float(x["slopes"][h]) * i)
            zmax = max(z)
            w = [math.exp(v - zmax) for v in z]
            tot = sum(w)
            for e in range(wl.D):
                acc = 0.0
                for i in range(L):
                    acc += w[i] / tot * float(vc[n, i, h // group, e])
                assert abs(acc - out[n, h, e]) < 1e-12


def test_beam1_identity_reduces_to_library_decode_attention():
    torch = pytest.importorskip("torch")
    wl = Workload("lib", B=3, W=1, Hq=8, Hkv=2, D=16, Lp=12, T=7, parents="identity", seed=31)
    x = _oracle_inputs(wl)
    out, _, _ = _run_oracle(wl, x)
    group = wl.Hq // wl.Hkv
    # ordinary decode attention: keys = prompt followed by the response rows
    k = np.concatenate([x["prompt_k"], x["resp_k"][: wl.T].transpose(1, 0, 2, 3)], axis=1)
    v = np.concatenate([x["prompt_v"], x["resp_v"][: wl.T].transpose(1, 0, 2, 3)], axis=1)
    kt = torch.from_numpy(k.astype(np.float64)).permute(0, 2, 1, 3).repeat_interleave(group, 1)
    vt = torch.from_numpy(v.astype(np.float64)).permute(0, 2, 1, 3).repeat_interleave(group, 1)
    qt = torch.from_numpy(x["q"].astype(np.float64)).unsqueeze(2)          # [B, Hq, 1, D]
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, scale=wl.scale)
    np.testing.assert_allclose(out, ref.squeeze(2).numpy(), rtol=0, atol=1e-12)


# ------------------------------------------------------------ closed forms ----
@pytest.mark.parametrize("wl", SMALL, ids=lambda w: w.name)
def test_softmax_rows_sum_to_one(wl):
    x = _oracle_inputs(wl)
    _, _, probs = _run_oracle(wl, x, want_probs=True)
    assert probs.shape == (wl.N * wl.Hq, wl.Lp + wl.T)
    assert np.all(probs >= 0)
    np.testing.assert_allclose(probs.sum(axis=1), 1.0, rtol=0, atol=1e-12)


def test_constant_values_give_constant_context():
    wl = SMALL[1]
    x = _oracle_inputs(wl)
    x["prompt_v"][:] = 1
    x["resp_v"][: wl.T] = 1
    out, _, _ = _run_oracle(wl, x)
    np.testing.assert_allclose(out, 1.0, rtol=0, atol=1e-12)


def test_zero_query_gives_mean_of_selected_rows():
    # q = 0 -> uniform weights -> context is the plain mean of the prompt rows
    # and of the response rows on the beam's own lineage (lineage given by hand).
    B, W, Hq, D, Lp, T = 1, 3, 1, 2, 2, 3
    parent = np.array([[0, 0, 0], [2, 0, 0], [1, 1, 0]], dtype=np.int32)
    # lineage of slot j: step2 -> j ; step1 -> parent[2][j] ; step0 -> parent[1][that]
    # j=0: 0 <- parent[2][0]=1 <- parent[1][1]=0 ; j=1: 1 <- 1 <- 0 ; j=2: 2 <- 0 <- parent[1][0]=2
    lineage = {0: (0, 1, 0), 1: (0, 1, 1), 2: (2, 0, 2)}      # (slot@0, slot@1, slot@2)
    rng = np.random.default_rng(3)
    prompt_v = rng.standard_normal((B, Lp, 1, D)).astype(np.float16)
    resp_v = np.zeros((16, W, 1, D), dtype=np.float16)
    resp_v[:T] = rng.standard_normal((T, W, 1, D)).astype(np.float16)
    zk_p = np.zeros_like(prompt_v)
    zk_r = np.zeros_like(resp_v)
    q = np.zeros((W, Hq, D), dtype=np.float16)
    out, anc, _ = oracle.sdpa_decode(q, zk_p, prompt_v, zk_r, resp_v, parent, W, T, 0.7)
    for j in range(W):
        rows = [prompt_v[0, i, 0].astype(np.float64) for i in range(Lp)]
        rows += [resp_v[s, lineage[j][s], 0].astype(np.float64) for s in range(T)]
        np.testing.assert_allclose(out[j, 0], np.mean(rows, axis=0), rtol=0, atol=1e-13)
        assert tuple(anc[:, j]) == lineage[j]


def test_alibi_closed_form_with_zero_query():
    # q = 0 and slope a: weight of the key at position p is e^{a p} / sum_p e^{a p},
    # positions 0..Lp-1 for the prompt and Lp..Lp+T-1 for the response.
    W, D, Lp, T, a = 1, 1, 3, 2, 0.25
    prompt_v = np.array([1, 2, 4], dtype=np.float16).reshape(1, Lp, 1, D)
    resp_v = np.zeros((16, 1, 1, D), dtype=np.float16)
    resp_v[:T, 0, 0, 0] = [8, 16]
    q = np.zeros((1, 1, D), dtype=np.float16)
    parent = np.zeros((T, 1), dtype=np.int32)
    out, _, probs = oracle.sdpa_decode(q, np.zeros_like(prompt_v), prompt_v, np.zeros_like(resp_v),
                                       resp_v, parent, W, T, 1.0,
                                       slopes=np.array([a]), want_probs=True)
    w = np.exp(a * np.arange(Lp + T))
    w /= w.sum()
    np.testing.assert_allclose(probs[0], w, rtol=0, atol=1e-14)
    np.testing.assert_allclose(out[0, 0, 0], np.dot(w, [1, 2, 4, 8, 16]), rtol=0, atol=1e-13)


def test_two_key_softmax_closed_form_and_scale():
    # one prompt key with logit scale*q.k = ln 3 and one response key with logit 0
    # -> weights 3/4 and 1/4.
    D = 2
    q = np.array([[[2.0, 1.0]]], dtype=np.float16)
    prompt_k = np.array([1.0, 0.5], dtype=np.float16).reshape(1, 1, 1, D)   # q.k = 2.5
    prompt_v = np.array([10.0, -2.0], dtype=np.float16).reshape(1, 1, 1, D)
    resp_k = np.zeros((16, 1, 1, D), dtype=np.float16)
    resp_v = np.zeros((16, 1, 1, D), dtype=np.float16)
    resp_v[0, 0, 0] = [2.0, 6.0]
    scale = math.log(3.0) / 2.5
    out, _, probs = oracle.sdpa_decode(q, prompt_k, prompt_v, resp_k, resp_v,
                                       np.zeros((1, 1), dtype=np.int32), 1, 1, scale,
                                       want_probs=True)
    np.testing.assert_allclose(probs[0], [0.75, 0.25], rtol=0, atol=1e-15)
    np.testing.assert_allclose(out[0, 0], [0.75 * 10 + 0.25 * 2, 0.75 * -2 + 0.25 * 6],
                               rtol=0, atol=1e-14)


def test_prompt_row_permutation_invariance_without_alibi():
    wl = SMALL[1]
    x = _oracle_inputs(wl)
    out, _, _ = _run_oracle(wl, x)
    perm = np.random.default_rng(9).permutation(wl.Lp)
    x["prompt_k"] = np.ascontiguousarray(x["prompt_k"][:, perm])
    x["prompt_v"] = np.ascontiguousarray(x["prompt_v"][:, perm])
    out2, _, _ = _run_oracle(wl, x)
    np.testing.assert_allclose(out2, out, rtol=0, atol=1e-13)


def test_alibi_absolute_and_relative_positions_agree():
    # softmax is shift invariant: slope*keypos and -slope*(qpos-keypos) differ by
    # a per-row constant.  Emulate the relative form by folding the constant
    # into an extra all-ones feature of q and k.
    wl = Workload("rel", B=1, W=2, Hq=2, Hkv=2, D=8, Lp=5, T=4, alibi=True, seed=41)
    x = _oracle_inputs(wl)
    out_abs, _, p_abs = _run_oracle(wl, x, want_probs=True)
    ref, p_ref = _run_dense(wl, {**x, "resp_k": np.nan_to_num(x["resp_k"]),
                                 "resp_v": np.nan_to_num(x["resp_v"])})
    L = wl.Lp + wl.T
    pos = np.arange(L, dtype=np.float64)
    rel = -x["slopes"].astype(np.float64)[:, None] * ((L - 1) - pos)[None, :]
    # relative-bias softmax computed directly from the dense logits
    kc = dense_gather.replay_standard_cache(x["prompt_k"], np.nan_to_num(x["resp_k"]),
                                            x["parent"], wl.W, wl.T)
    logits = wl.scale * np.einsum("nhd,nlhd->nhl", x["q"].astype(np.float64), kc) + rel[None]
    w = np.exp(logits - logits.max(-1, keepdims=True))
    w /= w.sum(-1, keepdims=True)
    np.testing.assert_allclose(p_abs.reshape(w.shape), w, rtol=0, atol=1e-13)
    np.testing.assert_allclose(out_abs, ref, rtol=0, atol=1e-12)


def test_rows_beyond_T_and_dead_slots_do_not_matter():
    wl = SMALL[1]
    x = _oracle_inputs(wl, poison=True)
    out, anc, _ = _run_oracle(wl, x)
    assert np.all(np.isfinite(out))
    # overwrite every response row that no beam descends from with the fp16 maximum
    N = wl.N
    used = np.zeros((wl.T, N), dtype=bool)
    offs = (np.arange(N) // wl.W) * wl.W
    for s in range(wl.T):
        used[s, offs + anc[s]] = True
    y = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in x.items()}
    y["resp_k"][: wl.T][~used] = 65504
    y["resp_v"][: wl.T][~used] = -65504
    out2, _, _ = _run_oracle(wl, y)
    assert np.array_equal(out, out2)


def test_sampled_pairs_equal_full_result():
    wl = SMALL[1]
    x = _oracle_inputs(wl)
    full, _, _ = _run_oracle(wl, x)
    pairs = np.array([[0, 0], [3, 5], [7, 7], [4, 2]], dtype=np.int32)
    part, _, _ = _run_oracle(wl, x, pairs=pairs)
    for r, (n, h) in enumerate(pairs):
        assert np.array_equal(part[r], full[n, h])


def test_half_decoding_is_exact_for_every_bit_pattern():
    # A lone key has weight 1, so the context is its value row, exactly: run
    # every finite fp16 bit pattern through as a value (zero, subnormals,
    # normals, both signs) and compare with numpy's own exact widening.
    vals = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    finite = vals[np.isfinite(vals)]
    D = 8
    n = finite.size // D
    assert n * D == finite.size
    rv = np.zeros((16, n, 1, D), dtype=np.float16)
    rv[0] = finite.reshape(n, 1, D)
    rk = np.zeros_like(rv)
    q = np.ones((n, 1, D), dtype=np.float16)
    empty = np.zeros((n, 0, 1, D), dtype=np.float16)
    out, _, probs = oracle.sdpa_decode(q, empty, empty, rk, rv, np.zeros((1, n), np.int32),
                                       1, 1, 1.0, want_probs=True)
    assert np.array_equal(probs, np.ones((n, 1)))
    assert np.array_equal(out[:, 0], rv[0, :, 0].astype(np.float64))


def test_ragged_prompt_lengths_reduce_to_the_batch_call():
    # per-request lengths: equal lengths reproduce the batch call exactly; shorter ones ignore
    # whatever sits in the padding rows
    wl = Workload("ragged", B=3, W=2, Hq=4, Hkv=2, D=8, Lp=9, T=4, alibi=True, seed=77)
    x = make_inputs(wl)
    rk, rv = x["resp_k"].copy(), x["resp_v"].copy()
    oracle.append_kv(rk, rv, x["k_new"], x["v_new"], wl.T - 1)
    full, anc, _ = oracle.sdpa_decode(x["q"], x["prompt_k"], x["prompt_v"], rk, rv, x["parent"], wl.W,
                                      wl.T, wl.scale, slopes=x["slopes"])
    same, anc2 = oracle.sdpa_decode_ragged(x["q"], x["prompt_k"], x["prompt_v"], rk, rv, x["parent"],
                                           wl.W, wl.T, wl.scale, np.full(wl.B, wl.Lp), slopes=x["slopes"])
    assert np.array_equal(anc, anc2)
    np.testing.assert_allclose(same, full, rtol=0, atol=1e-13)
    lens = np.array([9, 0, 5])
    a, _ = oracle.sdpa_decode_ragged(x["q"], x["prompt_k"], x["prompt_v"], rk, rv, x["parent"], wl.W,
                                     wl.T, wl.scale, lens, slopes=x["slopes"])
    pk2, pv2 = x["prompt_k"].copy(), x["prompt_v"].copy()
    for b, lb in enumerate(lens):
        pk2[b, lb:] = np.float16(np.nan)
        pv2[b, lb:] = np.float16(np.nan)
    b_, _ = oracle.sdpa_decode_ragged(x["q"], pk2, pv2, rk, rv, x["parent"], wl.W, wl.T, wl.scale, lens,
                                      slopes=x["slopes"])
    assert np.array_equal(a, b_) and np.isfinite(a).all()
    np.testing.assert_allclose(a[0:2], full[0:2], rtol=0, atol=1e-13)       # request 0 is at full length
    assert np.abs(a[2:] - full[2:]).max() > 1e-3                            # the others are not
