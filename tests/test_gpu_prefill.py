"""GPU parity of the prefill attention against the fp64 oracle, and hand-over of
its K/V to the decode kernel (prefill -> first decode step)."""
import numpy as np
import pytest

from paper_2401_05391_amd.workloads import alibi_slopes
from segkv_testlib import assert_parity

pytestmark = pytest.mark.gpu


def _draw(B, N0, Hq, Hkv, D, seed):
    rng = np.random.default_rng(seed)
    f = lambda *s: rng.standard_normal(s, dtype=np.float32).astype(np.float16)
    return f(B, N0, Hq, D), f(B, N0, Hkv, D), f(B, N0, Hkv, D)


def _run(q, k, v, scale, slopes=None):
    import torch
    import paper_2401_05391_amd as segkv
    dev = torch.device("cuda:0")
    B, N0, Hq, D = q.shape
    up = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    out = torch.full((B, N0, Hq, D), float("nan"), dtype=torch.float16, device=dev)
    dims = segkv.make_dims(B, 1, Hq, k.shape[2], D, N0, 1, 1)
    segkv.sdpa_prefill(out, up(q), up(k), up(v), dims, scale, alibi_slopes=up(slopes))
    torch.cuda.synchronize()
    return out.cpu().numpy()


CASES = [
    # B, N0, Hq, Hkv, D, alibi : several key tiles and query blocks, ragged tails
    (1, 1, 1, 1, 64, False),
    (2, 31, 2, 2, 64, False),
    (2, 33, 4, 2, 128, False),
    (1, 130, 4, 4, 128, True),
    (2, 257, 8, 2, 128, False),
    (1, 300, 2, 1, 256, False),
    (2, 521, 4, 2, 256, True),
    (3, 128, 2, 2, 64, True),
    (1, 515, 2, 2, 128, False),
]


@pytest.mark.parametrize("staging", ["direct", "regs"])
@pytest.mark.parametrize("B,N0,Hq,Hkv,D,alibi", CASES)
def test_prefill_matches_oracle(B, N0, Hq, Hkv, D, alibi, staging, planner_env):
    # D = 128 and 256 have two kernels: tiles copied straight into LDS (the default) and
    # tiles staged through registers (SEGKV_PREFILL=regs); D = 64 ignores the knob
    from oracle import segkv_oracle as oracle
    if staging == "regs" and D == 64:
        pytest.skip("one kernel only at this head dimension")
    planner_env(SEGKV_PREFILL=staging)
    print(f"\n[case] prefill B={B} N0={N0} Hq={Hq} Hkv={Hkv} D={D} alibi={alibi}", flush=True)
    q, k, v = _draw(B, N0, Hq, Hkv, D, 1000 + N0)
    slopes = alibi_slopes(Hq) if alibi else None
    scale = 1.0 / np.sqrt(D)
    ref = oracle.sdpa_prefill(q, k, v, scale, slopes=slopes)
    got = _run(q, k, v, scale, slopes)
    assert_parity(got, ref, f"prefill N0={N0} D={D}")


@pytest.mark.parametrize("staging", ["direct", "regs"])
@pytest.mark.parametrize("D,scale,alibi", [(128, -0.11, False), (128, 0.0, True), (128, 0.0, False), (128, 1e-36, True),
                                           (64, -0.2, True), (256, -0.07, False), (64, 0.0, True)])
def test_prefill_negative_and_zero_scale(D, scale, alibi, staging, planner_env):
    # the kernels keep the logits in the units of the raw products and move the sign of
    # the scale into Q; a zero scale leaves only the bias (uniform weights without one)
    from oracle import segkv_oracle as oracle
    if staging == "regs" and D == 64:
        pytest.skip("one kernel only at this head dimension")
    planner_env(SEGKV_PREFILL=staging)
    B, N0, Hq, Hkv = 2, 150, 4, 2
    print(f"\n[case] prefill scale={scale} D={D} alibi={alibi} {staging}", flush=True)
    q, k, v = _draw(B, N0, Hq, Hkv, D, 77)
    slopes = alibi_slopes(Hq) if alibi else None
    ref = oracle.sdpa_prefill(q, k, v, scale, slopes=slopes)
    got = _run(q, k, v, scale, slopes)
    assert_parity(got, ref, f"prefill scale={scale} D={D}")


def test_prefill_is_deterministic_and_ignores_future_keys():
    q, k, v = _draw(2, 200, 4, 2, 128, 7)
    a = _run(q, k, v, 0.088)
    b = _run(q, k, v, 0.088)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    k2, v2 = k.copy(), v.copy()
    k2[:, 150:] = 60000
    v2[:, 150:] = -60000
    c = _run(q, k2, v2, 0.088)
    # (not bit-identical: lanes that do see the huge keys move the wave's shared
    # rescale points, which changes the rounding of their neighbours)
    from oracle import segkv_oracle as oracle
    ref = oracle.sdpa_prefill(q, k, v, 0.088)
    assert_parity(c[:, :150], ref[:, :150], "tokens before the poisoned keys")
    assert np.max(np.abs(a[:, :150].astype(np.float64) - c[:, :150].astype(np.float64))) <= 1e-3


def _bench_prefill_shapes():
    from bench import PREFILL_SHAPES
    return PREFILL_SHAPES


@pytest.mark.parametrize("name,B,N0,Hq,Hkv,D", _bench_prefill_shapes(), ids=[c[0] for c in _bench_prefill_shapes()])
def test_benchmark_prompt_shapes_sampled_rows(name, B, N0, Hq, Hkv, D):
    # every shape `bench.py --prefill` quotes, at the batch size it times; the oracle
    # computes sampled (request, token, head) rows one by one: tile and query-block
    # boundaries, the first and the last token, every query head of one KV group
    # (grouped-query shapes), and random rows
    from oracle import segkv_oracle as oracle
    print(f"\n[case] prefill {name} B={B} N0={N0} Hq={Hq} Hkv={Hkv} D={D}", flush=True)
    q, k, v = _draw(B, N0, Hq, Hkv, D, 99)
    scale = 1.0 / np.sqrt(D)
    got = _run(q, k, v, scale)
    print("[gpu done]", flush=True)
    rng = np.random.default_rng(5)
    edges = sorted({t for t in (0, 1, 15, 16, 31, 32, 33, 127, 128, 255, 256, 257, N0 // 2 - 1, N0 // 2,
                                N0 - 129, N0 - 128, N0 - 33, N0 - 32, N0 - 2, N0 - 1) if 0 <= t < N0})
    G = Hq // Hkv
    fixed = [(b, t, h) for b in (0, B - 1) for t in edges for h in (0, Hq - 1)]
    fixed += [(B // 2, t, (Hkv // 2) * G + j) for t in (edges[3], edges[-1], N0 // 3) for j in range(G)]
    rnd = np.stack([rng.integers(0, B, 400), rng.integers(0, N0, 400), rng.integers(0, Hq, 400)], 1)
    rows = np.concatenate([np.asarray(fixed, dtype=np.int64), rnd]).astype(np.int32)
    ref = oracle.sdpa_prefill(q, k, v, scale, rows=rows)
    sel = got[rows[:, 0], rows[:, 1], rows[:, 2]]
    max_abs, rel_l2 = assert_parity(sel, ref, f"prefill {name} sampled")
    print(f"[parity] {name}: {len(rows)} rows, max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}", flush=True)
    assert np.all(np.isfinite(got.astype(np.float32))), "non-finite output outside the sampled rows"


WORK_ORDER_SHAPES = [
    # B, N0, Hq, Hkv, D: how the (request, head, query block) items fall on the XCDs
    (5, 700, 6, 3, 128),      # 30 heads: XCD shares of 4 and 3 heads, one group each
    (2, 1500, 56, 8, 256),    # 14 heads per XCD in three groups of 5, 5 and 4
    (1, 12837, 2, 1, 128),    # more query blocks per head (101) than work-group slots per XCD
    (3, 257, 1, 1, 64),       # fewer heads than XCDs: most shares are empty
    (1, 900, 9, 9, 128),      # 9 heads: one XCD with two, seven with one
]


@pytest.mark.parametrize("B,N0,Hq,Hkv,D", WORK_ORDER_SHAPES)
def test_every_query_block_of_every_head_is_computed(B, N0, Hq, Hkv, D):
    # the output starts as NaN: a (request, head, block) item that no work-group took, or
    # took twice with different operands, shows up in the finite check or in the sampled rows
    from oracle import segkv_oracle as oracle
    print(f"\n[case] prefill work order B={B} N0={N0} Hq={Hq} Hkv={Hkv} D={D}", flush=True)
    q, k, v = _draw(B, N0, Hq, Hkv, D, 4242)
    scale = 1.0 / np.sqrt(D)
    got = _run(q, k, v, scale)
    assert np.all(np.isfinite(got.astype(np.float32))), "rows left unwritten"
    rng = np.random.default_rng(9)
    blk = 256 if D == 256 else 128
    fixed = [(b, t, h) for b in range(B) for h in range(Hq)
             for t in sorted({0, min(N0 - 1, blk - 1), min(N0 - 1, blk), N0 - 1})]
    rnd = np.stack([rng.integers(0, B, 200), rng.integers(0, N0, 200), rng.integers(0, Hq, 200)], 1)
    rows = np.concatenate([np.asarray(fixed, dtype=np.int64), rnd]).astype(np.int32)
    if len(rows) > 700:
        rows = rows[rng.permutation(len(rows))[:700]]
    ref = oracle.sdpa_prefill(q, k, v, scale, rows=rows)
    assert_parity(got[rows[:, 0], rows[:, 1], rows[:, 2]], ref, f"prefill work order N0={N0} D={D}")


def _random_prefill_shapes(n, seed):
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(n):
        D = int(rng.choice([64, 128, 128, 256]))
        Hkv = int(rng.choice([1, 2, 3, 5, 8]))
        G = int(rng.choice([1, 1, 2, 4]))
        B = int(rng.integers(1, 5))
        N0 = int(rng.choice([rng.integers(1, 40), rng.integers(40, 300), rng.integers(300, 900)]))
        shapes.append((B, N0, Hkv * G, Hkv, D, bool(rng.integers(0, 2)), float(rng.choice([1.0, -1.0]))))
    return shapes


@pytest.mark.parametrize("B,N0,Hq,Hkv,D,alibi,sign", _random_prefill_shapes(16, 20240))
def test_prefill_random_shapes(B, N0, Hq, Hkv, D, alibi, sign):
    # seeded random dimensions: ragged lengths around the tile and block sizes, grouped heads,
    # head counts that do not divide among the XCDs, both signs of the scale
    from oracle import segkv_oracle as oracle
    print(f"\n[case] prefill random B={B} N0={N0} Hq={Hq} Hkv={Hkv} D={D} alibi={alibi} sign={sign}", flush=True)
    q, k, v = _draw(B, N0, Hq, Hkv, D, 31 * N0 + Hq)
    slopes = alibi_slopes(Hq) if alibi else None
    scale = sign / np.sqrt(D)
    ref = oracle.sdpa_prefill(q, k, v, scale, slopes=slopes)
    got = _run(q, k, v, scale, slopes)
    assert_parity(got, ref, f"prefill random N0={N0} D={D}")


def test_prefill_then_first_decode_step_share_the_prompt_segment():
    # K/V given to prefill are handed unchanged to the decode kernel as the
    # prompt segment; the decode step (beam 1, T = 1) at position N0 must match
    # the oracle's prefill over N0 + 1 tokens at its last token.
    import torch
    import paper_2401_05391_amd as segkv
    from oracle import segkv_oracle as oracle
    B, N0, Hq, Hkv, D = 2, 96, 4, 2, 128
    q, k, v = _draw(B, N0 + 1, Hq, Hkv, D, 11)
    scale = 1.0 / np.sqrt(D)
    ref = oracle.sdpa_prefill(q, k, v, scale)
    dev = torch.device("cuda:0")
    pk = torch.from_numpy(np.ascontiguousarray(k[:, :N0])).to(dev)
    pv = torch.from_numpy(np.ascontiguousarray(v[:, :N0])).to(dev)
    pq = torch.from_numpy(np.ascontiguousarray(q[:, :N0])).to(dev)
    out_p = torch.empty((B, N0, Hq, D), dtype=torch.float16, device=dev)
    segkv.sdpa_prefill(out_p, pq, pk, pv, segkv.make_dims(B, 1, Hq, Hkv, D, N0, 1, 1), scale)
    rk = torch.full((16, B, Hkv, D), float("nan"), dtype=torch.float16, device=dev)
    rv = torch.full((16, B, Hkv, D), float("nan"), dtype=torch.float16, device=dev)
    out_d = torch.empty((B, Hq, D), dtype=torch.float16, device=dev)
    dims = segkv.make_dims(B, 1, Hq, Hkv, D, N0, 1, 16)
    nb = segkv.workspace_bytes(dims)
    ws = torch.empty(max(nb, 16) // 4, dtype=torch.float32, device=dev) if nb else None
    segkv.sdpa_decode(out_d, torch.from_numpy(np.ascontiguousarray(q[:, N0])).to(dev), pk, pv, rk, rv,
                      None, dims, scale, k_new=torch.from_numpy(np.ascontiguousarray(k[:, N0])).to(dev),
                      v_new=torch.from_numpy(np.ascontiguousarray(v[:, N0])).to(dev), workspace=ws)
    torch.cuda.synchronize()
    assert_parity(out_p.cpu().numpy(), ref[:, :N0], "prefill part")
    assert_parity(out_d.cpu().numpy(), ref[:, N0], "first decode step")
