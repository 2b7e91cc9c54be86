"""The lineage list kept across decode steps, on the GPU: the per-step update
kernel against the oracle's list entry by entry, and the attention call that
reads the list against the call that resolves the raw parent table (same bits)
and against the fp64 oracle."""
import numpy as np
import pytest

from oracle import lineage as lineage_oracle
from oracle import segkv_oracle as oracle
from paper_2401_05391_amd.workloads import Workload, make_inputs
from segkv_testlib import assert_parity, same_bits

pytestmark = pytest.mark.gpu

HDR = 4     # 32-bit words ahead of a request's entries: {entries, steps covered, 0, 0}


def _assert_same_attention(from_list, from_table, T, what=""):
    """Same tiles, same arithmetic.  Up to 256 response steps the tiles are also dealt
    to the waves in the same order, so the bits are equal; beyond that the wave that
    prepares the list joins the deal earlier when it only has to copy it, and the
    fp32 partial sums are combined in a different order."""
    if T <= 256:
        assert same_bits(from_list, from_table), what
    else:
        diff = np.abs(from_list.astype(np.float64) - from_table.astype(np.float64)).max()
        assert diff <= 1e-3, (what, diff)


def _device_list(buf, b, cap):
    words = buf.cpu().numpy().view(np.uint32).reshape(-1, HDR + cap)[b]
    return int(words[1]), [int(x) for x in words[HDR:HDR + int(words[0])]]


@pytest.mark.parametrize("W,kind", [(1, "uniform"), (2, "uniform"), (4, "uniform"), (8, "uniform"),
                                    (4, "identity"), (3, "zeros")])
def test_update_kernel_keeps_the_oracles_list(W, kind):
    import torch
    import paper_2401_05391_amd as segkv
    B, T = 3, 300                                  # identity parents: 1200 entries, 5 passes of 256
    rng = np.random.default_rng(31 + W)
    if kind == "identity":
        parent = np.tile(np.arange(W, dtype=np.int32), (T, B))
    elif kind == "zeros":
        parent = np.zeros((T, B * W), dtype=np.int32)
    else:
        parent = rng.integers(0, W, (T, B * W)).astype(np.int32)
    cap = ((T * W + 3) // 4) * 4
    dims = segkv.make_dims(B, W, 1, 1, 64, 0, 1, 1)
    dev = torch.device("cuda:0")
    nbytes = segkv.lineage_bytes(dims, cap)
    assert nbytes == B * (HDR + cap) * 4
    buf = torch.full((nbytes // 4,), -1, dtype=torch.int32, device=dev)       # garbage: t == 0 starts the list
    pdev = torch.from_numpy(parent).to(dev)
    ref = [[] for _ in range(B)]
    for t in range(T):
        segkv.lineage_update(buf, cap, pdev[t] if t > 0 else None, t, dims)
        for b in range(B):
            ref[b] = lineage_oracle.update(ref[b], parent[t, b * W:(b + 1) * W], t, W)
        if t < 40 or t % 37 == 0 or t == T - 1:
            torch.cuda.synchronize()
            for b in range(B):
                steps, got = _device_list(buf, b, cap)
                assert steps == t + 1
                assert got == ref[b], f"step {t} request {b}"


def _lineage_for(parent, B, W, T, cap):
    import torch
    import paper_2401_05391_amd as segkv
    dims = segkv.make_dims(B, W, 1, 1, 64, 0, 1, 1)
    buf = torch.zeros(segkv.lineage_bytes(dims, cap) // 4, dtype=torch.int32, device="cuda:0")
    pdev = torch.from_numpy(np.ascontiguousarray(parent)).to("cuda:0")
    for t in range(T):
        segkv.lineage_update(buf, cap, pdev[t] if t > 0 else None, t, dims)
    return buf


CASES = [
    # workload, planner knobs, compare with the oracle as well
    (Workload("lin_single_launch", B=40, W=4, Hq=8, Hkv=8, D=128, Lp=64, T=37, seed=601), {}, True),
    (Workload("lin_few_units", B=2, W=4, Hq=8, Hkv=2, D=128, Lp=300, T=70, seed=602), {}, True),
    (Workload("lin_alibi_d64", B=3, W=3, Hq=4, Hkv=4, D=64, Lp=100, T=290, alibi=True, seed=603), {}, True),
    (Workload("lin_d256_w8", B=2, W=8, Hq=2, Hkv=2, D=256, Lp=40, T=33, seed=604), {}, True),
    (Workload("lin_no_prompt", B=2, W=4, Hq=4, Hkv=4, D=128, Lp=0, T=130, seed=605), {}, True),
    # a response too long for one work-group's list: chunks of the response, each
    # looking up its own range of the list
    (Workload("lin_response_chunks", B=1, W=4, Hq=4, Hkv=4, D=128, Lp=96, T=1300, seed=606), {}, True),
    (Workload("lin_greedy", B=4, W=1, Hq=8, Hkv=8, D=128, Lp=50, T=20, parents="identity", seed=607), {}, True),
    # two adjacent 64-wide heads per work-group
    (Workload("lin_head_pairs", B=2, W=4, Hq=4, Hkv=4, D=64, Lp=70, T=90, alibi=True, seed=608),
     dict(SEGKV_PAIR_HEADS=1), True),
]


@pytest.mark.parametrize("wl,knobs,with_oracle", CASES, ids=[c[0].name for c in CASES])
def test_attention_from_the_list_equals_attention_from_the_parent_table(wl, knobs, with_oracle, planner_env):
    import torch
    import paper_2401_05391_amd as segkv
    for k, v in knobs.items():
        planner_env(**{k: v})
    x = make_inputs(wl)
    dev = torch.device("cuda:0")
    up = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    dims = segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, wl.Lp, wl.T, wl.Tcap)
    cap = ((wl.Tcap * wl.W + 3) // 4) * 4
    lin = _lineage_for(x["parent"], wl.B, wl.W, wl.T, cap)
    nbytes = segkv.workspace_bytes(dims)
    outs = []
    for use_list in (False, True):
        rk, rv = up(x["resp_k"]), up(x["resp_v"])
        ws = torch.full((max(nbytes, 16) // 4,), float("nan"), dtype=torch.float32, device=dev) if nbytes else None
        out = torch.full((wl.N, wl.Hq, wl.D), float("nan"), dtype=torch.float16, device=dev)
        kw = dict(k_new=up(x["k_new"]), v_new=up(x["v_new"]), alibi_slopes=up(x["slopes"]), workspace=ws)
        if use_list:
            segkv.sdpa_decode_lineage(out, up(x["q"]), up(x["prompt_k"]), up(x["prompt_v"]), rk, rv, lin, cap,
                                      dims, wl.scale, **kw)
        else:
            segkv.sdpa_decode(out, up(x["q"]), up(x["prompt_k"]), up(x["prompt_v"]), rk, rv, up(x["parent"]),
                              dims, wl.scale, **kw)
        torch.cuda.synchronize()
        outs.append((out.cpu().numpy(), rk.cpu().numpy(), rv.cpu().numpy()))
    assert not np.isnan(outs[1][0].astype(np.float32)).any()
    _assert_same_attention(outs[1][0], outs[0][0], wl.T, wl.name)
    assert same_bits(outs[1][1], outs[0][1]) and same_bits(outs[1][2], outs[0][2])
    if with_oracle:
        ork, orv = x["resp_k"].copy(), x["resp_v"].copy()
        oracle.append_kv(ork, orv, x["k_new"], x["v_new"], wl.T - 1)
        ref, _, _ = oracle.sdpa_decode(x["q"], x["prompt_k"], x["prompt_v"], ork, orv, x["parent"],
                                       wl.W, wl.T, wl.scale, slopes=x["slopes"])
        assert_parity(outs[1][0], ref, wl.name)


@pytest.mark.parametrize("name", ["llama2_70b_gqa", "bloom176b_alibi"])
def test_full_size_list_against_parent_table(name):
    # benchmark configurations at full size, fused append: the same bits either way
    import torch
    import paper_2401_05391_amd as segkv
    from paper_2401_05391_amd.workloads import CONFIGS
    wl = CONFIGS[name]
    x = make_inputs(wl)
    dev = torch.device("cuda:0")
    up = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    dims = segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, wl.Lp, wl.T, wl.Tcap)
    cap = wl.Tcap * wl.W
    lin = _lineage_for(x["parent"], wl.B, wl.W, wl.T, cap)
    nbytes = segkv.workspace_bytes(dims)
    ws = torch.empty(max(nbytes, 16) // 4, dtype=torch.float32, device=dev) if nbytes else None
    q, pk, pv = up(x["q"]), up(x["prompt_k"]), up(x["prompt_v"])
    kn, vn, slopes = up(x["k_new"]), up(x["v_new"]), up(x["slopes"])
    outs = []
    for use_list in (False, True):
        rk, rv = up(x["resp_k"]), up(x["resp_v"])
        out = torch.full((wl.N, wl.Hq, wl.D), float("nan"), dtype=torch.float16, device=dev)
        if use_list:
            segkv.sdpa_decode_lineage(out, q, pk, pv, rk, rv, lin, cap, dims, wl.scale, k_new=kn, v_new=vn,
                                      alibi_slopes=slopes, workspace=ws)
        else:
            segkv.sdpa_decode(out, q, pk, pv, rk, rv, up(x["parent"]), dims, wl.scale, k_new=kn, v_new=vn,
                              alibi_slopes=slopes, workspace=ws)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
        assert same_bits(rk[wl.T - 1].cpu().numpy(), x["k_new"])
        del rk, rv
    assert same_bits(outs[1], outs[0])


def _random_beam_workloads(n, seed):
    """Seeded draw of small beam-search shapes across what the planner looks at."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        D = int(rng.choice([64, 128, 256]))
        W = int(rng.choice([2, 3, 4, 5, 8]))
        Hkv = int(rng.choice([1, 2, 4, 8]))
        G = int(rng.choice([1, 1, 2, 4, 8]))
        out.append(Workload(f"linrnd{seed}_{i}", B=int(rng.integers(1, 5)), W=W, Hq=Hkv * G, Hkv=Hkv, D=D,
                            Lp=int(rng.choice([0, 1, 33, 100, 257])), T=int(rng.choice([1, 2, 17, 64, 130, 300])),
                            alibi=bool(rng.integers(0, 2)),
                            parents=str(rng.choice(["uniform", "uniform", "identity", "zeros"])),
                            seed=2000 * seed + i))
    return out


@pytest.mark.parametrize("wl", _random_beam_workloads(24, 11), ids=lambda w: w.name)
def test_random_shapes_list_against_parent_table(wl):
    import torch
    import paper_2401_05391_amd as segkv
    x = make_inputs(wl)
    dev = torch.device("cuda:0")
    up = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    dims = segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, wl.Lp, wl.T, wl.Tcap)
    cap = ((wl.Tcap * wl.W + 3) // 4) * 4
    lin = _lineage_for(x["parent"], wl.B, wl.W, wl.T, cap)
    nbytes = segkv.workspace_bytes(dims)
    ws = torch.empty(max(nbytes, 16) // 4, dtype=torch.float32, device=dev) if nbytes else None
    rk, rv = up(x["resp_k"]), up(x["resp_v"])
    segkv.append_kv(rk, rv, up(x["k_new"]), up(x["v_new"]), wl.T - 1, dims)
    a = torch.empty((wl.N, wl.Hq, wl.D), dtype=torch.float16, device=dev)
    c = torch.full((wl.N, wl.Hq, wl.D), float("nan"), dtype=torch.float16, device=dev)
    args = (up(x["q"]), up(x["prompt_k"]), up(x["prompt_v"]), rk, rv)
    segkv.sdpa_decode(a, *args, up(x["parent"]), dims, wl.scale, alibi_slopes=up(x["slopes"]), workspace=ws)
    segkv.sdpa_decode_lineage(c, *args, lin, cap, dims, wl.scale, alibi_slopes=up(x["slopes"]), workspace=ws)
    torch.cuda.synchronize()
    _assert_same_attention(c.cpu().numpy(), a.cpu().numpy(), wl.T, wl.name)
    # and both against the oracle, which resolves the lineage from the parent table
    ork, orv = x["resp_k"].copy(), x["resp_v"].copy()
    oracle.append_kv(ork, orv, x["k_new"], x["v_new"], wl.T - 1)
    ref, _, _ = oracle.sdpa_decode(x["q"], x["prompt_k"], x["prompt_v"], ork, orv, x["parent"], wl.W, wl.T,
                                   wl.scale, slopes=x["slopes"])
    assert_parity(c.cpu().numpy(), ref, f"{wl.name}/list")
    assert_parity(a.cpu().numpy(), ref, f"{wl.name}/parent table")


def test_step_by_step_generation_with_the_list():
    # the list follows the beams through 60 steps; every step's attention from the
    # list is compared with attention from the table of all parent rows so far
    import torch
    import paper_2401_05391_amd as segkv
    B, W, Hq, Hkv, D, Lp, steps = 2, 4, 8, 2, 128, 45, 60
    N = B * W
    rng = np.random.default_rng(77)
    dev = torch.device("cuda:0")
    f16 = lambda *s: torch.from_numpy(rng.standard_normal(s).astype(np.float16)).to(dev)
    pk, pv = f16(B, Lp, Hkv, D), f16(B, Lp, Hkv, D)
    tcap = 64
    cap = tcap * W
    rk = torch.full((tcap, N, Hkv, D), float("nan"), dtype=torch.float16, device=dev)
    rv = torch.full((tcap, N, Hkv, D), float("nan"), dtype=torch.float16, device=dev)
    lin = torch.zeros(segkv.lineage_bytes(segkv.make_dims(B, W, Hq, Hkv, D, Lp, 1, tcap), cap) // 4,
                      dtype=torch.int32, device=dev)
    parent = torch.zeros((0, N), dtype=torch.int32, device=dev)
    for t in range(steps):
        dims = segkv.make_dims(B, W, Hq, Hkv, D, Lp, t + 1, tcap)
        row = torch.from_numpy(rng.integers(0, W, N).astype(np.int32)).to(dev)
        parent = torch.cat([parent, row[None]])
        segkv.lineage_update(lin, cap, row, t, dims)
        q, kn, vn = f16(N, Hq, D), f16(N, Hkv, D), f16(N, Hkv, D)
        segkv.append_kv(rk, rv, kn, vn, t, dims)
        nb = segkv.workspace_bytes(dims)
        ws = torch.empty(max(nb, 16) // 4, dtype=torch.float32, device=dev) if nb else None
        a = torch.empty(N, Hq, D, dtype=torch.float16, device=dev)
        c = torch.empty(N, Hq, D, dtype=torch.float16, device=dev)
        segkv.sdpa_decode(a, q, pk, pv, rk, rv, parent.contiguous(), dims, D ** -0.5, workspace=ws)
        segkv.sdpa_decode_lineage(c, q, pk, pv, rk, rv, lin, cap, dims, D ** -0.5, workspace=ws)
        torch.cuda.synchronize()
        assert same_bits(c.cpu().numpy(), a.cpu().numpy()), f"step {t}"


def test_lineage_arguments_are_checked():
    import torch
    import paper_2401_05391_amd as segkv
    dims = segkv.make_dims(2, 4, 4, 4, 64, 0, 10, 16)
    buf = torch.zeros(segkv.lineage_bytes(dims, 64) // 4, dtype=torch.int32, device="cuda:0")
    with pytest.raises(segkv.SegkvError):           # capacity not a multiple of 4
        segkv.lineage_update(buf, 62, None, 0, dims)
    with pytest.raises(segkv.SegkvError):           # 17 steps of 4 beams do not fit 64 entries
        segkv.lineage_update(buf, 64, buf, 16, dims)
    with pytest.raises(segkv.SegkvError):           # a parent row is required after step 0
        segkv.lineage_update(buf, 64, None, 3, dims)
    assert segkv.lineage_bytes(dims, 62) == 0
