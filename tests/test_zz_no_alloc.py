"""segkv_sdpa_decode_static_scratch (the entry point for callers that cannot
allocate: split-KV partials in the library's static device buffer) against
segkv_sdpa_decode with a caller workspace, through the C-ABI: same kernels and
plan, so the outputs must be the same bits; both are also held to the oracle's
tolerance.  Two calls in a row, the second on a smaller input, so that the
buffer still holds the first call's partials when the second one runs."""
import numpy as np
import pytest

from paper_2401_05391_amd.workloads import Workload, make_inputs
from segkv_testlib import assert_parity, oracle_reference, same_bits

pytestmark = pytest.mark.gpu


def _run_both(wl):
    import torch
    import paper_2401_05391_amd as segkv

    dev = torch.device("cuda:0")
    x = make_inputs(wl)
    up = lambda a: None if a is None else torch.from_numpy(a).to(dev)
    dims = segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, wl.Lp, wl.T, wl.Tcap)
    need = segkv.workspace_bytes(dims)
    assert 0 < need <= segkv.binding.STATIC_SCRATCH_BYTES, "the case must use the scratch buffer"
    res = {}
    for which in ("workspace", "static"):
        q, pk, pv = up(x["q"]), up(x["prompt_k"]), up(x["prompt_v"])
        rk, rv = up(x["resp_k"]), up(x["resp_v"])
        kn, vn, parent, slopes = up(x["k_new"]), up(x["v_new"]), up(x["parent"]), up(x["slopes"])
        out = torch.full((wl.N, wl.Hq, wl.D), float("nan"), dtype=torch.float16, device=dev)
        anc = torch.full((wl.T, wl.N), -1, dtype=torch.int32, device=dev)
        if which == "workspace":
            ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device=dev)
            segkv.sdpa_decode(out, q, pk, pv, rk, rv, parent, dims, wl.scale, k_new=kn, v_new=vn,
                              alibi_slopes=slopes, anc_out=anc, workspace=ws)
        else:
            segkv.sdpa_decode_static_scratch(out, q, pk, pv, rk, rv, parent, dims, wl.scale, k_new=kn,
                                             v_new=vn, alibi_slopes=slopes, anc_out=anc)
        torch.cuda.synchronize()
        res[which] = dict(out=out.cpu().numpy(), anc=anc.cpu().numpy(), rk=rk.cpu().numpy(),
                          rv=rv.cpu().numpy())
    ref_out, ref_anc, ref_rk, ref_rv = oracle_reference(wl, x)
    for which, r in res.items():
        assert np.array_equal(r["anc"], ref_anc), f"{wl.name}/{which}: ancestors"
        assert_parity(r["out"], ref_out, f"{wl.name}/{which}")
        assert same_bits(r["rk"], ref_rk) and same_bits(r["rv"], ref_rv)
    assert same_bits(res["static"]["out"], res["workspace"]["out"]), f"{wl.name}: outputs differ"


def test_static_scratch_equals_caller_workspace_twice_in_a_row():
    # few (request, head) units: the planner cuts each unit's keys into chunks whose
    # partial results pass through the scratch buffer; the second call is smaller
    print("\n[case] static scratch: first call, 16 units of 1500 + 40 keys", flush=True)
    _run_both(Workload("noalloc_a", B=2, W=4, Hq=8, Hkv=8, D=128, Lp=1500, T=40, seed=901))
    print("[case] static scratch: second call, 4 units of 700 + 12 keys, ALiBi, grouped heads", flush=True)
    _run_both(Workload("noalloc_b", B=1, W=3, Hq=8, Hkv=4, D=64, Lp=700, T=12, alibi=True, seed=902))


def test_static_scratch_call_replays_from_a_graph():
    # the callers this entry point is for: a decode step recorded into a HIP graph (no
    # allocation possible inside the capture).  The buffer's address is looked up by one
    # eager call first; the recorded step is replayed with new inputs, eager launches and
    # synchronisations in between, and every replay must give the bits of the eager
    # segkv_sdpa_decode call with a caller workspace.
    import torch
    import paper_2401_05391_amd as segkv

    dev = torch.device("cuda:0")
    B, W, Hq, Hkv, D, Lp, T = 1, 4, 8, 8, 128, 600, 11
    N = B * W
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    rnd = lambda *s: torch.randn(*s, generator=gen, device=dev, dtype=torch.float32).half()
    tcap = segkv.response_capacity(T)
    dims = segkv.make_dims(B, W, Hq, Hkv, D, Lp, T, tcap)
    need = segkv.workspace_bytes(dims)
    assert 0 < need <= segkv.binding.STATIC_SCRATCH_BYTES
    pk, pv = rnd(B, Lp, Hkv, D), rnd(B, Lp, Hkv, D)
    rk, rv = rnd(tcap, N, Hkv, D), rnd(tcap, N, Hkv, D)
    parent = torch.randint(0, W, (T, N), generator=gen, device=dev, dtype=torch.int32)
    q = torch.empty(N, Hq, D, dtype=torch.float16, device=dev)
    out_g = torch.full((N, Hq, D), float("nan"), dtype=torch.float16, device=dev)
    out_e = torch.full((N, Hq, D), float("nan"), dtype=torch.float16, device=dev)
    ws = torch.full((need // 4,), float("nan"), dtype=torch.float32, device=dev)
    scale = D ** -0.5

    q.copy_(rnd(N, Hq, D))
    print("\n[case] static scratch: eager call that looks the buffer up", flush=True)
    segkv.sdpa_decode_static_scratch(out_g, q, pk, pv, rk, rv, parent, dims, scale)
    torch.cuda.synchronize()
    print("[case] static scratch: capture", flush=True)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        segkv.sdpa_decode_static_scratch(out_g, q, pk, pv, rk, rv, parent, dims, scale)
    torch.cuda.synchronize()
    for i in range(4):
        print(f"[case] static scratch: replay {i}", flush=True)
        q.copy_(rnd(N, Hq, D))
        segkv.sdpa_decode(out_e, q, pk, pv, rk, rv, parent, dims, scale, workspace=ws)
        torch.cuda.synchronize()
        out_g.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert same_bits(out_g.cpu().numpy(), out_e.cpu().numpy()), f"replay {i}"
        assert not np.isnan(out_g.float().cpu().numpy()).any()
