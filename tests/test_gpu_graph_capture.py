"""The entry points enqueue kernels only (no allocation, no memset, no
synchronisation), so a decode step can be recorded into a HIP graph and
replayed: the launch-bound regime of small batches is where that matters.
One layer-step = RoPE + append (producer kernel) + attention (+ merge pass when
the plan splits the keys).  The graph is replayed several times with new
inputs written into the same buffers, with eager launches and
synchronisations in between, and every replay must give the bits of the eager
call on the same inputs."""
import numpy as np
import pytest

from segkv_testlib import same_bits

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,W,Hq,Hkv,D,Lp,T", [
    (1, 4, 8, 8, 128, 300, 9),      # few units: split-KV plan, workspace + merge kernel in the graph
    (40, 4, 8, 8, 128, 64, 20),     # 320 units: single launch, two work-groups per CU
    (2, 1, 4, 4, 256, 90, 5),       # greedy, D = 256
])
def test_decode_step_replays_from_a_graph(B, W, Hq, Hkv, D, Lp, T):
    import torch
    import paper_2401_05391_amd as segkv

    dev = torch.device("cuda:0")
    N = B * W
    gen = torch.Generator(device=dev)
    gen.manual_seed(17 + D + W)
    rnd = lambda *s: torch.randn(*s, generator=gen, device=dev, dtype=torch.float32).half()
    tcap = segkv.response_capacity(T)
    dims = segkv.make_dims(B, W, Hq, Hkv, D, Lp, T, tcap)
    pk, pv = rnd(B, Lp, Hkv, D), rnd(B, Lp, Hkv, D)
    rk0, rv0 = rnd(tcap, N, Hkv, D), rnd(tcap, N, Hkv, D)
    parent = torch.randint(0, W, (T, N), generator=gen, device=dev, dtype=torch.int32)
    nb = segkv.workspace_bytes(dims)
    scale = D ** -0.5

    def buffers():
        ws = torch.full((max(nb, 16) // 4,), float("nan"), dtype=torch.float32, device=dev) if nb else None
        return dict(q=torch.empty(N, Hq, D, dtype=torch.float16, device=dev),
                    kn=torch.empty(N, Hkv, D, dtype=torch.float16, device=dev),
                    vn=torch.empty(N, Hkv, D, dtype=torch.float16, device=dev),
                    rk=rk0.clone(), rv=rv0.clone(), ws=ws,
                    out=torch.full((N, Hq, D), float("nan"), dtype=torch.float16, device=dev))

    def step(b):
        segkv.rope_append(b["q"], b["kn"], b["vn"], b["rk"], b["rv"], T - 1, dims, 10000.0, D if D <= 128 else 64)
        segkv.sdpa_decode(b["out"], b["q"], pk, pv, b["rk"], b["rv"], parent, dims, scale, workspace=b["ws"])

    def load(b, inputs):
        b["q"].copy_(inputs[0]); b["kn"].copy_(inputs[1]); b["vn"].copy_(inputs[2])

    eager, graphed = buffers(), buffers()
    inputs = [(rnd(N, Hq, D), rnd(N, Hkv, D), rnd(N, Hkv, D)) for _ in range(4)]

    # record (the launches inside the capture are not executed)
    load(graphed, inputs[0])
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(graphed)
    torch.cuda.synchronize()

    for i, inp in enumerate(inputs):
        load(eager, inp)
        step(eager)
        torch.cuda.synchronize()
        load(graphed, inp)
        graphed["out"].fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert same_bits(graphed["out"].cpu().numpy(), eager["out"].cpu().numpy()), f"replay {i}"
        assert same_bits(graphed["rk"].cpu().numpy(), eager["rk"].cpu().numpy()), f"replay {i}: appended K row"
        assert same_bits(graphed["q"].cpu().numpy(), eager["q"].cpu().numpy()), f"replay {i}: rotated q"
        assert not np.isnan(graphed["out"].float().cpu().numpy()).any()
