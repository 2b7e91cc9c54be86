"""GPU parity of segkv_rope_append against the fp64 oracle (oracle/rope.py), and
of the whole step rope_append -> sdpa_decode against oracle rope -> oracle decode."""
import numpy as np
import pytest

from oracle import rope
from paper_2401_05391_amd.workloads import CONFIGS, Workload, make_inputs
from segkv_testlib import assert_parity, same_bits

pytestmark = pytest.mark.gpu

CASES = [
    # name, workload, rotary_dim, interleaved, per-request positions
    ("llama_half", Workload("r1", B=3, W=4, Hq=8, Hkv=2, D=128, Lp=300, T=9, seed=201), 128, False, False),
    ("gptj_interleaved_partial", Workload("r2", B=2, W=4, Hq=4, Hkv=4, D=256, Lp=77, T=5, seed=202), 64, True, False),
    ("d64_half_partial", Workload("r3", B=4, W=1, Hq=6, Hkv=3, D=64, Lp=1000, T=17, parents="identity", seed=203), 32, False, True),
    ("no_rotation", Workload("r4", B=2, W=2, Hq=2, Hkv=2, D=64, Lp=5, T=3, seed=204), 0, False, False),
    ("far_position", Workload("r5", B=1, W=4, Hq=4, Hkv=4, D=128, Lp=8100, T=92, seed=205), 128, False, False),
]


def _ulps(a16, b16):
    """Distance in fp16 representable steps between two finite fp16 arrays."""
    def key(x):
        u = x.view(np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a16) - key(b16))


def _run(wl, R, interleaved, ragged):
    import torch
    import paper_2401_05391_amd as segkv
    x = make_inputs(wl)
    dev = torch.device("cuda:0")
    t = wl.T - 1
    pos_np = None
    if ragged:
        pos_np = (np.random.default_rng(wl.seed).integers(0, wl.Lp + 1, size=wl.B) + t).astype(np.int32)
    q = torch.from_numpy(x["q"]).to(dev)
    kn, vn = torch.from_numpy(x["k_new"]).to(dev), torch.from_numpy(x["v_new"]).to(dev)
    rk, rv = torch.from_numpy(x["resp_k"]).to(dev), torch.from_numpy(x["resp_v"]).to(dev)
    pos = None if pos_np is None else torch.from_numpy(pos_np).to(dev)
    dims = segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, wl.Lp, wl.T, wl.Tcap)
    segkv.rope_append(q, kn, vn, rk, rv, t, dims, 10000.0, R, interleaved, positions=pos)
    torch.cuda.synchronize()
    ork, orv = x["resp_k"].copy(), x["resp_v"].copy()
    q_ref = rope.rope_append(x["q"], x["k_new"], x["v_new"], ork, orv, t, wl.W, wl.Lp, 10000.0, R,
                             interleaved, positions=pos_np)
    return x, dims, (q, rk, rv), (q_ref, ork, orv)


@pytest.mark.parametrize("name,wl,R,interleaved,ragged", CASES, ids=[c[0] for c in CASES])
def test_rope_append_matches_oracle(name, wl, R, interleaved, ragged):
    x, dims, (q, rk, rv), (q_ref, ork, orv) = _run(wl, R, interleaved, ragged)
    t = wl.T - 1
    q_gpu, rk_gpu, rv_gpu = q.cpu().numpy(), rk.cpu().numpy(), rv.cpu().numpy()
    # V row and all other rows: bit-exact (row t of V is a copy; the rest is untouched poison/history)
    assert same_bits(rv_gpu, orv)
    keep = np.ones(wl.Tcap, bool)
    keep[t] = False
    assert same_bits(rk_gpu[keep], ork[keep])
    # rotated values: fp32 arithmetic against fp64, both rounded to fp16 -> equal except
    # at rounding ties, where they may differ by one fp16 step
    for got, ref16 in ((rk_gpu[t], ork[t]), (q_gpu, q_ref.astype(np.float16))):
        assert np.isfinite(got.astype(np.float32)).all()
        d = _ulps(got, ref16)
        assert d.max() <= 1, f"{name}: {d.max()} fp16 steps"
        assert (d != 0).mean() < 2e-3, f"{name}: {(d != 0).mean():.2e} of elements off by one step"
    if R == 0:
        assert same_bits(q_gpu, x["q"]) and same_bits(rk_gpu[t], x["k_new"])
    if R < wl.D:
        assert same_bits(q_gpu[..., R:], x["q"][..., R:])
        assert same_bits(rk_gpu[t][..., R:], x["k_new"][..., R:])


def test_rope_append_then_decode_equals_oracle_chain():
    # the whole step as a framework would run it: producer kernel, then attention
    import torch
    import paper_2401_05391_amd as segkv
    from oracle import segkv_oracle as oracle
    name, wl, R, interleaved, ragged = CASES[0]
    x, dims, (q, rk, rv), (q_ref, ork, orv) = _run(wl, R, interleaved, ragged)
    dev = q.device
    out = torch.full((wl.N, wl.Hq, wl.D), float("nan"), dtype=torch.float16, device=dev)
    nbytes = segkv.workspace_bytes(dims)
    ws = torch.empty(max(nbytes, 16) // 4, dtype=torch.float32, device=dev) if nbytes else None
    segkv.sdpa_decode(out, q, torch.from_numpy(x["prompt_k"]).to(dev), torch.from_numpy(x["prompt_v"]).to(dev),
                      rk, rv, torch.from_numpy(x["parent"]).to(dev), dims, wl.scale, workspace=ws)
    torch.cuda.synchronize()
    # oracle chain: rotated query rounded to fp16 (what the kernel stored), rotated key row in ork
    ref, _, _ = oracle.sdpa_decode(q_ref.astype(np.float16), x["prompt_k"], x["prompt_v"], ork, orv,
                                   x["parent"], wl.W, wl.T, wl.scale)
    assert_parity(out.cpu().numpy(), ref, "rope_append -> sdpa_decode")


def test_rope_append_rejects_bad_arguments():
    import torch
    import paper_2401_05391_amd as segkv
    wl = CASES[0][1]
    dev = torch.device("cuda:0")
    z = lambda *s: torch.zeros(*s, dtype=torch.float16, device=dev)
    dims = segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, wl.Lp, wl.T, wl.Tcap)
    q, kn, vn = z(wl.N, wl.Hq, wl.D), z(wl.N, wl.Hkv, wl.D), z(wl.N, wl.Hkv, wl.D)
    rk, rv = z(wl.Tcap, wl.N, wl.Hkv, wl.D), z(wl.Tcap, wl.N, wl.Hkv, wl.D)
    for kw, status in ((dict(t=wl.Tcap), segkv.binding.SEGKV_INVALID_ARG),
                       (dict(rotary_dim=wl.D + 16), segkv.binding.SEGKV_INVALID_ARG),
                       (dict(rotary_dim=24), segkv.binding.SEGKV_UNSUPPORTED),
                       (dict(rope_base=0.0), segkv.binding.SEGKV_INVALID_ARG)):
        a = dict(t=0, rope_base=10000.0, rotary_dim=wl.D)
        a.update(kw)
        with pytest.raises(segkv.SegkvError) as e:
            segkv.rope_append(q, kn, vn, rk, rv, a["t"], dims, a["rope_base"], a["rotary_dim"])
        assert e.value.status == status
