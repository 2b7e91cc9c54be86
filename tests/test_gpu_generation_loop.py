"""The path as a framework would drive it, step after step, on the GPU:
prefill writes the prompt segment; every decode step runs the producer kernel
(RoPE + append into the response row) and the attention kernel; the response
buffers grow by 16 rows when they are full (Section 3.2); beams are re-ordered by
a fresh parent row every step.  Every step's output is compared with the fp64
oracle run on the state the oracle itself has accumulated."""
import numpy as np
import pytest

from oracle import rope
from oracle import segkv_oracle as oracle
from segkv_testlib import assert_parity, same_bits

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("B,W,Hq,Hkv,D,N0,steps,alibi", [
    (2, 4, 8, 2, 128, 70, 37, False),     # grouped queries, growth at steps 16 and 32
    (3, 1, 4, 4, 64, 33, 20, True),       # greedy, ALiBi on top of RoPE-free keys (rotary_dim 0)
    (1, 3, 4, 4, 256, 50, 18, False),     # odd beam width, D = 256, partial interleaved rotary
])
def test_prefill_then_many_decode_steps(B, W, Hq, Hkv, D, N0, steps, alibi):
    import torch
    import paper_2401_05391_amd as segkv
    from paper_2401_05391_amd.workloads import alibi_slopes

    rng = np.random.default_rng(1234 + D + W)
    f16 = lambda *s: rng.standard_normal(s).astype(np.float16)
    dev = torch.device("cuda:0")
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    scale = 1.0 / np.sqrt(D)
    slopes = alibi_slopes(Hq) if alibi else None
    R, interleaved = (0, False) if alibi else ((64, True) if D == 256 else (D, False))
    N = B * W

    # ---- prefill: keys are rotated by their positions before they enter the cache
    q0, k0, v0 = f16(B, N0, Hq, D), f16(B, N0, Hkv, D), f16(B, N0, Hkv, D)
    pos0 = np.tile(np.arange(N0), B)
    k0r = rope.rotate(k0.reshape(B * N0, Hkv, D), pos0, 10000.0, R, interleaved).astype(np.float16).reshape(k0.shape)
    q0r = rope.rotate(q0.reshape(B * N0, Hq, D), pos0, 10000.0, R, interleaved).astype(np.float16).reshape(q0.shape)
    pk, pv = up(k0r), up(v0)
    out_p = torch.empty((B, N0, Hq, D), dtype=torch.float16, device=dev)
    segkv.sdpa_prefill(out_p, up(q0r), pk, pv, segkv.make_dims(B, 1, Hq, Hkv, D, N0, 1, 1), scale,
                       alibi_slopes=None if slopes is None else up(slopes))
    torch.cuda.synchronize()
    assert_parity(out_p.cpu().numpy(), oracle.sdpa_prefill(q0r, k0r, v0, scale, slopes=slopes), "prefill")

    # ---- decode loop
    tcap = segkv.response_capacity(1)
    rk = torch.full((tcap, N, Hkv, D), float("nan"), dtype=torch.float16, device=dev)
    rv = torch.full((tcap, N, Hkv, D), float("nan"), dtype=torch.float16, device=dev)
    ork = np.full((tcap, N, Hkv, D), np.float16(np.nan))
    orv = np.full((tcap, N, Hkv, D), np.float16(np.nan))
    parent = np.zeros((0, N), dtype=np.int32)
    for t in range(steps):
        T = t + 1
        if T > tcap:                                   # grow by 16 rows, copy the valid ones
            new_cap = segkv.response_capacity(T)
            assert new_cap == tcap + 16
            nk = torch.full((new_cap, N, Hkv, D), float("nan"), dtype=torch.float16, device=dev)
            nv = torch.full((new_cap, N, Hkv, D), float("nan"), dtype=torch.float16, device=dev)
            segkv.grow_response(nk, nv, rk, rv, segkv.make_dims(B, W, Hq, Hkv, D, N0, t, tcap))
            rk, rv, tcap = nk, nv, new_cap
            ork = np.concatenate([ork, np.full((16, N, Hkv, D), np.float16(np.nan))])
            orv = np.concatenate([orv, np.full((16, N, Hkv, D), np.float16(np.nan))])
        row = np.tile(np.arange(W, dtype=np.int32), B) if W == 1 else rng.integers(0, W, N).astype(np.int32)
        parent = np.concatenate([parent, row[None]])
        q, kn, vn = f16(N, Hq, D), f16(N, Hkv, D), f16(N, Hkv, D)
        dims = segkv.make_dims(B, W, Hq, Hkv, D, N0, T, tcap)
        qd = up(q)
        segkv.rope_append(qd, up(kn), up(vn), rk, rv, t, dims, 10000.0, R, interleaved)
        out = torch.full((N, Hq, D), float("nan"), dtype=torch.float16, device=dev)
        anc = torch.full((T, N), -1, dtype=torch.int32, device=dev)
        nb = segkv.workspace_bytes(dims)
        ws = torch.full((max(nb, 16) // 4,), float("nan"), dtype=torch.float32, device=dev) if nb else None
        segkv.sdpa_decode(out, qd, pk, pv, rk, rv, up(parent), dims, scale,
                          alibi_slopes=None if slopes is None else up(slopes), anc_out=anc, workspace=ws)
        torch.cuda.synchronize()
        # oracle on its own state
        q_ref = rope.rope_append(q, kn, vn, ork, orv, t, W, N0, 10000.0, R, interleaved)
        ref, ref_anc, _ = oracle.sdpa_decode(q_ref.astype(np.float16), k0r, v0, ork, orv, parent, W, T, scale,
                                             slopes=slopes)
        assert np.array_equal(anc.cpu().numpy(), ref_anc), f"step {t}: ancestors"
        assert_parity(out.cpu().numpy(), ref, f"step {t}")
        # the cache the kernels have built equals the oracle's up to the rounding ties of the
        # rotated row; carry the GPU's row over so that both continue from identical bytes
        got_row = rk[t].cpu().numpy()
        d = np.abs(got_row.astype(np.float32) - ork[t].astype(np.float32))
        assert d.max() <= 2e-3 * max(1.0, float(np.abs(ork[t].astype(np.float32)).max()))
        ork[t] = got_row
        assert same_bits(rv[: T].cpu().numpy(), orv[: T])
    assert np.isnan(rk[steps:].cpu().numpy().astype(np.float32)).all()
