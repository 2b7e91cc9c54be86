"""Shared helpers of the GPU parity tests: upload, run through the C-ABI, compare."""
from __future__ import annotations

import numpy as np

MAX_ABS_TOL = 2e-3     # fp16 output vs fp64 oracle, element-wise
REL_L2_TOL = 1e-3      # ||gpu - ref||_2 / ||ref||_2 over the whole output


def oracle_reference(wl, x, pairs=None):
    """fp64 oracle on the same bytes; returns (out, anc, resp_k_after, resp_v_after)."""
    from oracle import segkv_oracle as oracle
    rk, rv = x["resp_k"].copy(), x["resp_v"].copy()
    oracle.append_kv(rk, rv, x["k_new"], x["v_new"], wl.T - 1)
    out, anc, _ = oracle.sdpa_decode(x["q"], x["prompt_k"], x["prompt_v"], rk, rv, x["parent"],
                                     wl.W, wl.T, wl.scale, slopes=x["slopes"], pairs=pairs)
    return out, anc, rk, rv


def run_gpu(wl, x, fused=True, want_anc=True, poison_workspace=True, repeats=1):
    """One decode step on cuda:0 through libsegkv.  Returns dict of numpy results."""
    import torch
    import paper_2401_05391_amd as segkv

    dev = torch.device("cuda:0")

    def up(a):
        return None if a is None else torch.from_numpy(a).to(dev)

    q, pk, pv = up(x["q"]), up(x["prompt_k"]), up(x["prompt_v"])
    rk, rv = up(x["resp_k"]), up(x["resp_v"])
    kn, vn = up(x["k_new"]), up(x["v_new"])
    parent = up(x["parent"])
    slopes = up(x["slopes"])
    dims = segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, wl.Lp, wl.T, wl.Tcap)
    nbytes = segkv.workspace_bytes(dims)
    ws = None
    if nbytes:
        ws = torch.empty(nbytes // 4, dtype=torch.float32, device=dev)
        if poison_workspace:
            ws.fill_(float("nan"))
    outs = []
    anc = torch.full((wl.T, wl.N), -1, dtype=torch.int32, device=dev) if want_anc else None
    for _ in range(repeats):
        out = torch.full((wl.N, wl.Hq, wl.D), float("nan"), dtype=torch.float16, device=dev)
        if fused:
            segkv.sdpa_decode(out, q, pk, pv, rk, rv, parent, dims, wl.scale, k_new=kn, v_new=vn,
                              alibi_slopes=slopes, anc_out=anc, workspace=ws)
        else:
            segkv.append_kv(rk, rv, kn, vn, wl.T - 1, dims)
            segkv.sdpa_decode(out, q, pk, pv, rk, rv, parent, dims, wl.scale,
                              alibi_slopes=slopes, anc_out=anc, workspace=ws)
        torch.cuda.synchronize()
        outs.append(out.cpu().numpy())
    return {
        "out": outs[0], "outs": outs,
        "anc": None if anc is None else anc.cpu().numpy(),
        "resp_k": rk.cpu().numpy(), "resp_v": rv.cpu().numpy(),
        "workspace_bytes": nbytes,
    }


def error_metrics(gpu_out, ref):
    g = gpu_out.astype(np.float64)
    diff = g - ref
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    rel_l2 = float(np.linalg.norm(diff.ravel()) / max(np.linalg.norm(ref.ravel()), 1e-300))
    return max_abs, rel_l2


def assert_parity(gpu_out, ref, what=""):
    assert np.all(np.isfinite(gpu_out.astype(np.float32))), f"{what}: non-finite output"
    max_abs, rel_l2 = error_metrics(gpu_out, ref)
    assert max_abs <= MAX_ABS_TOL, f"{what}: max abs err {max_abs:.3e} > {MAX_ABS_TOL}"
    assert rel_l2 <= REL_L2_TOL, f"{what}: rel L2 err {rel_l2:.3e} > {REL_L2_TOL}"
    return max_abs, rel_l2


def same_bits(a, b):
    """Bit-for-bit equality of fp16 arrays (NaN patterns included)."""
    return np.array_equal(a.view(np.uint16), b.view(np.uint16))
