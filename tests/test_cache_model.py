"""Segment-cache bookkeeping (Section 3.2, Eq. 1-3): oracle pinned by the paper's
printed numbers, library checked against the oracle; growth copy on the GPU."""
import os

import numpy as np
import pytest

import paper_2401_05391_amd as segkv
from oracle import cache_model


def _golden(golden_dir):
    kv = {}
    with open(os.path.join(golden_dir, "kv_cache_memory_worked_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, v = [t.strip() for t in line.split("=")]
                kv[k] = int(v) if v.lstrip("-").isdigit() else v
    return kv


def test_oracle_reproduces_the_papers_worked_numbers(golden_dir):
    g = _golden(golden_dir)
    tok = cache_model.cache_token(g["L"], g["H"], g["D"], g["sizeof_datatype"])
    assert tok == 512 * 1024                       # 0.5 MiB per token for this row of Table 1
    std = cache_model.cache_standard(g["BS"], g["BW"], g["N_prompt"], g["N_response"], tok)
    seg = cache_model.cache_segment(g["BS"], g["BW"], g["N_prompt"], g["N_response"], tok, g["step"])
    assert round(std / 1e9) == g["standard_GB"]
    assert round(seg / 1e9) == g["segment_GB"]
    assert round((std - seg) / 1e9) - g["saved_GB"] in (0, 1)   # 51.5 GB: printed as 51
    assert abs(100.0 * seg / std - g["segment_over_standard_percent"]) <= 0.5
    assert std == 128 * 2 ** 30 and seg == 80 * 2 ** 30


def test_capacity_grows_in_steps_of_sixteen():
    # Section 3.2: 16 rows at the 1st step, 32 at the 17th
    assert [cache_model.capacity(n) for n in (1, 16, 17, 32, 33, 128)] == [16, 16, 32, 32, 48, 128]
    assert cache_model.capacity(0) == 0


def test_library_matches_the_oracle():
    rng = np.random.default_rng(0)
    assert segkv.cache_token_bytes(32, 32, 128, 2) == cache_model.cache_token(32, 32, 128, 2)
    for _ in range(200):
        L, H, D = (int(x) for x in rng.integers(1, 200, 3))
        BS, BW = int(rng.integers(1, 300)), int(rng.integers(1, 9))
        npmt, nres = int(rng.integers(0, 5000)), int(rng.integers(0, 5000))
        tok = cache_model.cache_token(L, H, D, 2)
        assert segkv.cache_token_bytes(L, H, D, 2) == tok
        assert segkv.response_capacity(nres) == cache_model.capacity(nres)
        assert segkv.cache_standard_bytes(BS, BW, npmt, nres, tok) == \
            cache_model.cache_standard(BS, BW, npmt, nres, tok)
        assert segkv.cache_segment_bytes(BS, BW, npmt, nres, tok) == \
            cache_model.cache_segment(BS, BW, npmt, nres, tok)
    assert segkv.cache_token_bytes(0, 1, 1, 2) == 0
    assert segkv.response_capacity(-3) == 0


def test_growth_rule_keeps_exactly_the_valid_rows_hand_case():
    # Section 3.2: a longer buffer is allocated and the old rows are copied over.  Hand
    # case, written out: 3 valid rows of a 4-row buffer moved into 6 rows filled with -1.
    old = np.array([[10, 11], [20, 21], [30, 31], [99, 99]], dtype=np.int32)      # row 3 is not valid
    got = cache_model.grow(old, 3, 6, -1)
    want = [[10, 11], [20, 21], [30, 31], [-1, -1], [-1, -1], [-1, -1]]
    assert got.tolist() == want                       # row T itself is `fill`, not the stale row
    assert got.dtype == old.dtype and got.shape == (6, 2)
    assert old.tolist() == [[10, 11], [20, 21], [30, 31], [99, 99]]               # the old buffer is untouched
    # T = 0 copies nothing; T = capacity copies everything
    assert cache_model.grow(old, 0, 5, 7).tolist() == [[7, 7]] * 5
    assert cache_model.grow(old, 4, 5, 7).tolist() == old.tolist() + [[7, 7]]
    # higher-rank rows keep their shape, and fp16 NaN fill survives
    k = np.arange(2 * 3 * 2, dtype=np.float16).reshape(2, 3, 2)
    g = cache_model.grow(k, 1, 3, np.float16(np.nan))
    assert g.shape == (3, 3, 2) and np.array_equal(g[0], k[0]) and np.isnan(g[1:]).all()


def test_segment_never_exceeds_standard_by_more_than_the_growth_slack():
    tok = cache_model.cache_token(40, 40, 128, 2)
    for nres in range(1, 70):
        std = cache_model.cache_standard(4, 4, 1024, nres, tok)
        seg = cache_model.cache_segment(4, 4, 1024, nres, tok)
        # shared prompt saves (BW-1)*N_prompt rows; growth wastes < 16 rows per beam
        assert seg <= std - 4 * (3 * 1024 - 4 * 15) * tok


@pytest.mark.gpu
@pytest.mark.parametrize("T", [0, 1, 16, 23])
def test_grow_response_copies_exactly_the_valid_rows(T):
    import torch
    print(f"\n[case] grow_response T={T}", flush=True)
    rng = np.random.default_rng(T)
    B, W, Hkv, D, tcap_old, tcap_new = 3, 4, 2, 64, 32, 48
    old_k = rng.standard_normal((tcap_old, B * W, Hkv, D)).astype(np.float16)
    old_v = rng.standard_normal((tcap_old, B * W, Hkv, D)).astype(np.float16)
    poison = np.float16(np.nan)
    dev = torch.device("cuda:0")
    nk = torch.full((tcap_new, B * W, Hkv, D), float("nan"), dtype=torch.float16, device=dev)
    nv = torch.full((tcap_new, B * W, Hkv, D), float("nan"), dtype=torch.float16, device=dev)
    dims = segkv.make_dims(B, W, Hkv, Hkv, D, 0, T, tcap_old)
    segkv.grow_response(nk, nv, torch.from_numpy(old_k).to(dev), torch.from_numpy(old_v).to(dev), dims)
    torch.cuda.synchronize()
    want_k = cache_model.grow(old_k, T, tcap_new, poison)
    want_v = cache_model.grow(old_v, T, tcap_new, poison)
    assert np.array_equal(nk.cpu().numpy().view(np.uint16), want_k.view(np.uint16))
    assert np.array_equal(nv.cpu().numpy().view(np.uint16), want_v.view(np.uint16))


@pytest.mark.gpu
def test_decode_across_a_growth_boundary_matches_the_oracle():
    # step 17 of a response: the 16-row buffers are full, grow to 32, then decode
    import torch
    from paper_2401_05391_amd.workloads import Workload, make_inputs
    from segkv_testlib import assert_parity, oracle_reference
    print("\n[case] decode across growth boundary", flush=True)
    wl = Workload("grow17", B=2, W=4, Hq=4, Hkv=2, D=128, Lp=40, T=17, seed=77)
    x = make_inputs(wl)                       # Tcap = 32 buffers; rows 0..15 hold the past
    ref_out, ref_anc, ref_rk, ref_rv = oracle_reference(wl, x)
    dev = torch.device("cuda:0")
    old_k = torch.from_numpy(np.ascontiguousarray(x["resp_k"][:16])).to(dev)
    old_v = torch.from_numpy(np.ascontiguousarray(x["resp_v"][:16])).to(dev)
    cap = segkv.response_capacity(wl.T)
    assert cap == 32
    new_k = torch.full((cap, wl.N, wl.Hkv, wl.D), float("nan"), dtype=torch.float16, device=dev)
    new_v = torch.full((cap, wl.N, wl.Hkv, wl.D), float("nan"), dtype=torch.float16, device=dev)
    segkv.grow_response(new_k, new_v, old_k, old_v, segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, 0, 16, 16))
    up = lambda a: torch.from_numpy(a).to(dev)
    out = torch.empty((wl.N, wl.Hq, wl.D), dtype=torch.float16, device=dev)
    dims = segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, wl.Lp, wl.T, cap)
    nb = segkv.workspace_bytes(dims)
    ws = torch.empty(max(nb, 16) // 4, dtype=torch.float32, device=dev) if nb else None
    segkv.sdpa_decode(out, up(x["q"]), up(x["prompt_k"]), up(x["prompt_v"]), new_k, new_v,
                      up(x["parent"]), dims, wl.scale, k_new=up(x["k_new"]), v_new=up(x["v_new"]),
                      workspace=ws)
    torch.cuda.synchronize()
    assert_parity(out.cpu().numpy(), ref_out, "grow17")
    assert np.array_equal(new_k.cpu().numpy().view(np.uint16), ref_rk.view(np.uint16))
    assert np.array_equal(new_v.cpu().numpy().view(np.uint16), ref_rv.view(np.uint16))
