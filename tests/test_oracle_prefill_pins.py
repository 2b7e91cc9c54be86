"""Pins for the prefill oracle (CPU only): library causal attention, the decode
oracle (prefill is the special case without a response history), closed forms."""
import numpy as np
import pytest

from oracle import segkv_oracle as oracle
from paper_2401_05391_amd.workloads import alibi_slopes


def _draw(B, N0, Hq, Hkv, D, seed):
    rng = np.random.default_rng(seed)
    f = lambda *s: rng.standard_normal(s).astype(np.float16)
    return f(B, N0, Hq, D), f(B, N0, Hkv, D), f(B, N0, Hkv, D)


@pytest.mark.parametrize("B,N0,Hq,Hkv,D", [(2, 9, 4, 4, 8), (1, 33, 8, 2, 16), (3, 5, 6, 1, 32)])
def test_matches_library_causal_attention(B, N0, Hq, Hkv, D):
    torch = pytest.importorskip("torch")
    q, k, v = _draw(B, N0, Hq, Hkv, D, 1)
    scale = 0.37
    out = oracle.sdpa_prefill(q, k, v, scale)
    g = Hq // Hkv
    t = lambda a, rep: torch.from_numpy(a.astype(np.float64)).permute(0, 2, 1, 3).repeat_interleave(rep, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(t(q, 1), t(k, g), t(v, g), is_causal=True,
                                                           scale=scale)
    np.testing.assert_allclose(out, ref.permute(0, 2, 1, 3).numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("use_alibi", [False, True])
def test_every_token_equals_a_decode_step_over_its_prefix(use_alibi):
    # token i of the prefill == decode with prompt = keys 0..i-1 and a one-row
    # response holding key i (beam 1): the "special case" relation of Section 3.3
    B, N0, Hq, Hkv, D = 2, 7, 4, 2, 8
    q, k, v = _draw(B, N0, Hq, Hkv, D, 2)
    slopes = alibi_slopes(Hq) if use_alibi else None
    scale = 1.0 / np.sqrt(D)
    out = oracle.sdpa_prefill(q, k, v, scale, slopes=slopes)
    for i in range(N0):
        pk = np.ascontiguousarray(k[:, :i])
        pv = np.ascontiguousarray(v[:, :i])
        rk = np.zeros((16, B, Hkv, D), dtype=np.float16)
        rv = np.zeros((16, B, Hkv, D), dtype=np.float16)
        rk[0], rv[0] = k[:, i], v[:, i]
        dec, _, _ = oracle.sdpa_decode(np.ascontiguousarray(q[:, i]), pk, pv, rk, rv,
                                       np.zeros((1, B), np.int32), 1, 1, scale, slopes=slopes)
        np.testing.assert_allclose(out[:, i], dec, rtol=0, atol=1e-13)


def test_first_token_returns_its_own_value_and_constant_values_stay_constant():
    q, k, v = _draw(2, 6, 4, 2, 8, 3)
    out = oracle.sdpa_prefill(q, k, v, 0.5)
    g = 2
    for hq in range(4):
        assert np.array_equal(out[:, 0, hq], v[:, 0, hq // g].astype(np.float64))
    v1 = np.ones_like(v)
    np.testing.assert_allclose(oracle.sdpa_prefill(q, k, v1, 0.5), 1.0, rtol=0, atol=1e-13)


def test_zero_query_gives_running_mean_and_future_keys_do_not_matter():
    q, k, v = _draw(1, 8, 2, 2, 4, 4)
    q0 = np.zeros_like(q)
    out = oracle.sdpa_prefill(q0, k, v, 1.0)
    for i in range(8):
        np.testing.assert_allclose(out[0, i], v[0, : i + 1].astype(np.float64).mean(axis=0),
                                   rtol=0, atol=1e-13)
    base = oracle.sdpa_prefill(q, k, v, 1.0)
    k2, v2 = k.copy(), v.copy()
    k2[:, 5:] = 60000
    v2[:, 5:] = -60000
    changed = oracle.sdpa_prefill(q, k2, v2, 1.0)
    assert np.array_equal(base[:, :5], changed[:, :5])          # causal: tokens < 5 never see keys >= 5


def test_selected_rows_equal_full_result():
    q, k, v = _draw(2, 10, 4, 2, 8, 5)
    full = oracle.sdpa_prefill(q, k, v, 0.3)
    rows = np.array([[0, 0, 0], [1, 9, 3], [0, 4, 2]], dtype=np.int32)
    part = oracle.sdpa_prefill(q, k, v, 0.3, rows=rows)
    for r, (b, i, h) in enumerate(rows):
        assert np.array_equal(part[r], full[b, i, h])
