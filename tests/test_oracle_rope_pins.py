"""Pins for the RoPE + append oracle (CPU only).  The paper names the operation
but prints no formula, so the pins are the mathematics of the published
definition: complex multiplication, isometry, the relative-position property,
and a hand-computed value."""
import numpy as np
import pytest

from oracle import rope


def _draw(rows, H, D, seed):
    return np.random.default_rng(seed).standard_normal((rows, H, D)).astype(np.float16)


@pytest.mark.parametrize("interleaved", [False, True])
@pytest.mark.parametrize("D,R", [(8, 8), (16, 8), (64, 64), (256, 64)])
def test_equals_complex_multiplication(D, R, interleaved):
    # a pair (a, b) is the complex number a + ib multiplied by exp(i pos theta)
    x = _draw(5, 3, D, 1)
    pos = np.array([0, 1, 7, 1030, 4095])
    got = rope.rotate(x, pos, 10000.0, R, interleaved)
    ia, ib = rope.pair_indices(R, interleaved)
    z = x.astype(np.float64)[..., ia] + 1j * x.astype(np.float64)[..., ib]
    theta = 10000.0 ** (-2.0 * np.arange(R // 2) / R)
    z = z * np.exp(1j * pos.reshape(-1, 1, 1) * theta)
    want = x.astype(np.float64)
    want[..., ia] = z.real
    want[..., ib] = z.imag
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    if R < D:
        assert np.array_equal(got[..., R:], x.astype(np.float64)[..., R:])


def test_hand_value():
    # D = R = 2: theta_0 = 1, so position 1 turns (1, 0) by one radian
    x = np.array([[[1.0, 0.0]]])
    got = rope.rotate(x, np.array([1]), 10000.0, 2, False)
    np.testing.assert_allclose(got[0, 0], [0.5403023058681398, 0.8414709848078965], atol=1e-15)
    # position 0 is the identity
    x2 = rope.rotate(np.array([[[3.0, 4.0]]]), np.array([0]), 10000.0, 2, False)
    assert np.array_equal(x2[0, 0], [3.0, 4.0])
    # D = R = 4, second pair: theta_1 = base^(-1/2) = 1/100, position 50 -> half a radian
    got = rope.rotate(np.array([[[0.0, 2.0, 0.0, 0.0]]]), np.array([50]), 10000.0, 4, False)
    np.testing.assert_allclose(got[0, 0], [0.0, 2 * 0.8775825618903728, 0.0, 2 * 0.479425538604203],
                               atol=1e-15)


@pytest.mark.parametrize("interleaved", [False, True])
def test_isometry_and_relative_position(interleaved):
    q, k = _draw(4, 2, 32, 2), _draw(4, 2, 32, 3)
    m, n = np.array([5, 100, 2047, 12]), np.array([3, 40, 1000, 12])
    qm = rope.rotate(q, m, 10000.0, 32, interleaved)
    kn = rope.rotate(k, n, 10000.0, 32, interleaved)
    # each pair keeps its length
    ia, ib = rope.pair_indices(32, interleaved)
    np.testing.assert_allclose(qm[..., ia] ** 2 + qm[..., ib] ** 2,
                               q.astype(np.float64)[..., ia] ** 2 + q.astype(np.float64)[..., ib] ** 2,
                               rtol=1e-12)
    # <R_m q, R_n k> depends on m - n only
    lhs = np.einsum("rhd,rhd->rh", qm, kn)
    rhs = np.einsum("rhd,rhd->rh", rope.rotate(q, m - n, 10000.0, 32, interleaved), k.astype(np.float64))
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-10)


def test_interleaved_is_the_half_convention_on_permuted_coordinates():
    x = _draw(3, 2, 16, 4)
    pos = np.array([9, 300, 77])
    perm = np.concatenate([np.arange(0, 16, 2), np.arange(1, 16, 2)])   # pairs (2i,2i+1) -> (i,i+8)
    a = rope.rotate(x, pos, 10000.0, 16, True)[..., perm]
    b = rope.rotate(x[..., perm], pos, 10000.0, 16, False)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)


def test_rope_append_writes_only_row_t():
    B, W, Hq, Hkv, D, Lp, t, Tcap = 2, 3, 4, 2, 16, 11, 5, 16
    N = B * W
    q, k, v = _draw(N, Hq, D, 5), _draw(N, Hkv, D, 6), _draw(N, Hkv, D, 7)
    rk = np.full((Tcap, N, Hkv, D), np.float16(np.nan))
    rv = np.full((Tcap, N, Hkv, D), np.float16(np.nan))
    q_rot = rope.rope_append(q, k, v, rk, rv, t, W, Lp, 10000.0, D, False)
    pos = np.full(N, Lp + t)
    np.testing.assert_allclose(q_rot, rope.rotate(q, pos, 10000.0, D, False), atol=0)
    assert np.array_equal(rk[t], rope.rotate(k, pos, 10000.0, D, False).astype(np.float16))
    assert np.array_equal(rv[t].view(np.uint16), v.view(np.uint16))
    mask = np.ones(Tcap, bool)
    mask[t] = False
    assert np.isnan(rk[mask].astype(np.float32)).all() and np.isnan(rv[mask].astype(np.float32)).all()
    # per-request positions
    q2 = rope.rope_append(q, k, v, rk, rv, t, W, Lp, 10000.0, D, False, positions=np.array([3, 40]))
    np.testing.assert_allclose(q2, rope.rotate(q, np.repeat([3, 40], W), 10000.0, D, False), atol=0)
