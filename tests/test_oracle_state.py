"""Pins for the oracle's linear state (Eq. 2) and RoPE helper.  CPU only."""
import math

import numpy as np
import pytest

import oracle as orc


def _rng(seed):
    return np.random.default_rng(seed)


def _scalar_phi(x, kind):
    if kind == orc.PHI_RELU:
        return x if x > 0.0 else 0.0
    return x + 1.0 if x > 0.0 else math.exp(x)


@pytest.mark.parametrize("kind", [orc.PHI_RELU, orc.PHI_ELU1])
def test_state_equals_scalar_triple_loop(kind):
    # Eq. 2 written as scalar loops: L[i][j] += phi(k_t)[i] * v_t[j]; z[i] += phi(k_t)[i]
    r = _rng(1)
    n, d = 7, 4
    K = r.normal(size=(n, d))
    V = r.normal(size=(n, d))
    L = [[0.0] * d for _ in range(d)]
    z = [0.0] * d
    for t in range(n):
        for i in range(d):
            f = _scalar_phi(K[t, i], kind)
            z[i] += f
            for j in range(d):
                L[i][j] += f * V[t, j]
    L0, z0 = orc.state_zero(d)
    L1, z1 = orc.state_absorb(L0, z0, K, V, kind)
    np.testing.assert_allclose(L1, np.array(L), rtol=0, atol=1e-13)
    np.testing.assert_allclose(z1, np.array(z), rtol=0, atol=1e-13)
    # the state is not symmetric: a transposed operand would show
    assert np.abs(L1 - L1.T).max() > 1e-3


def test_state_with_rope_equals_scalar_loop():
    r = _rng(2)
    n, d = 5, 6
    K = r.normal(size=(n, d))
    V = r.normal(size=(n, d))
    ang = r.uniform(-3, 3, size=(n, d // 2))
    L = np.zeros((d, d))
    z = np.zeros(d)
    for t in range(n):
        f = [max(K[t, i], 0.0) for i in range(d)]
        rot = [0.0] * d
        for p in range(d // 2):
            c, s = math.cos(ang[t, p]), math.sin(ang[t, p])
            rot[2 * p] = f[2 * p] * c - f[2 * p + 1] * s
            rot[2 * p + 1] = f[2 * p] * s + f[2 * p + 1] * c
        for i in range(d):
            z[i] += f[i]  # the normaliser is never rotated
            for j in range(d):
                L[i, j] += rot[i] * V[t, j]
    L1, z1 = orc.state_absorb(*orc.state_zero(d), K, V, orc.PHI_RELU, np.cos(ang), np.sin(ang))
    np.testing.assert_allclose(L1, L, atol=1e-13)
    np.testing.assert_allclose(z1, z, atol=1e-13)


def test_state_one_hot_keys_closed_form():
    # keys that are positive one-hot vectors route each value row into one row of L;
    # negative entries are removed by ReLU.
    d = 5
    slots = [0, 3, 3, 1, 0, 3]
    K = -np.ones((len(slots), d))
    for t, a in enumerate(slots):
        K[t, a] = 2.0
    V = np.arange(len(slots) * d, dtype=float).reshape(len(slots), d)
    L, z = orc.state_absorb(*orc.state_zero(d), K, V)
    for a in range(d):
        rows = [t for t, s in enumerate(slots) if s == a]
        np.testing.assert_allclose(L[a], 2.0 * V[rows].sum(axis=0) if rows else np.zeros(d))
        assert z[a] == 2.0 * len(rows)


def test_state_chunked_oneshot_permuted_agree():
    r = _rng(3)
    n, d = 300, 16
    K = r.normal(size=(n, d))
    V = r.normal(size=(n, d))
    one = orc.state_absorb(*orc.state_zero(d), K, V)
    for chunk in (1, 64, 77):
        L, z = orc.state_zero(d)
        for s in range(0, n, chunk):
            L, z = orc.state_absorb(L, z, K[s:s + chunk], V[s:s + chunk])
        np.testing.assert_allclose(L, one[0], rtol=0, atol=1e-11)
        np.testing.assert_allclose(z, one[1], rtol=0, atol=1e-11)
    perm = r.permutation(n)
    Lp, zp = orc.state_absorb(*orc.state_zero(d), K[perm], V[perm])
    np.testing.assert_allclose(Lp, one[0], rtol=0, atol=1e-11)
    np.testing.assert_allclose(zp, one[1], rtol=0, atol=1e-11)


def test_absorb_does_not_modify_inputs_and_accumulates():
    r = _rng(4)
    d = 8
    K = r.normal(size=(10, d))
    V = r.normal(size=(10, d))
    L0 = r.normal(size=(d, d))
    z0 = r.normal(size=d)
    L0c, z0c = L0.copy(), z0.copy()
    L1, z1 = orc.state_absorb(L0, z0, K, V)
    assert np.array_equal(L0, L0c) and np.array_equal(z0, z0c)
    La, za = orc.state_absorb(*orc.state_zero(d), K, V)
    np.testing.assert_allclose(L1 - L0, La, atol=1e-12)
    np.testing.assert_allclose(z1 - z0, za, atol=1e-12)


def test_phi_special_values():
    x = np.array([-1e9, -1.0, 0.0, 1.0, 3.5])
    np.testing.assert_array_equal(orc.phi(x, orc.PHI_RELU), [0, 0, 0, 1.0, 3.5])
    e = orc.phi(x, orc.PHI_ELU1)
    np.testing.assert_allclose(e, [0.0, math.exp(-1.0), 1.0, 2.0, 4.5], atol=1e-15)
    assert (e >= 0).all()


def test_rope_quarter_turn_and_norm():
    x = np.array([[1.0, 2.0, -3.0, 0.5]])
    quarter = np.full((1, 2), math.pi / 2)
    y = orc.rope_rotate(x, np.cos(quarter), np.sin(quarter))
    np.testing.assert_allclose(y, [[-2.0, 1.0, -0.5, -3.0]], atol=1e-15)
    r = _rng(5)
    X = r.normal(size=(9, 8))
    ang = r.uniform(-4, 4, size=(9, 4))
    Y = orc.rope_rotate(X, np.cos(ang), np.sin(ang))
    np.testing.assert_allclose((Y ** 2).sum(1), (X ** 2).sum(1), rtol=1e-13)
    # pair norms too (rotation acts on adjacent pairs only)
    np.testing.assert_allclose(Y[:, 0::2] ** 2 + Y[:, 1::2] ** 2, X[:, 0::2] ** 2 + X[:, 1::2] ** 2, rtol=1e-12)


def test_rope_zero_angle_is_identity_and_none():
    r = _rng(6)
    X = r.normal(size=(4, 6))
    zero = np.zeros((4, 3))
    np.testing.assert_array_equal(orc.rope_rotate(X, np.cos(zero), np.sin(zero)), X)
    np.testing.assert_array_equal(orc.rope_rotate(X), X)


def test_rope_relative_shift_property():
    # <R_a x, R_b y> depends on a - b only: shifting query and key positions together
    # leaves every numerator weight of the linear attention unchanged.
    r = _rng(7)
    d = 8
    freq = 10000.0 ** (-2.0 * np.arange(d // 2) / d)
    x = np.abs(r.normal(size=(1, d)))
    y = np.abs(r.normal(size=(1, d)))

    def dot(pa, pb):
        a = np.array([[pa]]) * freq[None]
        b = np.array([[pb]]) * freq[None]
        return (orc.rope_rotate(x, np.cos(a), np.sin(a)) @ orc.rope_rotate(y, np.cos(b), np.sin(b)).T).item()

    assert abs(dot(5.0, 2.0) - dot(105.0, 102.0)) < 1e-11
    assert abs(dot(5.0, 2.0) - dot(3.0, 0.0)) < 1e-11
    assert abs(dot(5.0, 2.0) - dot(2.0, 5.0)) > 1e-3  # and it is not symmetric in the offset
