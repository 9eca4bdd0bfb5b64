"""Pins for the oracle's gradients of the hybrid attention (training algorithm of the supplement): central
differences of the pinned forward oracle, a library autograd in the dense case, closed-form sums.  CPU only."""
import numpy as np
import pytest
import torch

import oracle as orc


def _rng(seed):
    return np.random.default_rng(seed)


def _away_from_zero(x, margin=0.05):
    return np.where(np.abs(x) < margin, np.sign(x + 1e-30) * margin, x)


def _loss(fwd, G):
    return float((fwd * G).sum())


def _central(f, X, h=1e-6):
    """d f / d X by central differences, element by element."""
    g = np.zeros_like(X)
    for idx in np.ndindex(*X.shape):
        old = X[idx]
        X[idx] = old + h
        up = f()
        X[idx] = old - h
        dn = f()
        X[idx] = old
        g[idx] = (up - dn) / (2 * h)
    return g


@pytest.mark.parametrize("n_q,n_kv,b_q,b_kv,k", [(6, 10, 2, 3, 2), (5, 7, 4, 2, 3), (4, 8, 4, 4, 2)])
def test_sparse_attention_gradients_against_central_differences(n_q, n_kv, b_q, b_kv, k):
    r = _rng(n_q * 100 + n_kv)
    d = 4
    Q, K, V, G = r.normal(size=(n_q, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_q, d))
    idx, _ = orc.select_blocks(orc.block_scores(Q, K, b_q, b_kv), k)      # held fixed: the mask is piecewise constant
    dQ, dK, dV = orc.sparse_attention_bwd(Q, K, V, idx, b_q, b_kv, G, scale=0.7)
    f = lambda: _loss(orc.sparse_attention(Q, K, V, idx, b_q, b_kv, scale=0.7), G)
    np.testing.assert_allclose(dQ, _central(f, Q), atol=2e-8)
    np.testing.assert_allclose(dK, _central(f, K), atol=2e-8)
    np.testing.assert_allclose(dV, _central(f, V), atol=2e-8)
    # the gradients are not interchangeable: a swapped or transposed operand would show
    assert np.abs(dK - dV).max() > 1e-3


def test_dense_case_against_library_autograd():
    r = _rng(7)
    n_q, n_kv, d = 9, 14, 8
    Q, K, V, G = r.normal(size=(n_q, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_q, d))
    all_blocks = np.tile(np.arange(4), (3, 1))                              # b_q = 3, b_kv = 4 (ragged last block)
    dQ, dK, dV = orc.sparse_attention_bwd(Q, K, V, all_blocks, 3, 4, G)
    q, kk, v = (torch.tensor(x, dtype=torch.float64, requires_grad=True) for x in (Q, K, V))
    out = torch.softmax(q @ kk.T / d ** 0.5, dim=-1) @ v
    out.backward(torch.tensor(G))
    np.testing.assert_allclose(dQ, q.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dK, kk.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dV, v.grad.numpy(), atol=1e-13)


def test_closed_form_sums_and_unselected_blocks():
    r = _rng(9)
    n_q, n_kv, d, b = 8, 12, 4, 2
    Q, K, V, G = r.normal(size=(n_q, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_q, d))
    idx = np.array([[0, 1], [0, 1], [2, 5], [2, 5]])                        # blocks 3 and 4 are never selected
    dQ, dK, dV = orc.sparse_attention_bwd(Q, K, V, idx, b, b, G)
    # every softmax row sums to one: shifting all values by a constant shifts every output by it
    np.testing.assert_allclose(dV.sum(axis=0), G.sum(axis=0), atol=1e-13)
    # shifting every key by the same vector changes no softmax row: the key gradients of a block row's set cancel
    np.testing.assert_allclose(dK.sum(axis=0), 0.0, atol=1e-13)
    assert np.all(dK[6:10] == 0.0) and np.all(dV[6:10] == 0.0)
    assert np.abs(dK[:6]).min() > 0.0


@pytest.mark.parametrize("kind,rope,use_w", [(orc.PHI_RELU, False, False), (orc.PHI_RELU, True, True),
                                             (orc.PHI_ELU1, True, False), (orc.PHI_ELU1, False, True)])
def test_history_gradient_against_central_differences(kind, rope, use_w):
    r = _rng(11 + kind)
    n, d = 5, 6
    Q = _away_from_zero(r.normal(size=(n, d)))                               # away from the kink of ReLU
    L, z = orc.state_absorb(*orc.state_zero(d), r.normal(size=(9, d)), r.normal(size=(9, d)), kind)
    G = r.normal(size=(n, d))
    ang = r.uniform(-2, 2, size=(n, d // 2))
    cos, sin = (np.cos(ang), np.sin(ang)) if rope else (None, None)
    W = r.normal(size=(d, d)) if use_w else None
    dQ = orc.history_readout_bwd(Q, L, z, G, kind, cos, sin, 1e-3, 0.5, W)
    f = lambda: _loss(orc.history_readout(Q, L, z, kind, cos, sin, 1e-3, 0.5, W), G)
    np.testing.assert_allclose(dQ, _central(f, Q), atol=5e-8)
    if kind == orc.PHI_RELU:
        assert np.all(dQ[Q < 0] == 0.0)                                      # nothing flows through a clamped feature


def test_whole_path_gradient_is_the_sum_of_the_branches_and_splits_by_query_tensor():
    r = _rng(13)
    n_q, n_kv, d, b, k = 6, 12, 4, 3, 2
    Q = _away_from_zero(r.normal(size=(n_q, d)))
    Qh = _away_from_zero(r.normal(size=(n_q, d)))
    K, V, G = r.normal(size=(n_kv, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_q, d))
    st = orc.state_absorb(*orc.state_zero(d), r.normal(size=(7, d)), r.normal(size=(7, d)))
    idx, _ = orc.select_blocks(orc.block_scores(Q, K, b, b), k)
    # one tensor feeding both branches
    dQl, dQh, dK, dV = orc.hybrid_attention_bwd(Q, K, V, st, b, b, idx, G)
    f = lambda: _loss(orc.hybrid_attention(Q, K, V, st, b, b, k, block_idx=idx)[0], G)
    np.testing.assert_allclose(dQl + dQh, _central(f, Q), atol=5e-8)
    np.testing.assert_allclose(dK, _central(f, K), atol=5e-8)
    np.testing.assert_allclose(dV, _central(f, V), atol=5e-8)
    # split queries: each gradient belongs to its own tensor
    dQl2, dQh2, _, _ = orc.hybrid_attention_bwd(Q, K, V, st, b, b, idx, G, Q_hist=Qh)
    f2 = lambda: _loss(orc.hybrid_attention(Q, K, V, st, b, b, k, block_idx=idx, Q_hist=Qh)[0], G)
    np.testing.assert_allclose(dQl2, _central(f2, Q), atol=5e-8)
    np.testing.assert_allclose(dQh2, _central(f2, Qh), atol=5e-8)
    # no state: the history branch contributes nothing
    assert np.all(orc.hybrid_attention_bwd(Q, K, V, None, b, b, idx, G)[1] == 0.0)
