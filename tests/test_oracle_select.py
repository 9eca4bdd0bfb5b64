"""Pins for block scoring (Eq. 4) and top-K selection.  CPU only."""
import math

import numpy as np
import pytest

import oracle as orc
import workloads as wl


def test_select_k_for_the_named_configs():
    assert orc.select_k(0.25, 16) == 4          # "top-4 of 16" in the tiny case
    assert orc.select_k(0.25, 147) == 37        # ceil(36.75)
    assert [orc.select_k(r, 169) for r in (0.125, 0.25, 0.5, 1.0)] == [22, 43, 85, 169]
    assert orc.select_k(1e-9, 10) == 1          # never below one block
    assert orc.select_k(1.0, 7) == 7
    assert orc.select_k(0.5, 8) == 4            # exact products do not round up


def test_pool_blocks_ragged_tail_uses_true_length():
    X = np.arange(72 * 2, dtype=float).reshape(72, 2)
    P = orc.pool_blocks(X, 16)
    assert P.shape == (5, 2)
    for i in range(4):
        np.testing.assert_allclose(P[i], X[16 * i:16 * i + 16].mean(0))
    np.testing.assert_allclose(P[4], X[64:72].mean(0))  # eight real rows, not sixteen


def test_scores_and_selection_brute_force_tiny():
    w = wl.get("tiny_f32")
    Q, K, _ = wl.make_qkv(w)
    b, k = w.block, orc.select_k(w.keep_ratio, w.t_n)
    assert k == 4
    for h in range(w.heads):
        q = wl.to_f64(Q[0, h])
        kk = wl.to_f64(K[0, h])
        t_m, t_n, d = w.t_m, w.t_n, w.head_dim
        A = [[0.0] * t_n for _ in range(t_m)]
        for i in range(t_m):
            qm = [sum(q[i * b + r, c] for r in range(b)) / b for c in range(d)]
            for j in range(t_n):
                km = [sum(kk[j * b + r, c] for r in range(b)) / b for c in range(d)]
                A[i][j] = sum(qm[c] * km[c] for c in range(d))
        A = np.array(A)
        np.testing.assert_allclose(orc.block_scores(q, kk, b, b), A, atol=1e-13)
        idx, gap = orc.select_blocks(orc.block_scores(q, kk, b, b), k)
        assert idx.shape == (t_m, k)
        for i in range(t_m):
            full = np.argsort(-A[i], kind="stable")
            assert sorted(full[:k].tolist()) == idx[i].tolist()
            assert list(idx[i]) == sorted(set(idx[i]))            # ascending, distinct
            assert 0 <= idx[i][0] and idx[i][-1] < t_n
            srt = np.sort(A[i])[::-1]
            assert gap[i] == pytest.approx(srt[k - 1] - srt[k], abs=1e-15)
            # the algorithm listing selects on Softmax(pool(Q) pool(K)^T / sqrt(d)): same set
            s = A[i] / math.sqrt(d)
            p = np.exp(s - s.max())
            p /= p.sum()
            assert sorted(np.argsort(-p, kind="stable")[:k].tolist()) == idx[i].tolist()


def test_selection_ties_go_to_lower_index_and_gap():
    A = np.array([[1.0, 3.0, 3.0, 0.5, 3.0, 2.0],
                  [0.0, 0.0, 0.0, 0.0, 0.0, 0.0],
                  [5.0, 4.0, 3.0, 2.0, 1.0, 0.0]])
    idx, gap = orc.select_blocks(A, 2)
    assert idx.tolist() == [[1, 2], [0, 1], [0, 1]]
    assert gap.tolist() == [0.0, 0.0, 1.0]
    idx, gap = orc.select_blocks(A, 6)
    assert idx.tolist() == [list(range(6))] * 3
    assert np.isinf(gap).all()
    idx, _ = orc.select_blocks(A, 4)
    assert idx[0].tolist() == [1, 2, 4, 5]


def test_selection_picks_the_planted_blocks():
    # plant key blocks aligned with each query block's mean: they must be the ones kept
    r = np.random.default_rng(11)
    b, d, t_m, t_n, k = 4, 16, 3, 10, 2
    Q = r.normal(size=(t_m * b, d)) * 0.01
    K = r.normal(size=(t_n * b, d)) * 0.01
    planted = {0: (7, 2), 1: (0, 9), 2: (5, 4)}
    for i, js in planted.items():
        u = r.normal(size=d)
        Q[i * b:(i + 1) * b] += u
        for j in js:
            K[j * b:(j + 1) * b] += u
    idx, gap = orc.select_blocks(orc.block_scores(Q, K, b, b), k)
    for i, js in planted.items():
        assert idx[i].tolist() == sorted(js)
    assert (gap > 1.0).all()


def test_rectangular_blocks():
    r = np.random.default_rng(12)
    Q = r.normal(size=(20, 8))
    K = r.normal(size=(50, 8))
    A = orc.block_scores(Q, K, 8, 16)
    assert A.shape == (3, 4)
    np.testing.assert_allclose(A[2, 3], Q[16:20].mean(0) @ K[48:50].mean(0), atol=1e-14)
