"""Pins for the oracle's sparse window attention (Eq. 5), readout (Eq. 3) and sum (Eq. 6)."""
import math

import numpy as np
import pytest
import torch

import oracle as orc


def _rng(seed):
    return np.random.default_rng(seed)


def _sdpa(Q, K, V, mask=None, scale=None):
    q, k, v = (torch.from_numpy(np.ascontiguousarray(x))[None, None] for x in (Q, K, V))
    m = None if mask is None else torch.from_numpy(mask)[None, None]
    return torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=m, scale=scale)[0, 0].numpy()


# ----------------------------------------------------------------------------- Eq. 5
def test_dense_attention_matches_library_sdpa():
    r = _rng(21)
    Q, K, V = r.normal(size=(37, 16)), r.normal(size=(90, 16)), r.normal(size=(90, 16))
    np.testing.assert_allclose(orc.dense_attention(Q, K, V), _sdpa(Q, K, V), atol=1e-12)
    np.testing.assert_allclose(orc.dense_attention(Q, K, V, scale=0.3), _sdpa(Q, K, V, scale=0.3), atol=1e-12)


@pytest.mark.parametrize("n_q,n_kv,b", [(64, 256, 16), (50, 72, 16), (33, 130, 32)])
def test_keep_all_blocks_is_dense_attention(n_q, n_kv, b):
    r = _rng(22)
    d = 32
    Q, K, V = r.normal(size=(n_q, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_kv, d))
    t_m, t_n = -(-n_q // b), -(-n_kv // b)
    idx = np.tile(np.arange(t_n, dtype=np.int32), (t_m, 1))
    O = orc.sparse_attention(Q, K, V, idx, b, b)
    np.testing.assert_allclose(O, orc.dense_attention(Q, K, V), atol=1e-12)
    np.testing.assert_allclose(O, _sdpa(Q, K, V), atol=1e-12)


def test_sparse_attention_matches_library_sdpa_with_token_mask():
    # the block list, expanded by hand to a token-level boolean mask, through a library routine
    r = _rng(23)
    n_q, n_kv, d, b_q, b_kv, k = 44, 100, 16, 8, 16, 3
    Q, K, V = r.normal(size=(n_q, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_kv, d))
    t_m, t_n = -(-n_q // b_q), -(-n_kv // b_kv)
    idx = np.stack([np.sort(r.choice(t_n, size=k, replace=False)) for _ in range(t_m)]).astype(np.int32)
    idx[0] = [0, 3, t_n - 1]  # make sure the short last block is used
    mask = np.zeros((n_q, n_kv), dtype=bool)
    for row in range(n_q):
        for j in idx[row // b_q]:
            mask[row, j * b_kv:(j + 1) * b_kv] = True
    np.testing.assert_allclose(orc.sparse_attention(Q, K, V, idx, b_q, b_kv), _sdpa(Q, K, V, mask), atol=1e-12)


def test_single_key_and_uniform_logit_closed_forms():
    r = _rng(24)
    d = 8
    K, V = r.normal(size=(10, d)), r.normal(size=(10, d))
    Q = r.normal(size=(4, d))
    # blocks of one key: softmax over a single key returns that value row
    idx = np.array([[3], [7], [0], [9]], dtype=np.int32)
    O = orc.sparse_attention(Q, K, V, idx, 1, 1)
    np.testing.assert_allclose(O, V[[3, 7, 0, 9]], atol=1e-14)
    # zero queries: uniform weights -> mean of the selected value rows
    idx = np.array([[1, 4]], dtype=np.int32)
    O = orc.sparse_attention(np.zeros((2, d)), K, V, idx, 2, 2)
    np.testing.assert_allclose(O, np.tile(V[[2, 3, 8, 9]].mean(0), (2, 1)), atol=1e-14)


def test_softmax_invariants():
    r = _rng(25)
    n_q, n_kv, d, b, k = 32, 96, 16, 16, 3
    Q, K, V = r.normal(size=(n_q, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_kv, d))
    idx = np.array([[0, 2, 5], [1, 3, 4]], dtype=np.int32)
    O = orc.sparse_attention(Q, K, V, idx, b, b)
    # rows of P sum to one
    np.testing.assert_allclose(orc.sparse_attention(Q, K, np.ones_like(V), idx, b, b), 1.0, atol=1e-14)
    # adding one vector to every key shifts every logit of a row equally
    u = r.normal(size=d)
    np.testing.assert_allclose(orc.sparse_attention(Q, K + u, V, idx, b, b), O, atol=1e-12)
    # the order of the selected blocks does not matter
    np.testing.assert_allclose(orc.sparse_attention(Q, K, V, idx[:, ::-1], b, b), O, atol=1e-13)
    # but the selection does
    other = np.array([[0, 2, 4], [1, 3, 4]], dtype=np.int32)
    assert np.abs(orc.sparse_attention(Q, K, V, other, b, b)[:16] - O[:16]).max() > 1e-3
    # scale default is 1/sqrt(d)
    np.testing.assert_allclose(orc.sparse_attention(Q, K, V, idx, b, b, scale=1 / math.sqrt(d)), O, atol=1e-14)


def test_blockwise_attention_merges_by_log_sum_exp():
    """Softmax attention over a union of key sets is the mixture of the per-set attentions weighted by each set's
    share of the partition function: O = sum_j w_j O_j, w_j = exp(lse_j) / sum_j' exp(lse_j').  Each O_j and lse_j
    comes from the library's dense attention / logsumexp on ONE block, so the check shares nothing with the
    oracle's gather-and-softmax; large logits make the weights very unequal."""
    import torch
    r = _rng(26)
    n_q, n_kv, d, b = 16, 80, 8, 16
    Q, K, V = 6.0 * r.normal(size=(n_q, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_kv, d))
    idx = np.array([[4, 0, 2]], dtype=np.int32)
    tq = torch.from_numpy(Q)
    outs, lses = [], []
    for j in idx[0]:
        tk, tv = torch.from_numpy(K[j * b:(j + 1) * b]), torch.from_numpy(V[j * b:(j + 1) * b])
        outs.append(torch.nn.functional.scaled_dot_product_attention(tq[None], tk[None], tv[None])[0])
        lses.append(torch.logsumexp(tq @ tk.T / math.sqrt(d), dim=1))
    w = torch.softmax(torch.stack(lses), dim=0)             # [blocks, n_q]
    ref = sum(w[i][:, None] * outs[i] for i in range(len(outs))).numpy()
    assert float(w.min()) < 1e-3 < float(w.max())           # the merge is far from a plain average
    np.testing.assert_allclose(orc.sparse_attention(Q, K, V, idx, 16, b), ref, atol=1e-12)


def test_ragged_tail_equals_hand_masked_padding():
    r = _rng(27)
    n_q, n_kv, d, b = 40, 72, 8, 16   # 72 = 4*16 + 8, 40 = 2*16 + 8
    Q, K, V = r.normal(size=(n_q, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_kv, d))
    idx = np.array([[0, 4], [2, 4], [1, 4]], dtype=np.int32)
    O = orc.sparse_attention(Q, K, V, idx, b, b)
    Kp = np.concatenate([K, 1e3 * np.ones((8, d))])   # padding that would dominate if it leaked
    Vp = np.concatenate([V, 1e3 * np.ones((8, d))])
    for row in range(n_q):
        cols = np.concatenate([np.arange(j * b, (j + 1) * b) for j in idx[row // b]])
        s = Kp[cols] @ Q[row] / math.sqrt(d)
        s[cols >= n_kv] = -np.inf                      # masked by hand
        p = np.exp(s - s.max())
        np.testing.assert_allclose(O[row], (p / p.sum()) @ Vp[cols], atol=1e-12)


# ----------------------------------------------------------------------------- Eq. 3
@pytest.mark.parametrize("kind", [orc.PHI_RELU, orc.PHI_ELU1])
def test_readout_is_the_quadratic_linear_attention(kind):
    # o_hist = sum_t w_t v_t with w_t = R_q(phi q).R_t(phi k_t) / (sum_s phi q . phi k_s + eps)
    r = _rng(31)
    n_q, n_ev, d, eps = 6, 23, 8, 1e-6
    Q, K, V = r.normal(size=(n_q, d)), r.normal(size=(n_ev, d)), r.normal(size=(n_ev, d))
    aq, ak = r.uniform(-3, 3, size=(n_q, d // 2)), r.uniform(-3, 3, size=(n_ev, d // 2))
    L, z = orc.state_absorb(*orc.state_zero(d), K, V, kind, np.cos(ak), np.sin(ak))
    O = orc.history_readout(Q, L, z, kind, np.cos(aq), np.sin(aq), eps)

    def rot(x, a):
        y = x.copy()
        y[0::2] = x[0::2] * np.cos(a) - x[1::2] * np.sin(a)
        y[1::2] = x[0::2] * np.sin(a) + x[1::2] * np.cos(a)
        return y

    f = (lambda x: np.maximum(x, 0)) if kind == orc.PHI_RELU else (lambda x: np.where(x > 0, x + 1, np.exp(x)))
    for i in range(n_q):
        fq = f(Q[i])
        den = sum(fq @ f(K[s]) for s in range(n_ev)) + eps
        o = np.zeros(d)
        for t in range(n_ev):
            o += (rot(fq, aq[i]) @ rot(f(K[t]), ak[t])) / den * V[t]
        np.testing.assert_allclose(O[i], o, atol=1e-12)


def test_readout_invariants_identity_rope():
    r = _rng(32)
    n_q, n_ev, d, eps = 9, 40, 8, 1e-6
    Q, K, V = r.normal(size=(n_q, d)), r.normal(size=(n_ev, d)), r.normal(size=(n_ev, d))
    L, z = orc.state_absorb(*orc.state_zero(d), K, V)
    O = orc.history_readout(Q, L, z, eps=eps)
    den = np.maximum(Q, 0) @ z
    shrink = (den / (den + eps))[:, None]
    # convex combination of value rows (non-negative weights), up to the eps shrink
    lo, hi = V.min(0)[None], V.max(0)[None]
    assert (O >= np.minimum(lo * shrink, lo) - 1e-12).all() and (O <= np.maximum(hi * shrink, hi) + 1e-12).all()
    # constant values come back (times the shrink)
    Lc, zc = orc.state_absorb(*orc.state_zero(d), K, np.full_like(V, 2.5))
    np.testing.assert_allclose(orc.history_readout(Q, Lc, zc, eps=eps), 2.5 * shrink * np.ones((1, d)), atol=1e-12)
    # scaling L and z together changes nothing when eps -> 0
    np.testing.assert_allclose(orc.history_readout(Q, 7 * L, 7 * z, eps=0.0), orc.history_readout(Q, L, z, eps=0.0), rtol=1e-12)
    # z_scale = 1/n is the per-frame-mean reading of the normaliser
    np.testing.assert_allclose(orc.history_readout(Q, L, z, eps=0.0, z_scale=0.25), 4 * orc.history_readout(Q, L, z, eps=0.0), rtol=1e-12)


def test_readout_empty_state_and_dead_queries_give_zero():
    d = 8
    Q = np.random.default_rng(33).normal(size=(5, d))
    np.testing.assert_array_equal(orc.history_readout(Q, *orc.state_zero(d)), np.zeros((5, d)))
    L, z = orc.state_absorb(*orc.state_zero(d), np.abs(Q), Q)
    np.testing.assert_array_equal(orc.history_readout(-np.abs(Q), L, z), np.zeros((5, d)))


def test_linear_map_of_the_history_branch_and_its_fold_into_the_state():
    # Eq. 3 with a per-head d x d Linear (no bias): pinned by the quadratic form with projected values,
    # by the direct-sum state of projected values, and by special matrices
    r = _rng(34)
    n_q, n_ev, d, eps = 7, 19, 8, 1e-6
    Q, K, V = r.normal(size=(n_q, d)), r.normal(size=(n_ev, d)), r.normal(size=(n_ev, d))
    W = r.normal(size=(d, d))
    aq, ak = r.uniform(-3, 3, size=(n_q, d // 2)), r.uniform(-3, 3, size=(n_ev, d // 2))
    L, z = orc.state_absorb(*orc.state_zero(d), K, V, cos=np.cos(ak), sin=np.sin(ak))
    O = orc.history_readout(Q, L, z, cos=np.cos(aq), sin=np.sin(aq), eps=eps, W=W)
    # (a) the map acts on what the branch returns: weights of Eq. 3 times the PROJECTED value rows
    plain = orc.history_readout(Q, L, z, cos=np.cos(aq), sin=np.sin(aq), eps=eps)
    for i in range(n_q):
        np.testing.assert_allclose(O[i], sum(plain[i, j] * W[j] for j in range(d)), atol=1e-12)
    # (b) the same state as absorbing the projected values v_t W by direct sum (Eq. 2)
    Lp, zp = orc.state_absorb(*orc.state_zero(d), K, V @ W, cos=np.cos(ak), sin=np.sin(ak))
    np.testing.assert_allclose(orc.state_fold_linear(L, W), Lp, atol=1e-12)
    np.testing.assert_array_equal(z, zp)
    # (c) folding: the plain readout of the folded state is the mapped readout
    np.testing.assert_allclose(orc.history_readout(Q, orc.state_fold_linear(L, W), z, cos=np.cos(aq), sin=np.sin(aq), eps=eps),
                               O, atol=1e-12)
    # (d) identity, a feature permutation and a diagonal scaling
    np.testing.assert_array_equal(orc.history_readout(Q, L, z, eps=eps, W=np.eye(d)), orc.history_readout(Q, L, z, eps=eps))
    perm = r.permutation(d)
    np.testing.assert_allclose(orc.history_readout(Q, L, z, eps=eps, W=np.eye(d)[:, perm]),
                               orc.history_readout(Q, L, z, eps=eps)[:, perm], atol=1e-15)
    s = r.uniform(0.5, 2.0, size=d)
    np.testing.assert_allclose(orc.history_readout(Q, L, z, eps=eps, W=np.diag(s)),
                               orc.history_readout(Q, L, z, eps=eps) * s[None], rtol=1e-13)
    # (e) a transposed W is a different map (guards the operand order)
    assert not np.allclose(orc.history_readout(Q, L, z, eps=eps, W=W.T), O)
    # (f) the whole path: only the history term is mapped
    Kw, Vw = r.normal(size=(64, d)), r.normal(size=(64, d))
    Qw = r.normal(size=(16, d))
    Ow, Ol, Oh, _, _ = orc.hybrid_attention(Qw, Kw, Vw, (L, z), 16, 16, 2, W=W)
    O0, Ol0, Oh0, _, _ = orc.hybrid_attention(Qw, Kw, Vw, (L, z), 16, 16, 2)
    np.testing.assert_array_equal(Ol, Ol0)
    np.testing.assert_allclose(Oh, Oh0 @ W, atol=1e-13)
    np.testing.assert_allclose(Ow, Ol + Oh, atol=0)


# ----------------------------------------------------------------------------- Eq. 6
def test_hybrid_sum_and_null_state():
    r = _rng(41)
    n_q, n_kv, d, b, k = 32, 128, 16, 16, 3
    Q, K, V = r.normal(size=(n_q, d)), r.normal(size=(n_kv, d)), r.normal(size=(n_kv, d))
    Ke, Ve = r.normal(size=(50, d)), r.normal(size=(50, d))
    st = orc.state_absorb(*orc.state_zero(d), Ke, Ve)
    O, Ol, Oh, idx, gap = orc.hybrid_attention(Q, K, V, st, b, b, k)
    np.testing.assert_allclose(O - Ol, Oh, atol=1e-13)
    np.testing.assert_allclose(Oh, orc.history_readout(Q, *st), atol=0)
    idx2, gap2 = orc.select_blocks(orc.block_scores(Q, K, b, b), k)
    assert np.array_equal(idx, idx2) and np.array_equal(gap, gap2)
    np.testing.assert_allclose(Ol, orc.sparse_attention(Q, K, V, idx2, b, b), atol=0)
    O0, Ol0, Oh0, _, _ = orc.hybrid_attention(Q, K, V, None, b, b, k)
    assert np.array_equal(O0, Ol0) and not Oh0.any()
    # a supplied index list overrides the oracle's own selection
    forced = np.tile(np.array([0, 1, 2], dtype=np.int32), (2, 1))
    _, Olf, _, idxf, gapf = orc.hybrid_attention(Q, K, V, None, b, b, k, block_idx=forced)
    assert gapf is None and np.array_equal(idxf, forced)
    np.testing.assert_allclose(Olf, orc.dense_attention(Q, K[:48], V[:48]), atol=1e-12)


def test_hybrid_equals_full_history_linear_plus_window_softmax():
    # With every window block kept, the output is softmax attention over the window plus
    # kernelised (linear) attention over exactly the evicted tokens.
    r = _rng(42)
    d, b = 8, 8
    Q = r.normal(size=(16, d))
    hist_K, hist_V = r.normal(size=(24, d)), r.normal(size=(24, d))
    win_K, win_V = r.normal(size=(32, d)), r.normal(size=(32, d))
    st = orc.state_absorb(*orc.state_zero(d), hist_K, hist_V)
    O, *_ = orc.hybrid_attention(Q, win_K, win_V, st, b, b, 4, eps=0.0)
    fq, fk = np.maximum(Q, 0), np.maximum(hist_K, 0)
    W = fq @ fk.T
    lin = (W / W.sum(1, keepdims=True)) @ hist_V
    np.testing.assert_allclose(O, _sdpa(Q, win_K, win_V) + lin, atol=1e-12)
