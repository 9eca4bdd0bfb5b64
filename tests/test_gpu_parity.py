"""GPU parity: every stage of the HIP path, through the C ABI, against the fp64 oracle on the
same seeded inputs.  Bounds: block indices exact as sets except boundary ties closer than
1e-6 in the oracle; outputs rel-L2 <= 1e-2 and max-abs <= 2e-2 for bf16, rel-L2 <= 1e-5 for
fp32; fp32 state rel-L2 <= 1e-5 (bf16-exact products, fp32 accumulation) and <= 5e-3 when
rotated keys are rounded to bf16 for the matrix cores."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle as orc
import paper_2604_10103_amd as hf
import workloads as wl
from parity import (BF16_MAX_ABS, BF16_REL_L2, F32_REL_L2, check_block_idx, heads_of, max_abs, oracle_state,
                    rel_l2, split_state)

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def cfg_of(w, **kw):
    args = dict(batch=w.batch, heads=w.heads, head_dim=w.head_dim, dtype=w.dtype, block_q=w.block,
                block_kv=w.block, keep_ratio=w.keep_ratio)
    args.update(kw)
    return hf.make_config(**args)


def new_state(cfg):
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    st.fill_(float("nan"))          # init must overwrite everything
    hf.hf_state_init(cfg, st)
    return st


def absorb_ws(cfg, n):
    nbytes = hf.hf_absorb_workspace_bytes(cfg, n)
    return torch.empty(nbytes, dtype=torch.uint8, device=DEV) if nbytes else None


def new_workspace(cfg, n_q, n_kv):
    return torch.empty(hf.hf_workspace_bytes(cfg, n_q, n_kv), dtype=torch.uint8, device=DEV)


def out_bounds(w):
    return (BF16_REL_L2, BF16_MAX_ABS) if w.dtype == "bf16" else (F32_REL_L2, 1e-4)


def gpu_select(cfg, w, Q, K, want_scores=True):
    k = hf.hf_select_k(cfg, K.shape[2])
    t_m, t_n = -(-Q.shape[2] // cfg.block_q), -(-K.shape[2] // cfg.block_kv)
    idx = torch.full((w.batch, w.heads, t_m, k), -1, dtype=torch.int32, device=DEV)
    scores = torch.empty((w.batch, w.heads, t_m, t_n), dtype=torch.float32, device=DEV) if want_scores else None
    ws = new_workspace(cfg, Q.shape[2], K.shape[2])
    hf.hf_block_select(cfg, Q, K, idx, scores, ws)
    torch.cuda.synchronize()
    return idx, scores, k


# ------------------------------------------------------------------------------- state (Eq. 2)
@pytest.mark.parametrize("name", ["tiny_f32", "small_bf16", "small_f32_d128"])
def test_state_init_and_absorb_match_direct_sum(name):
    w = wl.get(name)
    cfg = cfg_of(w)
    st = new_state(cfg)
    assert not st.isnan().any() and float(st.abs().max()) == 0.0
    Ks, Vs = [], []
    for c in range(w.evicted_frames):       # one call per evicted frame
        K, V = wl.make_evicted(w, c, w.tokens_per_frame)
        Ks.append(K); Vs.append(V)
        hf.hf_absorb_evicted(cfg, st, K.to(DEV), V.to(DEV))
    torch.cuda.synchronize()
    ref = oracle_state(Ks, Vs, w.head_dim)
    L, z = split_state(st, w.batch * w.heads, w.head_dim)
    assert rel_l2(L, np.stack([r[0] for r in ref])) <= 1e-5
    assert rel_l2(z, np.stack([r[1] for r in ref])) <= 1e-5
    # order / chunking invariance on the GPU: one call with all tokens, partials through a workspace
    st2 = new_state(cfg)
    n_all = w.evicted_frames * w.tokens_per_frame
    hf.hf_absorb_evicted(cfg, st2, torch.cat(Ks, 2).to(DEV), torch.cat(Vs, 2).to(DEV),
                         workspace=absorb_ws(cfg, n_all))
    torch.cuda.synchronize()
    L2, z2 = split_state(st2, w.batch * w.heads, w.head_dim)
    assert rel_l2(L2, L) <= 2e-6 and rel_l2(z2, z) <= 2e-6


@pytest.mark.parametrize("name", ["tiny_f32", "small_bf16"])
@pytest.mark.parametrize("phi", [hf.HF_PHI_RELU, hf.HF_PHI_ELU1])
@pytest.mark.parametrize("use_ws", [False, True])
def test_absorb_with_rope_and_elu(name, phi, use_ws):
    w = wl.get(name)
    cfg = cfg_of(w, phi=phi)
    st = new_state(cfg)
    n = 3 * w.tokens_per_frame + 5   # ragged
    K, V = wl.make_evicted(w, 40, n)
    cos, sin = wl.rope_tables(n, w.head_dim, first_position=3.0, tokens_per_position=w.tokens_per_frame)
    hf.hf_absorb_evicted(cfg, st, K.to(DEV), V.to(DEV), cos.to(DEV), sin.to(DEV),
                         workspace=absorb_ws(cfg, n) if use_ws else None)
    torch.cuda.synchronize()
    ref = oracle_state([K], [V], w.head_dim, phi, [(cos, sin)])
    L, z = split_state(st, w.batch * w.heads, w.head_dim)
    tol = 5e-3 if w.dtype == "bf16" else 1e-5
    assert rel_l2(L, np.stack([r[0] for r in ref])) <= tol
    assert rel_l2(z, np.stack([r[1] for r in ref])) <= 1e-5


def test_absorb_long_run_uses_several_runs_per_slice():
    # more tokens than one workgroup requests at once, a ragged end, and a dirty workspace
    w = wl.get("small_bf16")
    cfg = cfg_of(w)
    n = 12 * 320 * 9 + 37
    K, V = wl.make_evicted(w, 42, n)
    ws = absorb_ws(cfg, n)
    ws.fill_(0x7f)
    st = new_state(cfg)
    hf.hf_absorb_evicted(cfg, st, K.to(DEV), V.to(DEV), workspace=ws)
    st2 = new_state(cfg)
    hf.hf_absorb_evicted(cfg, st2, K.to(DEV), V.to(DEV))
    torch.cuda.synchronize()
    ref = oracle_state([K], [V], w.head_dim)
    for s_ in (st, st2):
        L, z = split_state(s_, w.batch * w.heads, w.head_dim)
        assert rel_l2(L, np.stack([r[0] for r in ref])) <= 1e-5
        assert rel_l2(z, np.stack([r[1] for r in ref])) <= 1e-5


def test_absorb_single_token_and_accumulation():
    w = wl.get("small_bf16")
    cfg = cfg_of(w)
    st = new_state(cfg)
    K, V = wl.make_evicted(w, 41, 1)
    hf.hf_absorb_evicted(cfg, st, K.to(DEV), V.to(DEV))
    hf.hf_absorb_evicted(cfg, st, K.to(DEV), V.to(DEV), workspace=absorb_ws(cfg, 1))     # twice: the state accumulates
    torch.cuda.synchronize()
    ref = oracle_state([K, K], [V, V], w.head_dim)
    L, z = split_state(st, w.batch * w.heads, w.head_dim)
    assert rel_l2(L, np.stack([r[0] for r in ref])) <= 1e-6
    assert rel_l2(z, np.stack([r[1] for r in ref])) <= 1e-6


# ------------------------------------------------------------------------------- selection (Eq. 4)
@pytest.mark.parametrize("name", ["tiny_f32", "small_bf16", "small_b128", "small_f32_d128"])
def test_block_scores_and_indices(name):
    w = wl.get(name)
    cfg = cfg_of(w)
    Q, K, _ = wl.make_qkv(w)
    idx, scores, k = gpu_select(cfg, w, Q.to(DEV), K.to(DEV))
    assert k == orc.select_k(w.keep_ratio, w.t_n)
    idx, scores = idx.cpu().numpy(), wl.to_f64(scores)
    for h, (q, kk) in enumerate(zip(heads_of(Q), heads_of(K))):
        A = orc.block_scores(q, kk, w.block, w.block)
        assert np.abs(scores[0, h] - A).max() <= 1e-5 * max(1.0, np.abs(A).max())
        check_block_idx(idx[0, h], A, k)


def test_selection_over_many_blocks_takes_the_one_row_kernel():
    # 640 KV blocks: the three-rows-per-workgroup kernel's LDS need exceeds 64 KB, the one-row kernel serves
    w = dataclasses.replace(wl.get("tiny_f32"), heads=1, tokens_per_frame=16 * 64, chunk_frames=1, window_frames=10)
    assert w.t_n == 640 and w.t_m == 64
    cfg = cfg_of(w, keep_k=64)
    Q, K, _ = wl.make_qkv(w)
    idx, scores, k = gpu_select(cfg, w, Q.to(DEV), K.to(DEV))
    assert k == 64
    A = orc.block_scores(wl.to_f64(Q[0, 0]), wl.to_f64(K[0, 0]), w.block, w.block)
    assert np.abs(scores.cpu().numpy()[0, 0] - A).max() <= 1e-5 * max(1.0, np.abs(A).max())
    check_block_idx(idx.cpu().numpy()[0, 0], A, k)


def test_selection_ties_and_keep_all():
    # identical key blocks give exactly tied scores: the lower index must win
    w = wl.get("small_bf16")
    cfg = cfg_of(w, keep_k=3)
    Q, K, _ = wl.make_qkv(w)
    K[:, :, 64:128] = K[:, :, 0:64]
    K[:, :, 128:192] = K[:, :, 0:64]
    idx, scores, k = gpu_select(cfg, w, Q.to(DEV), K.to(DEV))
    idx = idx.cpu().numpy()
    for h, (q, kk) in enumerate(zip(heads_of(Q), heads_of(K))):
        A = orc.block_scores(q, kk, w.block, w.block)
        ref, _ = orc.select_blocks(A, 3)
        # ties are exact in fp32 as well (same pooled vectors), so the sets must agree outright
        assert np.array_equal(idx[0, h], ref)
    cfg = cfg_of(w, keep_ratio=1.0)
    idx, _, k = gpu_select(cfg, w, Q.to(DEV), K.to(DEV), want_scores=False)
    assert k == w.t_n
    assert np.array_equal(idx.cpu().numpy(), np.broadcast_to(np.arange(k, dtype=np.int32), idx.shape))


@pytest.mark.parametrize("name", ["small_bf16", "tiny_f32", "small_b128"])
def test_selection_with_reused_pooled_keys(name):
    # denoising steps of one chunk: the older half of the window is fixed, the chunk's own K changes;
    # the pooled means of the unchanged whole blocks are reused from the previous call's workspace
    w = wl.get(name)
    cfg = cfg_of(w)
    k = hf.hf_select_k(cfg, w.n_kv)
    ws = new_workspace(cfg, w.n_q, w.n_kv)
    idx = torch.full((w.batch, w.heads, w.t_m, k), -1, dtype=torch.int32, device=DEV)
    scores = torch.empty((w.batch, w.heads, w.t_m, w.t_n), dtype=torch.float32, device=DEV)
    Q0, K0, _ = wl.make_qkv(w, step=0)
    hf.hf_block_select(cfg, Q0.to(DEV), K0.to(DEV), idx, scores, ws)
    half = w.n_kv - w.n_q                      # tokens of the cached part
    reuse = half // w.block                    # its whole blocks (a straddling block is pooled again)
    assert 0 < reuse < w.t_n
    for step in (1, 2):
        Q, Kn, _ = wl.make_qkv(w, step=step)
        K = torch.cat([K0[:, :, :half], Kn[:, :, half:]], dim=2).contiguous()
        hf.hf_block_select_cached(cfg, Q.to(DEV), K.to(DEV), reuse, idx, scores, ws)
        torch.cuda.synchronize()
        got_idx, got_sc = idx.cpu().numpy().copy(), scores.cpu().numpy().copy()
        for h, (q, kk) in enumerate(zip(heads_of(Q), heads_of(K))):
            A = orc.block_scores(q, kk, w.block, w.block)
            assert np.abs(got_sc[0, h] - A).max() <= 1e-5 * max(1.0, np.abs(A).max())
            check_block_idx(got_idx[0, h], A, k)
        # bit for bit what the full pooling gives on the same window (in a fresh workspace)
        idx2, sc2, _ = gpu_select(cfg, w, Q.to(DEV), K.to(DEV))
        assert np.array_equal(got_idx, idx2.cpu().numpy())
        assert np.array_equal(got_sc, sc2.cpu().numpy())
    # reusing everything that is whole, with nothing changed, is the identity
    hf.hf_block_select_cached(cfg, Q.to(DEV), K.to(DEV), w.n_kv // w.block, idx, scores, ws)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), got_idx) and np.array_equal(scores.cpu().numpy(), got_sc)


# ------------------------------------------------------------------------------- cache eviction
@pytest.mark.parametrize("name,use_ws,rope", [("small_bf16", True, False), ("small_bf16", False, True),
                                              ("tiny_f32", False, False), ("small_b128", True, True)])
def test_window_advance_absorbs_the_oldest_chunk_and_compacts(name, use_ws, rope):
    # three rolls of the window buffers: every roll pops one chunk into the state (oracle: direct sum over
    # exactly those tokens), moves the rest to the front bit for bit, and leaves the freed tail to the caller
    w = wl.get(name)
    cfg = cfg_of(w)
    d, n_kv, n_ev = w.head_dim, w.n_kv, w.n_q
    assert n_kv - n_ev > n_ev                       # source and destination of the move overlap
    _, K, V = wl.make_qkv(w)
    Kd, Vd = K.to(DEV).clone(), V.to(DEV).clone()
    Kc, Vc = K.clone(), V.clone()                   # host mirror of the window
    st = new_state(cfg)
    aws = absorb_ws(cfg, n_ev) if use_ws else None
    states = [orc.state_zero(d) for _ in range(w.batch * w.heads)]
    for roll in range(3):
        tab = wl.rope_tables(n_ev, d, first_position=float(roll), tokens_per_position=w.tokens_per_frame) if rope \
            else (None, None)
        hf.hf_window_advance(cfg, Kd, Vd, n_ev, st, *(t.to(DEV) if t is not None else None for t in tab), workspace=aws)
        torch.cuda.synchronize()
        cos, sin = (None, None) if not rope else (wl.to_f64(tab[0]), wl.to_f64(tab[1]))
        ke, ve = heads_of(Kc[:, :, :n_ev]), heads_of(Vc[:, :, :n_ev])
        states = [orc.state_absorb(L, z, k_, v_, cfg.phi, cos, sin) for (L, z), k_, v_ in zip(states, ke, ve)]
        Lg, zg = split_state(st, w.batch * w.heads, d)
        bound = 5e-3 if (rope and w.dtype == "bf16" and d == 128) else 1e-5   # rotated keys rounded to bf16
        assert rel_l2(Lg, np.stack([s_[0] for s_ in states])) <= bound
        assert rel_l2(zg, np.stack([s_[1] for s_ in states])) <= 1e-5
        # the window moved to the front, the tail untouched
        Kc = torch.cat([Kc[:, :, n_ev:], Kc[:, :, n_kv - n_ev:]], dim=2)
        Vc = torch.cat([Vc[:, :, n_ev:], Vc[:, :, n_kv - n_ev:]], dim=2)
        assert torch.equal(Kd.cpu(), Kc) and torch.equal(Vd.cpu(), Vc)
        # the caller writes the next chunk into the freed slots
        Kn, Vn = wl.make_evicted(w, 40 + roll, n_ev)
        Kd[:, :, n_kv - n_ev:] = Kn.to(DEV); Vd[:, :, n_kv - n_ev:] = Vn.to(DEV)
        Kc[:, :, n_kv - n_ev:] = Kn; Vc[:, :, n_kv - n_ev:] = Vn
    # evicting the whole window is allowed: nothing moves
    hf.hf_window_advance(cfg, Kd, Vd, n_kv, st, workspace=None)
    torch.cuda.synchronize()
    assert torch.equal(Kd.cpu(), Kc)


# ------------------------------------------------------------------------------- Linear of Eq. 3
@pytest.mark.parametrize("name", ["small_bf16", "tiny_f32"])
def test_linear_map_folded_into_the_state(name):
    w = wl.get(name)
    cfg = cfg_of(w)
    d = w.head_dim
    Ke, Ve = wl.make_evicted(w, 0)
    st = new_state(cfg)
    hf.hf_absorb_evicted(cfg, st, Ke.to(DEV), Ve.to(DEV))
    W = wl.randn((w.heads, d, d), 91_000 + w.cfg, 1.0 / np.sqrt(d), torch.float32)
    st2 = torch.full_like(st, float("nan"))
    hf.hf_state_fold_linear(cfg, st, W.to(DEV), st2)
    torch.cuda.synchronize()
    Lg, zg = split_state(st, w.heads, d)
    L2, z2 = split_state(st2, w.heads, d)
    assert np.array_equal(z2, zg)                               # the normaliser is copied
    W64 = W.double().numpy()
    for h in range(w.heads):
        ref = orc.state_fold_linear(Lg[0, h] if Lg.ndim == 4 else Lg[h], W64[h])
        got = L2[0, h] if L2.ndim == 4 else L2[h]
        assert rel_l2(got, ref) <= 1e-6                         # fp32 FMA over d terms
    # the whole path on the folded state = oracle with the map applied to the history term
    Q, K, V = wl.make_qkv(w)
    idx, _, k = gpu_select(cfg, w, Q.to(DEV), K.to(DEV), want_scores=False)
    O = run_hybrid(cfg, w, Q, K, V, idx, st2)
    Og, idxc = wl.to_f64(O), idx.cpu().numpy()
    states = oracle_state([Ke], [Ve], d)
    bound_l2, bound_abs = out_bounds(w)
    for h in range(w.heads):
        ref, *_ = orc.hybrid_attention(wl.to_f64(Q[0, h]), wl.to_f64(K[0, h]), wl.to_f64(V[0, h]), states[h],
                                       w.block, w.block, k, eps=cfg.eps, block_idx=idxc[0, h], W=W64[h])
        assert rel_l2(Og[0, h], ref) <= bound_l2
        assert max_abs(Og[0, h], ref) <= bound_abs


# ------------------------------------------------------------------------------- attention (Eq. 5, 3, 6)
def run_hybrid(cfg, w, Q, K, V, idx, st, tables=None):
    O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
    ws = new_workspace(cfg, Q.shape[2], K.shape[2])
    cos, sin = (None, None) if tables is None else (tables[0].to(DEV), tables[1].to(DEV))
    hf.hf_hybrid_attn_fwd(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, st, O, ws, cos, sin)
    torch.cuda.synchronize()
    return O


@pytest.mark.parametrize("name,q_gain", [("tiny_f32", 1.0), ("tiny_f32", 6.0), ("small_bf16", 1.0),
                                         ("small_bf16", 8.0), ("small_bf16", 64.0), ("small_b128", 1.0),
                                         ("small_b128", 48.0), ("small_f32_d128", 3.0)])
def test_sparse_attention_alone_matches_oracle(name, q_gain):
    w = wl.get(name)
    cfg = cfg_of(w)
    Q, K, V = wl.make_qkv(w, q_gain=q_gain)
    idx, _, k = gpu_select(cfg, w, Q.to(DEV), K.to(DEV), want_scores=False)
    O = run_hybrid(cfg, w, Q, K, V, idx, None)
    assert not O.isnan().any()
    Og, idxc = wl.to_f64(O), idx.cpu().numpy()
    rl, ma = out_bounds(w)
    for h, (q, kk, v) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V))):
        ref = orc.sparse_attention(q, kk, v, idxc[0, h], w.block, w.block)   # the GPU's own index list
        assert rel_l2(Og[0, h], ref) <= rl, (name, h)
        assert max_abs(Og[0, h], ref) <= ma


@pytest.mark.parametrize("name", ["tiny_f32", "small_bf16", "small_b128"])
def test_dense_window_attention_matches_bruteforce(name):
    w = wl.get(name)
    cfg = cfg_of(w, keep_ratio=1.0)
    Q, K, V = wl.make_qkv(w, q_gain=2.0)
    O = wl.to_f64(run_hybrid(cfg, w, Q, K, V, None, None))
    rl, ma = out_bounds(w)
    for h, (q, kk, v) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V))):
        ref = orc.dense_attention(q, kk, v)
        assert rel_l2(O[0, h], ref) <= rl and max_abs(O[0, h], ref) <= ma


@pytest.mark.parametrize("name,phi,rope", [("tiny_f32", hf.HF_PHI_RELU, False), ("tiny_f32", hf.HF_PHI_ELU1, True),
                                           ("small_bf16", hf.HF_PHI_RELU, False), ("small_bf16", hf.HF_PHI_RELU, True),
                                           ("small_b128", hf.HF_PHI_ELU1, False), ("small_f32_d128", hf.HF_PHI_RELU, True)])
def test_full_hybrid_path_matches_oracle(name, phi, rope):
    w = wl.get(name)
    cfg = cfg_of(w, phi=phi)
    st = new_state(cfg)
    Ks, Vs, tabs = [], [], []
    for c in range(w.evicted_frames):
        K, V = wl.make_evicted(w, c, w.tokens_per_frame)
        tab = wl.rope_tables(w.tokens_per_frame, w.head_dim, first_position=float(c)) if rope else (None, None)
        Ks.append(K); Vs.append(V); tabs.append(tab)
        hf.hf_absorb_evicted(cfg, st, K.to(DEV), V.to(DEV), *(t.to(DEV) if t is not None else None for t in tab))
    Q, K, V = wl.make_qkv(w)
    qtab = wl.rope_tables(w.n_q, w.head_dim, first_position=float(w.evicted_frames + 2),
                          tokens_per_position=w.tokens_per_frame) if rope else None
    idx, _, k = gpu_select(cfg, w, Q.to(DEV), K.to(DEV), want_scores=False)
    O = wl.to_f64(run_hybrid(cfg, w, Q, K, V, idx, st, qtab))
    idxc = idx.cpu().numpy()
    ref_states = oracle_state(Ks, Vs, w.head_dim, phi, tabs if rope else None)
    rl, ma = out_bounds(w)
    cq = None if qtab is None else wl.to_f64(qtab[0])
    sq = None if qtab is None else wl.to_f64(qtab[1])
    for h, (q, kk, v) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V))):
        ref, ref_local, ref_hist, _, _ = orc.hybrid_attention(q, kk, v, ref_states[h], w.block, w.block, k, phi,
                                                             cq, sq, cfg.eps, cfg.z_scale, block_idx=idxc[0, h])
        assert np.abs(ref_hist).max() > 1e-4   # the history term is really there
        assert rel_l2(O[0, h], ref) <= rl, (name, h, rel_l2(O[0, h], ref))
        assert max_abs(O[0, h], ref) <= ma


def test_empty_state_gives_local_attention_only():
    w = wl.get("small_bf16")
    cfg = cfg_of(w)
    Q, K, V = wl.make_qkv(w)
    idx, _, _ = gpu_select(cfg, w, Q.to(DEV), K.to(DEV), want_scores=False)
    a = run_hybrid(cfg, w, Q, K, V, idx, None)
    b = run_hybrid(cfg, w, Q, K, V, idx, new_state(cfg))     # zero state: 0 / (0 + eps) = 0
    assert torch.equal(a, b)


@pytest.mark.parametrize("n_q,n_kv,b", [(1, 1, 64), (5, 70, 64), (64, 64, 64), (129, 257, 128), (33, 100, 16),
                                        (300, 1300, 256), (200, 1000, 192)])   # 192 / 256: wavefront-per-64-rows kernel
def test_ragged_and_degenerate_sizes(n_q, n_kv, b):
    dtype = torch.bfloat16
    cfg = hf.make_config(1, 2, 128, "bf16", b, b, 0.5)
    Q = wl.randn((1, 2, n_q, 128), 901, 0.7, dtype)
    K = wl.randn((1, 2, n_kv, 128), 902, 0.7, dtype)
    V = wl.randn((1, 2, n_kv, 128), 903, 0.7, dtype)
    Ke, Ve = wl.randn((1, 2, 37, 128), 904, 0.7, dtype), wl.randn((1, 2, 37, 128), 905, 0.7, dtype)
    st = new_state(cfg)
    hf.hf_absorb_evicted(cfg, st, Ke.to(DEV), Ve.to(DEV))
    k = hf.hf_select_k(cfg, n_kv)
    t_m = -(-n_q // b)
    idx = torch.empty((1, 2, t_m, k), dtype=torch.int32, device=DEV)
    ws = new_workspace(cfg, n_q, n_kv)
    hf.hf_block_select(cfg, Q.to(DEV), K.to(DEV), idx, None, ws)
    guard = torch.full((1, 2, n_q + 4, 128), 7.0, dtype=dtype, device=DEV)   # rows past n_q must stay untouched
    O = guard[:, :, :n_q].contiguous()
    hf.hf_hybrid_attn_fwd(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, st, O, ws)
    torch.cuda.synchronize()
    states = oracle_state([Ke], [Ve], 128)
    idxc = idx.cpu().numpy()
    for h, (q, kk, v) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V))):
        A = orc.block_scores(q, kk, b, b)
        check_block_idx(idxc[0, h], A, k)
        ref, *_ = orc.hybrid_attention(q, kk, v, states[h], b, b, k, block_idx=idxc[0, h])
        assert rel_l2(wl.to_f64(O)[0, h], ref) <= BF16_REL_L2
        assert max_abs(wl.to_f64(O)[0, h], ref) <= BF16_MAX_ABS


def test_out_of_range_block_index_is_ignored_not_read():
    w = wl.get("small_bf16")
    cfg = cfg_of(w)
    Q, K, V = wl.make_qkv(w)
    idx, _, k = gpu_select(cfg, w, Q.to(DEV), K.to(DEV), want_scores=False)
    bad = torch.cat([idx, torch.full_like(idx[..., :1], 1 << 20)], dim=-1).contiguous()
    a = run_hybrid(cfg, w, Q, K, V, idx, None)
    b = run_hybrid(cfg, w, Q, K, V, bad[..., : k + 1].contiguous() if k + 1 <= w.t_n else idx, None)
    assert torch.equal(a, b)


@pytest.mark.parametrize("name", ["small_bf16", "tiny_f32", "small_f32_d128"])
def test_query_block_with_no_valid_block_index_gives_zeros_on_every_kernel(name):
    """A row of the index list that names no existing block selects no key: its softmax is empty and O_local is
    defined as zero there (never NaN), by the matrix-core kernel and by the fp32-arithmetic kernel alike; the
    other query blocks are not affected."""
    w = wl.get(name)
    cfg = cfg_of(w)
    Q, K, V = wl.make_qkv(w)
    idx, _, k = gpu_select(cfg, w, Q.to(DEV), K.to(DEV), want_scores=False)
    bad = idx.clone()
    bad[:, :, 1, :] = 1 << 20                       # query block 1 of every head: nothing but invalid indices
    bad[:, 0, 0, :] = -7                            # and block 0 of head 0
    a = run_hybrid(cfg, w, Q, K, V, idx, None)
    b = run_hybrid(cfg, w, Q, K, V, bad, None)
    assert torch.isfinite(b.float()).all()
    rows1 = slice(w.block, min(2 * w.block, w.n_q))
    assert (b[:, :, rows1] == 0).all() and (b[:, 0, : w.block] == 0).all()
    keep = torch.ones(w.n_q, dtype=torch.bool, device=DEV)
    keep[rows1] = False
    assert torch.equal(a[:, 1:, keep], b[:, 1:, keep])


# ------------------------------------------------------------------------------- batch > 1
@pytest.mark.parametrize("name", ["small_bf16", "tiny_f32"])
def test_batch_of_two_every_stage(name):
    # (batch, head) pairs are independent: layouts [B, H, ...] with B = 2, the Linear weight shared by the batch
    w = dataclasses.replace(wl.get(name), batch=2, heads=3)
    cfg = cfg_of(w)
    d, B, H = w.head_dim, w.batch, w.heads
    Ke, Ve = wl.make_evicted(w, 1)
    st = new_state(cfg)
    hf.hf_absorb_evicted(cfg, st, Ke.to(DEV), Ve.to(DEV), workspace=absorb_ws(cfg, Ke.shape[2]))
    torch.cuda.synchronize()
    states = oracle_state([Ke], [Ve], d)                      # (b, h) order
    L, z = split_state(st, B * H, d)
    assert rel_l2(L, np.stack([s_[0] for s_ in states])) <= 1e-5
    assert rel_l2(z, np.stack([s_[1] for s_ in states])) <= 1e-5
    W = wl.randn((H, d, d), 92_000 + w.cfg, d ** -0.5, torch.float32)
    st2 = torch.empty_like(st)
    hf.hf_state_fold_linear(cfg, st, W.to(DEV), st2)
    Q, K, V = wl.make_qkv(w)
    idx, scores, k = gpu_select(cfg, w, Q.to(DEV), K.to(DEV))
    O = run_hybrid(cfg, w, Q, K, V, idx, st2)
    Og, idxc, sc = wl.to_f64(O), idx.cpu().numpy(), scores.cpu().numpy()
    rl, ma = out_bounds(w)
    W64 = W.double().numpy()
    for n, (q, kk, v) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V))):
        b, h = divmod(n, H)
        A = orc.block_scores(q, kk, w.block, w.block)
        assert np.abs(sc[b, h] - A).max() <= 1e-5 * max(1.0, np.abs(A).max())
        check_block_idx(idxc[b, h], A, k)
        ref, *_ = orc.hybrid_attention(q, kk, v, states[n], w.block, w.block, k, eps=cfg.eps,
                                       block_idx=idxc[b, h], W=W64[h])
        assert rel_l2(Og[b, h], ref) <= rl, (b, h)
        assert max_abs(Og[b, h], ref) <= ma


# ------------------------------------------------------------------------------- seeded random shapes
@pytest.mark.parametrize("seed", range(16))
def test_seeded_random_shapes_whole_path(seed):
    # every dispatch path (MFMA / generic attention, fused / stand-alone readout, MFMA / FMA absorb with and
    # without workspace, both selection kernels) on shapes drawn from a seeded generator
    r = np.random.default_rng(7_000 + seed)
    dtype = ["bf16", "f32"][int(r.integers(0, 2))]
    d = [64, 128][int(r.integers(0, 2))]
    b = [16, 32, 64, 128][int(r.integers(0, 4))]
    B, H = int(r.integers(1, 3)), int(r.integers(1, 4))
    n_q, n_kv, n_ev = int(r.integers(1, 300)), int(r.integers(1, 700)), int(r.integers(1, 200))
    phi = [hf.HF_PHI_RELU, hf.HF_PHI_ELU1][int(r.integers(0, 2))]
    rope = bool(r.integers(0, 2))
    keep = float(r.uniform(0.1, 1.0))
    use_ws = bool(r.integers(0, 2))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    cfg = hf.make_config(B, H, d, dtype, b, b, keep, phi=phi)
    mk = lambda n, s_: wl.randn((B, H, n, d), 8_000 + 10 * seed + s_, 0.6, tdt)
    Q, K, V, Ke, Ve = mk(n_q, 0), mk(n_kv, 1), mk(n_kv, 2), mk(n_ev, 3), mk(n_ev, 4)
    etab = wl.rope_tables(n_ev, d, first_position=3.0, tokens_per_position=7) if rope else (None, None)
    qtab = wl.rope_tables(n_q, d, first_position=40.0, tokens_per_position=5) if rope else None
    st = new_state(cfg)
    hf.hf_absorb_evicted(cfg, st, Ke.to(DEV), Ve.to(DEV), *(t.to(DEV) if t is not None else None for t in etab),
                         workspace=absorb_ws(cfg, n_ev) if use_ws else None)
    k = hf.hf_select_k(cfg, n_kv)
    t_m, t_n = -(-n_q // b), -(-n_kv // b)
    idx = torch.full((B, H, t_m, k), -1, dtype=torch.int32, device=DEV)
    scores = torch.empty((B, H, t_m, t_n), dtype=torch.float32, device=DEV)
    ws = new_workspace(cfg, n_q, n_kv)
    hf.hf_block_select(cfg, Q.to(DEV), K.to(DEV), idx, scores, ws)
    O = torch.full(Q.shape, float("nan"), dtype=tdt, device=DEV)
    hf.hf_hybrid_attn_fwd(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, st, O, ws,
                          *(() if qtab is None else (qtab[0].to(DEV), qtab[1].to(DEV))))
    torch.cuda.synchronize()
    assert not O.isnan().any()
    states = oracle_state([Ke], [Ve], d, phi, [etab] if rope else None)
    L, z = split_state(st, B * H, d)
    # rotated / ELU keys are rounded to bf16 before the matrix cores on the bf16 d = 128 path
    sb = 5e-3 if (dtype == "bf16" and d == 128 and (rope or phi != hf.HF_PHI_RELU)) else 1e-5
    assert rel_l2(L, np.stack([s_[0] for s_ in states])) <= sb
    assert rel_l2(z, np.stack([s_[1] for s_ in states])) <= 1e-5
    Og, idxc, sc = wl.to_f64(O), idx.cpu().numpy(), scores.cpu().numpy()
    rl, ma = (BF16_REL_L2, BF16_MAX_ABS) if dtype == "bf16" else (F32_REL_L2, 1e-4)
    cq = None if qtab is None else wl.to_f64(qtab[0])
    sq = None if qtab is None else wl.to_f64(qtab[1])
    for n, (q, kk, v) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V))):
        bi, h = divmod(n, H)
        A = orc.block_scores(q, kk, b, b)
        assert np.abs(sc[bi, h] - A).max() <= 1e-5 * max(1.0, np.abs(A).max())
        check_block_idx(idxc[bi, h], A, k)
        ref, *_ = orc.hybrid_attention(q, kk, v, states[n], b, b, k, phi, cq, sq, cfg.eps, cfg.z_scale,
                                       block_idx=idxc[bi, h])
        assert rel_l2(Og[bi, h], ref) <= rl, (seed, bi, h, rel_l2(Og[bi, h], ref))
        assert max_abs(Og[bi, h], ref) <= ma
