"""GPU parity of the backward pass (training algorithm of the supplement) against the fp64 oracle's gradients:
dQ, dK, dV of the block-sparse attention for the library's own index lists, the history branch's query gradient,
split queries, the dense window, a cache buffer with spare capacity.

Bounds.  fp32 storage: rel-L2 <= 5e-5 (fp32 exp2 and accumulation; dS = P (dP - D) subtracts two O(1) numbers, which
costs a few units over the forward's 1e-5).  bf16 storage: rel-L2 <= 1e-2 and max-abs <= 2e-2 of the largest
gradient magnitude, the forward's bounds (inputs are exact in both; the output rounding alone is 2^-9)."""

import numpy as np
import pytest
import torch

import oracle as orc
import paper_2604_10103_amd as hf
import workloads as wl
from parity import heads_of, max_abs, oracle_state, rel_l2

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def cfg_of(w, **kw):
    args = dict(batch=w.batch, heads=w.heads, head_dim=w.head_dim, dtype=w.dtype, block_q=w.block,
                block_kv=w.block, keep_ratio=w.keep_ratio)
    args.update(kw)
    return hf.make_config(**args)


def bounds(w):
    return (1e-2, 2e-2) if w.dtype == "bf16" else (5e-5, 1e-4)


def check(name, got, ref, w):
    rl, ma = bounds(w)
    scale = max(np.abs(ref).max(), 1e-3)      # a gradient that is exactly zero (one key: P = 1) is met to rounding
    e1, e2 = rel_l2(got, ref), max_abs(got, ref) / scale
    assert e1 <= rl and e2 <= ma, (name, e1, e2)
    return e1


def make_state(cfg, w, phi, rope):
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    Ks, Vs, tabs = [], [], []
    for c in range(w.evicted_frames):
        K, V = wl.make_evicted(w, c, w.tokens_per_frame)
        tab = wl.rope_tables(w.tokens_per_frame, w.head_dim, first_position=float(c)) if rope else (None, None)
        Ks.append(K); Vs.append(V); tabs.append(tab)
        hf.hf_absorb_evicted(cfg, st, K.to(DEV), V.to(DEV), *(None if t is None else t.to(DEV) for t in tab))
    return st, oracle_state(Ks, Vs, w.head_dim, phi, tabs if rope else None)


def run_bwd(cfg, w, Q, K, V, idx, st, dO, tables=None, Q_hist=None, n_kv=None):
    dQ = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
    dK = torch.full(K.shape, float("nan"), dtype=K.dtype, device=DEV)
    dV = torch.full(K.shape, float("nan"), dtype=K.dtype, device=DEV)
    dQh = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV) if Q_hist is not None else None
    nkv = K.shape[2] if n_kv is None else n_kv
    ws = torch.empty(hf.hf_bwd_workspace_bytes(cfg, Q.shape[2], nkv), dtype=torch.uint8, device=DEV)
    cos, sin = (None, None) if tables is None else (tables[0].to(DEV), tables[1].to(DEV))
    hf.hf_hybrid_attn_bwd(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, st, dO.to(DEV), dQ, dK, dV, ws, cos, sin,
                          None if Q_hist is None else Q_hist.to(DEV), dQh, n_kv=n_kv)
    torch.cuda.synchronize()
    return dQ, dK, dV, dQh


def select(cfg, w, Q, K):
    k = hf.hf_select_k(cfg, w.n_kv)
    idx = torch.full((w.batch, w.heads, w.t_m, k), -1, dtype=torch.int32, device=DEV)
    ws = torch.empty(hf.hf_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=DEV)
    hf.hf_block_select(cfg, Q.to(DEV), K.to(DEV), idx, None, ws)
    torch.cuda.synchronize()
    return idx, k


@pytest.mark.parametrize("name,phi,rope", [("tiny_f32", hf.HF_PHI_RELU, False), ("tiny_f32", hf.HF_PHI_ELU1, True),
                                           ("small_f32_d128", hf.HF_PHI_RELU, True), ("small_bf16", hf.HF_PHI_RELU, False),
                                           ("small_bf16", hf.HF_PHI_ELU1, True), ("small_b128", hf.HF_PHI_RELU, False)])
def test_gradients_of_the_whole_path_match_oracle(name, phi, rope):
    w = wl.get(name)
    cfg = cfg_of(w, phi=phi)
    st, ref_states = make_state(cfg, w, phi, rope)
    Q, K, V = wl.make_qkv(w, q_gain=2.0)
    dO = wl.randn(Q.shape, 91_000 + w.cfg, 1.0, w.torch_dtype)
    qtab = wl.rope_tables(w.n_q, w.head_dim, first_position=float(w.evicted_frames + 2),
                          tokens_per_position=w.tokens_per_frame) if rope else None
    idx, k = select(cfg, w, Q, K)
    dQ, dK, dV, _ = run_bwd(cfg, w, Q, K, V, idx, st, dO, qtab)
    idxc = idx.cpu().numpy()
    cq = None if qtab is None else wl.to_f64(qtab[0])
    sq = None if qtab is None else wl.to_f64(qtab[1])
    gq, gk, gv = wl.to_f64(dQ), wl.to_f64(dK), wl.to_f64(dV)
    for h, (q, kk, v, g) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V), heads_of(dO))):
        rql, rqh, rk, rv = orc.hybrid_attention_bwd(q, kk, v, ref_states[h], w.block, w.block, idxc[0, h], g, phi,
                                                    cq, sq, cfg.eps, cfg.z_scale)
        assert np.abs(rqh).max() > 1e-3 * np.abs(rql).max()        # the history branch's share is really there
        check("dQ", gq[0, h], rql + rqh, w)
        check("dK", gk[0, h], rk, w)
        check("dV", gv[0, h], rv, w)
        # blocks nobody selected: exact zeros
        unused = sorted(set(range(w.t_n)) - set(idxc[0, h].ravel().tolist()))
        for j in unused:
            assert not gk[0, h, j * w.block:(j + 1) * w.block].any() and not gv[0, h, j * w.block:(j + 1) * w.block].any()


@pytest.mark.parametrize("name", ["tiny_f32", "small_bf16"])
def test_split_queries_no_state_and_dense_window(name):
    w = wl.get(name)
    cfg = cfg_of(w)
    st, ref_states = make_state(cfg, w, hf.HF_PHI_RELU, False)
    Q, K, V = wl.make_qkv(w)
    Qh = wl.randn(Q.shape, 92_000 + w.cfg, w.scale, w.torch_dtype)
    dO = wl.randn(Q.shape, 93_000 + w.cfg, 1.0, w.torch_dtype)
    idx, k = select(cfg, w, Q, K)
    idxc = idx.cpu().numpy()
    # split queries: the two gradients go to the two tensors
    dQ, dK, dV, dQh = run_bwd(cfg, w, Q, K, V, idx, st, dO, Q_hist=Qh)
    for h, (q, qh, kk, v, g) in enumerate(zip(heads_of(Q), heads_of(Qh), heads_of(K), heads_of(V), heads_of(dO))):
        rql, rqh, rk, rv = orc.hybrid_attention_bwd(q, kk, v, ref_states[h], w.block, w.block, idxc[0, h], g,
                                                    eps=cfg.eps, z_scale=cfg.z_scale, Q_hist=qh)
        check("dQ", wl.to_f64(dQ)[0, h], rql, w)
        check("dQ_hist", wl.to_f64(dQh)[0, h], rqh, w)
        check("dK", wl.to_f64(dK)[0, h], rk, w)
    # no state: dQ_hist is zero, dQ is the softmax branch alone
    dQ0, _, _, dQh0 = run_bwd(cfg, w, Q, K, V, idx, None, dO, Q_hist=Qh)
    assert not dQh0.float().abs().max().item()
    assert torch.equal(dQ0, dQ)
    # dense window: no index list
    dQd, dKd, dVd, _ = run_bwd(cfg, w, Q, K, V, None, None, dO)
    all_blocks = np.tile(np.arange(w.t_n), (w.t_m, 1))
    for h, (q, kk, v, g) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V), heads_of(dO))):
        rq, rk, rv = orc.sparse_attention_bwd(q, kk, v, all_blocks, w.block, w.block, g)
        check("dQ dense", wl.to_f64(dQd)[0, h], rq, w)
        check("dK dense", wl.to_f64(dKd)[0, h], rk, w)
        check("dV dense", wl.to_f64(dVd)[0, h], rv, w)


def test_gradients_in_a_cache_buffer_layout():
    w = wl.get("small_bf16")
    cap = w.n_kv + 70
    packed, cached = cfg_of(w), cfg_of(w, kv_capacity=cap)
    Q, K, V = wl.make_qkv(w)
    dO = wl.randn(Q.shape, 94_000, 1.0, w.torch_dtype)
    idx, k = select(packed, w, Q, K)
    Kc = torch.zeros((w.batch, w.heads, cap, w.head_dim), dtype=K.dtype)
    Vc = torch.zeros_like(Kc)
    Kc[:, :, :w.n_kv] = K
    Vc[:, :, :w.n_kv] = V
    a = run_bwd(packed, w, Q, K, V, idx, None, dO)
    b = run_bwd(cached, w, Q, Kc, Vc, idx, None, dO, n_kv=w.n_kv)
    assert torch.equal(a[0], b[0])
    assert torch.equal(a[1], b[1][:, :, :w.n_kv]) and torch.equal(a[2], b[2][:, :, :w.n_kv])
    assert b[1][:, :, w.n_kv:].isnan().all()          # nothing behind the valid tokens is written


@pytest.mark.parametrize("name,block_kv,force_generic", [("small_bf16", 64, True), ("small_bf16", 100, False),
                                                         ("small_bf16", 32, False), ("small_b128", 200, False)])
def test_bf16_kernel_choices_and_key_blocks_that_are_no_multiple_of_a_tile(name, block_kv, force_generic):
    """bf16 through the fp32-arithmetic kernels as well, and KV blocks whose length is not a multiple of the
    32-key tile of the matrix-core kernels (a tile then ends inside the next block and must be cut)."""
    w = wl.get(name)
    cfg = cfg_of(w, block_kv=block_kv)
    st, ref_states = make_state(cfg, w, hf.HF_PHI_RELU, False)
    Q, K, V = wl.make_qkv(w, q_gain=1.5)
    dO = wl.randn(Q.shape, 95_000 + block_kv, 1.0, w.torch_dtype)
    k = hf.hf_select_k(cfg, w.n_kv)
    t_n = -(-w.n_kv // block_kv)
    idx = torch.full((w.batch, w.heads, w.t_m, k), -1, dtype=torch.int32, device=DEV)
    ws = torch.empty(hf.hf_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=DEV)
    hf.hf_block_select(cfg, Q.to(DEV), K.to(DEV), idx, None, ws)
    torch.cuda.synchronize()
    if force_generic:
        cfg.flags |= hf.HF_FLAG_BWD_FP32_KERNELS
    dQ, dK, dV, _ = run_bwd(cfg, w, Q, K, V, idx, st, dO)
    idxc = idx.cpu().numpy()
    assert idxc.max() < t_n
    for h, (q, kk, v, g) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V), heads_of(dO))):
        rql, rqh, rk, rv = orc.hybrid_attention_bwd(q, kk, v, ref_states[h], w.block, block_kv, idxc[0, h], g,
                                                    eps=cfg.eps, z_scale=cfg.z_scale)
        check("dQ", wl.to_f64(dQ)[0, h], rql + rqh, w)
        check("dK", wl.to_f64(dK)[0, h], rk, w)
        check("dV", wl.to_f64(dV)[0, h], rv, w)


@pytest.mark.parametrize("name", ["small_bf16", "small_b128", "step_832x480"])
def test_launch_order_of_the_key_side_kernel_changes_no_bit(name):
    """The dK/dV workgroups are launched longest list first, from records that also carry their first list
    entries; in index order (HF_FLAG_DKV_INDEX_ORDER) every workgroup finds the same entries by itself.  A workgroup's
    result does not depend on when it runs, so the two orders must agree bit for bit, and so must two runs."""
    w = wl.get(name)
    cfg = cfg_of(w)
    Q, K, V = wl.make_qkv(w)
    dO = wl.randn(Q.shape, 97_000, 1.0, w.torch_dtype)
    idx, _ = select(cfg, w, Q, K)
    a = run_bwd(cfg, w, Q, K, V, idx, None, dO)
    b = run_bwd(cfg, w, Q, K, V, idx, None, dO)
    cfg.flags |= hf.HF_FLAG_DKV_INDEX_ORDER
    c = run_bwd(cfg, w, Q, K, V, idx, None, dO)
    for x, y, z in zip(a[:3], b[:3], c[:3]):
        assert torch.isfinite(x.float()).all()
        assert torch.equal(x, y) and torch.equal(x, z)


@pytest.mark.parametrize("n_q,n_kv,b", [(1, 1, 64), (5, 70, 64), (64, 64, 64), (129, 257, 128), (33, 100, 16),
                                        (200, 1000, 192)])
def test_backward_ragged_and_degenerate_sizes(n_q, n_kv, b):
    dtype = torch.bfloat16
    cfg = hf.make_config(1, 2, 128, "bf16", b, b, 0.5)
    Q = wl.randn((1, 2, n_q, 128), 911, 0.7, dtype)
    K = wl.randn((1, 2, n_kv, 128), 912, 0.7, dtype)
    V = wl.randn((1, 2, n_kv, 128), 913, 0.7, dtype)
    dO = wl.randn((1, 2, n_q, 128), 914, 1.0, dtype)
    Ke, Ve = wl.randn((1, 2, 37, 128), 915, 0.7, dtype), wl.randn((1, 2, 37, 128), 916, 0.7, dtype)
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    hf.hf_absorb_evicted(cfg, st, Ke.to(DEV), Ve.to(DEV))
    k = hf.hf_select_k(cfg, n_kv)
    t_m = -(-n_q // b)
    idx = torch.empty((1, 2, t_m, k), dtype=torch.int32, device=DEV)
    ws = torch.empty(hf.hf_workspace_bytes(cfg, n_q, n_kv), dtype=torch.uint8, device=DEV)
    hf.hf_block_select(cfg, Q.to(DEV), K.to(DEV), idx, None, ws)
    # rows past the tensors' ends must stay untouched
    gq = torch.full((1, 2, n_q + 3, 128), 7.0, dtype=dtype, device=DEV)
    dQ = gq[:, :, :n_q].contiguous()
    dK = torch.full((1, 2, n_kv, 128), float("nan"), dtype=dtype, device=DEV)
    dV = torch.full((1, 2, n_kv, 128), float("nan"), dtype=dtype, device=DEV)
    bws = torch.empty(hf.hf_bwd_workspace_bytes(cfg, n_q, n_kv), dtype=torch.uint8, device=DEV)
    hf.hf_hybrid_attn_bwd(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, st, dO.to(DEV), dQ, dK, dV, bws)
    torch.cuda.synchronize()
    assert not dK.isnan().any() and not dV.isnan().any()
    states = oracle_state([Ke], [Ve], 128)
    idxc = idx.cpu().numpy()

    class W:          # the bounds helper only looks at the storage type
        dtype = "bf16"
    for h, (q, kk, v, g) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V), heads_of(dO))):
        rql, rqh, rk, rv = orc.hybrid_attention_bwd(q, kk, v, states[h], b, b, idxc[0, h], g)
        check("dQ", wl.to_f64(dQ)[0, h], rql + rqh, W)
        check("dK", wl.to_f64(dK)[0, h], rk, W)
        check("dV", wl.to_f64(dV)[0, h], rv, W)


@pytest.mark.parametrize("seed", range(10))
def test_backward_seeded_random_shapes(seed):
    # every dispatch path of the backward pass (matrix-core and fp32-arithmetic kernels, both feature maps, with and
    # without rotation, split queries, batch > 1, block_q != block_kv) on shapes drawn from a seeded generator
    r = np.random.default_rng(8_000 + seed)
    dtype = ["bf16", "f32"][int(r.integers(0, 2))]
    d = [64, 128][int(r.integers(0, 2))]
    bq = [16, 64, 128][int(r.integers(0, 3))]
    bkv = [16, 48, 64, 128][int(r.integers(0, 4))]
    B, H = int(r.integers(1, 3)), int(r.integers(1, 4))
    n_q, n_kv, n_ev = int(r.integers(1, 260)), int(r.integers(1, 600)), int(r.integers(1, 150))
    phi = [hf.HF_PHI_RELU, hf.HF_PHI_ELU1][int(r.integers(0, 2))]
    rope, split = bool(r.integers(0, 2)), bool(r.integers(0, 2))
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    cfg = hf.make_config(B, H, d, dtype, bq, bkv, float(r.uniform(0.2, 1.0)), phi=phi, z_scale=float(r.uniform(0.3, 2.0)))
    Q = wl.randn((B, H, n_q, d), 8_100 + seed, 0.8, tdt)
    Qh = wl.randn((B, H, n_q, d), 8_200 + seed, 0.8, tdt) if split else None
    K = wl.randn((B, H, n_kv, d), 8_300 + seed, 0.8, tdt)
    V = wl.randn((B, H, n_kv, d), 8_400 + seed, 0.8, tdt)
    dO = wl.randn((B, H, n_q, d), 8_500 + seed, 1.0, tdt)
    Ke, Ve = wl.randn((B, H, n_ev, d), 8_600 + seed, 0.8, tdt), wl.randn((B, H, n_ev, d), 8_700 + seed, 0.8, tdt)
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    hf.hf_absorb_evicted(cfg, st, Ke.to(DEV), Ve.to(DEV))
    tab = wl.rope_tables(n_q, d, first_position=2.0, tokens_per_position=7) if rope else None
    k = hf.hf_select_k(cfg, n_kv)
    t_m = -(-n_q // bq)
    idx = torch.empty((B, H, t_m, k), dtype=torch.int32, device=DEV)
    ws = torch.empty(hf.hf_workspace_bytes(cfg, n_q, n_kv), dtype=torch.uint8, device=DEV)
    hf.hf_block_select(cfg, Q.to(DEV), K.to(DEV), idx, None, ws)

    class W:
        pass
    W.dtype, W.batch, W.heads = dtype, B, H
    dQ, dK, dV, dQh = run_bwd(cfg, W, Q, K, V, idx, st, dO, tab, Qh)
    states = oracle_state([Ke], [Ve], d, phi)
    idxc = idx.cpu().numpy()
    cq = None if tab is None else wl.to_f64(tab[0])
    sq = None if tab is None else wl.to_f64(tab[1])
    qh_heads = heads_of(Qh) if split else [None] * (B * H)
    for n, (q, qh, kk, v, g) in enumerate(zip(heads_of(Q), qh_heads, heads_of(K), heads_of(V), heads_of(dO))):
        b_, h_ = divmod(n, H)
        rql, rqh, rk, rv = orc.hybrid_attention_bwd(q, kk, v, states[n], bq, bkv, idxc[b_, h_], g, phi, cq, sq,
                                                    cfg.eps, cfg.z_scale, Q_hist=qh)
        if split:
            check("dQ", wl.to_f64(dQ)[b_, h_], rql, W)
            check("dQ_hist", wl.to_f64(dQh)[b_, h_], rqh, W)
        else:
            check("dQ", wl.to_f64(dQ)[b_, h_], rql + rqh, W)
        check("dK", wl.to_f64(dK)[b_, h_], rk, W)
        check("dV", wl.to_f64(dV)[b_, h_], rv, W)


def run_fwd_save(cfg, Q, K, V, idx, st, tables=None, Q_hist=None):
    n_q, n_kv = Q.shape[2], K.shape[2]
    O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
    Ol = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
    lse = torch.full((cfg.batch * cfg.heads, n_q), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(hf.hf_workspace_bytes(cfg, n_q, n_kv), dtype=torch.uint8, device=DEV)
    cos, sin = (None, None) if tables is None else (tables[0].to(DEV), tables[1].to(DEV))
    hf.hf_hybrid_attn_fwd_save(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, st, O, Ol, lse, ws, cos, sin,
                               None if Q_hist is None else Q_hist.to(DEV))
    torch.cuda.synchronize()
    return O, Ol, lse


def oracle_lse2(q, kk, idx_rows, block, scale):
    """log2 of the softmax denominator of every query row over the keys of its selected blocks (Eq. 5), written out."""
    out = np.empty(q.shape[0])
    for i in range(q.shape[0]):
        keys = np.concatenate([np.arange(j * block, min((j + 1) * block, kk.shape[0])) for j in idx_rows[i // block]])
        s = (kk[keys] @ q[i]) * scale * np.log2(np.e)
        out[i] = s.max() + np.log2(np.exp2(s - s.max()).sum())
    return out


@pytest.mark.parametrize("name,phi,rope,split,with_state", [("small_bf16", hf.HF_PHI_RELU, False, False, True),
                                                            ("small_bf16", hf.HF_PHI_ELU1, True, True, True),
                                                            ("small_b128", hf.HF_PHI_RELU, False, False, True),
                                                            ("small_bf16", hf.HF_PHI_RELU, False, False, False)])
def test_saving_forward_and_backward_from_saved_statistics(name, phi, rope, split, with_state):
    """The training forward writes the same O as the plain forward plus O_local and the row statistic; the backward
    pass fed with them meets the oracle to the same bounds as the recomputing one."""
    w = wl.get(name)
    cfg = cfg_of(w, phi=phi)
    st, ref_states = make_state(cfg, w, phi, rope) if with_state else (None, [orc.state_zero(w.head_dim)] * w.heads)
    Q, K, V = wl.make_qkv(w, q_gain=2.0)
    Qh = wl.randn(Q.shape, 94_000 + w.cfg, w.scale, w.torch_dtype) if split else None
    dO = wl.randn(Q.shape, 95_000 + w.cfg, 1.0, w.torch_dtype)
    qtab = wl.rope_tables(w.n_q, w.head_dim, first_position=float(w.evicted_frames + 2),
                          tokens_per_position=w.tokens_per_frame) if rope else None
    idx, k = select(cfg, w, Q, K)
    idxc = idx.cpu().numpy()
    O, Ol, lse = run_fwd_save(cfg, Q, K, V, idx, st, qtab, Qh)
    # the plain forward gives the same O, bit for bit
    O2 = torch.empty_like(O)
    ws = torch.empty(hf.hf_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=DEV)
    cos, sin = (None, None) if qtab is None else (qtab[0].to(DEV), qtab[1].to(DEV))
    hf.hf_hybrid_attn_fwd(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, st, O2, ws, cos, sin, None if Qh is None else Qh.to(DEV))
    torch.cuda.synchronize()
    assert torch.equal(O, O2)
    scale = 1.0 / np.sqrt(w.head_dim)
    lse_c = lse.cpu().numpy().astype(np.float64)
    for h, (q, kk, v) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V))):
        ref_l = orc.sparse_attention(q, kk, v, idxc[0, h], w.block, w.block)
        check("O_local", wl.to_f64(Ol)[0, h], ref_l, w)
        assert np.abs(lse_c[h] - oracle_lse2(q, kk, idxc[0, h], w.block, scale)).max() <= 2e-5 * max(1.0, np.abs(lse_c[h]).max())
    if not with_state:
        assert torch.equal(O, Ol)
    # backward from the saved by-products
    dQ = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
    dK, dV = torch.full(K.shape, float("nan"), dtype=K.dtype, device=DEV), torch.full(K.shape, float("nan"), dtype=K.dtype, device=DEV)
    dQh = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV) if split else None
    bws = torch.empty(hf.hf_bwd_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=DEV)
    hf.hf_hybrid_attn_bwd_saved(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, st, dO.to(DEV), Ol, lse, dQ, dK, dV, bws, cos, sin,
                                None if Qh is None else Qh.to(DEV), dQh)
    torch.cuda.synchronize()
    cq = None if qtab is None else wl.to_f64(qtab[0])
    sq = None if qtab is None else wl.to_f64(qtab[1])
    for h, (q, kk, v, g) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V), heads_of(dO))):
        qh = None if Qh is None else heads_of(Qh)[h]
        rql, rqh, rk, rv = orc.hybrid_attention_bwd(q, kk, v, ref_states[h], w.block, w.block, idxc[0, h], g, phi,
                                                    cq, sq, cfg.eps, cfg.z_scale, Q_hist=qh)
        if split:
            check("dQ", wl.to_f64(dQ)[0, h], rql, w)
            check("dQ_hist", wl.to_f64(dQh)[0, h], rqh, w)
        else:
            check("dQ", wl.to_f64(dQ)[0, h], rql + (rqh if with_state else 0.0), w)
        check("dK", wl.to_f64(dK)[0, h], rk, w)
        check("dV", wl.to_f64(dV)[0, h], rv, w)


def test_saving_entry_points_refuse_what_they_do_not_cover():
    w = wl.get("tiny_f32")
    cfg = cfg_of(w)
    Q, K, V = wl.make_qkv(w)
    idx, k = select(cfg, w, Q, K)
    O, Ol = torch.empty_like(Q, device=DEV), torch.empty_like(Q, device=DEV)
    lse = torch.empty((w.batch * w.heads, w.n_q), dtype=torch.float32, device=DEV)
    with pytest.raises(hf.HFError, match="bf16"):
        hf.hf_hybrid_attn_fwd_save(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, None, O, Ol, lse)
    dQ, dK, dV = torch.empty_like(O), torch.empty_like(K, device=DEV), torch.empty_like(K, device=DEV)
    bws = torch.empty(hf.hf_bwd_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=DEV)
    with pytest.raises(hf.HFError, match="bf16"):
        hf.hf_hybrid_attn_bwd_saved(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, None, O, Ol, lse, dQ, dK, dV, bws)
