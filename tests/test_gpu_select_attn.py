"""GPU parity of the one-launch path: Top-K selection (Eq. 4) in the prologue of the attention workgroups
(hf_pool_keys + hf_select_attn_fwd) against the fp64 oracle.  Bounds as for the two-call path: scores within 1e-5,
block lists exact as sets except boundary ties closer than 1e-6 in the oracle, outputs rel-L2 <= 1e-2 and max-abs
<= 2e-2 (bf16) against the oracle's attention over the GPU's own list."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle as orc
import paper_2604_10103_amd as hf
import workloads as wl
from parity import BF16_MAX_ABS, BF16_REL_L2, check_block_idx, heads_of, max_abs, oracle_state, rel_l2

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def cfg_of(w, **kw):
    args = dict(batch=w.batch, heads=w.heads, head_dim=w.head_dim, dtype=w.dtype, block_q=w.block,
                block_kv=w.block, keep_ratio=w.keep_ratio)
    args.update(kw)
    return hf.make_config(**args)


def make_state(cfg, w, rope=False):
    """GPU state (+ its planes) after the workload's evicted frames, and the oracle's states per head."""
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    Ks, Vs = [], []
    for c in range(w.evicted_frames):
        K, V = wl.make_evicted(w, c, w.tokens_per_frame)
        Ks.append(K); Vs.append(V)
        hf.hf_absorb_evicted(cfg, st, K.to(DEV), V.to(DEV))
    planes = torch.empty(hf.hf_state_planes_bytes(cfg), dtype=torch.uint8, device=DEV)
    hf.hf_state_planes(cfg, st, planes)
    return st, planes, oracle_state(Ks, Vs, w.head_dim, cfg.phi)


def run_one_launch(cfg, w, Q, K, V, st, planes, want_scores=True, tables=None, Q_hist=None, n_cached=0, pooled=None):
    n_q, n_kv = Q.shape[2], K.shape[2]
    k = hf.hf_select_k(cfg, n_kv)
    t_m, t_n = -(-n_q // cfg.block_q), -(-n_kv // cfg.block_kv)
    if pooled is None:
        pooled = torch.full((hf.hf_pooled_keys_bytes(cfg, n_kv),), 0xFF, dtype=torch.uint8, device=DEV)   # NaN bytes
    idx = torch.full((w.batch, w.heads, t_m, k), -1, dtype=torch.int32, device=DEV)
    scores = torch.full((w.batch, w.heads, t_m, t_n), float("nan"), dtype=torch.float32, device=DEV) if want_scores else None
    O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
    Kd = K.to(DEV)
    hf.hf_pool_keys(cfg, Kd, pooled, n_cached)
    cos, sin = (None, None) if tables is None else (tables[0].to(DEV), tables[1].to(DEV))
    hf.hf_select_attn_fwd(cfg, Q.to(DEV), Kd, V.to(DEV), pooled, st, planes, O, idx, scores, cos, sin,
                          None if Q_hist is None else Q_hist.to(DEV))
    torch.cuda.synchronize()
    return O, idx, scores, k, pooled


def check_against_oracle(cfg, w, Q, K, V, O, idx, scores, k, states, tables=None, Q_hist=None, block=None):
    b = block or w.block
    Og, idxc = wl.to_f64(O), idx.cpu().numpy()
    sc = None if scores is None else scores.cpu().numpy().astype(np.float64)
    cq = None if tables is None else wl.to_f64(tables[0])
    sq = None if tables is None else wl.to_f64(tables[1])
    qh = heads_of(Q_hist) if Q_hist is not None else [None] * len(heads_of(Q))
    assert not O.isnan().any()
    for h, (q, kk, v) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V))):
        A = orc.block_scores(q, kk, b, b)
        if sc is not None:
            assert np.abs(sc[0, h] - A).max() <= 1e-5 * max(1.0, np.abs(A).max())
        check_block_idx(idxc[0, h], A, k)
        if states is None:
            ref = orc.sparse_attention(q, kk, v, idxc[0, h], b, b)
        elif qh[h] is None:
            ref, *_ = orc.hybrid_attention(q, kk, v, states[h], b, b, k, cfg.phi, cq, sq, cfg.eps, cfg.z_scale,
                                           block_idx=idxc[0, h])
        else:
            ref = orc.sparse_attention(q, kk, v, idxc[0, h], b, b) + orc.history_readout(
                qh[h], states[h][0], states[h][1], cfg.phi, cq, sq, cfg.eps, cfg.z_scale)
        assert rel_l2(Og[0, h], ref) <= BF16_REL_L2, (h, rel_l2(Og[0, h], ref))
        assert max_abs(Og[0, h], ref) <= BF16_MAX_ABS


@pytest.mark.parametrize("name", ["small_bf16", "small_b128"])
@pytest.mark.parametrize("with_state", [False, True])
def test_selection_inside_the_attention_launch(name, with_state):
    w = wl.get(name)
    cfg = cfg_of(w)
    st, planes, states = make_state(cfg, w) if with_state else (None, None, None)
    Q, K, V = wl.make_qkv(w, q_gain=2.0)
    O, idx, scores, k, _ = run_one_launch(cfg, w, Q, K, V, st, planes)
    assert k == orc.select_k(w.keep_ratio, w.t_n)
    check_against_oracle(cfg, w, Q, K, V, O, idx, scores, k, states)


def test_one_launch_equals_the_two_call_path_on_its_own_list():
    """Fed with the list the one-launch path chose, hf_hybrid_attn_fwd_planes gives the same output bit for bit:
    the prologue changes which blocks are read, nothing in the arithmetic behind it."""
    w = wl.get("small_bf16")
    cfg = cfg_of(w)
    st, planes, _ = make_state(cfg, w)
    Q, K, V = wl.make_qkv(w)
    O, idx, _, k, _ = run_one_launch(cfg, w, Q, K, V, st, planes, want_scores=False)
    O2 = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
    hf.hf_hybrid_attn_fwd_planes(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), idx, st, planes, O2)
    torch.cuda.synchronize()
    assert torch.equal(O, O2)
    # and the stand-alone selection chooses the same sets (no boundary ties in this draw)
    idx2 = torch.empty_like(idx)
    ws = torch.empty(hf.hf_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=DEV)
    hf.hf_block_select(cfg, Q.to(DEV), K.to(DEV), idx2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2)


def test_one_launch_with_rotation_elu_and_split_queries():
    w = wl.get("small_bf16")
    cfg = cfg_of(w, phi=hf.HF_PHI_ELU1)
    st, planes, states = make_state(cfg, w)
    Q, K, V = wl.make_qkv(w)
    Qh = wl.randn(Q.shape, 97_000 + w.cfg, w.scale, w.torch_dtype)
    qtab = wl.rope_tables(w.n_q, w.head_dim, first_position=float(w.evicted_frames + 2),
                          tokens_per_position=w.tokens_per_frame)
    O, idx, scores, k, _ = run_one_launch(cfg, w, Q, K, V, st, planes, tables=qtab, Q_hist=Qh)
    check_against_oracle(cfg, w, Q, K, V, O, idx, scores, k, states, tables=qtab, Q_hist=Qh)


def test_one_launch_exact_ties_and_keep_all():
    # identical key blocks give exactly tied scores: the lower index must win
    w = wl.get("small_bf16")
    cfg = cfg_of(w, keep_k=3)
    Q, K, V = wl.make_qkv(w)
    K[:, :, 64:128] = K[:, :, 0:64]
    K[:, :, 128:192] = K[:, :, 0:64]
    O, idx, scores, k, _ = run_one_launch(cfg, w, Q, K, V, None, None)
    idxc = idx.cpu().numpy()
    for h, (q, kk) in enumerate(zip(heads_of(Q), heads_of(K))):
        ref, _ = orc.select_blocks(orc.block_scores(q, kk, w.block, w.block), 3)
        assert np.array_equal(idxc[0, h], ref)
    check_against_oracle(cfg, w, Q, K, V, O, idx, scores, k, None)
    cfg = cfg_of(w, keep_ratio=1.0)
    O, idx, _, k, _ = run_one_launch(cfg, w, Q, K, V, None, None, want_scores=False)
    assert k == w.t_n
    assert np.array_equal(idx.cpu().numpy(), np.broadcast_to(np.arange(k, dtype=np.int32), idx.shape))
    for h, (q, kk, v) in enumerate(zip(heads_of(Q), heads_of(K), heads_of(V))):
        assert rel_l2(wl.to_f64(O)[0, h], orc.dense_attention(q, kk, v)) <= BF16_REL_L2


@pytest.mark.parametrize("n_q,n_kv,b", [(1, 1, 64), (5, 70, 64), (64, 64, 64), (129, 257, 128), (200, 1000, 64),
                                        (520, 4100, 64), (300, 2100, 128), (130, 12000, 64), (70, 19300, 64),
                                        (300, 40000, 128)])
def test_one_launch_ragged_and_degenerate_sizes(n_q, n_kv, b):
    base = wl.get("small_bf16")
    w = dataclasses.replace(base, heads=2, block=b)
    cfg = cfg_of(w, keep_ratio=0.3)
    Q = wl.randn((1, 2, n_q, 128), 71_000 + n_q, 0.5, torch.bfloat16)
    K = wl.randn((1, 2, n_kv, 128), 72_000 + n_kv, 0.5, torch.bfloat16)
    V = wl.randn((1, 2, n_kv, 128), 73_000 + n_kv, 0.5, torch.bfloat16)
    O, idx, scores, k, _ = run_one_launch(cfg, w, Q, K, V, None, None)
    check_against_oracle(cfg, w, Q, K, V, O, idx, scores, k, None, block=b)


def test_one_launch_with_reused_pooled_keys():
    # denoising steps of one chunk: the pooled keys of the older whole blocks stay in the caller's buffer
    w = wl.get("small_bf16")
    cfg = cfg_of(w)
    st, planes, states = make_state(cfg, w)
    Q0, K0, V0 = wl.make_qkv(w, step=0)
    _, _, _, k, pooled = run_one_launch(cfg, w, Q0, K0, V0, st, planes)
    half = w.n_kv - w.n_q
    reuse = half // w.block
    assert 0 < reuse < w.t_n
    for step in (1, 2):
        Q, Kn, Vn = wl.make_qkv(w, step=step)
        K = torch.cat([K0[:, :, :half], Kn[:, :, half:]], dim=2).contiguous()
        V = torch.cat([V0[:, :, :half], Vn[:, :, half:]], dim=2).contiguous()
        O, idx, scores, k, pooled = run_one_launch(cfg, w, Q, K, V, st, planes, n_cached=reuse, pooled=pooled)
        check_against_oracle(cfg, w, Q, K, V, O, idx, scores, k, states)


def test_one_launch_rejects_what_it_does_not_cover():
    w = wl.get("tiny_f32")
    cfg = cfg_of(w)
    Q, K, V = (t.to(DEV) for t in wl.make_qkv(w))
    pooled = torch.empty(hf.hf_pooled_keys_bytes(cfg, w.n_kv), dtype=torch.uint8, device=DEV)
    hf.hf_pool_keys(cfg, K, pooled)          # pooling itself covers every configuration
    k = hf.hf_select_k(cfg, w.n_kv)
    idx = torch.empty((w.batch, w.heads, w.t_m, k), dtype=torch.int32, device=DEV)
    with pytest.raises(hf.HFError):
        hf.hf_select_attn_fwd(cfg, Q, K, V, pooled, None, None, torch.empty_like(Q), idx)
    # more KV blocks than the kernel ranks in its tile space
    w = dataclasses.replace(wl.get("small_bf16"), heads=1, block=64)
    cfg = cfg_of(w)
    n_kv = 64 * 1025
    Q = torch.zeros((1, 1, 64, 128), dtype=torch.bfloat16, device=DEV)
    K = torch.zeros((1, 1, n_kv, 128), dtype=torch.bfloat16, device=DEV)
    pooled = torch.empty(hf.hf_pooled_keys_bytes(cfg, n_kv), dtype=torch.uint8, device=DEV)
    idx = torch.empty((1, 1, 1, hf.hf_select_k(cfg, n_kv)), dtype=torch.int32, device=DEV)
    with pytest.raises(hf.HFError):
        hf.hf_select_attn_fwd(cfg, Q, K, K, pooled, None, None, torch.empty_like(Q), idx)


def test_one_launch_832x480_all_heads():
    """The launch configuration bench.py times: every head of the 832x480 layer step against the oracle."""
    w = wl.get("step_832x480")
    cfg = cfg_of(w)
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    planes = torch.empty(hf.hf_state_planes_bytes(cfg), dtype=torch.uint8, device=DEV)
    aws = torch.empty(hf.hf_absorb_workspace_bytes(cfg, w.n_q), dtype=torch.uint8, device=DEV)
    Ks, Vs = [], []
    for c in range(w.evicted_frames // w.chunk_frames):
        K, V = wl.make_evicted(w, c)
        Ks.append(K); Vs.append(V)
        hf.hf_absorb_evicted_planes(cfg, st, K.to(DEV), V.to(DEV), planes, workspace=aws)
    states = oracle_state(Ks, Vs, w.head_dim)
    Q, K, V = wl.make_qkv(w)
    O, idx, scores, k, _ = run_one_launch(cfg, w, Q, K, V, st, planes)
    assert k == 37 and w.t_m == 74 and w.t_n == 147
    check_against_oracle(cfg, w, Q, K, V, O, idx, scores, k, states)


def test_one_launch_large_shape_head_subset():
    """1280x720-like shape (block 128, four wavefronts per workgroup, several rounds of workgroups: the list is read
    back from memory for the tiles behind the first 64)."""
    w = wl.get("large_1280x720")
    heads = (0, 13, 39)
    sub = dataclasses.replace(w, heads=len(heads))
    cfg = cfg_of(sub)
    Q, K, V = wl.make_qkv(w)
    Q, K, V = (t[:, list(heads)].contiguous() for t in (Q, K, V))
    O, idx, scores, k, _ = run_one_launch(cfg, sub, Q, K, V, None, None)
    assert k == 43
    check_against_oracle(cfg, sub, Q, K, V, O, idx, scores, k, None)


# ------------------------------------------------------------------ Eq. 2 in workgroups of the same launch
def run_step(cfg, w, Q, K, V, st, planes, Ke, Ve, n_ev=None, scores=False):
    n_q, n_kv = Q.shape[2], K.shape[2]
    k = hf.hf_select_k(cfg, n_kv)
    t_m, t_n = -(-n_q // cfg.block_q), -(-n_kv // cfg.block_kv)
    pooled = torch.empty(hf.hf_pooled_keys_bytes(cfg, n_kv), dtype=torch.uint8, device=DEV)
    idx = torch.full((w.batch, w.heads, t_m, k), -1, dtype=torch.int32, device=DEV)
    sc = torch.empty((w.batch, w.heads, t_m, t_n), dtype=torch.float32, device=DEV) if scores else None
    O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
    st_out = torch.full((hf.hf_state_bytes(cfg) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    pl_out = torch.full((hf.hf_state_planes_bytes(cfg),), 0xFF, dtype=torch.uint8, device=DEV)
    ne = Ke.shape[2] if n_ev is None else n_ev
    ws = torch.full((hf.hf_step_workspace_bytes(cfg, n_q, ne),), 0xFF, dtype=torch.uint8, device=DEV)   # needs no init
    Kd = K.to(DEV)
    hf.hf_pool_keys(cfg, Kd, pooled)
    hf.hf_step_fwd(cfg, Q.to(DEV), Kd, V.to(DEV), pooled, st, planes, O, idx, Ke.to(DEV), Ve.to(DEV), st_out, pl_out, ws,
                   scores=sc, n_ev=n_ev)
    torch.cuda.synchronize()
    return O, idx, sc, k, st_out, pl_out, pooled


def check_state(cfg, w, st_out, pl_out, ref_states):
    from parity import split_state
    Lg, zg = split_state(st_out, w.batch * w.heads, w.head_dim)
    assert rel_l2(Lg, np.stack([s[0] for s in ref_states])) <= 1e-5
    assert rel_l2(zg, np.stack([s[1] for s in ref_states])) <= 1e-5
    # the planes are the planes of exactly that state
    ref_pl = torch.empty_like(pl_out)
    hf.hf_state_planes(cfg, st_out, ref_pl)
    torch.cuda.synchronize()
    assert torch.equal(pl_out, ref_pl)


@pytest.mark.parametrize("name", ["small_bf16", "small_b128"])
@pytest.mark.parametrize("with_state", [True, False])
def test_step_absorbs_next_to_the_attention(name, with_state):
    w = wl.get(name)
    cfg = cfg_of(w)
    st, planes, states = make_state(cfg, w) if with_state else (None, None, None)
    Q, K, V = wl.make_qkv(w, q_gain=2.0)
    Ke, Ve = wl.make_evicted(w, w.evicted_frames + 1, w.n_q)          # the chunk the next eviction removes
    before = None if st is None else st.clone()
    O, idx, sc, k, st_out, pl_out, pooled = run_step(cfg, w, Q, K, V, st, planes, Ke, Ve, scores=True)
    # the attention of this launch read the OLD state
    check_against_oracle(cfg, w, Q, K, V, O, idx, sc, k, states)
    if st is not None:
        assert torch.equal(st, before)
    # ... and is bit for bit the launch without the absorbing workgroups
    O2 = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
    idx2 = torch.empty_like(idx)
    hf.hf_select_attn_fwd(cfg, Q.to(DEV), K.to(DEV), V.to(DEV), pooled, st, planes, O2, idx2)
    torch.cuda.synchronize()
    assert torch.equal(O, O2) and torch.equal(idx, idx2)
    # the new state holds the old one plus the chunk
    base = states if states is not None else [orc.state_zero(w.head_dim) for _ in range(w.batch * w.heads)]
    ref = [orc.state_absorb(L, z, kk, vv) for (L, z), kk, vv in zip(base, heads_of(Ke), heads_of(Ve))]
    check_state(cfg, w, st_out, pl_out, ref)


@pytest.mark.parametrize("n_ev,stride", [(1, 1), (17, 40), (333, 333), (1000, 1200)])
def test_step_absorbs_ragged_token_counts_of_a_strided_buffer(n_ev, stride):
    w = wl.get("small_bf16")
    cfg = cfg_of(w)
    st, planes, states = make_state(cfg, w)
    Q, K, V = wl.make_qkv(w)
    Ke = wl.randn((w.batch, w.heads, stride, w.head_dim), 98_000 + n_ev, w.scale, w.torch_dtype)
    Ve = wl.randn((w.batch, w.heads, stride, w.head_dim), 98_500 + n_ev, w.scale, w.torch_dtype)
    O, idx, _, k, st_out, pl_out, _ = run_step(cfg, w, Q, K, V, st, planes, Ke, Ve, n_ev=n_ev)
    ref = [orc.state_absorb(L, z, kk[:n_ev], vv[:n_ev]) for (L, z), kk, vv in zip(states, heads_of(Ke), heads_of(Ve))]
    check_state(cfg, w, st_out, pl_out, ref)
    check_against_oracle(cfg, w, Q, K, V, O, idx, None, k, states)


def test_step_rejects_overlapping_state_buffers_and_other_feature_maps():
    w = wl.get("small_bf16")
    cfg = cfg_of(w)
    st, planes, _ = make_state(cfg, w)
    Q, K, V = (t.to(DEV) for t in wl.make_qkv(w))
    Ke, Ve = (t.to(DEV) for t in wl.make_evicted(w, 9, w.n_q))
    k = hf.hf_select_k(cfg, w.n_kv)
    pooled = torch.empty(hf.hf_pooled_keys_bytes(cfg, w.n_kv), dtype=torch.uint8, device=DEV)
    hf.hf_pool_keys(cfg, K, pooled)
    idx = torch.empty((w.batch, w.heads, w.t_m, k), dtype=torch.int32, device=DEV)
    O = torch.empty_like(Q)
    ws = torch.empty(hf.hf_step_workspace_bytes(cfg, w.n_q, w.n_q), dtype=torch.uint8, device=DEV)
    pl2 = torch.empty_like(planes)
    with pytest.raises(hf.HFError):   # in place: the attention would read a state that is being written
        hf.hf_step_fwd(cfg, Q, K, V, pooled, st, planes, O, idx, Ke, Ve, st, pl2, ws)
    with pytest.raises(hf.HFError):
        hf.hf_step_fwd(cfg, Q, K, V, pooled, st, planes, O, idx, Ke, Ve, torch.empty_like(st), planes, ws)
    with pytest.raises(hf.HFError):   # workspace too small
        hf.hf_step_fwd(cfg, Q, K, V, pooled, st, planes, O, idx, Ke, Ve, torch.empty_like(st), pl2, ws[:1024])
    cfg_elu = cfg_of(w, phi=hf.HF_PHI_ELU1)
    with pytest.raises(hf.HFError):
        hf.hf_step_fwd(cfg_elu, Q, K, V, pooled, st, planes, O, idx, Ke, Ve, torch.empty_like(st), pl2, ws)


def test_step_832x480_state_and_output_twice():
    """The launch bench.py times: select + attend on the old state, absorb a 4680-token chunk into the new one.  Two
    launches on the same workspace give the same bits (the partials meet in slice order; the arrival counters need
    no reset)."""
    w = wl.get("step_832x480")
    cfg = cfg_of(w)
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    planes = torch.empty(hf.hf_state_planes_bytes(cfg), dtype=torch.uint8, device=DEV)
    aws = torch.empty(hf.hf_absorb_workspace_bytes(cfg, w.n_q), dtype=torch.uint8, device=DEV)
    Ks, Vs = [], []
    for c in range(2):
        K, V = wl.make_evicted(w, c)
        Ks.append(K); Vs.append(V)
        hf.hf_absorb_evicted_planes(cfg, st, K.to(DEV), V.to(DEV), planes, workspace=aws)
    states = oracle_state(Ks, Vs, w.head_dim)
    Ke, Ve = wl.make_evicted(w, 2)
    Q, K, V = wl.make_qkv(w)
    n_q, n_kv = w.n_q, w.n_kv
    k = hf.hf_select_k(cfg, n_kv)
    pooled = torch.empty(hf.hf_pooled_keys_bytes(cfg, n_kv), dtype=torch.uint8, device=DEV)
    idx = torch.empty((w.batch, w.heads, w.t_m, k), dtype=torch.int32, device=DEV)
    ws = torch.empty(hf.hf_step_workspace_bytes(cfg, n_q, w.n_q), dtype=torch.uint8, device=DEV)
    Qd, Kd, Vd, Ked, Ved = (t.to(DEV) for t in (Q, K, V, Ke, Ve))
    hf.hf_pool_keys(cfg, Kd, pooled)
    outs = []
    for rep in range(2):
        O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
        st_out = torch.full_like(st, float("nan"))
        pl_out = torch.empty_like(planes)
        hf.hf_step_fwd(cfg, Qd, Kd, Vd, pooled, st, planes, O, idx, Ked, Ved, st_out, pl_out, ws)
        torch.cuda.synchronize()
        outs.append((O, st_out, pl_out, idx.clone()))
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)
    O, st_out, pl_out, idxc = outs[0]
    check_against_oracle(cfg, w, Q, K, V, O, idxc, None, k, states)
    ref = [orc.state_absorb(L, z, kk, vv) for (L, z), kk, vv in zip(states, heads_of(Ke), heads_of(Ve))]
    check_state(cfg, w, st_out, pl_out, ref)


def test_streaming_200_chunks_through_the_two_launch_step():
    """200 chunks at the 832x480 shape with the state carried by hf_step_fwd alone: every chunk's step attends with the
    current state and absorbs the chunk that the next arrival evicts into the other of two state buffers, which then
    swap.  The state is compared with the oracle's after every chunk (fp32 accumulation of exact bf16 products: far
    below the bound and not growing with the stream); lists and outputs on sampled chunks."""
    from parity import split_state
    w = wl.get("step_832x480")
    cfg = cfg_of(w)
    n_chunk, n_chunks, pool_size = w.n_q, 200, 8
    pool = [wl.make_evicted(w, 200 + i) for i in range(pool_size)]
    pool_dev = [(k.to(DEV), v.to(DEV)) for k, v in pool]
    pool64 = [([wl.to_f64(k[0, h]) for h in range(w.heads)], [wl.to_f64(v[0, h]) for h in range(w.heads)])
              for k, v in pool]
    win = [0, 1]                      # window = [older chunk | current chunk]
    states = [orc.state_zero(w.head_dim) for _ in range(w.heads)]
    st = [torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV) for _ in range(2)]
    pl = [torch.empty(hf.hf_state_planes_bytes(cfg), dtype=torch.uint8, device=DEV) for _ in range(2)]
    hf.hf_state_init(cfg, st[0])
    hf.hf_state_planes(cfg, st[0], pl[0])
    cur = 0
    k = hf.hf_select_k(cfg, w.n_kv)
    pooled = torch.empty(hf.hf_pooled_keys_bytes(cfg, w.n_kv), dtype=torch.uint8, device=DEV)
    sws = torch.empty(hf.hf_step_workspace_bytes(cfg, n_chunk, n_chunk), dtype=torch.uint8, device=DEV)
    idx = torch.empty((w.batch, w.heads, w.t_m, k), dtype=torch.int32, device=DEV)
    O = torch.empty((w.batch, w.heads, n_chunk, w.head_dim), dtype=w.torch_dtype, device=DEV)
    q_pool = [wl.randn(O.shape, 76_000 + i, w.scale, w.torch_dtype).to(DEV) for i in range(3)]
    sampled = {1, 2, 50, 100, 200}
    errs_L, errs_z = [], []
    Kw = torch.cat([pool_dev[win[0]][0], pool_dev[win[1]][0]], dim=2).contiguous()
    Vw = torch.cat([pool_dev[win[0]][1], pool_dev[win[1]][1]], dim=2).contiguous()
    for c in range(1, n_chunks + 1):
        Q = wl.randn(O.shape, 77_000 + c, w.scale, w.torch_dtype) if c in sampled else None
        hf.hf_pool_keys(cfg, Kw, pooled)
        # the older half of the window is what the next chunk's arrival evicts: absorbed beside this chunk's attention
        Kev, Vev = pool_dev[win[0]]
        hf.hf_step_fwd(cfg, q_pool[c % 3] if Q is None else Q.to(DEV), Kw, Vw, pooled, st[cur], pl[cur], O, idx, Kev, Vev,
                       st[1 - cur], pl[1 - cur], sws)
        torch.cuda.synchronize()
        if Q is not None:
            Kc = torch.cat([pool[win[0]][0], pool[win[1]][0]], dim=2)
            Vc = torch.cat([pool[win[0]][1], pool[win[1]][1]], dim=2)
            heads = [c % w.heads, (c + 5) % w.heads]
            Og, idxc = wl.to_f64(O), idx.cpu().numpy()
            for h in heads:
                q, kk, v = wl.to_f64(Q[0, h]), wl.to_f64(Kc[0, h]), wl.to_f64(Vc[0, h])
                check_block_idx(idxc[0, h], orc.block_scores(q, kk, w.block, w.block), k)
                ref, *_ = orc.hybrid_attention(q, kk, v, states[h], w.block, w.block, k, eps=cfg.eps, block_idx=idxc[0, h])
                assert rel_l2(Og[0, h], ref) <= BF16_REL_L2 and max_abs(Og[0, h], ref) <= BF16_MAX_ABS
        k64, v64 = pool64[win[0]]
        states = [orc.state_absorb(Ls, zs, k64[h], v64[h]) for h, (Ls, zs) in enumerate(states)]
        cur = 1 - cur
        win = [win[1], (win[1] + 1) % pool_size]
        Kw[:, :, :n_chunk] = pool_dev[win[0]][0]
        Vw[:, :, :n_chunk] = pool_dev[win[0]][1]
        Kw[:, :, n_chunk:] = pool_dev[win[1]][0]
        Vw[:, :, n_chunk:] = pool_dev[win[1]][1]
        Lg, zg = split_state(st[cur], w.heads, w.head_dim)
        errs_L.append(rel_l2(Lg, np.stack([s[0] for s in states])))
        errs_z.append(rel_l2(zg, np.stack([s[1] for s in states])))
    assert max(errs_L) <= 1e-5 and max(errs_z) <= 1e-5, (max(errs_L), max(errs_z))
    assert errs_L[-1] <= 4 * max(errs_L[:20]) + 1e-7
    ref_pl = torch.empty_like(pl[cur])
    hf.hf_state_planes(cfg, st[cur], ref_pl)
    torch.cuda.synchronize()
    assert torch.equal(pl[cur], ref_pl)


def test_step_large_shape_head_subset():
    """1280x720-like shape, three heads: four wavefronts per workgroup, the list read back from memory behind the first
    64 tiles, and three frames (10 800 tokens per head) absorbed beside the attention."""
    w = wl.get("large_1280x720")
    heads = (0, 13, 39)
    sub = dataclasses.replace(w, heads=len(heads))
    cfg = cfg_of(sub)
    Q, K, V = wl.make_qkv(w)
    Q, K, V = (t[:, list(heads)].contiguous() for t in (Q, K, V))
    Ke0, Ve0 = (t[:, list(heads)].contiguous() for t in wl.make_evicted(w, 0))
    Ke1, Ve1 = (t[:, list(heads)].contiguous() for t in wl.make_evicted(w, 1))
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    planes = torch.empty(hf.hf_state_planes_bytes(cfg), dtype=torch.uint8, device=DEV)
    hf.hf_absorb_evicted_planes(cfg, st, Ke0.to(DEV), Ve0.to(DEV), planes)
    states = oracle_state([Ke0], [Ve0], w.head_dim)
    O, idx, _, k, st_out, pl_out, _ = run_step(cfg, sub, Q, K, V, st, planes, Ke1, Ve1)
    assert k == 43 and Ke1.shape[2] == 10800
    check_against_oracle(cfg, sub, Q, K, V, O, idx, None, k, states)
    ref = [orc.state_absorb(L, z, kk, vv) for (L, z), kk, vv in zip(states, heads_of(Ke1), heads_of(Ve1))]
    check_state(cfg, sub, st_out, pl_out, ref)
