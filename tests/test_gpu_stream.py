"""The rolling KV cache of the inference algorithm of the supplement as library calls: a cache buffer with
spare capacity, sink frames that are never evicted, eviction into the linear state when a chunk does not fit,
several denoising steps per chunk.  Checked step by step against an oracle loop that keeps the cache as lists."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2604_10103_amd as hf
import workloads as wl
from parity import BF16_MAX_ABS, BF16_REL_L2, F32_REL_L2, check_block_idx, max_abs, rel_l2, split_state

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def cfg_of(w, **kw):
    args = dict(batch=w.batch, heads=w.heads, head_dim=w.head_dim, dtype=w.dtype, block_q=w.block,
                block_kv=w.block, keep_ratio=w.keep_ratio)
    args.update(kw)
    return hf.make_config(**args)


@pytest.mark.parametrize("name", ["tiny_f32", "small_bf16", "small_b128"])
def test_cache_buffer_with_spare_capacity_equals_the_packed_window(name):
    w = wl.get(name)
    Q, K, V = wl.make_qkv(w)
    cap = w.n_kv + 3 * w.block + 5
    packed, cached = cfg_of(w), cfg_of(w, kv_capacity=cap)
    Kc = torch.full((w.batch, w.heads, cap, w.head_dim), float("nan"), dtype=K.dtype)
    Vc = torch.full_like(Kc, float("nan"))            # whatever lies behind the valid tokens is never read
    Kc[:, :, :w.n_kv] = K
    Vc[:, :, :w.n_kv] = V
    st = torch.empty(hf.hf_state_bytes(packed) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(packed, st)
    Ke, Ve = wl.make_evicted(w, 0)
    hf.hf_absorb_evicted(packed, st, Ke.to(DEV), Ve.to(DEV))
    k = hf.hf_select_k(packed, w.n_kv)
    outs = []
    for cfg, Kd, Vd, n in ((packed, K.to(DEV), V.to(DEV), None), (cached, Kc.to(DEV), Vc.to(DEV), w.n_kv)):
        idx = torch.full((w.batch, w.heads, w.t_m, k), -1, dtype=torch.int32, device=DEV)
        ws = torch.empty(hf.hf_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=DEV)
        O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
        hf.hf_block_select(cfg, Q.to(DEV), Kd, idx, None, ws, n_kv=n)
        hf.hf_hybrid_attn_fwd(cfg, Q.to(DEV), Kd, Vd, idx, st, O, ws, n_kv=n)
        torch.cuda.synchronize()
        outs.append((idx.cpu(), O.cpu()))
    assert torch.equal(outs[0][0], outs[1][0])
    assert torch.equal(outs[0][1], outs[1][1]) and not outs[1][1].isnan().any()


@pytest.mark.parametrize("name,sink_frames,rope", [("small_bf16", 1, False), ("small_bf16", 0, True),
                                                   ("tiny_f32", 2, True), ("small_b128", 1, False)])
def test_stream_with_sink_frames_matches_the_oracle_loop(name, sink_frames, rope):
    w = wl.get(name)
    H, d, tpf = w.heads, w.head_dim, w.tokens_per_frame
    n_chunk = w.n_q
    n_sink = sink_frames * tpf
    cap = n_sink + 2 * n_chunk + tpf            # sink + two cached chunks and a frame + ... : evictions are ragged
    cfg = cfg_of(w, kv_capacity=cap)
    win = hf.hf_window(n_sink, n_sink)
    Kw = torch.zeros((w.batch, H, cap, d), dtype=w.torch_dtype, device=DEV)
    Vw = torch.zeros_like(Kw)
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    aws_n = hf.hf_absorb_workspace_bytes(cfg, n_chunk)
    aws = torch.empty(aws_n, dtype=torch.uint8, device=DEV) if aws_n else None
    ws = torch.empty(hf.hf_workspace_bytes(cfg, n_chunk, cap), dtype=torch.uint8, device=DEV)
    O = torch.empty((w.batch, H, n_chunk, d), dtype=w.torch_dtype, device=DEV)

    # oracle side: the cache as per-head lists of fp64 rows, the state as (L, z) per head
    cacheK = [np.zeros((0, d)) for _ in range(H)]
    cacheV = [np.zeros((0, d)) for _ in range(H)]
    states = [orc.state_zero(d) for _ in range(H)]
    if n_sink:
        Ks, Vs = wl.make_evicted(w, 900, n_sink)
        Kw[:, :, :n_sink] = Ks.to(DEV)
        Vw[:, :, :n_sink] = Vs.to(DEV)
        for h in range(H):
            cacheK[h], cacheV[h] = wl.to_f64(Ks[0, h]), wl.to_f64(Vs[0, h])
    rl, ma = (BF16_REL_L2, BF16_MAX_ABS) if w.dtype == "bf16" else (F32_REL_L2, 1e-4)
    total_evicted = 0
    for c in range(6):
        over = max(0, win.n_tokens + n_chunk - cap)
        tab_ev = wl.rope_tables(over, d, first_position=3.0 + c) if (rope and over) else (None, None)
        first, n_ev = hf.hf_stream_open_chunk(cfg, win, n_chunk, Kw, Vw, st, *(None if t is None else t.to(DEV) for t in tab_ev),
                                              workspace=aws)
        assert n_ev == over
        total_evicted += n_ev
        for h in range(H):                   # pop(0) behind the sink, update the linear state
            if over:
                ek, ev = cacheK[h][n_sink:n_sink + over], cacheV[h][n_sink:n_sink + over]
                states[h] = orc.state_absorb(*states[h], ek, ev, orc.PHI_RELU,
                                             None if tab_ev[0] is None else wl.to_f64(tab_ev[0]),
                                             None if tab_ev[1] is None else wl.to_f64(tab_ev[1]))
                cacheK[h] = np.concatenate([cacheK[h][:n_sink], cacheK[h][n_sink + over:]])
                cacheV[h] = np.concatenate([cacheV[h][:n_sink], cacheV[h][n_sink + over:]])
            assert first == cacheK[h].shape[0]
        n_kv = win.n_tokens
        k = hf.hf_select_k(cfg, n_kv)
        idx = torch.full((w.batch, H, w.t_m, k), -1, dtype=torch.int32, device=DEV)
        tab_q = wl.rope_tables(n_chunk, d, first_position=9.0) if rope else (None, None)
        for step in range(3):               # the chunk's own K, V change with every denoising step
            Kn, Vn = wl.make_evicted(w, 1000 + 10 * c + step, n_chunk)
            Q = wl.randn((w.batch, H, n_chunk, d), 88_000 + 10 * c + step, w.scale, w.torch_dtype)
            Kw[:, :, first:first + n_chunk] = Kn.to(DEV)
            Vw[:, :, first:first + n_chunk] = Vn.to(DEV)
            hf.hf_stream_step(cfg, win, Q.to(DEV), Kw, Vw, step, idx, st, O, ws,
                              *(None if t is None else t.to(DEV) for t in tab_q))
            torch.cuda.synchronize()
            Og, idxc = wl.to_f64(O), idx.cpu().numpy()
            for h in range(H):
                kk = np.concatenate([cacheK[h], wl.to_f64(Kn[0, h])])
                vv = np.concatenate([cacheV[h], wl.to_f64(Vn[0, h])])
                assert kk.shape[0] == n_kv
                q = wl.to_f64(Q[0, h])
                check_block_idx(idxc[0, h], orc.block_scores(q, kk, w.block, w.block), k)
                ref = orc.hybrid_attention(q, kk, vv, states[h], w.block, w.block, k, orc.PHI_RELU,
                                           None if tab_q[0] is None else wl.to_f64(tab_q[0]),
                                           None if tab_q[1] is None else wl.to_f64(tab_q[1]),
                                           cfg.eps, cfg.z_scale, block_idx=idxc[0, h])[0]
                assert rel_l2(Og[0, h], ref) <= rl, (c, step, h, rel_l2(Og[0, h], ref))
                assert max_abs(Og[0, h], ref) <= ma
        # the last step's K, V are the clean ones that stay in the cache
        for h in range(H):
            cacheK[h] = np.concatenate([cacheK[h], wl.to_f64(Kn[0, h])])
            cacheV[h] = np.concatenate([cacheV[h], wl.to_f64(Vn[0, h])])
        # the buffer holds exactly the oracle's cache, sink frames untouched in front
        for h in range(H):
            assert np.array_equal(wl.to_f64(Kw[0, h, :win.n_tokens]), cacheK[h])
            assert np.array_equal(wl.to_f64(Vw[0, h, :win.n_tokens]), cacheV[h])
    assert total_evicted > 2 * n_chunk           # the cache did overflow several times
    Lg, zg = split_state(st, H, d)
    assert rel_l2(Lg, np.stack([s[0] for s in states])) <= (5e-3 if (rope and w.dtype == "bf16") else 1e-5)
    assert rel_l2(zg, np.stack([s[1] for s in states])) <= 1e-5


@pytest.mark.parametrize("name,sink_frames,rope,ahead", [("small_bf16", 1, False, False), ("small_bf16", 0, True, False),
                                                         ("tiny_f32", 2, False, False), ("small_b128", 1, True, False),
                                                         ("small_bf16", 1, False, True), ("small_b128", 0, False, True),
                                                         ("small_bf16", 0, True, True), ("tiny_f32", 1, False, True)])
def test_ring_cache_evicts_without_moving_a_token_and_matches_the_oracle_loop(name, sink_frames, rope, ahead):
    """The cache as a ring of chunk slots: opening a chunk absorbs the oldest chunk where it lies and changes no
    other byte of the cache (nothing is copied).  The oracle keeps the cache as a list of chunks (pop(0) / append);
    the window it is asked about is that list laid out in the ring's storage order, which is what the library
    defines the blocks of Eq. 4 on (softmax attention itself does not depend on the order of its keys).
    ahead: the last denoising step of every chunk is hf_ring_last_step, which absorbs the chunk that the next
    hf_ring_open_chunk would evict into a second state buffer while the step still attends with the old state (in
    workgroups of the attention launch where that applies, by launches of their own for fp32 or rotated keys); the
    oracle's loop keeps the literal order, and every output and the final state must still agree."""
    w = wl.get(name)
    H, d, tpf = w.heads, w.head_dim, w.tokens_per_frame
    n_chunk, n_sink, slots = w.n_q, sink_frames * tpf, 3
    cap = n_sink + slots * n_chunk
    cfg = cfg_of(w, kv_capacity=cap)
    ring = hf.make_ring(n_sink, n_chunk)
    Kc = torch.zeros((w.batch, H, cap, d), dtype=w.torch_dtype, device=DEV)
    Vc = torch.zeros_like(Kc)
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    st_other = torch.full_like(st, float("nan"))
    aws_n = hf.hf_absorb_workspace_bytes(cfg, n_chunk)
    aws = torch.empty(aws_n, dtype=torch.uint8, device=DEV) if aws_n else None
    sws = torch.empty(max(hf.hf_step_workspace_bytes(cfg, n_chunk, n_chunk), aws_n, 256), dtype=torch.uint8, device=DEV)
    ws = torch.empty(hf.hf_workspace_bytes(cfg, n_chunk, cap), dtype=torch.uint8, device=DEV)
    O = torch.empty((w.batch, H, n_chunk, d), dtype=w.torch_dtype, device=DEV)
    done_ahead = False

    sinkK = [np.zeros((0, d)) for _ in range(H)]
    sinkV = [np.zeros((0, d)) for _ in range(H)]
    if n_sink:
        Ks, Vs = wl.make_evicted(w, 900, n_sink)
        Kc[:, :, :n_sink] = Ks.to(DEV)
        Vc[:, :, :n_sink] = Vs.to(DEV)
        sinkK = [wl.to_f64(Ks[0, h]) for h in range(H)]
        sinkV = [wl.to_f64(Vs[0, h]) for h in range(H)]
    chunks = []                       # oracle: list of (chunk number, K [H][n,d], V) oldest first
    states = [orc.state_zero(d) for _ in range(H)]
    rl, ma = (BF16_REL_L2, BF16_MAX_ABS) if w.dtype == "bf16" else (F32_REL_L2, 1e-4)
    evictions = 0
    for c in range(8):
        before_K, before_V = Kc.clone(), Vc.clone()
        full = len(chunks) == slots
        tab_ev = wl.rope_tables(n_chunk, d, first_position=3.0 + c) if (rope and full) else (None, None)
        st_before = st.clone()
        first, n_ev = hf.hf_ring_open_chunk(cfg, ring, Kc, Vc, st, *(None if t is None else t.to(DEV) for t in tab_ev),
                                            workspace=aws)
        torch.cuda.synchronize()
        assert first == n_sink + (c % slots) * n_chunk and n_ev == (n_chunk if full else 0)
        if done_ahead:                # the chunk went into the state during the last step before: nothing was added now
            assert torch.equal(st, st_before) and ring.absorbed_ahead == 0
        # zero bytes copied: the cache is bit for bit what it was (the new chunk's slot still holds the old chunk)
        assert torch.equal(Kc, before_K) and torch.equal(Vc, before_V)
        if full:                      # pop(0): the oldest chunk goes into the linear state
            _, ek, ev = chunks.pop(0)
            for h in range(H):
                states[h] = orc.state_absorb(*states[h], ek[h], ev[h], orc.PHI_RELU,
                                             None if tab_ev[0] is None else wl.to_f64(tab_ev[0]),
                                             None if tab_ev[1] is None else wl.to_f64(tab_ev[1]))
            evictions += 1
        n_kv = n_sink + ring.n_filled * n_chunk
        k = hf.hf_select_k(cfg, n_kv)
        t_m = -(-n_chunk // w.block)
        idx = torch.full((w.batch, H, t_m, k), -1, dtype=torch.int32, device=DEV)
        tab_q = wl.rope_tables(n_chunk, d, first_position=9.0) if rope else (None, None)
        for step in range(3):
            Kn, Vn = wl.make_evicted(w, 2000 + 10 * c + step, n_chunk)
            Q = wl.randn((w.batch, H, n_chunk, d), 89_000 + 10 * c + step, w.scale, w.torch_dtype)
            Kc[:, :, first:first + n_chunk] = Kn.to(DEV)
            Vc[:, :, first:first + n_chunk] = Vn.to(DEV)
            if ahead and step == 2:
                # the chunk evicted next is absorbed now, with the tables the oracle's loop will use when it pops it
                will_evict = len(chunks) + 1 > slots - 1 and len(chunks) == slots - 1
                tab_nx = wl.rope_tables(n_chunk, d, first_position=3.0 + c + 1) if (rope and will_evict) else (None, None)
                st_old = st.clone()
                done_ahead = hf.hf_ring_last_step(cfg, ring, Q.to(DEV), Kc, Vc, step, idx, st, O, ws, st_other, sws,
                                                  *(None if t is None else t.to(DEV) for t in tab_q),
                                                  rope_cos_ev=None if tab_nx[0] is None else tab_nx[0].to(DEV),
                                                  rope_sin_ev=None if tab_nx[1] is None else tab_nx[1].to(DEV))
                torch.cuda.synchronize()
                assert done_ahead == will_evict and torch.equal(st, st_old)      # this step read the old state
            else:
                hf.hf_ring_step(cfg, ring, Q.to(DEV), Kc, Vc, step, idx, st, O, ws,
                                *(None if t is None else t.to(DEV) for t in tab_q))
            torch.cuda.synchronize()
            Og, idxc = wl.to_f64(O), idx.cpu().numpy()
            # the oracle's list, laid out in storage order: slot s holds the newest chunk with number = s mod slots
            cur = (c, [wl.to_f64(Kn[0, h]) for h in range(H)], [wl.to_f64(Vn[0, h]) for h in range(H)])
            by_slot = {num % slots: (kk, vv) for num, kk, vv in chunks + [cur]}
            for h in range(H):
                kk = np.concatenate([sinkK[h]] + [by_slot[s][0][h] for s in sorted(by_slot)])
                vv = np.concatenate([sinkV[h]] + [by_slot[s][1][h] for s in sorted(by_slot)])
                assert kk.shape[0] == n_kv
                assert np.array_equal(wl.to_f64(Kc[0, h, :n_kv]), kk)          # the buffer IS that window
                q = wl.to_f64(Q[0, h])
                check_block_idx(idxc[0, h], orc.block_scores(q, kk, w.block, w.block), k)
                ref = orc.hybrid_attention(q, kk, vv, states[h], w.block, w.block, k, orc.PHI_RELU,
                                           None if tab_q[0] is None else wl.to_f64(tab_q[0]),
                                           None if tab_q[1] is None else wl.to_f64(tab_q[1]),
                                           cfg.eps, cfg.z_scale, block_idx=idxc[0, h])[0]
                assert rel_l2(Og[0, h], ref) <= rl, (c, step, h, rel_l2(Og[0, h], ref))
                assert max_abs(Og[0, h], ref) <= ma
        chunks.append(cur)
        if done_ahead:                # the second buffer is the state from the next chunk on
            st, st_other = st_other, st
    assert evictions == 8 - slots
    if done_ahead:                    # the chunk absorbed ahead of an open that this loop no longer performs
        _, ek, ev = chunks[0]
        tab_nx = wl.rope_tables(n_chunk, d, first_position=3.0 + 8) if rope else (None, None)
        for h in range(H):
            states[h] = orc.state_absorb(*states[h], ek[h], ev[h], orc.PHI_RELU,
                                         None if tab_nx[0] is None else wl.to_f64(tab_nx[0]),
                                         None if tab_nx[1] is None else wl.to_f64(tab_nx[1]))
    Lg, zg = split_state(st, H, d)
    assert rel_l2(Lg, np.stack([s[0] for s in states])) <= (5e-3 if (rope and w.dtype == "bf16") else 1e-5)
    assert rel_l2(zg, np.stack([s[1] for s in states])) <= 1e-5


def test_ring_arguments_are_checked():
    cfg = hf.make_config(1, 2, 128, "bf16", 64, 64, 0.25, kv_capacity=1000)
    K = torch.zeros((1, 2, 1000, 128), dtype=torch.bfloat16, device=DEV)
    st = torch.zeros(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    with pytest.raises(hf.HFError) as e:                 # 1000 - 100 is no multiple of 400
        hf.hf_ring_open_chunk(cfg, hf.make_ring(100, 400), K, K.clone(), st)
    assert "multiple" in str(e.value)
    ring = hf.make_ring(200, 400)
    with pytest.raises(hf.HFError) as e:                 # no chunk open yet
        hf.hf_ring_step(cfg, ring, K[:, :, :400].contiguous(), K, K, 0, torch.zeros((1, 2, 7, 1), dtype=torch.int32, device=DEV), st,
                        torch.empty((1, 2, 400, 128), dtype=torch.bfloat16, device=DEV),
                        torch.empty(1 << 20, dtype=torch.uint8, device=DEV))
    assert "open" in str(e.value)
