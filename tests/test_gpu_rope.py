"""GPU parity of the relative RoPE calls (Sec. 3.3, Eq. 7) against the fp64 oracle: table construction,
rotation of Q / K, and the attention call whose two branches read differently prepared queries."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_2604_10103_amd as hf
import workloads as wl
from parity import BF16_MAX_ABS, BF16_REL_L2, F32_REL_L2, check_block_idx, heads_of, max_abs, oracle_state, rel_l2

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
T0 = 21          # cap of the temporal index (Sec. 4.1)


def cfg_of(w, **kw):
    args = dict(batch=w.batch, heads=w.heads, head_dim=w.head_dim, dtype=w.dtype, block_q=w.block,
                block_kv=w.block, keep_ratio=w.keep_ratio)
    args.update(kw)
    return hf.make_config(**args)


def gpu_tables(frames, hh, ww, pairs, temporal_only=False):
    n = len(frames) * hh * ww
    cos = torch.full((n, sum(pairs)), float("nan"), dtype=torch.float32, device=DEV)
    sin = torch.full((n, sum(pairs)), float("nan"), dtype=torch.float32, device=DEV)
    hf.hf_rope_tables(frames, hh, ww, pairs, cos, sin, temporal_only=temporal_only)
    torch.cuda.synchronize()
    return cos, sin


def as_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.float32)


@pytest.mark.parametrize("frames,hh,ww,pairs,temporal_only", [
    ([0], 1, 1, (1, 0, 0), False),
    ([3, 4, 5], 3, 5, (3, 2, 3), False),
    ([-3, -3], 4, 4, (22, 21, 21), True),
    (list(range(16, 22)), 30, 52, (22, 21, 21), False),        # the window of the 832x480 step beyond the cap
    (list(range(-40, 24)), 2, 3, (44, 42, 42), False),         # most frames and pairs one call takes
])
def test_tables_match_oracle(frames, hh, ww, pairs, temporal_only):
    cos, sin = gpu_tables(frames, hh, ww, pairs, temporal_only)
    rc, rs = orc.rope_tables_3d(frames, hh, ww, pairs, temporal_only=temporal_only)
    # fp64 on both sides, one rounding to fp32: at most one unit in the last place of a value <= 1
    assert np.abs(wl.to_f64(cos) - rc).max() <= 1.2e-7
    assert np.abs(wl.to_f64(sin) - rs).max() <= 1.2e-7
    assert float((cos == as_f32(rc).to(DEV)).float().mean()) > 0.999


def test_window_indices_and_tables_of_a_capped_stream_stay_put():
    w = wl.get("small_bf16")
    hh, ww = wl.frame_grid(w)
    pairs = orc.default_axis_pairs(w.head_dim)
    a = gpu_tables(hf.hf_rope_window_indices(50, w.window_frames, T0), hh, ww, pairs)
    b = gpu_tables(hf.hf_rope_window_indices(53, w.window_frames, T0), hh, ww, pairs)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def rotated_ref(X, cos64, sin64):
    """Oracle rotation of every head from the stored values, in fp64."""
    x = wl.to_f64(X)
    out = np.empty_like(x)
    for b in range(x.shape[0]):
        for h in range(x.shape[1]):
            out[b, h] = orc.rope_rotate(x[b, h], cos64, sin64)
    return out


@pytest.mark.parametrize("name,which", [("tiny_f32", "K"), ("small_bf16", "Q"), ("small_bf16", "K"),
                                        ("small_f32_d128", "K"), ("step_832x480", "K")])
def test_rotation_matches_oracle(name, which):
    w = wl.get(name)
    cfg = cfg_of(w)
    hh, ww = wl.frame_grid(w)
    pairs = orc.default_axis_pairs(w.head_dim)
    Q, K, _ = wl.make_qkv(w)
    X = Q if which == "Q" else K
    nf = w.chunk_frames if which == "Q" else w.window_frames
    frames = orc.window_temporal_indices(40, nf, T0)
    cos, sin = (as_f32(t) for t in orc.rope_tables_3d(frames, hh, ww, pairs))    # stored fp32 tables: inputs
    ref = rotated_ref(X, wl.to_f64(cos), wl.to_f64(sin))
    Xd = X.to(DEV)
    Y = torch.full_like(Xd, float("nan"))
    hf.hf_rope_apply(cfg, Xd, cos.to(DEV), sin.to(DEV), Y)
    torch.cuda.synchronize()
    y = wl.to_f64(Y)
    if w.dtype == "bf16":
        # fp32 arithmetic, one rounding to bf16: within half a unit in the last place of the exact value (8
        # significant bits: 2^(e-9) for a value in [2^(e-1), 2^e)), and nearly always the very value the oracle's
        # result rounds to
        half_ulp = np.ldexp(1.0, np.frexp(np.abs(ref))[1] - 9)
        assert np.all(np.abs(y - ref) <= half_ulp * 1.01 + 1e-6)
        same = Y.cpu() == torch.from_numpy(ref).to(torch.bfloat16)
        assert float(same.float().mean()) > 0.999
    else:
        assert rel_l2(y, ref) <= 1e-6 and max_abs(y, ref) <= 1e-5
    # in place gives the same bits
    hf.hf_rope_apply(cfg, Xd, cos.to(DEV), sin.to(DEV), Xd)
    torch.cuda.synchronize()
    assert torch.equal(Xd, Y)


@pytest.mark.parametrize("name,phi", [("tiny_f32", hf.HF_PHI_RELU), ("small_bf16", hf.HF_PHI_RELU),
                                      ("small_bf16", hf.HF_PHI_ELU1), ("small_b128", hf.HF_PHI_RELU),
                                      ("small_f32_d128", hf.HF_PHI_ELU1)])
def test_rotated_local_branch_unrotated_history_branch(name, phi):
    """One chunk of a stream far beyond the cap, every stage on the library's side: tables from frame indices,
    evicted frames absorbed with their rotation, q and k rotated for Eq. 4 / 5, the un-rotated q through phi
    into Eq. 3.  The oracle does the same from its own tables; the attention stage is fed the oracle's rotated
    tensors so that a legal one-unit rounding difference in a rotated value cannot move a block boundary."""
    w = wl.get(name)
    cfg = cfg_of(w, phi=phi)
    hh, ww = wl.frame_grid(w)
    pairs = orc.default_axis_pairs(w.head_dim)
    i_now = 200
    win_idx = hf.hf_rope_window_indices(i_now, w.window_frames, T0)
    assert win_idx == orc.window_temporal_indices(i_now, w.window_frames, T0).tolist()
    q_idx = win_idx[-w.chunk_frames:]
    ev_idx = [win_idx[0] - 1]                      # a frame leaves the window one step behind its oldest frame

    # state: evicted frames, rotated at that index, library side and oracle side
    st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    ev_cos, ev_sin = gpu_tables(ev_idx, hh, ww, pairs)
    ev_ref = tuple(as_f32(t) for t in orc.rope_tables_3d(ev_idx, hh, ww, pairs))
    Ks, Vs = [], []
    for c in range(w.evicted_frames):
        Ke, Ve = wl.make_evicted(w, c, w.tokens_per_frame)
        Ks.append(Ke); Vs.append(Ve)
        hf.hf_absorb_evicted(cfg, st, Ke.to(DEV), Ve.to(DEV), ev_cos, ev_sin)
    ref_states = oracle_state(Ks, Vs, w.head_dim, phi, [ev_ref] * w.evicted_frames)

    Q, K, V = wl.make_qkv(w)
    q_cos, q_sin = gpu_tables(q_idx, hh, ww, pairs)
    k_cos, k_sin = gpu_tables(win_idx, hh, ww, pairs)
    qc64, qs64 = orc.rope_tables_3d(q_idx, hh, ww, pairs)
    kc64, ks64 = orc.rope_tables_3d(win_idx, hh, ww, pairs)
    Qrot_ref = torch.from_numpy(rotated_ref(Q, qc64, qs64)).to(w.torch_dtype)      # stored in the path's type
    Krot_ref = torch.from_numpy(rotated_ref(K, kc64, ks64)).to(w.torch_dtype)
    # the library's own rotation agrees with that, up to rare one-unit differences
    Qrot = torch.empty_like(Q, device=DEV)
    Krot = torch.empty_like(K, device=DEV)
    hf.hf_rope_apply(cfg, Q.to(DEV), q_cos, q_sin, Qrot)
    hf.hf_rope_apply(cfg, K.to(DEV), k_cos, k_sin, Krot)
    torch.cuda.synchronize()
    if w.dtype == "bf16":
        assert float((Qrot.cpu() == Qrot_ref).float().mean()) > 0.999
        assert float((Krot.cpu() == Krot_ref).float().mean()) > 0.999
    assert rel_l2(wl.to_f64(Qrot), wl.to_f64(Qrot_ref)) < (1e-3 if w.dtype == "bf16" else 1e-6)
    assert rel_l2(wl.to_f64(Krot), wl.to_f64(Krot_ref)) < (1e-3 if w.dtype == "bf16" else 1e-6)

    # selection and attention on the rotated tensors, history from the un-rotated queries
    k = hf.hf_select_k(cfg, w.n_kv)
    idx = torch.full((w.batch, w.heads, w.t_m, k), -1, dtype=torch.int32, device=DEV)
    ws = torch.empty(hf.hf_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=DEV)
    Qr, Kr = Qrot_ref.to(DEV), Krot_ref.to(DEV)
    hf.hf_block_select(cfg, Qr, Kr, idx, None, ws)
    O = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
    hf.hf_hybrid_attn_fwd(cfg, Qr, Kr, V.to(DEV), idx, st, O, ws, q_cos, q_sin, Q_hist=Q.to(DEV))
    torch.cuda.synchronize()
    Og, idxc = wl.to_f64(O), idx.cpu().numpy()
    rl, ma = (BF16_REL_L2, BF16_MAX_ABS) if w.dtype == "bf16" else (F32_REL_L2, 1e-4)
    for h, (q, qr, kr, v) in enumerate(zip(heads_of(Q), heads_of(Qrot_ref), heads_of(Krot_ref), heads_of(V))):
        check_block_idx(idxc[0, h], orc.block_scores(qr, kr, w.block, w.block), k)
        ref, _, ref_hist, _, _ = orc.hybrid_attention(qr, kr, v, ref_states[h], w.block, w.block, k, phi, qc64, qs64,
                                                     cfg.eps, cfg.z_scale, block_idx=idxc[0, h], Q_hist=q)
        assert np.abs(ref_hist).max() > 1e-4
        assert rel_l2(Og[0, h], ref) <= rl, (name, h, rel_l2(Og[0, h], ref))
        assert max_abs(Og[0, h], ref) <= ma
        # feeding the rotated queries to the history branch as well is a different result, further from what the
        # library returned: the split is live
        wrong = orc.hybrid_attention(qr, kr, v, ref_states[h], w.block, w.block, k, phi, qc64, qs64, cfg.eps,
                                     cfg.z_scale, block_idx=idxc[0, h])[0]
        assert rel_l2(Og[0, h], wrong) > 2 * rel_l2(Og[0, h], ref)


@pytest.mark.parametrize("name,rotate,capacity", [("small_bf16", True, 0), ("small_bf16", False, 0), ("small_bf16", True, 1200),
                                                  ("tiny_f32", True, 0), ("small_b128", True, 0), ("small_f32_d128", True, 0)])
def test_new_keys_are_rotated_into_the_window_and_pooled_in_one_pass(name, rotate, capacity):
    """hf_rope_append_keys: the chunk's un-rotated keys become the last n_q tokens of the window buffer (rotated by
    their tables) and the pooled keys of the KV blocks they touch are rewritten, the chunk's first block sharing
    tokens with the cached part (first is not a multiple of the block size).  Expected: the oracle's rotation, rounded
    to the storage type, laid behind the cached part, and the oracle's pooled means of that window."""
    w = wl.get(name)
    cfg = cfg_of(w, kv_capacity=capacity)
    hh, ww = wl.frame_grid(w)
    pairs = orc.default_axis_pairs(w.head_dim)
    _, K, _ = wl.make_qkv(w)                      # the cached part: its first tokens, as they lie in the cache
    first = w.n_kv - w.n_q
    assert first % w.block != 0 or name == "tiny_f32"
    K_new = wl.randn((w.batch, w.heads, w.n_q, w.head_dim), 99_000 + w.cfg, w.scale, w.torch_dtype)
    frames = orc.window_temporal_indices(40, w.chunk_frames, T0)
    cos, sin = (as_f32(t) for t in orc.rope_tables_3d(frames, hh, ww, pairs))
    if rotate:
        new_ref = torch.from_numpy(rotated_ref(K_new, wl.to_f64(cos), wl.to_f64(sin))).to(w.torch_dtype)
    else:
        new_ref = K_new
    window_ref = torch.cat([K[:, :, :first], new_ref], dim=2)
    cap = capacity or w.n_kv
    Kwin = torch.full((w.batch, w.heads, cap, w.head_dim), float("nan"), dtype=w.torch_dtype, device=DEV)
    Kwin[:, :, :first] = K[:, :, :first].to(DEV)
    pooled = torch.empty(hf.hf_pooled_keys_bytes(cfg, w.n_kv), dtype=torch.uint8, device=DEV)
    # the cached part is pooled once (its last, shared block from the stale tail: the append call rewrites it)
    Kwin[:, :, first:w.n_kv] = 0
    hf.hf_pool_keys(cfg, Kwin, pooled, n_kv=w.n_kv if capacity else None)
    before = pooled.clone()
    hf.hf_rope_append_keys(cfg, K_new.to(DEV), cos.to(DEV) if rotate else None, sin.to(DEV) if rotate else None, Kwin,
                           first, pooled, n_kv=w.n_kv if capacity else None)
    torch.cuda.synchronize()
    got = Kwin[:, :, :w.n_kv].cpu()
    assert torch.equal(got[:, :, :first], K[:, :, :first])                 # the cached part is untouched
    if w.dtype == "bf16":
        assert float((got == window_ref).float().mean()) > 0.999           # rare one-unit differences of the rotation
        assert rel_l2(wl.to_f64(got), wl.to_f64(window_ref)) < 1e-3
    else:
        assert rel_l2(wl.to_f64(got), wl.to_f64(window_ref)) <= 1e-6
    # pooled keys [B*H][d/4][T_n][4]: the touched blocks hold the means of the window, the others what they held
    t_n, d = w.t_n, w.head_dim
    pk = pooled.view(torch.float32)[: w.batch * w.heads * t_n * d].view(w.batch * w.heads, d // 4, t_n, 4)
    pb = before.view(torch.float32)[: w.batch * w.heads * t_n * d].view(w.batch * w.heads, d // 4, t_n, 4)
    pk = pk.permute(0, 2, 1, 3).reshape(w.batch * w.heads, t_n, d).cpu().double().numpy()
    pb = pb.permute(0, 2, 1, 3).reshape(w.batch * w.heads, t_n, d).cpu().double().numpy()
    b0 = first // w.block
    assert np.array_equal(pk[:, :b0], pb[:, :b0])
    for h, kk in enumerate(heads_of(window_ref)):
        ref = orc.pool_blocks(kk, w.block)
        diff = np.abs(pk[h, b0:] - ref[b0:])
        # a one-unit difference of a rotated value (fewer than one in a thousand, above) moves the mean it enters
        # by that unit over the block length; a mean gathers `block` values, so up to block/1000 of the means
        assert diff.max() <= (1e-4 if w.dtype == "bf16" else 1e-6)
        assert (diff <= 1e-6).mean() > 1.0 - w.block / 1000.0
    # and the pooled keys are those of the stand-alone pooling of the buffer as it now stands, to fp32 summation order
    again = torch.empty_like(pooled)
    hf.hf_pool_keys(cfg, Kwin, again, n_kv=w.n_kv if capacity else None)
    torch.cuda.synchronize()
    pa = again.view(torch.float32)[: w.batch * w.heads * t_n * d]
    torch.testing.assert_close(pooled.view(torch.float32)[: w.batch * w.heads * t_n * d], pa, rtol=0, atol=1e-6)
