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
