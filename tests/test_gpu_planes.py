"""The state's bf16 planes kept by the caller: hf_absorb_evicted_planes writes them from the kernel that
writes the state, hf_hybrid_attn_fwd_planes reads them instead of converting the state on every call.
Nothing about the arithmetic changes, so everything is compared bit for bit with the ordinary calls
(whose parity with the oracle the other GPU tests establish)."""
import pytest
import torch

import paper_2604_10103_amd as hf
import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def cfg_of(w, **kw):
    args = dict(batch=w.batch, heads=w.heads, head_dim=w.head_dim, dtype=w.dtype, block_q=w.block,
                block_kv=w.block, keep_ratio=w.keep_ratio)
    args.update(kw)
    return hf.make_config(**args)


def new_state(cfg):
    st = torch.full((hf.hf_state_bytes(cfg) // 4,), float("nan"), dtype=torch.float32, device=DEV)
    hf.hf_state_init(cfg, st)
    return st


def planes_buf(cfg):
    return torch.full((hf.hf_state_planes_bytes(cfg),), 0xAB, dtype=torch.uint8, device=DEV)


@pytest.mark.parametrize("name,phi,rope,with_ws", [
    ("small_bf16", hf.HF_PHI_RELU, False, True),      # slices summed by the reduce kernel: planes leave it
    ("small_bf16", hf.HF_PHI_RELU, True, True),       # rotated keys: the other absorb kernel, same reduce kernel
    ("small_bf16", hf.HF_PHI_ELU1, False, True),
    ("small_bf16", hf.HF_PHI_RELU, False, False),     # atomics: a conversion launch follows
    ("small_b128", hf.HF_PHI_RELU, False, True),
    ("step_832x480", hf.HF_PHI_RELU, False, True),
])
def test_kept_planes_change_no_bit(name, phi, rope, with_ws):
    w = wl.get(name)
    cfg = cfg_of(w, phi=phi)
    n_ev = w.tokens_per_frame * w.chunk_frames
    nb = hf.hf_absorb_workspace_bytes(cfg, n_ev)
    aws = torch.empty(nb, dtype=torch.uint8, device=DEV) if (nb and with_ws) else None
    Q, K, V = (t.to(DEV) for t in wl.make_qkv(w))
    k = hf.hf_select_k(cfg, w.n_kv)
    idx = torch.full((w.batch, w.heads, w.t_m, k), -1, dtype=torch.int32, device=DEV)
    ws = torch.empty(hf.hf_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=DEV)
    hf.hf_block_select(cfg, Q, K, idx, None, ws)
    tq = tuple(t.to(DEV) for t in wl.rope_tables(w.n_q, w.head_dim, first_position=9.0,
                                                 tokens_per_position=w.tokens_per_frame)) if rope else (None, None)
    st_a, st_b = new_state(cfg), new_state(cfg)
    planes, ref_planes = planes_buf(cfg), planes_buf(cfg)
    for c in range(3):
        Ke, Ve = (t.to(DEV) for t in wl.make_evicted(w, c, n_ev))
        te = tuple(t.to(DEV) for t in wl.rope_tables(n_ev, w.head_dim, first_position=float(c),
                                                     tokens_per_position=w.tokens_per_frame)) if rope else (None, None)
        hf.hf_absorb_evicted_planes(cfg, st_b, Ke, Ve, planes, te[0], te[1], workspace=aws)
        # the state itself is compared where its sums have a fixed order: the streamed kernel of the plain case with a
        # workspace (the register-staged kernel adds its wavefronts' shares of z with LDS atomics, the path without a
        # workspace adds slices with global ones: a last bit may differ between two calls there)
        if with_ws and phi == hf.HF_PHI_RELU and not rope:
            hf.hf_absorb_evicted(cfg, st_a, Ke, Ve, te[0], te[1], workspace=aws)
            torch.cuda.synchronize()
            assert torch.equal(st_a, st_b)
        # the planes are those of the state as it stands
        hf.hf_state_planes(cfg, st_b, ref_planes)
        torch.cuda.synchronize()
        assert torch.equal(planes, ref_planes)
        O_a = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
        O_b = torch.full(Q.shape, float("nan"), dtype=Q.dtype, device=DEV)
        hf.hf_hybrid_attn_fwd(cfg, Q, K, V, idx, st_b, O_a, ws, tq[0], tq[1])
        hf.hf_hybrid_attn_fwd_planes(cfg, Q, K, V, idx, st_b, planes, O_b, tq[0], tq[1])
        torch.cuda.synchronize()
        assert torch.isfinite(O_a.float()).all()
        assert torch.equal(O_a, O_b)


def test_kept_planes_are_refused_where_the_path_does_not_exist():
    w = wl.get("tiny_f32")
    cfg = cfg_of(w)
    assert hf.hf_state_planes_bytes(cfg) == 0
    st = new_state(cfg)
    buf = torch.empty(1024, dtype=torch.uint8, device=DEV)
    with pytest.raises(hf.HFError):
        hf.hf_state_planes(cfg, st, buf)
