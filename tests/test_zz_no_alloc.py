"""The entry point that allocates nothing: hf_block_select_static keeps the pooled block means in a buffer built
into the library instead of a caller workspace.  Called through the C ABI and compared with hf_block_select,
bit for bit (integer indices; the scores are the same kernels on the same inputs), on two calls in a row, the
second with a smaller input, so that whatever the first call left in the shared buffer must not matter."""
import pytest
import torch

import paper_2604_10103_amd as hf
import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _both(cfg, Q, K):
    n_q, n_kv = Q.shape[2], K.shape[2]
    k = hf.hf_select_k(cfg, n_kv)
    t_m, t_n = -(-n_q // cfg.block_q), -(-n_kv // cfg.block_kv)
    out = []
    for static in (False, True):
        idx = torch.full((cfg.batch, cfg.heads, t_m, k), -1, dtype=torch.int32, device=DEV)
        scores = torch.full((cfg.batch, cfg.heads, t_m, t_n), float("nan"), dtype=torch.float32, device=DEV)
        if static:
            hf.hf_block_select_static(cfg, Q, K, idx, scores)
        else:
            ws = torch.empty(hf.hf_workspace_bytes(cfg, n_q, n_kv), dtype=torch.uint8, device=DEV)
            hf.hf_block_select(cfg, Q, K, idx, scores, ws)
        torch.cuda.synchronize()
        out.append((idx, scores))
    return out


def test_static_scratch_selection_equals_workspace_selection_twice_in_a_row():
    w = wl.get("step_832x480")
    cfg = hf.make_config(w.batch, w.heads, w.head_dim, w.dtype, w.block, w.block, w.keep_ratio)
    Q, K, _ = wl.make_qkv(w)
    Q, K = Q.to(DEV), K.to(DEV)
    (ia, sa), (ib, sb) = _both(cfg, Q, K)
    assert int(ia.min()) >= 0 and torch.equal(ia, ib) and torch.equal(sa, sb)
    # a smaller call right behind it, ragged in both directions, other block size: the buffer still holds the
    # first call's pooled means beyond what this call overwrites
    cfg2 = hf.make_config(1, 5, 128, "bf16", 128, 128, 0.5)
    Q2, K2 = Q[:, :5, :1000].contiguous(), K[:, :5, :2100].contiguous()
    (ia, sa), (ib, sb) = _both(cfg2, Q2, K2)
    assert int(ia.min()) >= 0 and torch.equal(ia, ib) and torch.equal(sa, sb)
    # and the first shape again
    (ia, sa), (ib, sb) = _both(cfg, Q, K)
    assert torch.equal(ia, ib) and torch.equal(sa, sb)


def test_static_scratch_refuses_sizes_beyond_its_buffer():
    cfg = hf.make_config(1, 64, 128, "bf16", 16, 16, 0.25)
    n_q, n_kv = 16 * 128, 16 * 256        # 64 heads x (128 + 256) blocks x 128 x 4 B = 12.6 MB > 8 MiB
    Q = torch.zeros((1, 64, n_q, 128), dtype=torch.bfloat16, device=DEV)
    K = torch.zeros((1, 64, n_kv, 128), dtype=torch.bfloat16, device=DEV)
    idx = torch.empty((1, 64, 128, hf.hf_select_k(cfg, n_kv)), dtype=torch.int32, device=DEV)
    with pytest.raises(hf.HFError) as e:
        hf.hf_block_select_static(cfg, Q, K, idx)
    assert e.value.code == -5 and "built-in buffer" in str(e.value)
