"""The whole step as a captured HIP graph (the ordinary calls, and the calls bench.py launches, which keep the
state's bf16 planes with the caller), and a two-stream variant
in which the evicted chunk is absorbed on a second stream while the blocks are selected.

Every replay is compared with the same step run eagerly on one stream on buffers of its own;
between replays the process does eager work and synchronises, so that a node whose effect
survived only the first replay would show.  The captured calls hold no memset (buffers are
cleared by fill kernels) and allocate nothing.
"""
import pytest
import torch

import paper_2604_10103_amd as hf
import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


class Buffers:
    def __init__(self, cfg, w, Q, K, V, Ke, Ve):
        self.cfg = cfg
        self.Q, self.K, self.V, self.Ke, self.Ve = (t.to(DEV) for t in (Q, K, V, Ke, Ve))
        k = hf.hf_select_k(cfg, w.n_kv)
        self.idx = torch.full((w.batch, w.heads, w.t_m, k), -1, dtype=torch.int32, device=DEV)
        self.O = torch.zeros(Q.shape, dtype=Q.dtype, device=DEV)
        self.ws = torch.empty(hf.hf_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=DEV)
        nb = hf.hf_absorb_workspace_bytes(cfg, Ke.shape[2])
        self.aws = torch.empty(nb, dtype=torch.uint8, device=DEV) if nb else None
        self.st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=DEV)
        hf.hf_state_init(cfg, self.st)
        hf.hf_absorb_evicted(cfg, self.st, self.Ke, self.Ve, workspace=self.aws)   # a non-empty history
        nb = hf.hf_state_planes_bytes(cfg)
        self.planes = torch.empty(nb, dtype=torch.uint8, device=DEV) if nb else None
        if nb:
            hf.hf_state_planes(cfg, self.st, self.planes)

    def kept_planes_step(self):
        """The step as bench.py launches it: the state's bf16 planes travel with the state."""
        hf.hf_absorb_evicted_planes(self.cfg, self.st, self.Ke, self.Ve, self.planes, workspace=self.aws)
        hf.hf_block_select(self.cfg, self.Q, self.K, self.idx, None, self.ws)
        hf.hf_hybrid_attn_fwd_planes(self.cfg, self.Q, self.K, self.V, self.idx, self.st, self.planes, self.O)

    def eager_step(self):
        hf.hf_absorb_evicted(self.cfg, self.st, self.Ke, self.Ve, workspace=self.aws)
        hf.hf_block_select(self.cfg, self.Q, self.K, self.idx, None, self.ws)
        hf.hf_hybrid_attn_fwd(self.cfg, self.Q, self.K, self.V, self.idx, self.st, self.O, self.ws)

    def capture(self, two_streams):
        g = torch.cuda.CUDAGraph()
        if not two_streams:
            with torch.cuda.graph(g):
                self.eager_step()
            return g
        side = torch.cuda.Stream()
        with torch.cuda.graph(g):
            main = torch.cuda.current_stream()
            side.wait_stream(main)
            with torch.cuda.stream(side):
                hf.hf_absorb_evicted(self.cfg, self.st, self.Ke, self.Ve, workspace=self.aws)
            hf.hf_block_select(self.cfg, self.Q, self.K, self.idx, None, self.ws)
            main.wait_stream(side)
            hf.hf_hybrid_attn_fwd(self.cfg, self.Q, self.K, self.V, self.idx, self.st, self.O, self.ws)
        return g


@pytest.mark.parametrize("name,two_streams", [("small_bf16", False), ("small_bf16", True), ("tiny_f32", False),
                                              ("step_832x480", False), ("step_832x480", True)])
def test_captured_step_replays_match_eager(name, two_streams):
    w = wl.get(name)
    cfg = hf.make_config(batch=w.batch, heads=w.heads, head_dim=w.head_dim, dtype=w.dtype, block_q=w.block,
                         block_kv=w.block, keep_ratio=w.keep_ratio)
    Q, K, V = wl.make_qkv(w)
    Ke, Ve = wl.make_evicted(w, 0)
    ref = Buffers(cfg, w, Q, K, V, Ke, Ve)
    cap = Buffers(cfg, w, Q, K, V, Ke, Ve)
    torch.cuda.synchronize()
    before = cap.st.clone()
    g = cap.capture(two_streams)            # capturing runs nothing: cap.st still holds one absorbed chunk
    torch.cuda.synchronize()
    assert torch.equal(before, cap.st)
    scratch = torch.zeros(1 << 20, device=DEV)
    for rep in range(4):
        ref.eager_step()
        scratch.add_(1.0)        # the program's own eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(cap.idx, ref.idx), rep
        # the normaliser z is summed with LDS float atomics, whose order is not fixed: the state agrees
        # to fp32 rounding, the output to one rounding step of its type
        torch.testing.assert_close(cap.st, ref.st, rtol=1e-5, atol=1e-6)
        if w.dtype == "bf16":
            torch.testing.assert_close(cap.O.float(), ref.O.float(), rtol=1e-2, atol=1e-3)
        else:
            torch.testing.assert_close(cap.O, ref.O, rtol=1e-4, atol=1e-5)
        assert torch.isfinite(cap.O.float()).all()


@pytest.mark.parametrize("name", ["small_bf16", "step_832x480"])
def test_captured_step_with_kept_planes_replays_match_eager(name):
    """The same for the calls that keep the state's bf16 planes with the caller; the eager reference runs the
    ordinary calls.  In the plain case with a workspace every sum has a fixed order: bit for bit."""
    w = wl.get(name)
    cfg = hf.make_config(batch=w.batch, heads=w.heads, head_dim=w.head_dim, dtype=w.dtype, block_q=w.block,
                         block_kv=w.block, keep_ratio=w.keep_ratio)
    Q, K, V = wl.make_qkv(w)
    Ke, Ve = wl.make_evicted(w, 0)
    ref = Buffers(cfg, w, Q, K, V, Ke, Ve)
    cap = Buffers(cfg, w, Q, K, V, Ke, Ve)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        cap.kept_planes_step()
    scratch = torch.zeros(1 << 20, device=DEV)
    for rep in range(4):
        ref.eager_step()
        scratch.add_(1.0)        # the program's own eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(cap.idx, ref.idx), rep
        assert torch.equal(cap.st, ref.st), rep
        assert torch.equal(cap.O, ref.O), rep
        assert torch.isfinite(cap.O.float()).all()



@pytest.mark.parametrize("name", ["small_bf16", "step_832x480"])
def test_captured_two_launch_step_replays_match_eager(name):
    """hf_pool_keys + hf_step_fwd as a captured graph, one graph per direction of the state's two buffers (as bench.py
    replays them).  Every replay carries the same counter tag; the last workgroup of a head leaves its arrival counter
    at zero, so the replays count from zero again.  The eager reference makes the same calls on buffers of its own:
    every sum has a fixed order, so state, planes, lists and outputs agree bit for bit."""
    w = wl.get(name)
    cfg = hf.make_config(batch=w.batch, heads=w.heads, head_dim=w.head_dim, dtype=w.dtype, block_q=w.block,
                         block_kv=w.block, keep_ratio=w.keep_ratio)
    Q, K, V = wl.make_qkv(w)
    Ke, Ve = wl.make_evicted(w, 0)

    class Two(Buffers):
        def __init__(self):
            super().__init__(cfg, w, Q, K, V, Ke, Ve)
            self.st2, self.planes2 = torch.zeros_like(self.st), torch.zeros_like(self.planes)
            self.pooled = torch.empty(hf.hf_pooled_keys_bytes(cfg, w.n_kv), dtype=torch.uint8, device=DEV)
            self.sws = torch.empty(hf.hf_step_workspace_bytes(cfg, w.n_q, Ke.shape[2]), dtype=torch.uint8, device=DEV)

        def step(self, phase):
            a, b = ((self.st, self.planes), (self.st2, self.planes2))[::1 if phase == 0 else -1]
            hf.hf_pool_keys(cfg, self.K, self.pooled)
            hf.hf_step_fwd(cfg, self.Q, self.K, self.V, self.pooled, a[0], a[1], self.O, self.idx, self.Ke, self.Ve,
                           b[0], b[1], self.sws)

    ref, cap = Two(), Two()
    torch.cuda.synchronize()
    graphs = []
    for phase in (0, 1):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            cap.step(phase)
        graphs.append(g)
    scratch = torch.zeros(1 << 20, device=DEV)
    for rep in range(6):
        ref.step(rep % 2)
        scratch.add_(1.0)        # the program's own eager work between replays
        torch.cuda.synchronize()
        graphs[rep % 2].replay()
        torch.cuda.synchronize()
        assert torch.equal(cap.idx, ref.idx), rep
        assert torch.equal(cap.O, ref.O), rep
        for x, y in ((cap.st, ref.st), (cap.st2, ref.st2), (cap.planes, ref.planes), (cap.planes2, ref.planes2)):
            assert torch.equal(x, y), rep
        assert torch.isfinite(cap.O.float()).all()
    # the state grew by one chunk per step: six absorbed chunks on top of the first
    assert float(cap.st.abs().sum()) > 0 and not torch.equal(cap.st, cap.st2)
