#!/usr/bin/env python3
"""Benchmark of the hybrid-attention hot path on one MI355X.

A step is one pass of the whole path for one layer and one chunk of the 832x480 streaming
workload: block selection (Eq. 4), block-sparse flash forward (Eq. 5), history readout and sum
(Eq. 3, 6), and the state update for one evicted chunk (Eq. 2).  By default it runs as TWO
launches: hf_pool_keys, then hf_step_fwd (every query block's workgroup selects its blocks
itself, attends and adds the history term; workgroups of their own absorb the evicted chunk into
the other of two state buffers, which becomes the state of the next step).  --separate-launches
times the four launches of hf_block_select + hf_hybrid_attn_fwd_planes + hf_absorb_evicted_planes
instead (also reported next to the default as ms_per_step_separate_launches).  Inputs are seeded
synthetic tensors already resident in HBM; several layers' worth of tensors are rotated so that
consecutive steps do not find their inputs in the 256 MB Infinity Cache.

Prints ONE JSON line: metric = query tokens/s per layer, plus the roofline of the dominant
kernel (the sparse flash forward, bf16 MFMA bound), HBM figures for absorb/readout, the
speedup over the in-repo dense window kernel, and the fp64 oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def profile_value(workload: str, kind: str, key: str):
    """`key=value` line of profiles/bench_<workload>_<kind>.txt, as written by
    `python -m paper_2604_10103_amd.profile_summary` from rocprofv3 runs of this file; None if there is no such
    profile (the figure then stays out of the JSON line rather than being kept by hand)."""
    path = os.path.join(ROOT, "profiles", f"bench_{workload}_{kind}.txt")
    try:
        for line in open(path):
            if line.startswith(key + "="):
                v = float(line.split("=", 1)[1])
                return v if v == v else None
    except (OSError, ValueError):
        pass
    return None


def parse():
    p = argparse.ArgumentParser()
    p.add_argument("--gpus", type=int, default=1)
    p.add_argument("--steps", type=int, default=300)
    p.add_argument("--warmup", type=int, default=12)
    p.add_argument("--workload", default="step_832x480")
    p.add_argument("--layers", type=int, default=6, help="distinct layer tensor sets rotated through")
    p.add_argument("--keep-ratio", type=float, default=None)
    p.add_argument("--no-cpu-baseline", action="store_true")
    p.add_argument("--rope", action="store_true",
                   help="rotate phi(k) / phi(q) of the history branch with synthetic per-token tables (default: none)")
    p.add_argument("--no-dense", action="store_true",
                   help="skip the dense comparator launches (they share the sparse kernel's name in a profile)")
    p.add_argument("--no-backward", action="store_true", help="skip the timing of the backward pass (training step)")
    p.add_argument("--converted-planes", action="store_true",
                   help="let every attention call convert the state to its bf16 planes (hf_hybrid_attn_fwd) instead "
                        "of keeping them next to the state (hf_absorb_evicted_planes / hf_hybrid_attn_fwd_planes)")
    p.add_argument("--separate-launches", action="store_true",
                   help="the step as hf_block_select + hf_hybrid_attn_fwd_planes + hf_absorb_evicted_planes (four "
                        "launches) instead of hf_pool_keys + hf_step_fwd (two)")
    p.add_argument("--eager", action="store_true",
                   help="time eager single-stream launches instead of one captured HIP graph per step")
    p.add_argument("--cpu-heads", type=int, default=0, help="heads per layer the oracle is timed on (0 = all)")
    p.add_argument("--cpu-layers", type=int, default=6, help="layer sets the oracle is timed on")
    p.add_argument("--no-extras", action="store_true",
                   help="skip the layer-stack run (30 layers x 4 steps) and the keep-ratio sweep at the large shape")
    p.add_argument("--calibration-copy-mib", type=int, default=0,
                   help="also run one plain device copy of this size (reference for HBM byte counters)")
    return p.parse_args()


def algorithmic_flops(idx_cpu, w):
    """4 * d * sum over (head, query block) of real rows * real selected keys."""
    import numpy as np
    idx = idx_cpu.numpy().astype(np.int64)
    b = w.block
    rows = np.minimum(b, w.n_q - np.arange(w.t_m) * b)                       # [T_m]
    keys = np.minimum(b, w.n_kv - idx * b).sum(axis=-1)                      # [B,H,T_m]
    return float(4.0 * w.head_dim * (keys * rows[None, None, :]).sum())


def run_extras(hf, wl, torch, np, dev):
    """Two further measurements, outside the timed step: the attention stack of one denoising pass (30 layers x 4
    steps of the 832x480 layer call on 30 distinct layer sets, cached window half and state frozen across the
    steps of a layer) and the keep-ratio sweep at the 1280x720 shape.  Inputs are drawn on the GPU from seeded
    generators (no oracle runs on them; the parity tests cover these shapes with the CPU-seeded inputs)."""
    out = {}

    def gpu_randn(shape, seed, scale, dtype):
        g = torch.Generator(device=dev).manual_seed(int(seed))
        return (torch.randn(shape, generator=g, device=dev, dtype=torch.float32) * scale).to(dtype)

    # ---- layer stack: 30 layers x 4 denoising steps = 120 select + attention calls
    w = wl.get("step_832x480")
    cfg = hf.make_config(w.batch, w.heads, w.head_dim, w.dtype, w.block, w.block, w.keep_ratio)
    k = hf.hf_select_k(cfg, w.n_kv)
    n_layers, n_steps = 30, 4
    shape_q = (w.batch, w.heads, w.n_q, w.head_dim)
    shape_kv = (w.batch, w.heads, w.n_kv, w.head_dim)
    n_old = w.n_kv - w.n_q
    aws = torch.empty(hf.hf_absorb_workspace_bytes(cfg, w.n_q), dtype=torch.uint8, device=dev)
    layers = []
    for l in range(n_layers):
        K = gpu_randn(shape_kv, 40_000 + 100 * l + 1, w.scale, w.torch_dtype)
        V = gpu_randn(shape_kv, 40_000 + 100 * l + 2, w.scale, w.torch_dtype)
        st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=dev)
        hf.hf_state_init(cfg, st)
        planes = torch.empty(hf.hf_state_planes_bytes(cfg), dtype=torch.uint8, device=dev)
        hf.hf_absorb_evicted_planes(cfg, st, gpu_randn(shape_q, 45_000 + l, w.scale, w.torch_dtype),
                                    gpu_randn(shape_q, 47_500 + l, w.scale, w.torch_dtype), planes, workspace=aws)
        steps = []
        for s in range(n_steps):   # per (layer, step): new queries and the chunk's own keys and values
            steps.append((gpu_randn(shape_q, 40_000 + 100 * l + 10 * s, w.scale, w.torch_dtype),
                          gpu_randn(shape_q, 40_000 + 100 * l + 10 * s + 3, w.scale, w.torch_dtype),
                          gpu_randn(shape_q, 40_000 + 100 * l + 10 * s + 4, w.scale, w.torch_dtype)))
        layers.append(dict(K=K, V=V, st=st, planes=planes, steps=steps,
                           idx=torch.empty((w.batch, w.heads, w.t_m, k), dtype=torch.int32, device=dev),
                           O=torch.empty(shape_q, dtype=w.torch_dtype, device=dev),
                           pooled=torch.empty(hf.hf_pooled_keys_bytes(cfg, w.n_kv), dtype=torch.uint8, device=dev)))
    reuse = n_old // w.block

    def layer_call(L, s, events=None):
        Q, Kc, Vc = L["steps"][s]
        # the chunk's own K, V of this step take their place behind the cached half (the model's write, not timed)
        L["K"][:, :, n_old:].copy_(Kc)
        L["V"][:, :, n_old:].copy_(Vc)
        if events is not None:
            events[0].record()
        # the pooled keys of the frozen half are reused after a layer's first step; selection, attention and the
        # history term are one launch
        hf.hf_pool_keys(cfg, L["K"], L["pooled"], reuse if s > 0 else 0)
        hf.hf_select_attn_fwd(cfg, Q, L["K"], L["V"], L["pooled"], L["st"], L["planes"], L["O"], L["idx"])
        if events is not None:
            events[1].record()

    for s in range(n_steps):          # warm-up pass (also leaves the pooled keys of every layer in its workspace)
        for L in layers:
            layer_call(L, s)
    torch.cuda.synchronize()
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in layers]
           for _ in range(n_steps)]
    for s in range(n_steps):
        for i, L in enumerate(layers):
            layer_call(L, s, evs[s][i])
    torch.cuda.synchronize()
    ts = np.array([[e[0].elapsed_time(e[1]) for e in row] for row in evs])   # [steps, layers] ms
    out["stack_30x4"] = {
        "workload": "30 layers x 4 denoising steps of the step_832x480 layer call (hf_pool_keys + hf_select_attn_fwd), 30 distinct "
                    "layer sets (1.7 GB of K, V), cached window half and state frozen across a layer's steps",
        "calls": int(ts.size), "total_ms": float(ts.sum()), "mean_ms": float(ts.mean()), "min_ms": float(ts.min()),
        "max_ms": float(ts.max()), "first_step_mean_ms": float(ts[0].mean()), "later_steps_mean_ms": float(ts[1:].mean()),
        "query_tokens_per_s": float(w.n_q * ts.size / (ts.sum() * 1e-3)), "timing": "HIP events around each call, eager launches"}
    del layers

    # ---- keep-ratio sweep at the 1280x720 shape
    w = wl.get("large_1280x720")
    shape_q = (w.batch, w.heads, w.n_q, w.head_dim)
    shape_kv = (w.batch, w.heads, w.n_kv, w.head_dim)
    sets = [(gpu_randn(shape_q, 50_000 + 10 * l, w.scale, w.torch_dtype), gpu_randn(shape_kv, 50_001 + 10 * l, w.scale, w.torch_dtype),
             gpu_randn(shape_kv, 50_002 + 10 * l, w.scale, w.torch_dtype)) for l in range(2)]
    O = torch.empty(shape_q, dtype=w.torch_dtype, device=dev)
    sweep = []
    for keep in (0.125, 0.25, 0.5, 1.0):
        cfg = hf.make_config(w.batch, w.heads, w.head_dim, w.dtype, w.block, w.block, keep)
        k = hf.hf_select_k(cfg, w.n_kv)
        ws = torch.empty(hf.hf_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=dev)
        idxs = [torch.empty((w.batch, w.heads, w.t_m, k), dtype=torch.int32, device=dev) for _ in sets]

        def timed(fn, reps=3):
            for i in range(len(sets)):
                fn(i)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                for i in range(len(sets)):
                    fn(i)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / (reps * len(sets))

        sel_ms = timed(lambda i: hf.hf_block_select(cfg, sets[i][0], sets[i][1], idxs[i], None, ws))
        dense = keep >= 1.0
        att_ms = timed(lambda i: hf.hf_hybrid_attn_fwd(cfg, sets[i][0], sets[i][1], sets[i][2], None if dense else idxs[i],
                                                       None, O, ws))
        fl = float(np.mean([algorithmic_flops(ix.cpu(), w) for ix in idxs]))
        sweep.append({"keep_ratio": keep, "k": k, "select_ms": sel_ms, "sparse_flash_fwd_ms": att_ms,
                      "tflops": fl / (att_ms * 1e-3) / 1e12, "frac_of_bf16_peak": fl / (att_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS})
    base = sweep[-1]["sparse_flash_fwd_ms"]
    for r in sweep:
        r["speedup_over_dense_incl_select"] = base / (r["sparse_flash_fwd_ms"] + (0.0 if r["keep_ratio"] >= 1.0 else r["select_ms"]))
    out["large_1280x720_keep_sweep"] = {"heads": w.heads, "n_q": w.n_q, "n_kv": w.n_kv, "block": w.block, "rows": sweep}
    return out


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (heads are independent in every "
              "step and would shard without exchange); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2604_10103_amd as hf
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    hf.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = wl.get(a.workload)
    keep = w.keep_ratio if a.keep_ratio is None else a.keep_ratio
    cfg = hf.make_config(w.batch, w.heads, w.head_dim, w.dtype, w.block, w.block, keep)
    cfg_dense = hf.make_config(w.batch, w.heads, w.head_dim, w.dtype, w.block, w.block, 1.0)
    k = hf.hf_select_k(cfg, w.n_kv)
    nl = max(1, a.layers)
    esz = 2 if w.dtype == "bf16" else 4

    # ---- resident inputs
    sets = []
    chunk_frames = w.chunk_frames
    n_prefill_calls = max(1, w.evicted_frames // chunk_frames)
    prefill = [tuple(t.to(dev) for t in wl.make_evicted(w, c)) for c in range(n_prefill_calls)]
    ws_bytes = hf.hf_workspace_bytes(cfg, w.n_q, w.n_kv)
    aws_bytes = hf.hf_absorb_workspace_bytes(cfg, w.n_q)
    aws = torch.empty(aws_bytes, dtype=torch.uint8, device=dev) if aws_bytes else None
    keep_planes = (not a.converted_planes) and hf.hf_state_planes_bytes(cfg) > 0
    # the two-launch step: bf16 / head_dim 128 shapes with kept planes, ReLU, no rotation of the absorbed keys
    one_launch = keep_planes and not a.separate_launches and not a.rope
    for l in range(nl):
        Q, K, V = wl.make_qkv(w, layer=l)
        Ke, Ve = wl.make_evicted(w, 100 + l)
        st = torch.empty(hf.hf_state_bytes(cfg) // 4, dtype=torch.float32, device=dev)
        hf.hf_state_init(cfg, st)
        for (pk, pv) in prefill:
            hf.hf_absorb_evicted(cfg, st, pk, pv, workspace=aws)
        planes = None
        if keep_planes:   # the bf16 planes of the state, kept current by the absorb call from here on
            planes = torch.empty(hf.hf_state_planes_bytes(cfg), dtype=torch.uint8, device=dev)
            hf.hf_state_planes(cfg, st, planes)
        sets.append(dict(
            Q=Q.to(dev), K=K.to(dev), V=V.to(dev), Ke=Ke.to(dev), Ve=Ve.to(dev), st=st, planes=planes,
            idx=torch.empty((w.batch, w.heads, w.t_m, k), dtype=torch.int32, device=dev),
            O=torch.empty(Q.shape, dtype=Q.dtype, device=dev),
            ws=torch.empty(ws_bytes, dtype=torch.uint8, device=dev), Qc=Q, Kc=K, Vc=V))
        if keep_planes and not a.rope:   # second state buffer, pooled keys and workspace of the two-launch step
            sets[-1].update(
                st2=torch.empty_like(st), planes2=torch.empty_like(planes), phase=0,
                pooled=torch.empty(hf.hf_pooled_keys_bytes(cfg, w.n_kv), dtype=torch.uint8, device=dev),
                sws=torch.empty(hf.hf_step_workspace_bytes(cfg, w.n_q, w.n_q), dtype=torch.uint8, device=dev))
    del prefill
    torch.cuda.synchronize()

    rq = re_ = (None, None)
    if a.rope:   # caller-side tables (positions in frames); shared by heads and layer sets
        rq = tuple(t.to(dev) for t in wl.rope_tables(w.n_q, w.head_dim, first_position=21.0,
                                                     tokens_per_position=w.tokens_per_frame))
        re_ = tuple(t.to(dev) for t in wl.rope_tables(w.n_q, w.head_dim, first_position=3.0,
                                                      tokens_per_position=w.tokens_per_frame))

    def step_fused(s, events=None):
        """hf_pool_keys + hf_step_fwd: the state alternates between the set's two buffers."""
        ph = s["phase"]
        st_in, pl_in = (s["st"], s["planes"]) if ph == 0 else (s["st2"], s["planes2"])
        st_out, pl_out = (s["st2"], s["planes2"]) if ph == 0 else (s["st"], s["planes"])
        if events is not None:
            events[0].record()
        hf.hf_pool_keys(cfg, s["K"], s["pooled"])
        if events is not None:
            events[1].record()
        hf.hf_step_fwd(cfg, s["Q"], s["K"], s["V"], s["pooled"], st_in, pl_in, s["O"], s["idx"], s["Ke"], s["Ve"],
                       st_out, pl_out, s["sws"])
        if events is not None:
            events[2].record()
            events[3].record()
        s["phase"] = 1 - ph

    def step_separate(s, events=None):
        if events is not None:
            events[0].record()
        hf.hf_block_select(cfg, s["Q"], s["K"], s["idx"], None, s["ws"])
        if events is not None:
            events[1].record()
        if keep_planes:
            hf.hf_hybrid_attn_fwd_planes(cfg, s["Q"], s["K"], s["V"], s["idx"], s["st"], s["planes"], s["O"], rq[0], rq[1])
        else:
            hf.hf_hybrid_attn_fwd(cfg, s["Q"], s["K"], s["V"], s["idx"], s["st"], s["O"], s["ws"], rq[0], rq[1])
        if events is not None:
            events[2].record()
        if keep_planes:
            hf.hf_absorb_evicted_planes(cfg, s["st"], s["Ke"], s["Ve"], s["planes"], re_[0], re_[1], workspace=aws)
        else:
            hf.hf_absorb_evicted(cfg, s["st"], s["Ke"], s["Ve"], re_[0], re_[1], workspace=aws)
        if events is not None:
            events[3].record()

    step = step_fused if one_launch else step_separate

    if a.calibration_copy_mib > 0:   # a copy of known size: what FETCH_SIZE / WRITE_SIZE read for it scales the rest
        src = torch.empty(a.calibration_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        src.fill_(1)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(max(a.warmup, nl if not a.eager else 0)):
        step(sets[i % nl])
    torch.cuda.synchronize()

    # ---- per-call times: eager launches with HIP events on the launch stream
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(a.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(a.steps):
        step(sets[i % nl], evs[i])
    torch.cuda.synchronize()
    wall_eager = time.perf_counter() - t0
    step_calls_ms = None
    if one_launch:
        # per-call times of the two launches, then those of the separate calls (selection, attention with the
        # history term, absorb) from eager steps of their own
        step_calls_ms = {"pool_keys": float(np.mean([e[0].elapsed_time(e[1]) for e in evs])),
                         "step_fwd": float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))}
        for i in range(nl):
            step_separate(sets[i % nl])
        torch.cuda.synchronize()
        for i in range(a.steps):
            step_separate(sets[i % nl], evs[i])
        torch.cuda.synchronize()
    sel_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    fwd_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
    abs_ms = float(np.mean([e[2].elapsed_time(e[3]) for e in evs]))

    # ---- timed region: exactly `steps` steps, launched as captured HIP graphs (same kernels, same
    # order, same stream as the eager step; what goes away is the host's launch gap between the six
    # kernels of a step).  One graph holds one pass over the rotated layer sets; a remainder of
    # steps runs from single-step graphs.
    def timed_graphs(step_fn, phases):
        """`a.steps` steps of step_fn from captured graphs of one pass over the rotated sets each (`phases` of them,
        replayed in turn: the two-launch step alternates its state buffers, so its second pass is a graph of its
        own); a remainder of steps runs from single-step graphs.  Warm-up: whole passes."""
        def capture(group):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for s in group:
                    step_fn(s)
            return g
        torch.cuda.synchronize()
        g_pass = [capture(sets) for _ in range(phases)]          # (capturing runs the host side: the phases advance)
        n_pass, rem = a.steps // nl, a.steps % nl
        # the remainder follows n_pass + warm-up passes: capture it in the phase the sets will have then
        warm = -(-max(a.warmup, nl) // nl)
        for _ in range((warm + n_pass) % phases):
            for s in sets:
                if "phase" in s:
                    s["phase"] = 1 - s["phase"]
        g_one = [capture([s]) for s in sets[:rem]]
        for i in range(warm):
            g_pass[i % phases].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_pass):
            g_pass[(warm + i) % phases].replay()
        for g in g_one:
            g.replay()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    ms_separate = None
    if a.eager:
        wall, mode = wall_eager, "eager launches"
    else:
        wall = timed_graphs(step, 2 if one_launch else 1)
        mode = f"HIP graphs of {nl} steps"
        if one_launch:   # the four-launch step next to it, same sets, same way of launching
            ms_separate = timed_graphs(step_separate, 1) * 1e3 / a.steps
    ms_per_step = wall * 1e3 / a.steps

    # ---- the sparse flash forward alone (no state => only that kernel runs), same inputs
    def time_calls(fn, n):
        """Mean and best time of one call: events bracket passes of back-to-back calls over the rotated
        layer sets (a pair of events around a single ~100 us launch would add its own few us)."""
        passes = max(1, n // nl)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(passes)]
        for s in sets[:min(3, nl)]:
            fn(s)
        torch.cuda.synchronize()
        for e0, e1 in ev:
            e0.record()
            for s in sets:
                fn(s)
            e1.record()
        torch.cuda.synchronize()
        ts = [x.elapsed_time(y) / nl for x, y in ev]
        return float(np.mean(ts)), float(np.min(ts))

    pool_ms = stepf_ms = selattn_ms = None
    if "pooled" in sets[0]:
        pool_ms, _ = time_calls(lambda s: hf.hf_pool_keys(cfg, s["K"], s["pooled"]), a.steps)
        selattn_ms, _ = time_calls(lambda s: hf.hf_select_attn_fwd(cfg, s["Q"], s["K"], s["V"], s["pooled"], s["st"],
                                                                   s["planes"], s["O"], s["idx"]), a.steps)
        stepf_ms, _ = time_calls(lambda s: hf.hf_step_fwd(cfg, s["Q"], s["K"], s["V"], s["pooled"], s["st"], s["planes"],
                                                          s["O"], s["idx"], s["Ke"], s["Ve"], s["st2"], s["planes2"],
                                                          s["sws"]), a.steps)
        for s in sets:   # (the state of the timed steps' last phase is the one the later measurements read)
            if s["phase"]:
                s["st"], s["st2"], s["planes"], s["planes2"], s["phase"] = s["st2"], s["st"], s["planes2"], s["planes"], 0
    a4_ms, a4_min = time_calls(
        lambda s: hf.hf_hybrid_attn_fwd(cfg, s["Q"], s["K"], s["V"], s["idx"], None, s["O"], s["ws"]), a.steps)
    # selection on the later denoising steps of a chunk: pooled keys of the unchanged older half reused
    reuse = (w.n_kv - w.n_q) // w.block
    selc_ms, _ = time_calls(
        lambda s: hf.hf_block_select_cached(cfg, s["Q"], s["K"], reuse, s["idx"], None, s["ws"]), a.steps)
    dense_ms = None
    if not a.no_dense:
        dense_ms, _ = time_calls(
            lambda s: hf.hf_hybrid_attn_fwd(cfg_dense, s["Q"], s["K"], s["V"], None, None, s["O"], s["ws"]),
            max(3, min(a.steps, 10)))
    # the history readout as a kernel of its own (two-kernel path of hf_hybrid_attn_fwd) for its HBM roofline;
    # the default path adds the history term in the attention epilogue
    cfg_two = hf.make_config(w.batch, w.heads, w.head_dim, w.dtype, w.block, w.block, keep,
                             flags=hf.HF_FLAG_READOUT_KERNEL)
    fwd2_ms, _ = time_calls(
        lambda s: hf.hf_hybrid_attn_fwd(cfg_two, s["Q"], s["K"], s["V"], s["idx"], s["st"], s["O"], s["ws"], rq[0], rq[1]),
        a.steps)
    a5_ms = max(fwd2_ms - a4_ms, 0.0)

    # practical HBM ceiling at this size: a plain device copy of the readout's byte count (read + written)
    n_copy = (3 * w.batch * w.heads * w.n_q * w.head_dim * esz) // 2
    cp_src = [torch.empty(n_copy, dtype=torch.uint8, device=dev).fill_(l) for l in range(nl)]
    cp_dst = torch.empty(n_copy, dtype=torch.uint8, device=dev)
    it = iter(range(1 << 30))
    copy_ms, _ = time_calls(lambda s: cp_dst.copy_(cp_src[next(it) % nl]), a.steps)
    del cp_src, cp_dst

    # preparation of Sec. 3.3 around the step, once per chunk and so outside the timed step: cos/sin tables of the
    # window from its re-based frame indices, and the rotated copy of the window's keys that the softmax branch reads
    rows, cols = wl.frame_grid(w)
    pairs = (w.head_dim // 2 - 2 * (w.head_dim // 6), w.head_dim // 6, w.head_dim // 6)
    win_idx = hf.hf_rope_window_indices(200, w.window_frames, 21)
    kc = torch.empty((w.n_kv, w.head_dim // 2), dtype=torch.float32, device=dev)
    ks = torch.empty_like(kc)
    k_rot = torch.empty_like(sets[0]["K"])
    tab_ms, _ = time_calls(lambda s: hf.hf_rope_tables(win_idx, rows, cols, pairs, kc, ks), a.steps)
    ropek_ms, _ = time_calls(lambda s: hf.hf_rope_apply(cfg, s["K"], kc, ks, k_rot), a.steps)
    rope_bytes = 2 * w.batch * w.heads * w.n_kv * w.head_dim * esz + 2 * kc.numel() * 4
    # per denoising step of a model that rotates its keys: the chunk's own keys rotated into the window and their
    # KV blocks pooled in the same pass (no pooling launch on that step)
    append_ms = None
    if "pooled" in sets[0]:
        n_old = w.n_kv - w.n_q
        qc_tab, qs_tab = kc[n_old:].contiguous(), ks[n_old:].contiguous()
        append_ms, _ = time_calls(lambda s: hf.hf_rope_append_keys(cfg, s["Q"], qc_tab, qs_tab, k_rot, n_old, s["pooled"]),
                                  a.steps)   # (Q stands in for the chunk's new keys: same shape and type)
        for s in sets:
            hf.hf_pool_keys(cfg, s["K"], s["pooled"])
    del k_rot

    # the training algorithm's gradient step (outside the timed step, which is the inference path): dQ, dK, dV of
    # one layer call, row statistics recomputed
    bwd_ms = None
    if not a.no_backward:
        bws = torch.empty(hf.hf_bwd_workspace_bytes(cfg, w.n_q, w.n_kv), dtype=torch.uint8, device=dev)
        dO = wl.randn(sets[0]["Q"].shape, 96_000, 1.0, w.torch_dtype).to(dev)
        dQ, dK, dV = torch.empty_like(sets[0]["Q"]), torch.empty_like(sets[0]["K"]), torch.empty_like(sets[0]["V"])
        bwd_ms, _ = time_calls(lambda s: hf.hf_hybrid_attn_bwd(cfg, s["Q"], s["K"], s["V"], s["idx"], s["st"], dO, dQ, dK,
                                                               dV, bws), max(3, min(a.steps, 12)))
        # the same from the by-products of the saving forward: O_local and the softmax row statistic
        Ol = torch.empty_like(sets[0]["Q"])
        lse = torch.empty((w.batch * w.heads, w.n_q), dtype=torch.float32, device=dev)
        fwd_save_ms, _ = time_calls(lambda s: hf.hf_hybrid_attn_fwd_save(cfg, s["Q"], s["K"], s["V"], s["idx"], s["st"],
                                                                         s["O"], Ol, lse, s["ws"]), max(3, min(a.steps, 12)))
        bwd_saved_ms, _ = time_calls(lambda s: hf.hf_hybrid_attn_bwd_saved(cfg, s["Q"], s["K"], s["V"], s["idx"], s["st"],
                                                                           dO, Ol, lse, dQ, dK, dV, bws),
                                     max(3, min(a.steps, 12)))
        del bws, dO, dQ, dK, dV, Ol, lse

    # ---- what the matrix cores sustain when they do nothing else: the MFMA of the attention kernels, two wavefronts
    # per SIMD, non-trivial operands (a practical ceiling next to the nominal peak)
    scratch4 = torch.zeros(4, dtype=torch.float32, device=dev)
    probe_flops = hf.hf_probe_mfma_bf16(2000, scratch4)
    torch.cuda.synchronize()
    pe = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    pe[0].record()
    for _ in range(3):
        hf.hf_probe_mfma_bf16(2000, scratch4)
    pe[1].record()
    torch.cuda.synchronize()
    mfma_ceiling_tflops = 3 * probe_flops / (pe[0].elapsed_time(pe[1]) * 1e-3) / 1e12

    extras = {}
    if not a.no_extras:
        extras = run_extras(hf, wl, torch, np, dev)

    flops = float(np.mean([algorithmic_flops(s["idx"].cpu(), w) for s in sets]))
    dense_flops = 4.0 * w.head_dim * w.n_q * w.n_kv * w.heads * w.batch
    bh = w.batch * w.heads
    state_bytes = hf.hf_state_bytes(cfg)
    absorb_bytes = 2 * bh * w.n_q * w.head_dim * esz + 2 * state_bytes
    readout_bytes = 3 * bh * w.n_q * w.head_dim * esz + state_bytes
    select_bytes = bh * (w.n_q + w.n_kv) * w.head_dim * esz + bh * w.t_m * k * 4
    a4_tflops = flops / (a4_ms * 1e-3) / 1e12

    out = {
        "metric": "hybrid-attn query tokens/s per layer (select + sparse flash fwd + readout + absorb)",
        "step": ("hf_pool_keys + hf_step_fwd (2 launches: selection in the attention workgroups' prologue, absorb in "
                 "workgroups of their own)") if one_launch else
                "hf_block_select + hf_hybrid_attn_fwd + hf_absorb_evicted (4 launches)",
        "ms_per_step_separate_launches": ms_separate,
        "value": w.n_q * w.batch / (ms_per_step * 1e-3),
        "unit": "query tokens/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": ms_per_step,
        "launch": mode,
        "ms_per_step_eager": wall_eager * 1e3 / a.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "heads": w.heads, "head_dim": w.head_dim,
                   "n_q": w.n_q, "n_kv": w.n_kv, "block": w.block, "keep_ratio": keep, "k": k,
                   "t_n": w.t_n, "evicted_tokens_in_state": w.n_evicted, "rotated_layer_sets": nl,
                   "history_rope": bool(a.rope), "state_planes": "kept by the absorb call" if keep_planes else "converted per attention call"},
        "roofline": {"kernel": "sparse flash forward (Eq. 5)", "bound": "mfma", "achieved": a4_tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": a4_tflops / PEAK_BF16_TFLOPS,
                     # HBM-side bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size) and the
                     # kernel's average duration in the rocprofv3 trace, both read from profiles/ (null without)
                     "traffic": profile_value(w.name, "hbm_traffic", "a4_hbm_bytes_per_launch") if a.keep_ratio is None else None,
                     "flops_per_launch": flops, "avg_ms": a4_ms, "min_ms": a4_min,
                     "avg_ms_timing": "HIP events around back-to-back launches over the rotated layer sets (gaps included)",
                     "avg_ms_rocprofv3": (lambda v: None if v is None else v * 1e-3)(
                         profile_value(w.name, "kernel_trace", "a4_avg_us") if a.keep_ratio is None else None),
                     "mfma_issue_ceiling_tflops": mfma_ceiling_tflops,
                     "frac_of_issue_ceiling": a4_tflops / mfma_ceiling_tflops},
        "kernels_ms": {"block_select": sel_ms, "block_select_cached_half": selc_ms, "attn_fwd_total": fwd_ms, "sparse_flash_fwd": a4_ms,
                       "readout_combine_unfused": a5_ms, "fused_epilogue_extra": max(fwd_ms - a4_ms, 0.0), "absorb": abs_ms,
                       "dense_window_fwd": dense_ms, "rope_tables_window": tab_ms, "rope_apply_k_window": ropek_ms,
                       "pool_keys": pool_ms, "select_attn_fwd": selattn_ms, "step_fwd": stepf_ms,
                       "in_step_eager": step_calls_ms, "rope_append_keys_chunk": append_ms},
        "hbm": {"absorb_GBs": absorb_bytes / (abs_ms * 1e-3) / 1e9,
                "absorb_frac": absorb_bytes / (abs_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                "readout_GBs": (readout_bytes / (a5_ms * 1e-3) / 1e9) if a5_ms > 0 else None,
                "readout_frac": (readout_bytes / (a5_ms * 1e-3) / 1e9 / PEAK_HBM_GBS) if a5_ms > 0 else None,
                "select_GBs": select_bytes / (sel_ms * 1e-3) / 1e9,
                "rope_apply_GBs": rope_bytes / (ropek_ms * 1e-3) / 1e9,
                "device_copy_GBs": 2 * n_copy / (copy_ms * 1e-3) / 1e9,
                "peak_GBs": PEAK_HBM_GBS,
                "bytes": {"absorb": absorb_bytes, "readout": readout_bytes, "select": select_bytes,
                          "rope_apply": rope_bytes}},
    }
    if bwd_ms is not None:
        # five products of the forward's size (S, dP, dV, dK, dQ) count; the recomputation does not
        out["backward"] = {"ms": bwd_ms, "tflops": 2.5 * flops / (bwd_ms * 1e-3) / 1e12,
                           "frac_of_bf16_peak": 2.5 * flops / (bwd_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                           # training pair: the forward that also writes O_local and the row statistic, and the
                           # backward pass that starts from them (2 algorithmic products less: no recomputed forward)
                           "fwd_save_ms": fwd_save_ms, "saved_ms": bwd_saved_ms}
    out.update(extras)
    if dense_ms is not None:
        out["dense"] = {"tflops": dense_flops / (dense_ms * 1e-3) / 1e12,
                        "speedup_sparse_incl_select": dense_ms / (sel_ms + a4_ms),
                        "speedup_kernel_only": dense_ms / a4_ms, "ideal": w.t_n / k}

    if not a.no_cpu_baseline:
        import oracle as orc
        heads = list(range(w.heads if a.cpu_heads <= 0 else min(a.cpu_heads, w.heads)))
        layers = list(range(min(max(1, a.cpu_layers), nl)))
        Ke, Ve = wl.make_evicted(w, 0)
        t0 = time.perf_counter()
        for l in layers:
            s0 = sets[l]
            for h in heads:
                q, kk, v = (wl.to_f64(s0[n][0, h]) for n in ("Qc", "Kc", "Vc"))
                st = orc.state_absorb(*orc.state_zero(w.head_dim), wl.to_f64(Ke[0, h]), wl.to_f64(Ve[0, h]))
                orc.hybrid_attention(q, kk, v, st, w.block, w.block, k)
        t_cpu = time.perf_counter() - t0
        per_layer = t_cpu / (len(heads) * len(layers)) * w.heads * w.batch
        try:
            cores = len(os.sched_getaffinity(0))
        except AttributeError:
            cores = os.cpu_count()
        out["cpu_baseline"] = {
            "value": w.n_q * w.batch / per_layer, "unit": "query tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"fp64 NumPy oracle, {len(heads)} of {w.heads} heads of {len(layers)} layer steps at the full "
                      f"chunk shape (scores, top-k, sparse attention, readout, one absorb), {t_cpu:.1f} s of "
                      f"CPU work, scaled to one {w.heads}-head layer step"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
