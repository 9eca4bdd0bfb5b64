"""Workload shapes and seeded generators.

The paper evaluates a Wan2.1-1.3B-based streaming generator at 832x480 (Sec. 4.1): 30x52 =
1560 patch tokens per latent frame, chunks of three latent frames, 12 heads of width 128.
Its prompts, weights and evaluation suites are not used; i.i.d. Gaussians of these shapes
stand in for Q, K, V.  Values are drawn in fp32 on the CPU from ``torch.Generator`` with a
documented seed, scaled, and rounded to the workload's storage dtype.  Both the oracle
(after an exact up-cast to fp64) and the GPU path read these same stored values.
"""
from __future__ import annotations

import dataclasses

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    cfg: int               # index used in seeds
    dtype: str             # "bf16" | "f32": storage type of Q, K, V, O (state is always f32)
    batch: int
    heads: int
    head_dim: int
    tokens_per_frame: int
    chunk_frames: int
    window_frames: int     # window includes the current chunk
    block: int             # b_q == b_kv
    keep_ratio: float
    evicted_frames: int    # frames already absorbed into the linear state
    scale: float           # input standard deviation

    @property
    def n_q(self) -> int:
        return self.tokens_per_frame * self.chunk_frames

    @property
    def n_kv(self) -> int:
        return self.tokens_per_frame * self.window_frames

    @property
    def n_evicted(self) -> int:
        return self.tokens_per_frame * self.evicted_frames

    @property
    def t_m(self) -> int:
        return -(-self.n_q // self.block)

    @property
    def t_n(self) -> int:
        return -(-self.n_kv // self.block)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32


WORKLOADS = {
    # tiny fp32 streaming case
    "tiny_f32": Workload("tiny_f32", 1, "f32", 1, 2, 64, 64, 1, 4, 16, 0.25, 8, 1.0),
    # one layer of the 832x480 step
    "step_832x480": Workload("step_832x480", 2, "bf16", 1, 12, 128, 1560, 3, 6, 64, 0.25, 15, 0.5),
    # large-model shape, 1280x720-like frames
    "large_1280x720": Workload("large_1280x720", 5, "bf16", 1, 40, 128, 3600, 3, 6, 128, 0.25, 30, 0.5),
    # reduced shapes for element-by-element parity (several tiles + ragged tails, oracle in seconds)
    "small_bf16": Workload("small_bf16", 6, "bf16", 1, 3, 128, 200, 2, 5, 64, 0.25, 4, 0.5),
    "small_b128": Workload("small_b128", 7, "bf16", 1, 2, 128, 300, 2, 5, 128, 0.5, 3, 0.5),
    "small_f32_d128": Workload("small_f32_d128", 8, "f32", 1, 2, 128, 100, 2, 5, 32, 0.3, 3, 1.0),
}


def get(name: str) -> Workload:
    return WORKLOADS[name]


_ROLE = {"Q": 0, "K": 1, "V": 2}


def seed_for(cfg: int, role: str, layer: int = 0, step: int = 0) -> int:
    """S = 10000*cfg + 100*layer + 10*step + {Q:0, K:1, V:2}."""
    return 10_000 * cfg + 100 * layer + 10 * step + _ROLE[role]


def randn(shape, seed: int, scale: float, dtype) -> torch.Tensor:
    g = torch.Generator(device="cpu").manual_seed(int(seed))
    x = torch.randn(tuple(shape), generator=g, dtype=torch.float32) * float(scale)
    return x.to(dtype).contiguous()


def make_qkv(w: Workload, layer: int = 0, step: int = 0, q_gain: float = 1.0):
    """Q [B,H,n_q,d] and the window K, V [B,H,n_kv,d] (older frames first, chunk last).

    ``q_gain`` > 1 gives the 'peaky' variant whose logits exercise the online-softmax rescale.
    """
    d = w.head_dim
    Q = randn((w.batch, w.heads, w.n_q, d), seed_for(w.cfg, "Q", layer, step), w.scale * q_gain, w.torch_dtype)
    K = randn((w.batch, w.heads, w.n_kv, d), seed_for(w.cfg, "K", layer, step), w.scale, w.torch_dtype)
    V = randn((w.batch, w.heads, w.n_kv, d), seed_for(w.cfg, "V", layer, step), w.scale, w.torch_dtype)
    return Q, K, V


def make_evicted(w: Workload, chunk_index: int, n_tokens: int | None = None):
    """K, V [B,H,n,d] of one evicted run of tokens; seed 10000*cfg + 5000 + chunk_index (+2500 for V)."""
    n = w.n_q if n_tokens is None else int(n_tokens)
    base = 10_000 * w.cfg + 5_000 + int(chunk_index)
    K = randn((w.batch, w.heads, n, w.head_dim), base, w.scale, w.torch_dtype)
    V = randn((w.batch, w.heads, n, w.head_dim), base + 2_500, w.scale, w.torch_dtype)
    return K, V


def rope_tables(n_tokens: int, head_dim: int, first_position: float = 0.0,
                tokens_per_position: int = 1, theta: float = 10_000.0):
    """Synthetic per-token rotation tables cos, sin [n_tokens, d/2] in fp32.

    Token t sits at position first_position + t // tokens_per_position; pair i turns by
    position * theta^(-2i/d).  INPUT GENERATION ONLY: these tables are data that a caller hands to the library
    and to the oracle alike (like Q, K, V); neither side's rotary arithmetic lives here (the oracle's is
    oracle/rope.py, pinned by its own tests; the library's is csrc/hf_rope.hip), and nothing of the method may be
    added to this module.
    """
    pos = first_position + np.floor(np.arange(n_tokens, dtype=np.float64) / tokens_per_position)
    freq = theta ** (-2.0 * np.arange(head_dim // 2, dtype=np.float64) / head_dim)
    ang = pos[:, None] * freq[None, :]
    cos = torch.from_numpy(np.cos(ang)).to(torch.float32).contiguous()
    sin = torch.from_numpy(np.sin(ang)).to(torch.float32).contiguous()
    return cos, sin


_FRAME_GRID = {64: (8, 8), 100: (10, 10), 200: (10, 20), 300: (15, 20), 1560: (30, 52), 3600: (45, 80)}


def frame_grid(w: Workload):
    """(rows, columns) of the latent token grid of one frame (832x480 -> 30 x 52 tokens)."""
    return _FRAME_GRID[w.tokens_per_frame]


def to_f64(t) -> np.ndarray:
    """Exact up-cast of a stored tensor (bf16/f32/int) to a float64 NumPy array on the host."""
    if t is None:
        return None
    return t.detach().to("cpu").to(torch.float64).numpy()
