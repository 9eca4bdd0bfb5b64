"""ctypes binding of libhf.so: same names as the C ABI, argument marshalling only.

Every function takes torch tensors that already live on the GPU, checks dtype / shape /
contiguity, and passes raw device pointers plus the current HIP stream.  No step of the
method runs in Python or in torch; torch is used for device memory and streams.
There is no fallback: a missing library or a failed call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

HF_BF16, HF_F32 = 0, 1
HF_PHI_RELU, HF_PHI_ELU1 = 0, 1
HF_FLAG_READOUT_KERNEL, HF_FLAG_HISTORY_TWO_PLANES, HF_FLAG_BWD_FP32_KERNELS, HF_FLAG_DKV_INDEX_ORDER = 1, 2, 4, 8
HF_OK = 0

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhf.so")
_lib = None


class HFError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"hf error {code}: {msg}")
        self.code = code


class hf_config(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32),
        ("heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("block_q", ctypes.c_int32),
        ("block_kv", ctypes.c_int32),
        ("keep_ratio", ctypes.c_float),
        ("keep_k", ctypes.c_int32),
        ("phi", ctypes.c_int32),
        ("eps", ctypes.c_float),
        ("z_scale", ctypes.c_float),
        ("softmax_scale", ctypes.c_float),
        ("kv_capacity", ctypes.c_int32),
        ("flags", ctypes.c_int32),
    ]


class hf_window(ctypes.Structure):
    _fields_ = [("n_sink", ctypes.c_int32), ("n_tokens", ctypes.c_int32)]


class hf_ring(ctypes.Structure):
    _fields_ = [("n_sink", ctypes.c_int32), ("n_chunk", ctypes.c_int32), ("n_filled", ctypes.c_int32),
                ("next_slot", ctypes.c_int32), ("cur_slot", ctypes.c_int32), ("absorbed_ahead", ctypes.c_int32)]


def make_config(batch, heads, head_dim, dtype, block_q, block_kv, keep_ratio=1.0, keep_k=0,
                phi=HF_PHI_RELU, eps=1e-6, z_scale=1.0, softmax_scale=0.0, kv_capacity=0, flags=0) -> hf_config:
    if isinstance(dtype, str):
        dtype = {"bf16": HF_BF16, "f32": HF_F32}[dtype]
    elif isinstance(dtype, torch.dtype):
        dtype = {torch.bfloat16: HF_BF16, torch.float32: HF_F32}[dtype]
    return hf_config(batch, heads, head_dim, dtype, block_q, block_kv, keep_ratio, keep_k, phi, eps,
                     z_scale, softmax_scale, kv_capacity, flags)


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load libhf.so (built in-tree by ``python -m paper_2604_10103_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2604_10103_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    P, I, SZ = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    CP = ctypes.POINTER(hf_config)
    lib.hf_last_error.restype = ctypes.c_char_p
    lib.hf_last_error.argtypes = []
    lib.hf_version.restype = ctypes.c_char_p
    lib.hf_version.argtypes = []
    lib.hf_state_bytes.argtypes = [CP, ctypes.POINTER(SZ)]
    lib.hf_state_init.argtypes = [CP, P, P]
    lib.hf_state_fold_linear.argtypes = [CP, P, P, P, P]
    lib.hf_absorb_evicted.argtypes = [CP, P, P, P, I, P, P, P, SZ, P]
    lib.hf_absorb_workspace_bytes.argtypes = [CP, I, ctypes.POINTER(SZ)]
    lib.hf_state_planes_bytes.argtypes = [CP, ctypes.POINTER(SZ)]
    lib.hf_state_planes.argtypes = [CP, P, P, P]
    lib.hf_absorb_evicted_planes.argtypes = [CP, P, P, P, I, P, P, P, SZ, P, P]
    lib.hf_hybrid_attn_fwd_planes.argtypes = [CP, P, P, I, P, P, I, P, I, P, P, P, P, P, P]
    lib.hf_window_advance.argtypes = [CP, P, P, I, I, P, P, P, P, SZ, P]
    lib.hf_window_evict.argtypes = [CP, P, P, I, I, I, P, P, P, P, SZ, P]
    WP = ctypes.POINTER(hf_window)
    lib.hf_stream_open_chunk.argtypes = [CP, WP, I, P, P, P, P, P, P, SZ, ctypes.POINTER(I), ctypes.POINTER(I), P]
    lib.hf_stream_step.argtypes = [CP, WP, P, P, I, P, P, I, P, P, P, P, P, P, SZ, P]
    RP = ctypes.POINTER(hf_ring)
    lib.hf_ring_open_chunk.argtypes = [CP, RP, P, P, P, P, P, P, SZ, ctypes.POINTER(I), ctypes.POINTER(I), P]
    lib.hf_ring_step.argtypes = [CP, RP, P, P, P, P, I, P, P, P, P, P, P, SZ, P]
    lib.hf_select_k.argtypes = [CP, I, ctypes.POINTER(I)]
    lib.hf_workspace_bytes.argtypes = [CP, I, I, ctypes.POINTER(SZ)]
    lib.hf_block_select.argtypes = [CP, P, I, P, I, P, P, P, SZ, P]
    lib.hf_block_select_cached.argtypes = [CP, P, I, P, I, I, P, P, P, SZ, P]
    lib.hf_block_select_static.argtypes = [CP, P, I, P, I, P, P, P]
    lib.hf_pooled_keys_bytes.argtypes = [CP, I, ctypes.POINTER(ctypes.c_size_t)]
    lib.hf_pool_keys.argtypes = [CP, P, I, I, P, P]
    lib.hf_select_attn_fwd.argtypes = [CP, P, P, I, P, P, I, P, P, P, P, P, P, P, P, P]
    lib.hf_ring_last_step.argtypes = [CP, ctypes.POINTER(hf_ring), P, P, P, P, I, P, P, P, P, P, P, SZ, P, P, P, P, SZ,
                                      ctypes.POINTER(ctypes.c_int32), P]
    lib.hf_step_workspace_bytes.argtypes = [CP, I, I, ctypes.POINTER(SZ)]
    lib.hf_step_fwd.argtypes = [CP, P, P, I, P, P, I, P, P, P, P, P, P, P, P, P, P, I, I, P, P, P, SZ, P]
    lib.hf_hybrid_attn_fwd.argtypes = [CP, P, I, P, P, I, P, I, P, P, P, P, P, SZ, P]
    lib.hf_hybrid_attn_fwd_split.argtypes = [CP, P, P, I, P, P, I, P, I, P, P, P, P, P, SZ, P]
    lib.hf_hybrid_attn_fwd_save.argtypes = [CP, P, P, I, P, P, I, P, I, P, P, P, P, P, P, P, SZ, P]
    lib.hf_bwd_workspace_bytes.argtypes = [CP, I, I, ctypes.POINTER(SZ)]
    lib.hf_hybrid_attn_bwd.argtypes = [CP, P, P, I, P, P, I, P, I, P, P, P, P, P, P, P, P, P, SZ, P]
    lib.hf_hybrid_attn_bwd_saved.argtypes = [CP, P, P, I, P, P, I, P, I, P, P, P, P, P, P, P, P, P, P, P, SZ, P]
    lib.hf_rope_window_indices.argtypes = [I, I, I, ctypes.POINTER(I)]
    lib.hf_rope_tables.argtypes = [ctypes.POINTER(I), I, I, I, I, I, I, ctypes.c_double, I, P, P, P]
    lib.hf_rope_apply.argtypes = [CP, P, I, P, P, P, P]
    lib.hf_rope_append_keys.argtypes = [CP, P, I, P, P, P, I, I, P, P]
    lib.hf_probe_mfma_bf16.argtypes = [I, P, ctypes.POINTER(ctypes.c_double), P]
    for name in ("hf_state_bytes", "hf_state_init", "hf_state_fold_linear", "hf_window_advance", "hf_absorb_evicted", "hf_absorb_workspace_bytes", "hf_select_k",
                 "hf_workspace_bytes",
                 "hf_block_select", "hf_block_select_cached", "hf_block_select_static", "hf_hybrid_attn_fwd",
                 "hf_hybrid_attn_fwd_split",
                 "hf_rope_window_indices", "hf_rope_tables", "hf_rope_apply", "hf_window_evict", "hf_stream_open_chunk",
                 "hf_stream_step", "hf_bwd_workspace_bytes", "hf_hybrid_attn_bwd", "hf_state_planes_bytes",
                 "hf_state_planes", "hf_absorb_evicted_planes", "hf_hybrid_attn_fwd_planes", "hf_probe_mfma_bf16",
                 "hf_ring_open_chunk", "hf_ring_step", "hf_pooled_keys_bytes", "hf_pool_keys", "hf_select_attn_fwd",
                 "hf_step_workspace_bytes", "hf_step_fwd", "hf_rope_append_keys", "hf_ring_last_step"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(code: int):
    if code != HF_OK:
        raise HFError(code, load().hf_last_error().decode())


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t, name, dtype=None, shape=None):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr()


def _kv_len(cfg: hf_config, K_win, n_kv):
    """Valid tokens of a window tensor: its length when packed, the caller's n_kv in a cache buffer."""
    if cfg.kv_capacity > 0:
        if n_kv is None:
            raise ValueError("n_kv must be given when cfg.kv_capacity is set")
        if K_win.shape[2] != cfg.kv_capacity:
            raise ValueError(f"K_win must hold kv_capacity={cfg.kv_capacity} tokens per head")
        return int(n_kv)
    if n_kv is not None and n_kv != K_win.shape[2]:
        raise ValueError("n_kv differs from the packed window length")
    return K_win.shape[2]


def _tdtype(cfg: hf_config):
    return torch.bfloat16 if cfg.dtype == HF_BF16 else torch.float32


def _cdiv(a, b):
    return -(-a // b)


# ------------------------------------------------------------------------------ host helpers
def hf_version() -> str:
    return load().hf_version().decode()


def hf_state_bytes(cfg: hf_config) -> int:
    out = ctypes.c_size_t(0)
    _check(load().hf_state_bytes(ctypes.byref(cfg), ctypes.byref(out)))
    return out.value


def hf_window_advance(cfg: hf_config, K_win, V_win, n_evict: int, state, rope_cos=None, rope_sin=None,
                      workspace=None, n_sink: int = 0, n_kv=None) -> None:
    """Absorb the oldest n_evict tokens behind the first n_sink of the window buffers into the state and move
    the rest down (hf_window_evict; n_sink = 0 is hf_window_advance)."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_kv = _kv_len(cfg, K_win, n_kv)
    ns = hf_state_bytes(cfg) // 4
    tab = (int(n_evict), d // 2)
    _check(load().hf_window_evict(
        ctypes.byref(cfg), _dev(K_win, "K_win", _tdtype(cfg), (B, H, K_win.shape[2], d)),
        _dev(V_win, "V_win", _tdtype(cfg), (B, H, K_win.shape[2], d)), n_kv, int(n_sink), int(n_evict),
        _dev(state, "state", torch.float32, (ns,)), _dev(rope_cos, "rope_cos", torch.float32, tab),
        _dev(rope_sin, "rope_sin", torch.float32, tab), _dev(workspace, "workspace", torch.uint8),
        0 if workspace is None else workspace.numel(), _stream()))


def hf_select_k(cfg: hf_config, n_kv: int) -> int:
    out = ctypes.c_int32(0)
    _check(load().hf_select_k(ctypes.byref(cfg), n_kv, ctypes.byref(out)))
    return out.value


def hf_absorb_workspace_bytes(cfg: hf_config, n_tokens: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().hf_absorb_workspace_bytes(ctypes.byref(cfg), n_tokens, ctypes.byref(out)))
    return out.value


def hf_workspace_bytes(cfg: hf_config, n_q: int, n_kv: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().hf_workspace_bytes(ctypes.byref(cfg), n_q, n_kv, ctypes.byref(out)))
    return out.value


# ------------------------------------------------------------------------------ device calls
def hf_state_init(cfg: hf_config, state: torch.Tensor) -> None:
    """state: fp32 GPU tensor of hf_state_bytes(cfg)/4 elements, zeroed in place."""
    n = hf_state_bytes(cfg) // 4
    _check(load().hf_state_init(ctypes.byref(cfg), _dev(state, "state", torch.float32, (n,)), _stream()))


def hf_state_fold_linear(cfg: hf_config, state_in, W, state_out) -> None:
    """state_out = state_in with L[b,h] replaced by L[b,h] @ W[h]; W: fp32 GPU tensor [H, d, d]."""
    n = hf_state_bytes(cfg) // 4
    d = cfg.head_dim
    _check(load().hf_state_fold_linear(
        ctypes.byref(cfg), _dev(state_in, "state_in", torch.float32, (n,)),
        _dev(W, "W", torch.float32, (cfg.heads, d, d)), _dev(state_out, "state_out", torch.float32, (n,)), _stream()))


def hf_absorb_evicted(cfg: hf_config, state, K_ev, V_ev, rope_cos=None, rope_sin=None, workspace=None) -> None:
    """workspace: optional uint8 GPU buffer of hf_absorb_workspace_bytes(cfg, n) bytes (atomic-free path)."""
    n = hf_state_bytes(cfg) // 4
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    if K_ev.dim() != 4:
        raise ValueError("K_ev must be [B, H, n, d]")
    nt = K_ev.shape[2]
    shp = (B, H, nt, d)
    tab = (nt, d // 2)
    _check(load().hf_absorb_evicted(
        ctypes.byref(cfg), _dev(state, "state", torch.float32, (n,)),
        _dev(K_ev, "K_ev", _tdtype(cfg), shp), _dev(V_ev, "V_ev", _tdtype(cfg), shp), nt,
        _dev(rope_cos, "rope_cos", torch.float32, tab), _dev(rope_sin, "rope_sin", torch.float32, tab),
        _dev(workspace, "workspace", torch.uint8), 0 if workspace is None else workspace.numel(), _stream()))


def hf_state_planes_bytes(cfg: hf_config) -> int:
    """Bytes of the caller-kept bf16 planes of the state (0: the configuration has no such path)."""
    out = ctypes.c_size_t(0)
    _check(load().hf_state_planes_bytes(ctypes.byref(cfg), ctypes.byref(out)))
    return out.value


def hf_state_planes(cfg: hf_config, state, planes_out) -> None:
    """planes_out (uint8 GPU buffer of hf_state_planes_bytes(cfg) bytes) = the bf16 planes of state."""
    n = hf_state_bytes(cfg) // 4
    _check(load().hf_state_planes(ctypes.byref(cfg), _dev(state, "state", torch.float32, (n,)),
                                  _dev(planes_out, "planes_out", torch.uint8), _stream()))


def hf_absorb_evicted_planes(cfg: hf_config, state, K_ev, V_ev, planes_out, rope_cos=None, rope_sin=None,
                             workspace=None) -> None:
    """hf_absorb_evicted that also writes the planes of the updated state into planes_out."""
    n = hf_state_bytes(cfg) // 4
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    if K_ev.dim() != 4:
        raise ValueError("K_ev must be [B, H, n, d]")
    nt = K_ev.shape[2]
    shp = (B, H, nt, d)
    tab = (nt, d // 2)
    _check(load().hf_absorb_evicted_planes(
        ctypes.byref(cfg), _dev(state, "state", torch.float32, (n,)),
        _dev(K_ev, "K_ev", _tdtype(cfg), shp), _dev(V_ev, "V_ev", _tdtype(cfg), shp), nt,
        _dev(rope_cos, "rope_cos", torch.float32, tab), _dev(rope_sin, "rope_sin", torch.float32, tab),
        _dev(workspace, "workspace", torch.uint8), 0 if workspace is None else workspace.numel(),
        _dev(planes_out, "planes_out", torch.uint8), _stream()))


def hf_block_select(cfg: hf_config, Q, K_win, block_idx, scores=None, workspace=None, n_kv=None) -> None:
    """block_idx: int32 [B,H,T_m,k] out; scores: optional fp32 [B,H,T_m,T_n] out; workspace: uint8 buffer."""
    hf_block_select_cached(cfg, Q, K_win, 0, block_idx, scores, workspace, _entry="hf_block_select", n_kv=n_kv)


HF_STATIC_SCRATCH_BYTES = 8 << 20


def hf_block_select_static(cfg: hf_config, Q, K_win, block_idx, scores=None, n_kv=None) -> None:
    """hf_block_select without a workspace: the pooled means live in the library's built-in per-GPU buffer."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_q, n_kv = Q.shape[2], _kv_len(cfg, K_win, n_kv)
    t_m, t_n = _cdiv(n_q, cfg.block_q), _cdiv(n_kv, cfg.block_kv)
    k = hf_select_k(cfg, n_kv)
    _check(load().hf_block_select_static(
        ctypes.byref(cfg), _dev(Q, "Q", _tdtype(cfg), (B, H, n_q, d)), n_q,
        _dev(K_win, "K_win", _tdtype(cfg), (B, H, K_win.shape[2], d)), n_kv,
        _dev(block_idx, "block_idx", torch.int32, (B, H, t_m, k)),
        _dev(scores, "scores", torch.float32, (B, H, t_m, t_n)), _stream()))


def hf_block_select_cached(cfg: hf_config, Q, K_win, n_cached_kv_blocks: int, block_idx, scores=None,
                           workspace=None, _entry="hf_block_select_cached", n_kv=None) -> None:
    """As hf_block_select; the pooled means of the first n_cached_kv_blocks KV blocks are reused from the
    previous call on the same workspace (the caller guarantees those tokens did not change)."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_q, n_kv = Q.shape[2], _kv_len(cfg, K_win, n_kv)
    t_m, t_n = _cdiv(n_q, cfg.block_q), _cdiv(n_kv, cfg.block_kv)
    k = hf_select_k(cfg, n_kv)
    ws_ptr = _dev(workspace, "workspace", torch.uint8)
    extra = () if _entry == "hf_block_select" else (int(n_cached_kv_blocks),)
    _check(getattr(load(), _entry)(
        ctypes.byref(cfg), _dev(Q, "Q", _tdtype(cfg), (B, H, n_q, d)), n_q,
        _dev(K_win, "K_win", _tdtype(cfg), (B, H, K_win.shape[2], d)), n_kv, *extra,
        _dev(block_idx, "block_idx", torch.int32, (B, H, t_m, k)),
        _dev(scores, "scores", torch.float32, (B, H, t_m, t_n)),
        ws_ptr, 0 if workspace is None else workspace.numel(), _stream()))


def hf_hybrid_attn_fwd(cfg: hf_config, Q, K_win, V_win, block_idx, state, O, workspace=None,
                       rope_cos_q=None, rope_sin_q=None, Q_hist=None, n_kv=None) -> None:
    """block_idx None = dense window attention; state None = no history term; Q_hist: the history branch's
    queries when they are not Q (hf_hybrid_attn_fwd_split)."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_q, n_kv = Q.shape[2], _kv_len(cfg, K_win, n_kv)
    t_m = _cdiv(n_q, cfg.block_q)
    k = 0
    if block_idx is not None:
        if block_idx.dim() != 4:
            raise ValueError("block_idx must be [B, H, T_m, k]")
        k = block_idx.shape[3]
    tab = (n_q, d // 2)
    ns = hf_state_bytes(cfg) // 4
    split = () if Q_hist is None else (_dev(Q_hist, "Q_hist", _tdtype(cfg), (B, H, n_q, d)),)
    entry = load().hf_hybrid_attn_fwd if Q_hist is None else load().hf_hybrid_attn_fwd_split
    _check(entry(
        ctypes.byref(cfg), _dev(Q, "Q", _tdtype(cfg), (B, H, n_q, d)), *split, n_q,
        _dev(K_win, "K_win", _tdtype(cfg), (B, H, K_win.shape[2], d)),
        _dev(V_win, "V_win", _tdtype(cfg), (B, H, K_win.shape[2], d)), n_kv,
        _dev(block_idx, "block_idx", torch.int32, (B, H, t_m, k)), k,
        _dev(state, "state", torch.float32, (ns,)),
        _dev(rope_cos_q, "rope_cos_q", torch.float32, tab), _dev(rope_sin_q, "rope_sin_q", torch.float32, tab),
        _dev(O, "O", _tdtype(cfg), (B, H, n_q, d)),
        _dev(workspace, "workspace", torch.uint8), 0 if workspace is None else workspace.numel(), _stream()))


def hf_hybrid_attn_fwd_planes(cfg: hf_config, Q, K_win, V_win, block_idx, state, planes, O, rope_cos_q=None,
                              rope_sin_q=None, Q_hist=None, n_kv=None) -> None:
    """hf_hybrid_attn_fwd with the state's planes kept by the caller (hf_absorb_evicted_planes /
    hf_state_planes): no workspace, no conversion launch."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_q, n_kv = Q.shape[2], _kv_len(cfg, K_win, n_kv)
    t_m = _cdiv(n_q, cfg.block_q)
    k = 0
    if block_idx is not None:
        if block_idx.dim() != 4:
            raise ValueError("block_idx must be [B, H, T_m, k]")
        k = block_idx.shape[3]
    tab = (n_q, d // 2)
    qs = (B, H, n_q, d)
    _check(load().hf_hybrid_attn_fwd_planes(
        ctypes.byref(cfg), _dev(Q, "Q", _tdtype(cfg), qs), _dev(Q_hist, "Q_hist", _tdtype(cfg), qs), n_q,
        _dev(K_win, "K_win", _tdtype(cfg), (B, H, K_win.shape[2], d)),
        _dev(V_win, "V_win", _tdtype(cfg), (B, H, K_win.shape[2], d)), n_kv,
        _dev(block_idx, "block_idx", torch.int32, (B, H, t_m, k)), k,
        _dev(state, "state", torch.float32, (hf_state_bytes(cfg) // 4,)), _dev(planes, "planes", torch.uint8),
        _dev(rope_cos_q, "rope_cos_q", torch.float32, tab), _dev(rope_sin_q, "rope_sin_q", torch.float32, tab),
        _dev(O, "O", _tdtype(cfg), qs), _stream()))


def hf_pooled_keys_bytes(cfg: hf_config, n_kv: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().hf_pooled_keys_bytes(ctypes.byref(cfg), n_kv, ctypes.byref(out)))
    return out.value


def hf_pool_keys(cfg: hf_config, K_win, pooled_K, n_cached_kv_blocks: int = 0, n_kv=None) -> None:
    """Pooled keys of the window (Eq. 4's k-bar) for hf_select_attn_fwd; the first n_cached_kv_blocks keep their values."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_kv = _kv_len(cfg, K_win, n_kv)
    _check(load().hf_pool_keys(ctypes.byref(cfg), _dev(K_win, "K_win", _tdtype(cfg), (B, H, K_win.shape[2], d)), n_kv,
                               n_cached_kv_blocks, _dev(pooled_K, "pooled_K", torch.uint8), _stream()))


def hf_select_attn_fwd(cfg: hf_config, Q, K_win, V_win, pooled_K, state, planes, O, block_idx_out, scores=None,
                       rope_cos_q=None, rope_sin_q=None, Q_hist=None, n_kv=None) -> None:
    """Top-K selection (Eq. 4), sparse attention (Eq. 5) and history term (Eq. 3, 6) in one launch; the chosen
    blocks are written to block_idx_out [B, H, T_m, k]."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_q, n_kv = Q.shape[2], _kv_len(cfg, K_win, n_kv)
    t_m, t_n = _cdiv(n_q, cfg.block_q), _cdiv(n_kv, cfg.block_kv)
    if block_idx_out.dim() != 4:
        raise ValueError("block_idx_out must be [B, H, T_m, k]")
    k = block_idx_out.shape[3]
    if k != hf_select_k(cfg, n_kv):
        raise ValueError("block_idx_out must hold hf_select_k(cfg, n_kv) entries per row")
    tab = (n_q, d // 2)
    qs = (B, H, n_q, d)
    _check(load().hf_select_attn_fwd(
        ctypes.byref(cfg), _dev(Q, "Q", _tdtype(cfg), qs), _dev(Q_hist, "Q_hist", _tdtype(cfg), qs), n_q,
        _dev(K_win, "K_win", _tdtype(cfg), (B, H, K_win.shape[2], d)),
        _dev(V_win, "V_win", _tdtype(cfg), (B, H, K_win.shape[2], d)), n_kv,
        _dev(pooled_K, "pooled_K", torch.uint8),
        None if state is None else _dev(state, "state", torch.float32, (hf_state_bytes(cfg) // 4,)),
        _dev(planes, "planes", torch.uint8),
        _dev(rope_cos_q, "rope_cos_q", torch.float32, tab), _dev(rope_sin_q, "rope_sin_q", torch.float32, tab),
        _dev(O, "O", _tdtype(cfg), qs), _dev(block_idx_out, "block_idx_out", torch.int32, (B, H, t_m, k)),
        _dev(scores, "scores", torch.float32, (B, H, t_m, t_n)), _stream()))


def hf_step_workspace_bytes(cfg: hf_config, n_q: int, n_ev: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().hf_step_workspace_bytes(ctypes.byref(cfg), n_q, n_ev, ctypes.byref(out)))
    return out.value


def hf_step_fwd(cfg: hf_config, Q, K_win, V_win, pooled_K, state_in, planes, O, block_idx_out, K_ev, V_ev, state_out,
                planes_out, workspace, scores=None, rope_cos_q=None, rope_sin_q=None, Q_hist=None, n_kv=None,
                n_ev=None) -> None:
    """hf_select_attn_fwd with workgroups of their own that absorb K_ev, V_ev (Eq. 2) into state_out / planes_out
    = state_in + their contribution, in the same launch.  n_ev: tokens of every head of K_ev to absorb (default:
    all of its third dimension, which is also the head stride)."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_q, n_kv = Q.shape[2], _kv_len(cfg, K_win, n_kv)
    t_m, t_n = _cdiv(n_q, cfg.block_q), _cdiv(n_kv, cfg.block_kv)
    if block_idx_out.dim() != 4:
        raise ValueError("block_idx_out must be [B, H, T_m, k]")
    k = block_idx_out.shape[3]
    if k != hf_select_k(cfg, n_kv):
        raise ValueError("block_idx_out must hold hf_select_k(cfg, n_kv) entries per row")
    ev_stride = K_ev.shape[2]
    n_ev = ev_stride if n_ev is None else int(n_ev)
    tab = (n_q, d // 2)
    qs = (B, H, n_q, d)
    ns = hf_state_bytes(cfg) // 4
    _check(load().hf_step_fwd(
        ctypes.byref(cfg), _dev(Q, "Q", _tdtype(cfg), qs), _dev(Q_hist, "Q_hist", _tdtype(cfg), qs), n_q,
        _dev(K_win, "K_win", _tdtype(cfg), (B, H, K_win.shape[2], d)),
        _dev(V_win, "V_win", _tdtype(cfg), (B, H, K_win.shape[2], d)), n_kv,
        _dev(pooled_K, "pooled_K", torch.uint8),
        _dev(state_in, "state_in", torch.float32, (ns,)), _dev(planes, "planes", torch.uint8),
        _dev(rope_cos_q, "rope_cos_q", torch.float32, tab), _dev(rope_sin_q, "rope_sin_q", torch.float32, tab),
        _dev(O, "O", _tdtype(cfg), qs), _dev(block_idx_out, "block_idx_out", torch.int32, (B, H, t_m, k)),
        _dev(scores, "scores", torch.float32, (B, H, t_m, t_n)),
        _dev(K_ev, "K_ev", _tdtype(cfg), (B, H, ev_stride, d)), _dev(V_ev, "V_ev", _tdtype(cfg), (B, H, ev_stride, d)),
        n_ev, ev_stride, _dev(state_out, "state_out", torch.float32, (ns,)), _dev(planes_out, "planes_out", torch.uint8),
        _dev(workspace, "workspace", torch.uint8), 0 if workspace is None else workspace.numel(), _stream()))


def hf_hybrid_attn_fwd_save(cfg: hf_config, Q, K_win, V_win, block_idx, state, O, O_local_out, lse2_out, workspace=None,
                            rope_cos_q=None, rope_sin_q=None, Q_hist=None, n_kv=None) -> None:
    """hf_hybrid_attn_fwd that also writes O_local and the softmax row statistic lse2 [B*H, n_q] (fp32) for
    hf_hybrid_attn_bwd_saved."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_q, n_kv = Q.shape[2], _kv_len(cfg, K_win, n_kv)
    t_m = _cdiv(n_q, cfg.block_q)
    k = 0
    if block_idx is not None:
        if block_idx.dim() != 4:
            raise ValueError("block_idx must be [B, H, T_m, k]")
        k = block_idx.shape[3]
    tab = (n_q, d // 2)
    qs = (B, H, n_q, d)
    _check(load().hf_hybrid_attn_fwd_save(
        ctypes.byref(cfg), _dev(Q, "Q", _tdtype(cfg), qs), _dev(Q_hist, "Q_hist", _tdtype(cfg), qs), n_q,
        _dev(K_win, "K_win", _tdtype(cfg), (B, H, K_win.shape[2], d)),
        _dev(V_win, "V_win", _tdtype(cfg), (B, H, K_win.shape[2], d)), n_kv,
        _dev(block_idx, "block_idx", torch.int32, (B, H, t_m, k)), k,
        _dev(state, "state", torch.float32, (hf_state_bytes(cfg) // 4,)),
        _dev(rope_cos_q, "rope_cos_q", torch.float32, tab), _dev(rope_sin_q, "rope_sin_q", torch.float32, tab),
        _dev(O, "O", _tdtype(cfg), qs), _dev(O_local_out, "O_local_out", _tdtype(cfg), qs),
        _dev(lse2_out, "lse2_out", torch.float32, (B * H, n_q)),
        _dev(workspace, "workspace", torch.uint8), 0 if workspace is None else workspace.numel(), _stream()))


def hf_probe_mfma_bf16(iters: int, scratch) -> float:
    """Enqueue the MFMA issue-rate probe; returns the floating-point operations of the launch (time it with events)."""
    flops = ctypes.c_double(0.0)
    _check(load().hf_probe_mfma_bf16(int(iters), _dev(scratch, "scratch4", torch.float32), ctypes.byref(flops), _stream()))
    return flops.value


def hf_rope_window_indices(i_newest: int, n_frames: int, t0: int) -> list:
    """Eq. 7 with the cache re-based to the current chunk: temporal indices of the last n_frames frames."""
    out = (ctypes.c_int32 * n_frames)()
    _check(load().hf_rope_window_indices(int(i_newest), int(n_frames), int(t0), out))
    return list(out)


def hf_rope_tables(frame_idx, height: int, width: int, pairs, cos_out, sin_out, theta: float = 10000.0,
                   temporal_only: bool = False) -> None:
    """cos_out, sin_out: fp32 GPU tensors [len(frame_idx) * height * width, sum(pairs)]."""
    nf = len(frame_idx)
    arr = (ctypes.c_int32 * max(nf, 1))(*[int(x) for x in frame_idx])
    shp = (nf * height * width, int(sum(pairs)))
    _check(load().hf_rope_tables(arr, nf, int(height), int(width), int(pairs[0]), int(pairs[1]), int(pairs[2]),
                                 float(theta), 1 if temporal_only else 0,
                                 _dev(cos_out, "cos_out", torch.float32, shp),
                                 _dev(sin_out, "sin_out", torch.float32, shp), _stream()))


def hf_rope_append_keys(cfg: hf_config, K_new, rope_cos, rope_sin, K_win, first: int, pooled_K, n_kv=None) -> None:
    """K_new [B, H, n_new, d], rotated by its tables (None: copied), becomes tokens first .. first + n_new - 1 of the
    window buffer K_win; the pooled keys of the KV blocks those tokens touch are rewritten in pooled_K."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_new = K_new.shape[2]
    n_kv = _kv_len(cfg, K_win, n_kv)
    tab = (n_new, d // 2)
    _check(load().hf_rope_append_keys(
        ctypes.byref(cfg), _dev(K_new, "K_new", _tdtype(cfg), (B, H, n_new, d)), n_new,
        _dev(rope_cos, "rope_cos", torch.float32, tab), _dev(rope_sin, "rope_sin", torch.float32, tab),
        _dev(K_win, "K_win", _tdtype(cfg), (B, H, K_win.shape[2], d)), first, n_kv,
        _dev(pooled_K, "pooled_K", torch.uint8), _stream()))


def hf_rope_apply(cfg: hf_config, X, rope_cos, rope_sin, Y) -> None:
    """Y = X with adjacent feature pairs of every token turned by the tables [n, d/2]; Y may be X."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n = X.shape[2]
    _check(load().hf_rope_apply(
        ctypes.byref(cfg), _dev(X, "X", _tdtype(cfg), (B, H, n, d)), n,
        _dev(rope_cos, "rope_cos", torch.float32, (n, d // 2)), _dev(rope_sin, "rope_sin", torch.float32, (n, d // 2)),
        _dev(Y, "Y", _tdtype(cfg), (B, H, n, d)), _stream()))


def hf_stream_open_chunk(cfg: hf_config, win: hf_window, n_chunk: int, K_win, V_win, state, rope_cos_ev=None,
                         rope_sin_ev=None, workspace=None):
    """Evict what the next chunk of n_chunk tokens pushes out of the cache into the state and reserve the
    chunk's slot; returns (token offset of the slot, tokens evicted) and updates ``win``."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    cap = cfg.kv_capacity
    over = max(0, win.n_tokens + int(n_chunk) - cap)
    tab = (over, d // 2)
    first, n_ev = ctypes.c_int32(-1), ctypes.c_int32(-1)
    _check(load().hf_stream_open_chunk(
        ctypes.byref(cfg), ctypes.byref(win), int(n_chunk), _dev(K_win, "K_win", _tdtype(cfg), (B, H, cap, d)),
        _dev(V_win, "V_win", _tdtype(cfg), (B, H, cap, d)),
        _dev(state, "state", torch.float32, (hf_state_bytes(cfg) // 4,)),
        _dev(rope_cos_ev, "rope_cos_ev", torch.float32, tab), _dev(rope_sin_ev, "rope_sin_ev", torch.float32, tab),
        _dev(workspace, "workspace", torch.uint8), 0 if workspace is None else workspace.numel(),
        ctypes.byref(first), ctypes.byref(n_ev), _stream()))
    return first.value, n_ev.value


def hf_stream_step(cfg: hf_config, win: hf_window, Q, K_win, V_win, step_in_chunk: int, block_idx, state, O,
                   workspace, rope_cos_q=None, rope_sin_q=None, Q_hist=None) -> None:
    """Selection (pooled keys of the unchanged blocks reused after the chunk's first step) and hybrid attention
    over the valid tokens of the cache."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    cap, n_q = cfg.kv_capacity, Q.shape[2]
    t_m = _cdiv(n_q, cfg.block_q)
    k = hf_select_k(cfg, win.n_tokens)
    tab = (n_q, d // 2)
    _check(load().hf_stream_step(
        ctypes.byref(cfg), ctypes.byref(win), _dev(Q, "Q", _tdtype(cfg), (B, H, n_q, d)),
        _dev(Q_hist, "Q_hist", _tdtype(cfg), (B, H, n_q, d)), n_q,
        _dev(K_win, "K_win", _tdtype(cfg), (B, H, cap, d)), _dev(V_win, "V_win", _tdtype(cfg), (B, H, cap, d)),
        int(step_in_chunk), _dev(block_idx, "block_idx", torch.int32, (B, H, t_m, k)),
        _dev(state, "state", torch.float32, (hf_state_bytes(cfg) // 4,)),
        _dev(rope_cos_q, "rope_cos_q", torch.float32, tab), _dev(rope_sin_q, "rope_sin_q", torch.float32, tab),
        _dev(O, "O", _tdtype(cfg), (B, H, n_q, d)), _dev(workspace, "workspace", torch.uint8),
        0 if workspace is None else workspace.numel(), _stream()))


def make_ring(n_sink: int, n_chunk: int) -> hf_ring:
    return hf_ring(int(n_sink), int(n_chunk), 0, 0, -1, 0)


def hf_ring_open_chunk(cfg: hf_config, ring: hf_ring, K_cache, V_cache, state, rope_cos_ev=None, rope_sin_ev=None,
                       workspace=None):
    """Hand the next chunk slot of the ring to a new chunk; the chunk it held (if any) goes into the state where it
    lies.  Returns (token offset of the slot, tokens evicted) and updates ``ring``."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    cap = cfg.kv_capacity
    tab = (ring.n_chunk, d // 2)
    first, n_ev = ctypes.c_int32(-1), ctypes.c_int32(-1)
    _check(load().hf_ring_open_chunk(
        ctypes.byref(cfg), ctypes.byref(ring), _dev(K_cache, "K_cache", _tdtype(cfg), (B, H, cap, d)),
        _dev(V_cache, "V_cache", _tdtype(cfg), (B, H, cap, d)),
        _dev(state, "state", torch.float32, (hf_state_bytes(cfg) // 4,)),
        _dev(rope_cos_ev, "rope_cos_ev", torch.float32, tab), _dev(rope_sin_ev, "rope_sin_ev", torch.float32, tab),
        _dev(workspace, "workspace", torch.uint8), 0 if workspace is None else workspace.numel(),
        ctypes.byref(first), ctypes.byref(n_ev), _stream()))
    return first.value, n_ev.value


def hf_ring_last_step(cfg: hf_config, ring: hf_ring, Q, K_cache, V_cache, step_in_chunk: int, block_idx, state, O, workspace,
                      state_out, step_workspace, rope_cos_q=None, rope_sin_q=None, Q_hist=None, rope_cos_ev=None,
                      rope_sin_ev=None) -> bool:
    """hf_ring_step for the chunk's last denoising step; if the next hf_ring_open_chunk would evict a chunk, that chunk
    is absorbed now into state_out (= state + its contribution) and True is returned: state_out is the state from the
    next chunk on."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    cap, n_q = cfg.kv_capacity, ring.n_chunk
    n_kv = ring.n_sink + ring.n_filled * ring.n_chunk
    t_m = _cdiv(n_q, cfg.block_q)
    k = hf_select_k(cfg, n_kv)
    tab = (n_q, d // 2)
    qs = (B, H, n_q, d)
    ns = hf_state_bytes(cfg) // 4
    done = ctypes.c_int32(0)
    _check(load().hf_ring_last_step(
        ctypes.byref(cfg), ctypes.byref(ring), _dev(Q, "Q", _tdtype(cfg), qs), _dev(Q_hist, "Q_hist", _tdtype(cfg), qs),
        _dev(K_cache, "K_cache", _tdtype(cfg), (B, H, cap, d)), _dev(V_cache, "V_cache", _tdtype(cfg), (B, H, cap, d)),
        step_in_chunk, _dev(block_idx, "block_idx", torch.int32, (B, H, t_m, k)),
        None if state is None else _dev(state, "state", torch.float32, (ns,)),
        _dev(rope_cos_q, "rope_cos_q", torch.float32, tab), _dev(rope_sin_q, "rope_sin_q", torch.float32, tab),
        _dev(O, "O", _tdtype(cfg), qs), _dev(workspace, "workspace", torch.uint8), workspace.numel(),
        _dev(state_out, "state_out", torch.float32, (ns,)),
        _dev(rope_cos_ev, "rope_cos_ev", torch.float32, tab), _dev(rope_sin_ev, "rope_sin_ev", torch.float32, tab),
        _dev(step_workspace, "step_workspace", torch.uint8), 0 if step_workspace is None else step_workspace.numel(),
        ctypes.byref(done), _stream()))
    return bool(done.value)


def hf_ring_step(cfg: hf_config, ring: hf_ring, Q, K_cache, V_cache, step_in_chunk: int, block_idx, state, O, workspace,
                 rope_cos_q=None, rope_sin_q=None, Q_hist=None) -> None:
    """Selection and hybrid attention of one denoising step over the ring's valid tokens, in storage order."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    cap, n_q = cfg.kv_capacity, ring.n_chunk
    n_kv = ring.n_sink + ring.n_filled * ring.n_chunk
    t_m = _cdiv(n_q, cfg.block_q)
    k = hf_select_k(cfg, n_kv)
    tab = (n_q, d // 2)
    _check(load().hf_ring_step(
        ctypes.byref(cfg), ctypes.byref(ring), _dev(Q, "Q", _tdtype(cfg), (B, H, n_q, d)),
        _dev(Q_hist, "Q_hist", _tdtype(cfg), (B, H, n_q, d)),
        _dev(K_cache, "K_cache", _tdtype(cfg), (B, H, cap, d)), _dev(V_cache, "V_cache", _tdtype(cfg), (B, H, cap, d)),
        int(step_in_chunk), _dev(block_idx, "block_idx", torch.int32, (B, H, t_m, k)),
        _dev(state, "state", torch.float32, (hf_state_bytes(cfg) // 4,)),
        _dev(rope_cos_q, "rope_cos_q", torch.float32, tab), _dev(rope_sin_q, "rope_sin_q", torch.float32, tab),
        _dev(O, "O", _tdtype(cfg), (B, H, n_q, d)), _dev(workspace, "workspace", torch.uint8),
        0 if workspace is None else workspace.numel(), _stream()))


def hf_bwd_workspace_bytes(cfg: hf_config, n_q: int, n_kv: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().hf_bwd_workspace_bytes(ctypes.byref(cfg), n_q, n_kv, ctypes.byref(out)))
    return out.value


def hf_hybrid_attn_bwd(cfg: hf_config, Q, K_win, V_win, block_idx, state, dO, dQ, dK, dV, workspace,
                       rope_cos_q=None, rope_sin_q=None, Q_hist=None, dQ_hist=None, n_kv=None) -> None:
    """Gradients of hf_hybrid_attn_fwd's output with respect to Q (and Q_hist), K_win, V_win for a fixed mask
    and a constant state.  dK, dV are laid out like K_win, V_win."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_q, n_kv = Q.shape[2], _kv_len(cfg, K_win, n_kv)
    t_m = _cdiv(n_q, cfg.block_q)
    k = 0
    if block_idx is not None:
        k = block_idx.shape[3]
    tab = (n_q, d // 2)
    qs, ks = (B, H, n_q, d), (B, H, K_win.shape[2], d)
    _check(load().hf_hybrid_attn_bwd(
        ctypes.byref(cfg), _dev(Q, "Q", _tdtype(cfg), qs), _dev(Q_hist, "Q_hist", _tdtype(cfg), qs), n_q,
        _dev(K_win, "K_win", _tdtype(cfg), ks), _dev(V_win, "V_win", _tdtype(cfg), ks), n_kv,
        _dev(block_idx, "block_idx", torch.int32, (B, H, t_m, k)), k,
        _dev(state, "state", torch.float32, (hf_state_bytes(cfg) // 4,)),
        _dev(rope_cos_q, "rope_cos_q", torch.float32, tab), _dev(rope_sin_q, "rope_sin_q", torch.float32, tab),
        _dev(dO, "dO", _tdtype(cfg), qs), _dev(dQ, "dQ", _tdtype(cfg), qs), _dev(dQ_hist, "dQ_hist", _tdtype(cfg), qs),
        _dev(dK, "dK", _tdtype(cfg), ks), _dev(dV, "dV", _tdtype(cfg), ks),
        _dev(workspace, "workspace", torch.uint8), 0 if workspace is None else workspace.numel(), _stream()))


def hf_hybrid_attn_bwd_saved(cfg: hf_config, Q, K_win, V_win, block_idx, state, dO, O_local, lse2, dQ, dK, dV, workspace,
                             rope_cos_q=None, rope_sin_q=None, Q_hist=None, dQ_hist=None, n_kv=None) -> None:
    """hf_hybrid_attn_bwd from O_local and lse2 as hf_hybrid_attn_fwd_save wrote them (no recomputed forward)."""
    B, H, d = cfg.batch, cfg.heads, cfg.head_dim
    n_q, n_kv = Q.shape[2], _kv_len(cfg, K_win, n_kv)
    t_m = _cdiv(n_q, cfg.block_q)
    k = 0
    if block_idx is not None:
        k = block_idx.shape[3]
    tab = (n_q, d // 2)
    qs, ks = (B, H, n_q, d), (B, H, K_win.shape[2], d)
    _check(load().hf_hybrid_attn_bwd_saved(
        ctypes.byref(cfg), _dev(Q, "Q", _tdtype(cfg), qs), _dev(Q_hist, "Q_hist", _tdtype(cfg), qs), n_q,
        _dev(K_win, "K_win", _tdtype(cfg), ks), _dev(V_win, "V_win", _tdtype(cfg), ks), n_kv,
        _dev(block_idx, "block_idx", torch.int32, (B, H, t_m, k)), k,
        _dev(state, "state", torch.float32, (hf_state_bytes(cfg) // 4,)),
        _dev(rope_cos_q, "rope_cos_q", torch.float32, tab), _dev(rope_sin_q, "rope_sin_q", torch.float32, tab),
        _dev(dO, "dO", _tdtype(cfg), qs), _dev(O_local, "O_local", _tdtype(cfg), qs),
        _dev(lse2, "lse2", torch.float32, (B * H, n_q)),
        _dev(dQ, "dQ", _tdtype(cfg), qs), _dev(dQ_hist, "dQ_hist", _tdtype(cfg), qs),
        _dev(dK, "dK", _tdtype(cfg), ks), _dev(dV, "dV", _tdtype(cfg), ks),
        _dev(workspace, "workspace", torch.uint8), 0 if workspace is None else workspace.numel(), _stream()))
