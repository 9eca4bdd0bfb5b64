"""Host-side checks of the C-ABI library: it loads, exports what the header declares, and its
host-only helpers and argument checks behave.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

import oracle as orc
import paper_2604_10103_amd as hf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hf.lib_path()):
        from paper_2604_10103_amd import build
        build.build()
    return hf.load()


def _declared():
    src = open(os.path.join(ROOT, "include", "hf.h")).read()
    return re.findall(r"HF_API\s+[\w\s\*]+?\b(hf_\w+)\s*\(", src)


def test_every_declared_symbol_is_exported(lib):
    names = _declared()
    assert set(names) >= {"hf_state_bytes", "hf_state_init", "hf_absorb_evicted", "hf_select_k",
                          "hf_workspace_bytes", "hf_block_select", "hf_hybrid_attn_fwd", "hf_last_error",
                          "hf_version", "hf_absorb_workspace_bytes"}
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in hf.h but not exported"


def test_config_struct_layout():
    assert ctypes.sizeof(hf.hf_config) == 14 * 4
    assert hf.hf_config.flags.offset == 52
    assert hf.hf_config.keep_ratio.offset == 24 and hf.hf_config.softmax_scale.offset == 44
    assert hf.hf_config.kv_capacity.offset == 48
    assert ctypes.sizeof(hf.hf_window) == 8 and hf.hf_window.n_tokens.offset == 4


def test_library_reads_no_environment_variable(lib):
    """Kernel choices are hf_config.flags; nothing in the library's sources consults the process environment."""
    csrc = os.path.join(ROOT, "paper_2604_10103_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        text = open(os.path.join(csrc, name)).read()
        assert "getenv" not in text and "environ" not in text, name
    cfg = hf.make_config(1, 1, 128, "bf16", 64, 64, 0.25, flags=1 << 20)
    with pytest.raises(hf.HFError) as e:
        hf.hf_state_bytes(cfg)
    assert "flags" in str(e.value)


def test_version_and_state_bytes(lib):
    assert hf.hf_version().startswith("hf-gfx950")
    cfg = hf.make_config(1, 12, 128, "bf16", 64, 64, 0.25)
    assert hf.hf_state_bytes(cfg) == 12 * (128 * 128 + 128) * 4 == 792576
    cfg = hf.make_config(2, 3, 64, "f32", 16, 16, 0.25)
    assert hf.hf_state_bytes(cfg) == 6 * (64 * 64 + 64) * 4


@pytest.mark.parametrize("ratio,n_kv,b", [(0.25, 256, 16), (0.25, 9360, 64), (0.125, 21600, 128), (0.25, 21600, 128),
                                          (0.5, 21600, 128), (1.0, 21600, 128), (0.3, 500, 32), (1e-6, 100, 10),
                                          # ratio * T_n an integer with a ratio that float32 cannot hold exactly
                                          (0.1, 100, 10), (0.2, 1500, 10), (0.3, 100, 10), (0.6, 50, 10),
                                          (0.1, 1500, 10), (0.7, 100, 10), (0.9, 300, 10), (0.05, 2000, 10)])
def test_select_k_matches_oracle(lib, ratio, n_kv, b):
    cfg = hf.make_config(1, 1, 128, "bf16", b, b, ratio)
    t_n = -(-n_kv // b)
    assert hf.hf_select_k(cfg, n_kv) == orc.select_k(ratio, t_n)


def test_absorb_workspace_holds_one_partial_per_slice(lib):
    cfg = hf.make_config(1, 12, 128, "bf16", 64, 64, 0.25)
    part = (128 * 128 + 128) * 4
    got = hf.hf_absorb_workspace_bytes(cfg, 4680)
    assert got % (12 * part) == 0 and 1 <= got // (12 * part) <= 4680 // 64 + 1
    assert hf.hf_absorb_workspace_bytes(hf.make_config(1, 2, 64, "f32", 16, 16, 0.25), 512) == 0


def test_keep_k_override_and_bounds(lib):
    cfg = hf.make_config(1, 1, 128, "bf16", 64, 64, 0.25, keep_k=5)
    assert hf.hf_select_k(cfg, 9360) == 5
    cfg = hf.make_config(1, 1, 128, "bf16", 64, 64, 0.25, keep_k=148)
    with pytest.raises(hf.HFError) as e:
        hf.hf_select_k(cfg, 9360)
    assert e.value.code == -2


def test_workspace_covers_pooled_means_local_output_and_state_planes(lib):
    cfg = hf.make_config(1, 12, 128, "bf16", 64, 64, 0.25)
    need = 12 * (74 + 147) * 128 * 4 + 12 * 4680 * 128 * 2 + 12 * 2 * 128 * 128 * 2
    got = hf.hf_workspace_bytes(cfg, 4680, 9360)
    assert need <= got <= need + 4 * 256


@pytest.mark.parametrize("kw,code", [
    (dict(head_dim=96), -2), (dict(dtype=7), -3), (dict(phi=9), -3), (dict(block_q=0), -2),
    (dict(keep_ratio=0.0), -2), (dict(keep_ratio=1.5), -2), (dict(batch=0), -2), (dict(eps=-1.0), -2),
])
def test_bad_config_is_rejected(lib, kw, code):
    base = dict(batch=1, heads=2, head_dim=128, dtype=hf.HF_BF16, block_q=64, block_kv=64, keep_ratio=0.25)
    base.update(kw)
    cfg = hf.make_config(**base)
    with pytest.raises(hf.HFError) as e:
        hf.hf_state_bytes(cfg)
    assert e.value.code == code
    assert hf.load().hf_last_error()


def test_null_and_misaligned_pointers_are_rejected_before_any_launch(lib):
    cfg = hf.make_config(1, 2, 128, "bf16", 64, 64, 0.25)
    c = ctypes.byref(cfg)
    assert lib.hf_state_init(c, None, None) == -1
    assert lib.hf_state_init(None, None, None) == -1
    assert lib.hf_state_fold_linear(c, 4096, None, 1 << 24, None) == -1
    assert lib.hf_state_fold_linear(c, 4096, 1 << 20, 4096 + 256, None) == -2      # state_out overlaps state_in
    assert lib.hf_absorb_evicted(c, 4096, None, 4096, 10, None, None, None, 0, None) == -1
    assert lib.hf_absorb_evicted(c, 4096, 4096, 4100, 10, None, None, None, 0, None) == -4
    assert lib.hf_absorb_evicted(c, 4096, 4096, 4096, 0, None, None, None, 0, None) == -2
    assert lib.hf_absorb_evicted(c, 4096, 4096, 4096, 10, 4096, None, None, 0, None) == -1   # cos without sin
    assert lib.hf_absorb_evicted(c, 4096, 4096, 4096, 10, None, None, 4096 + 16, 1 << 20, None) == -4   # workspace alignment
    assert lib.hf_window_advance(c, 4096, 8192, 200, 300, 1 << 20, None, None, None, 0, None) == -2   # evicts more than it holds
    assert lib.hf_window_advance(c, 4096, None, 200, 100, 1 << 20, None, None, None, 0, None) == -1
    assert lib.hf_window_advance(c, 4096, 8192, 200, 100, 1 << 20, 4096, None, None, 0, None) == -1  # cos without sin
    assert lib.hf_block_select(c, 4096, 100, 4096, 200, 4096, None, None, 0, None) == -5
    assert lib.hf_block_select(c, 4096, 100, 4096, 200, 4096, None, 4096 + 16, 1 << 30, None) == -4
    # reused pooled keys: whole blocks of the window only (200 tokens = 3 whole blocks of 64)
    assert lib.hf_block_select_cached(c, 4096, 100, 4096, 200, 4, 4096, None, 4096, 1 << 30, None) == -2
    assert lib.hf_block_select_cached(c, 4096, 100, 4096, 200, -1, 4096, None, 4096, 1 << 30, None) == -2
    assert lib.hf_block_select_cached(c, 4096, 100, 4096, 200, 3, 4096, None, None, 0, None) == -5
    # O aliases Q
    assert lib.hf_hybrid_attn_fwd(c, 4096, 100, 8192, 8192, 200, None, 0, None, None, None, 4096, None, 0, None) == -2
    # k out of range with an index list
    assert lib.hf_hybrid_attn_fwd(c, 4096, 100, 8192, 8192, 200, 4096, 9, None, None, None, 16384, None, 0, None) == -2
    # state given but no workspace
    assert lib.hf_hybrid_attn_fwd(c, 4096, 100, 8192, 8192, 200, None, 0, 4096, None, None, 16384, None, 0, None) == -5
    assert b"workspace" in lib.hf_last_error()


def test_rope_window_indices_follow_eq7(lib):
    # host-only helper against the oracle's reading of Eq. 7 and of the re-based cache
    for t0 in (5, 21):
        for n in (1, 3, 6, 9, 30):
            for i in (0, 2, 5, 20, 21, 22, 23, 1000):
                assert hf.hf_rope_window_indices(i, n, t0) == orc.window_temporal_indices(i, n, t0).tolist()
    assert hf.hf_rope_window_indices(30, 3, 21) == orc.chunk_temporal_indices(30, 3, 21).tolist()


def test_rope_calls_reject_bad_arguments(lib):
    cfg = hf.make_config(1, 2, 128, "bf16", 64, 64, 0.25)
    c = ctypes.byref(cfg)
    I = ctypes.c_int32
    idx = (I * 70)(*range(70))
    assert lib.hf_rope_window_indices(5, 0, 21, idx) == -2
    assert lib.hf_rope_window_indices(5, 3, 21, None) == -1
    assert lib.hf_rope_tables(None, 3, 4, 4, 22, 21, 21, 1e4, 0, 4096, 8192, None) == -1
    assert lib.hf_rope_tables(idx, 65, 4, 4, 22, 21, 21, 1e4, 0, 4096, 8192, None) == -2     # too many frames
    assert lib.hf_rope_tables(idx, 3, 4, 4, 64, 64, 1, 1e4, 0, 4096, 8192, None) == -2       # too many pairs
    assert lib.hf_rope_tables(idx, 3, 0, 4, 22, 21, 21, 1e4, 0, 4096, 8192, None) == -2
    assert lib.hf_rope_tables(idx, 3, 4, 4, 22, 21, 21, -1.0, 0, 4096, 8192, None) == -2
    assert lib.hf_rope_tables(idx, 3, 4, 4, 22, 21, 21, 1e4, 0, None, 8192, None) == -1
    assert lib.hf_rope_apply(c, 4096, 100, None, 4096, 1 << 20, None) == -1
    assert lib.hf_rope_apply(c, 4096, 100, 4096, 4096, 4096 + 512, None) == -2              # partial overlap
    assert lib.hf_rope_apply(c, 4096, 0, 4096, 4096, 1 << 20, None) == -2
    # the split call checks the second query pointer like the first
    assert lib.hf_hybrid_attn_fwd_split(c, 4096, 4100, 100, 8192, 8192, 200, None, 0, None, None, None, 16384,
                                        None, 0, None) == -4
    assert lib.hf_hybrid_attn_fwd_split(c, 4096, 16384, 100, 8192, 8192, 200, None, 0, None, None, None, 16384,
                                        None, 0, None) == -2                                  # O aliases Q_hist


def test_cache_capacity_and_stream_bookkeeping_are_checked(lib):
    cfg = hf.make_config(1, 2, 128, "bf16", 64, 64, 0.25, kv_capacity=300)
    c = ctypes.byref(cfg)
    # a window longer than the cache buffer
    assert lib.hf_block_select(c, 4096, 100, 4096, 301, 4096, None, 4096, 1 << 30, None) == -2
    assert b"kv_capacity" in lib.hf_last_error()
    assert lib.hf_hybrid_attn_fwd(c, 4096, 100, 8192, 8192, 301, None, 0, None, None, None, 16384, None, 0, None) == -2
    assert lib.hf_window_evict(c, 4096, 8192, 301, 0, 100, 1 << 20, None, None, None, 0, None) == -2
    # eviction must stay behind the sink
    assert lib.hf_window_evict(c, 4096, 8192, 300, 250, 100, 1 << 20, None, None, None, 0, None) == -2
    assert lib.hf_window_evict(c, 4096, 8192, 300, -1, 100, 1 << 20, None, None, None, 0, None) == -2
    # stream calls: bookkeeping out of range, chunk larger than the room behind the sink, no capacity at all
    win = hf.hf_window(100, 50)
    first = ctypes.c_int32(0)
    assert lib.hf_stream_open_chunk(c, ctypes.byref(win), 100, 4096, 8192, 1 << 20, None, None, None, 0,
                                    ctypes.byref(first), None, None) == -2
    win = hf.hf_window(100, 100)
    assert lib.hf_stream_open_chunk(c, ctypes.byref(win), 201, 4096, 8192, 1 << 20, None, None, None, 0,
                                    ctypes.byref(first), None, None) == -2
    assert lib.hf_stream_open_chunk(c, None, 100, 4096, 8192, 1 << 20, None, None, None, 0, None, None, None) == -1
    packed = hf.make_config(1, 2, 128, "bf16", 64, 64, 0.25)
    assert lib.hf_stream_open_chunk(ctypes.byref(packed), ctypes.byref(win), 100, 4096, 8192, 1 << 20, None, None,
                                    None, 0, None, None, None) == -2
    # a chunk that fits without eviction launches nothing: pure bookkeeping on the host
    win = hf.hf_window(100, 100)
    n_ev = ctypes.c_int32(-1)
    assert lib.hf_stream_open_chunk(c, ctypes.byref(win), 150, 4096, 8192, 1 << 20, None, None, None, 0,
                                    ctypes.byref(first), ctypes.byref(n_ev), None) == 0
    assert (first.value, n_ev.value, win.n_tokens) == (100, 0, 250)
    # a step on a window shorter than the chunk
    win = hf.hf_window(0, 50)
    assert lib.hf_stream_step(c, ctypes.byref(win), 4096, None, 100, 8192, 8192, 0, 4096, None, None, None, 16384,
                              4096, 1 << 30, None) == -2


def test_backward_call_rejects_bad_arguments(lib):
    cfg = hf.make_config(1, 2, 128, "bf16", 64, 64, 0.25)
    c = ctypes.byref(cfg)
    a = [4096 * i for i in range(1, 12)]          # distinct aligned fake addresses; nothing is launched on an error
    Q, K, V, dO, dQ, dK, dV, dQh, Qh, ws = a[:10]
    ok_tail = (ws << 8, 1 << 40, None)
    # Q_hist of its own needs dQ_hist; a single query tensor must not get one
    assert lib.hf_hybrid_attn_bwd(c, Q, Qh, 100, K, V, 200, None, 0, None, None, None, dO, dQ, None, dK, dV, *ok_tail) == -1
    assert lib.hf_hybrid_attn_bwd(c, Q, None, 100, K, V, 200, None, 0, None, None, None, dO, dQ, dQh, dK, dV, *ok_tail) == -2
    # outputs aliasing inputs or each other
    assert lib.hf_hybrid_attn_bwd(c, Q, None, 100, K, V, 200, None, 0, None, None, None, dO, Q, None, dK, dV, *ok_tail) == -2
    assert lib.hf_hybrid_attn_bwd(c, Q, None, 100, K, V, 200, None, 0, None, None, None, dO, dQ, None, dK, dK, *ok_tail) == -2
    # missing gradient input, k out of range, workspace too small
    assert lib.hf_hybrid_attn_bwd(c, Q, None, 100, K, V, 200, None, 0, None, None, None, None, dQ, None, dK, dV, *ok_tail) == -1
    assert lib.hf_hybrid_attn_bwd(c, Q, None, 100, K, V, 200, 4096 * 20, 9, None, None, None, dO, dQ, None, dK, dV, *ok_tail) == -2
    assert lib.hf_hybrid_attn_bwd(c, Q, None, 100, K, V, 200, None, 0, None, None, None, dO, dQ, None, dK, dV, ws << 8, 16, None) == -5
    n = ctypes.c_size_t(0)
    assert lib.hf_bwd_workspace_bytes(c, 100, 200, ctypes.byref(n)) == 0
    # two row statistics per query row, the fp32 history gradient, the inverse index lists (counts + T_n x T_m entries)
    assert n.value >= 2 * 2 * 100 * 4 + 2 * 100 * 128 * 4 + 2 * 4 * 4 + 2 * 4 * 2 * 4


def test_saving_forward_and_saved_backward_reject_bad_arguments(lib):
    cfg = hf.make_config(1, 2, 128, "bf16", 64, 64, 0.25)
    c = ctypes.byref(cfg)
    a = [4096 * i for i in range(1, 14)]          # distinct aligned fake addresses; nothing is launched on an error
    Q, K, V, dO, dQ, dK, dV, O, Ol, lse, ws = a[:11]
    ok_tail = (ws << 8, 1 << 40, None)
    # both by-products are required and must be buffers of their own
    assert lib.hf_hybrid_attn_fwd_save(c, Q, None, 100, K, V, 200, None, 0, None, None, None, O, None, lse, *ok_tail) == -1
    assert lib.hf_hybrid_attn_fwd_save(c, Q, None, 100, K, V, 200, None, 0, None, None, None, O, Ol, None, *ok_tail) == -1
    assert lib.hf_hybrid_attn_fwd_save(c, Q, None, 100, K, V, 200, None, 0, None, None, None, O, O, lse, *ok_tail) == -2
    assert lib.hf_hybrid_attn_fwd_save(c, Q, None, 100, K, V, 200, None, 0, None, None, None, O, Ol, Ol, *ok_tail) == -2
    assert lib.hf_hybrid_attn_bwd_saved(c, Q, None, 100, K, V, 200, None, 0, None, None, None, dO, None, lse, dQ, None, dK,
                                        dV, *ok_tail) == -1
    assert lib.hf_hybrid_attn_bwd_saved(c, Q, None, 100, K, V, 200, None, 0, None, None, None, dO, Ol, None, dQ, None, dK,
                                        dV, *ok_tail) == -1
    assert lib.hf_hybrid_attn_bwd_saved(c, Q, None, 100, K, V, 200, None, 0, None, None, None, dO, Ol, lse, Ol, None, dK,
                                        dV, *ok_tail) == -2          # an output over a saved input
    # configurations outside the matrix-core path have no saving pair
    for other in (hf.make_config(1, 2, 128, "f32", 64, 64, 0.25), hf.make_config(1, 2, 64, "bf16", 64, 64, 0.25),
                  hf.make_config(1, 2, 128, "bf16", 32, 64, 0.25)):
        co = ctypes.byref(other)
        assert lib.hf_hybrid_attn_fwd_save(co, Q, None, 100, K, V, 200, None, 0, None, None, None, O, Ol, lse, *ok_tail) == -2
        assert lib.hf_hybrid_attn_bwd_saved(co, Q, None, 100, K, V, 200, None, 0, None, None, None, dO, Ol, lse, dQ, None,
                                            dK, dV, *ok_tail) == -2
        assert b"hf_hybrid_attn_bwd" in lib.hf_last_error() or b"recomput" in lib.hf_last_error()


def test_kept_planes_entry_points_reject_bad_arguments():
    """Argument checks of the calls that keep the state's bf16 planes with the caller (no GPU needed)."""
    import ctypes
    lib = hf.load()
    cfg32 = hf.make_config(1, 2, 64, "f32", 16, 16, 0.25)
    assert hf.hf_state_planes_bytes(cfg32) == 0
    cfg = hf.make_config(1, 12, 128, "bf16", 64, 64, 0.25)
    assert hf.hf_state_planes_bytes(cfg) == 12 * 2 * 128 * 128 * 2
    out = ctypes.c_size_t(0)
    assert lib.hf_state_planes_bytes(None, ctypes.byref(out)) != 0
    assert lib.hf_state_planes_bytes(ctypes.byref(cfg), None) != 0
    fake = ctypes.c_void_p(0x1000)
    # unsupported configuration, NULL planes, misaligned planes
    assert lib.hf_state_planes(ctypes.byref(cfg32), fake, fake, None) != 0
    assert lib.hf_state_planes(ctypes.byref(cfg), fake, None, None) != 0
    assert b"planes_out" in lib.hf_last_error()
    assert lib.hf_state_planes(ctypes.byref(cfg), fake, ctypes.c_void_p(0x1010), None) != 0
    assert b"aligned" in lib.hf_last_error()
    assert lib.hf_absorb_evicted_planes(ctypes.byref(cfg), fake, fake, fake, 64, None, None, None, 0, None, None) != 0
    assert lib.hf_absorb_evicted_planes(ctypes.byref(cfg), fake, fake, fake, 64, None, None, None, 0, fake, None) != 0
    assert b"alias" in lib.hf_last_error()
    assert lib.hf_hybrid_attn_fwd_planes(ctypes.byref(cfg), fake, None, 64, fake, fake, 64, None, 0, None, fake,
                                         None, None, fake, None) != 0
    assert b"state" in lib.hf_last_error()
    assert lib.hf_hybrid_attn_fwd_planes(ctypes.byref(cfg32), fake, None, 64, fake, fake, 64, None, 0, fake, fake,
                                         None, None, fake, None) != 0



def test_one_launch_entry_points_reject_bad_arguments(lib):
    """hf_pool_keys / hf_select_attn_fwd / hf_step_fwd: sizes and argument checks on the host, nothing launched."""
    class E:   # error codes of hf.h
        HF_ERR_NULL, HF_ERR_SHAPE, HF_ERR_DTYPE, HF_ERR_ALIGN, HF_ERR_WORKSPACE = -1, -2, -3, -4, -5
    cfg = hf.make_config(1, 12, 128, "bf16", 64, 64, 0.25)
    cfg32 = hf.make_config(1, 2, 64, "f32", 16, 16, 0.25)
    fake = ctypes.c_void_p(0x1000)
    # pooled keys: B*H*T_n*d floats, rounded up to 256 bytes
    assert hf.hf_pooled_keys_bytes(cfg, 9360) == 12 * 147 * 128 * 4
    assert hf.hf_pooled_keys_bytes(cfg32, 100) == (2 * 7 * 64 * 4 + 255) // 256 * 256
    # the step's workspace: counters + one partial of the state per (head, slice), at least one slice
    part = (128 * 128 + 128) * 4
    got = hf.hf_step_workspace_bytes(cfg, 4680, 4680)
    assert got > 12 * part and (got - 256) % (12 * part) == 0 and 1 <= (got - 256) // (12 * part) <= 8
    assert hf.hf_step_workspace_bytes(cfg32, 64, 64) == 0          # no such path for this configuration
    assert lib.hf_pool_keys(ctypes.byref(cfg), None, 9360, 0, fake, None) == E.HF_ERR_NULL
    assert lib.hf_pool_keys(ctypes.byref(cfg), fake, 9360, 0, ctypes.c_void_p(0x1010), None) == E.HF_ERR_ALIGN
    assert lib.hf_pool_keys(ctypes.byref(cfg), fake, 9360, 147, fake, None) == E.HF_ERR_SHAPE   # whole blocks only: 146
    # selection inside the attention launch: bf16 / head_dim 128 only, window of at most 1024 blocks, planes with a state
    args = lambda c, n_kv=9360, pooled=fake, state=None, planes=None, idx=fake: (
        ctypes.byref(c), fake, None, 4680, fake, fake, n_kv, pooled, state, planes, None, None, ctypes.c_void_p(0x2000),
        idx, None, None)
    assert lib.hf_select_attn_fwd(*args(cfg32)) == E.HF_ERR_SHAPE
    assert lib.hf_select_attn_fwd(*args(cfg, pooled=None)) == E.HF_ERR_NULL
    assert lib.hf_select_attn_fwd(*args(cfg, idx=None)) == E.HF_ERR_NULL
    assert lib.hf_select_attn_fwd(*args(cfg, n_kv=64 * 1025)) == E.HF_ERR_SHAPE
    assert lib.hf_select_attn_fwd(*args(cfg, state=fake, planes=None)) == E.HF_ERR_NULL
    # the step: state_out is required and must not overlap what the attention reads; phi = ReLU only
    st_in, st_out = ctypes.c_void_p(0x100000), ctypes.c_void_p(0x400000)
    pl_in, pl_out = ctypes.c_void_p(0x800000), ctypes.c_void_p(0xC00000)
    wsp = ctypes.c_void_p(0x1000000)
    def step(c=cfg, K_ev=fake, V_ev=fake, n_ev=4680, stride=0, so=st_out, po=pl_out, ws=wsp, wb=1 << 30):
        return lib.hf_step_fwd(ctypes.byref(c), fake, None, 4680, fake, fake, 9360, fake, st_in, pl_in, None, None,
                               ctypes.c_void_p(0x2000), fake, None, K_ev, V_ev, n_ev, stride, so, po, ws, wb, None)
    assert step(K_ev=None) == E.HF_ERR_NULL
    assert step(V_ev=None) == E.HF_ERR_NULL
    assert step(so=None) == E.HF_ERR_NULL
    assert step(so=st_in) == E.HF_ERR_SHAPE
    assert step(po=pl_in) == E.HF_ERR_SHAPE
    assert step(so=ctypes.c_void_p(0x100000 + 4096)) == E.HF_ERR_SHAPE           # overlaps state_in
    assert step(stride=100) == E.HF_ERR_SHAPE                                     # head stride below n_ev
    assert step(wb=1024) == E.HF_ERR_WORKSPACE
    assert step(ws=None) == E.HF_ERR_WORKSPACE
    assert step(c=hf.make_config(1, 12, 128, "bf16", 64, 64, 0.25, phi=hf.HF_PHI_ELU1)) == E.HF_ERR_SHAPE


def test_rope_append_keys_rejects_bad_arguments(lib):
    cfg = hf.make_config(1, 12, 128, "bf16", 64, 64, 0.25)
    fake, win, pooled = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x10000000), ctypes.c_void_p(0x40000000)
    call = lambda K_new=fake, n_new=4680, cos=fake, sin=fake, K_win=win, first=4680, n_kv=9360, pk=pooled: \
        lib.hf_rope_append_keys(ctypes.byref(cfg), K_new, n_new, cos, sin, K_win, first, n_kv, pk, None)
    assert call(K_new=None) == -1 and call(K_win=None) == -1 and call(pk=None) == -1
    assert call(sin=None) == -1                              # one table without the other
    assert call(first=4681) == -2 and call(first=-1) == -2   # the new tokens must lie inside the window
    assert call(n_new=0) == -2
    assert call(pk=ctypes.c_void_p(0x40000010)) == -4
    assert call(K_new=ctypes.c_void_p(0x10000100)) == -2     # overlaps the window buffer


def test_ring_struct_layout_and_last_step_arguments(lib):
    assert ctypes.sizeof(hf.hf_ring) == 6 * 4 and hf.hf_ring.absorbed_ahead.offset == 20
    cfg = hf.make_config(1, 2, 128, "bf16", 64, 64, 0.25, kv_capacity=1400)
    fake = ctypes.c_void_p(0x100000)
    ring = hf.make_ring(200, 400)
    args = lambda r, so=ctypes.c_void_p(0x900000): (ctypes.byref(cfg), ctypes.byref(r), fake, None, fake, fake, 2, fake, fake,
                                                    None, None, fake, fake, 1 << 30, so, None, None, fake, 1 << 30, None, None)
    assert lib.hf_ring_last_step(*args(ring)) == -2                 # no chunk is open
    full = hf.hf_ring(200, 400, 3, 0, 2, 0)
    assert lib.hf_ring_last_step(*args(full, so=None)) == -1        # a full ring needs somewhere to put the new state
    assert lib.hf_ring_last_step(*args(full, so=fake)) == -2        # ... other than the state it reads
    assert lib.hf_ring_last_step(*args(hf.hf_ring(200, 400, 3, 0, 2, 7))) == -2   # bookkeeping out of range
