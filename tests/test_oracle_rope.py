"""Pins for the oracle's relative, capped temporal RoPE (Sec. 3.3, Eq. 7).  CPU only."""
import cmath
import math
import os

import numpy as np
import pytest

import oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "eq7_temporal_indices.txt")


def test_eq7_values_written_out_by_hand():
    rows = [ln.split() for ln in open(GOLDEN) if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 6
    for r in rows:
        i, t0, want = int(r[0]), int(r[1]), [int(x) for x in r[2:]]
        assert orc.chunk_temporal_indices(i, 3, t0).tolist() == want


def test_window_indices_keep_offsets_and_stop_at_the_cap():
    t0, c, nwin = 21, 3, 9
    for i in (8, 14, 21, 22, 50, 1000):
        w = orc.window_temporal_indices(i, nwin, t0)
        assert np.all(np.diff(w) == 1)                       # offsets between frames are kept
        assert w[-c:].tolist() == orc.chunk_temporal_indices(i, c, t0).tolist()
        assert w[-1] == min(i, t0)
    # below the cap a new chunk moves every index by the chunk length, beyond it nothing moves
    assert (orc.window_temporal_indices(14, nwin, t0) - orc.window_temporal_indices(11, nwin, t0)).tolist() == [3] * nwin
    assert orc.window_temporal_indices(40, nwin, t0).tolist() == orc.window_temporal_indices(43, nwin, t0).tolist()
    # a window longer than the cap reaches below zero instead of folding frames onto each other
    assert orc.window_temporal_indices(100, 30, t0)[0] == t0 - 29


def test_default_split_covers_all_pairs():
    assert orc.default_axis_pairs(128) == (22, 21, 21)
    for d in (8, 64, 96, 128, 256):
        assert sum(orc.default_axis_pairs(d)) == d // 2


def test_tables_against_complex_exponentials():
    # rotating the pair (x0, x1) by the table equals multiplying x0 + i x1 by exp(i * pos * omega),
    # with omega spelled out per pair here (theta = 10000): time pairs 1, 1e-2; row pair 1; column pairs 1, 1e-2
    pairs = (2, 1, 2)
    frames, hh, ww = [4, 7], 3, 2
    cos, sin = orc.rope_tables_3d(frames, hh, ww, pairs)
    assert cos.shape == (2 * 3 * 2, 5)
    omega = [(0, 1.0), (0, 1e-2), (1, 1.0), (2, 1.0), (2, 1e-2)]       # (axis, frequency) per pair
    r = np.random.default_rng(3)
    X = r.normal(size=(cos.shape[0], 10))
    Y = orc.rope_rotate(X, cos, sin)
    n = 0
    for fi, f in enumerate(frames):
        for y in range(hh):
            for x in range(ww):
                pos = (f, y, x)
                for p, (axis, om) in enumerate(omega):
                    zc = complex(X[n, 2 * p], X[n, 2 * p + 1]) * cmath.exp(1j * pos[axis] * om)
                    assert abs(zc.real - Y[n, 2 * p]) < 1e-12 and abs(zc.imag - Y[n, 2 * p + 1]) < 1e-12
                n += 1


def test_table_special_values():
    pairs = orc.default_axis_pairs(128)
    cos, sin = orc.rope_tables_3d([0, 1, 21], 2, 3, pairs)
    np.testing.assert_allclose(cos * cos + sin * sin, 1.0, atol=1e-14)
    # token (frame index 0, row 0, column 0) is not rotated at all
    assert np.all(cos[0] == 1.0) and np.all(sin[0] == 0.0)
    # the first pair of each axis turns by one radian per position
    tok = 2 * 6 + 1 * 3 + 2          # frame index 21, row 1, column 2
    assert cos[tok, 0] == pytest.approx(math.cos(21.0), abs=1e-15)
    assert sin[tok, pairs[0]] == pytest.approx(math.sin(1.0), abs=1e-15)
    assert sin[tok, pairs[0] + pairs[1]] == pytest.approx(math.sin(2.0), abs=1e-15)
    # the slowest pair of the time axis: 10000 ** (-21 / 22)
    assert cos[tok, pairs[0] - 1] == pytest.approx(math.cos(21.0 * 10000.0 ** (-21.0 / 22.0)), abs=1e-15)
    # temporal_only leaves the spatial pairs alone
    c2, s2 = orc.rope_tables_3d([0, 1, 21], 2, 3, pairs, temporal_only=True)
    assert np.all(c2[:, pairs[0]:] == 1.0) and np.all(s2[:, pairs[0]:] == 0.0)
    np.testing.assert_array_equal(c2[:, :pairs[0]], cos[:, :pairs[0]])


def test_logits_depend_on_position_differences_only():
    # q.k after rotation is unchanged when query and key frames move by the same number of frames
    pairs = (3, 2, 3)
    r = np.random.default_rng(5)
    hh, ww = 2, 2
    q = r.normal(size=(hh * ww, 16))
    k = r.normal(size=(hh * ww, 16))

    def logits(tq, tk):
        cq, sq = orc.rope_tables_3d([tq], hh, ww, pairs)
        ck, sk = orc.rope_tables_3d([tk], hh, ww, pairs)
        return orc.rope_rotate(q, cq, sq) @ orc.rope_rotate(k, ck, sk).T

    np.testing.assert_allclose(logits(5, 2), logits(21, 18), atol=1e-12)
    assert np.abs(logits(5, 2) - logits(5, 3)).max() > 1e-3           # and does depend on the difference


def test_capped_streaming_logits_are_stationary():
    # beyond the cap the logits between the chunk's queries and the window's keys no longer change with i
    pairs, t0, c, nwin, hh, ww = (2, 1, 1), 21, 3, 9, 1, 2
    r = np.random.default_rng(6)
    q = r.normal(size=(c * hh * ww, 8))
    k = r.normal(size=(nwin * hh * ww, 8))

    def logits(i):
        cq, sq = orc.rope_tables_3d(orc.chunk_temporal_indices(i, c, t0), hh, ww, pairs)
        ck, sk = orc.rope_tables_3d(orc.window_temporal_indices(i, nwin, t0), hh, ww, pairs)
        return orc.rope_rotate(q, cq, sq) @ orc.rope_rotate(k, ck, sk).T

    np.testing.assert_allclose(logits(30), logits(300), atol=1e-12)
    np.testing.assert_allclose(logits(12), logits(30), atol=1e-12)    # the same offsets below the cap


def test_rebasing_rotated_keys_by_a_temporal_offset():
    # keys rotated at frame index t, turned again by a temporal-only table of -3 frames, equal keys rotated at t - 3
    pairs, hh, ww = (3, 2, 3), 2, 3
    r = np.random.default_rng(7)
    k = r.normal(size=(2 * hh * ww, 16))
    c0, s0 = orc.rope_tables_3d([10, 11], hh, ww, pairs)
    cd, sd = orc.rope_tables_3d([-3, -3], hh, ww, pairs, temporal_only=True)
    c1, s1 = orc.rope_tables_3d([7, 8], hh, ww, pairs)
    np.testing.assert_allclose(orc.rope_rotate(orc.rope_rotate(k, c0, s0), cd, sd), orc.rope_rotate(k, c1, s1), atol=1e-12)


def test_split_queries_feed_the_two_branches():
    # Q_hist replaces Q in the history branch only
    r = np.random.default_rng(8)
    n, d = 12, 8
    Q, Qh, K, V = (r.normal(size=(n, d)) for _ in range(4))
    L, z = orc.state_absorb(*orc.state_zero(d), r.normal(size=(20, d)), r.normal(size=(20, d)))
    O, Ol, Oh, _, _ = orc.hybrid_attention(Q, K, V, (L, z), 4, 4, 2, Q_hist=Qh)
    np.testing.assert_allclose(Ol, orc.hybrid_attention(Q, K, V, None, 4, 4, 2)[0], atol=1e-14)
    np.testing.assert_allclose(Oh, orc.history_readout(Qh, L, z), atol=1e-14)
    np.testing.assert_allclose(O, Ol + Oh, atol=1e-14)
