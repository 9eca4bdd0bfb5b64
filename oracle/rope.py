"""Plain fp64 NumPy oracle of the relative, capped temporal RoPE (Hybrid Forcing, Sec. 3.3, Eq. 7).

TEST INFRASTRUCTURE ONLY: shares nothing with, is not imported by and does not import the HIP
library.  It builds the per-token cos/sin tables that ``rope_rotate`` of the attention oracle
consumes.

What the paper fixes: the temporal index of the chunk being generated follows the running frame
index until it reaches the cap T0 and stays at the cap afterwards (Eq. 7); frames in the KV cache
are indexed by their offset to the current chunk; spatial coordinates are untouched.

Readings where the paper is silent ("parity unpinned" by the paper itself; each is a convention of
the pretrained video-diffusion family the paper starts from, restated here):

* ``i`` of Eq. 7 is the running index of the newest latent frame of the chunk; a chunk of c frames
  takes the c consecutive indices that end there (the paper prints c = 3).
* A cached frame that lies ``delta`` frames before the newest frame takes the newest frame's
  (capped) index minus ``delta``.
* Rotary features are split over three axes: of the d/2 adjacent feature pairs the first
  ``pairs_t`` turn with the frame index, the next ``pairs_h`` with the row and the last
  ``pairs_w`` with the column of the token; pair p of an axis with n pairs turns by
  ``position * theta ** (-p / n)`` radians, theta = 10000.
* Tokens are ordered frame-major, then row, then column.
"""
from __future__ import annotations

import numpy as np

_F = np.float64


def default_axis_pairs(d: int):
    """(pairs_t, pairs_h, pairs_w): rows and columns take d // 6 pairs each, time takes the rest."""
    if d % 2:
        raise ValueError("head_dim must be even")
    s = d // 6
    return d // 2 - 2 * s, s, s


def chunk_temporal_indices(i: int, chunk_frames: int, t0: int) -> np.ndarray:
    """Eq. 7: indices of the chunk whose newest frame has running index ``i``, capped at ``t0``."""
    last = i if i <= t0 else t0
    return np.arange(last - chunk_frames + 1, last + 1, dtype=np.int64)


def window_temporal_indices(i: int, n_window_frames: int, t0: int) -> np.ndarray:
    """Indices of the last ``n_window_frames`` frames up to and including running index ``i``
    (cached frames followed by the current chunk): each frame's offset to the newest frame is
    kept, the newest frame takes the capped index."""
    last = i if i <= t0 else t0
    delta = np.arange(n_window_frames - 1, -1, -1, dtype=np.int64)
    return last - delta


def axis_frequencies(n_pairs: int, theta: float = 10000.0) -> np.ndarray:
    p = np.arange(n_pairs, dtype=_F)
    return np.asarray(theta, dtype=_F) ** (-p / max(n_pairs, 1))


def rope_tables_3d(frame_idx, height: int, width: int, pairs, theta: float = 10000.0,
                   temporal_only: bool = False):
    """cos, sin ``[len(frame_idx) * height * width, pairs_t + pairs_h + pairs_w]`` (fp64).

    ``temporal_only`` zeroes the spatial angles: such a table turns keys that already carry their
    rotation by a change of temporal index alone (re-basing a cached chunk)."""
    pt, ph, pw = pairs
    frame_idx = np.asarray(frame_idx, dtype=_F)
    f = frame_idx.shape[0]
    ang = np.zeros((f, height, width, pt + ph + pw), dtype=_F)
    ang[..., :pt] = frame_idx[:, None, None, None] * axis_frequencies(pt, theta)
    if not temporal_only:
        rows = np.arange(height, dtype=_F)
        cols = np.arange(width, dtype=_F)
        ang[..., pt:pt + ph] = rows[None, :, None, None] * axis_frequencies(ph, theta)
        ang[..., pt + ph:] = cols[None, None, :, None] * axis_frequencies(pw, theta)
    ang = ang.reshape(f * height * width, pt + ph + pw)
    return np.cos(ang), np.sin(ang)
