"""Plain fp64 NumPy oracle of the per-chunk hybrid attention (Hybrid Forcing, Sec. 3.2).

TEST INFRASTRUCTURE ONLY.  Slow, un-tiled, un-fused, written from the paper's
definitions (Eq. 2-6 and the "Hybrid Attention" algorithm of the supplement) so a
reader can check it by eye.  Nothing here is shared with, imported by, or imports
the HIP library.  All arithmetic is float64; callers pass the *stored* input values
(e.g. bf16 numbers up-cast exactly).

Every function works on ONE head: 2-D arrays ``[tokens, d]``.  Heads and batch
entries are independent in every step of the method, so callers loop over them.

Readings of the paper taken where it is silent or ambiguous (each is a convention,
"parity unpinned" by the paper itself, and is repeated in the design notes):

* phi ("the activation function" of Eq. 2) is ReLU by default; ``elu(x)+1`` is offered.
* H of Eq. 2 is read as z = sum over evicted tokens of phi(k_t) (a d-vector); a
  constant ``z_scale`` at readout reproduces the per-frame-mean reading.
* ``phi(Q) H`` in Eq. 3 is the inner product phi(q).z, one scalar per query row.
* The ``Linear`` map around Eq. 3 is the identity by default; when a weight is given it is read as a
  per-head d x d matrix without bias acting on the value features (``x -> x W``).
* RoPE is given by caller-built per-token cos/sin tables ``[tokens, d/2]`` acting on
  adjacent feature pairs (2i, 2i+1); it is applied after phi, on the numerator only.
* The readout divides by ``z_scale * phi(q).z + eps``.
* Blocks are consecutive runs of b tokens; a short last block is pooled over its real
  length and contributes only its real keys.
* Top-K is per query-block row on the raw Eq. 4 scores; ties go to the lower index.
* No causal mask inside the window and no forced (sink/diagonal) blocks.

Pins (see tests/test_oracle_*.py): dense limit vs brute-force softmax attention and a
library SDPA; state vs scalar triple loop; order/chunking invariance; brute-force
scoring/selection; quadratic form of linear attention; RoPE relative-shift property;
softmax invariants; hand-masked ragged tails.
"""
from __future__ import annotations

import math

import numpy as np

PHI_RELU = 0
PHI_ELU1 = 1

_F = np.float64


def _as2d(x) -> np.ndarray:
    a = np.asarray(x, dtype=_F)
    if a.ndim != 2:
        raise ValueError("oracle functions take one head: a 2-D [tokens, d] array")
    return a


# --------------------------------------------------------------------------- feature map
def phi(x, kind: int = PHI_RELU) -> np.ndarray:
    """Feature map of Eq. 2/3.  ReLU (default) or elu(x)+1."""
    x = np.asarray(x, dtype=_F)
    if kind == PHI_RELU:
        return np.maximum(x, 0.0)
    if kind == PHI_ELU1:
        return np.where(x > 0.0, x + 1.0, np.exp(np.minimum(x, 0.0)))
    raise ValueError("unknown phi")


def rope_rotate(x, cos=None, sin=None) -> np.ndarray:
    """Rotate adjacent feature pairs (2i, 2i+1) of each token by its own angle.

    ``cos``/``sin`` are ``[tokens, d/2]``; ``None`` means the identity rotation.
    (Sec. 3.3 only fixes which *indices* feed RoPE; the tables are the caller's.)
    """
    x = _as2d(x)
    if cos is None and sin is None:
        return x.copy()
    c = np.asarray(cos, dtype=_F)
    s = np.asarray(sin, dtype=_F)
    n, d = x.shape
    if c.shape != (n, d // 2) or s.shape != (n, d // 2):
        raise ValueError("rope tables must be [tokens, d/2]")
    even = x[:, 0::2]
    odd = x[:, 1::2]
    out = np.empty_like(x)
    out[:, 0::2] = even * c - odd * s
    out[:, 1::2] = even * s + odd * c
    return out


# --------------------------------------------------------------------------- linear state, Eq. 2
def state_zero(d: int):
    """Empty linear state (the inference algorithm's 'Initialize Linear State cache')."""
    return np.zeros((d, d), dtype=_F), np.zeros((d,), dtype=_F)


def state_absorb(L, z, K_ev, V_ev, phi_kind: int = PHI_RELU, cos=None, sin=None):
    """Eq. 2: L += sum_t R_t(phi(k_t))^T v_t ;  z += sum_t phi(k_t).

    L[i, j] pairs key feature i with value feature j.  The sum over tokens is written
    as one matrix product (a library primitive standing for the sum); the tests pin it
    to the scalar triple loop.  Returns new arrays; inputs are not modified.
    """
    K_ev = _as2d(K_ev)
    V_ev = _as2d(V_ev)
    if K_ev.shape != V_ev.shape:
        raise ValueError("K_ev and V_ev must have the same shape")
    fk = phi(K_ev, phi_kind)
    rk = rope_rotate(fk, cos, sin)
    L_new = np.asarray(L, dtype=_F) + rk.T @ V_ev
    z_new = np.asarray(z, dtype=_F) + fk.sum(axis=0)
    return L_new, z_new


# --------------------------------------------------------------------------- block scoring, Eq. 4
def pool_blocks(X, b: int) -> np.ndarray:
    """Mean of each consecutive run of ``b`` rows; the last run may be short."""
    X = _as2d(X)
    n, d = X.shape
    t = -(-n // b)
    out = np.empty((t, d), dtype=_F)
    for i in range(t):
        rows = X[i * b : min((i + 1) * b, n)]
        out[i] = rows.sum(axis=0) / rows.shape[0]
    return out


def block_scores(Q, K, b_q: int, b_kv: int) -> np.ndarray:
    """Eq. 4: A[i, j] = Mean(q_i) . Mean(k_j), raw (no scale, no softmax)."""
    return pool_blocks(Q, b_q) @ pool_blocks(K, b_kv).T


def select_k(keep_ratio: float, t_n: int) -> int:
    """Number of KV blocks kept per query-block row for a keep ratio in (0, 1]."""
    k = int(math.ceil(float(keep_ratio) * t_n - 1e-9))
    return max(1, min(t_n, k))


def select_blocks(A, k: int):
    """Top-K mask of the algorithm's 'M_c' as index lists.

    For each row of ``A`` keep the ``k`` largest entries (ties: lower index first) and
    return their indices ascending, plus the gap between the k-th and (k+1)-th largest
    score of the row (+inf when every block is kept).
    """
    A = np.asarray(A, dtype=_F)
    t_m, t_n = A.shape
    if not (1 <= k <= t_n):
        raise ValueError("k out of range")
    idx = np.empty((t_m, k), dtype=np.int32)
    gap = np.empty((t_m,), dtype=_F)
    for i in range(t_m):
        order = sorted(range(t_n), key=lambda j: (-A[i, j], j))
        idx[i] = np.sort(np.asarray(order[:k], dtype=np.int32))
        gap[i] = np.inf if k == t_n else A[i, order[k - 1]] - A[i, order[k]]
    return idx, gap


# --------------------------------------------------------------------------- sparse window attention, Eq. 5
def sparse_attention(Q, K, V, block_idx, b_q: int, b_kv: int, scale=None) -> np.ndarray:
    """Eq. 5 by two-pass softmax over the keys of the selected blocks only.

    ``block_idx`` is ``[T_m, k]``: for query block i the KV blocks with M[i, j] = 1.
    Keys of a short last block are just the tokens that exist.
    """
    Q = _as2d(Q)
    K = _as2d(K)
    V = _as2d(V)
    n_q, d = Q.shape
    n_kv = K.shape[0]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    block_idx = np.asarray(block_idx)
    t_m = -(-n_q // b_q)
    if block_idx.shape[0] != t_m:
        raise ValueError("block_idx needs one row per query block")
    O = np.empty((n_q, d), dtype=_F)
    for i in range(t_m):
        keys = []
        for j in block_idx[i]:
            keys.extend(range(int(j) * b_kv, min((int(j) + 1) * b_kv, n_kv)))
        keys = np.asarray(keys, dtype=np.int64)
        Ks = K[keys]
        Vs = V[keys]
        rows = slice(i * b_q, min((i + 1) * b_q, n_q))  # all rows of a block share its key set
        S = (Q[rows] @ Ks.T) * scale
        P = np.exp(S - S.max(axis=1, keepdims=True))
        O[rows] = (P / P.sum(axis=1, keepdims=True)) @ Vs
    return O


def dense_attention(Q, K, V, scale=None) -> np.ndarray:
    """Plain softmax(Q K^T / sqrt(d)) V over the whole window (Eq. 1 restricted to one
    window / Eq. 5 with an all-ones mask).  Written separately from sparse_attention."""
    Q = _as2d(Q)
    K = _as2d(K)
    V = _as2d(V)
    if scale is None:
        scale = 1.0 / math.sqrt(Q.shape[1])
    S = (Q @ K.T) * scale
    S = S - S.max(axis=1, keepdims=True)
    P = np.exp(S)
    P /= P.sum(axis=1, keepdims=True)
    return P @ V


# --------------------------------------------------------------------------- history readout, Eq. 3
def history_readout(Q, L, z, phi_kind: int = PHI_RELU, cos=None, sin=None,
                    eps: float = 1e-6, z_scale: float = 1.0, W=None) -> np.ndarray:
    """Eq. 3: Linear( R_q(phi(q)) L / (z_scale * phi(q).z + eps) ); Linear = identity when W is None,
    else right-multiplication of every output row by the d x d matrix W."""
    Q = _as2d(Q)
    fq = phi(Q, phi_kind)
    num = rope_rotate(fq, cos, sin) @ np.asarray(L, dtype=_F)
    den = z_scale * (fq @ np.asarray(z, dtype=_F)) + eps
    out = num / den[:, None]
    if W is not None:
        out = out @ np.asarray(W, dtype=_F)
    return out


def state_fold_linear(L, W) -> np.ndarray:
    """The state whose plain readout equals Linear(readout of L): the row-wise division of Eq. 3
    commutes with a right-multiplication, so the map can be applied to L once: L W."""
    return np.asarray(L, dtype=_F) @ np.asarray(W, dtype=_F)


# --------------------------------------------------------------------------- Eq. 6
def hybrid_attention(Q, K_win, V_win, state, b_q: int, b_kv: int, k: int,
                     phi_kind: int = PHI_RELU, cos_q=None, sin_q=None,
                     eps: float = 1e-6, z_scale: float = 1.0, scale=None,
                     block_idx=None, W=None, Q_hist=None):
    """The whole per-chunk path for one head: score, select, sparse attention,
    history readout, sum (Eq. 4, 5, 3, 6).

    ``Q_hist``: the queries the history branch reads, when they differ from the ones of the
    softmax branch (a model that rotates q for Eq. 4/5 while Eq. 3 applies phi to the
    un-rotated q and rotates afterwards); ``None`` = the same ``Q``.

    ``state`` is ``(L, z)`` or ``None`` (no history yet: O_history = 0).  If
    ``block_idx`` is given it is used instead of the oracle's own selection (stage-wise
    parity: a legal tie difference must not poison the output check).
    Returns ``(O, O_local, O_history, block_idx, gap)``.
    """
    gap = None
    if block_idx is None:
        A = block_scores(Q, K_win, b_q, b_kv)
        block_idx, gap = select_blocks(A, k)
    O_local = sparse_attention(Q, K_win, V_win, block_idx, b_q, b_kv, scale)
    if state is None:
        O_hist = np.zeros_like(O_local)
    else:
        O_hist = history_readout(Q if Q_hist is None else Q_hist, state[0], state[1], phi_kind, cos_q, sin_q, eps, z_scale, W)
    return O_local + O_hist, O_local, O_hist, np.asarray(block_idx), gap
