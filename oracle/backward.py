"""Plain fp64 NumPy oracle of the gradients of the per-chunk hybrid attention (the step of the training
algorithm of the supplement that runs with gradients enabled).

TEST INFRASTRUCTURE ONLY: shares nothing with, is not imported by and does not import the HIP library.

The training algorithm computes the KV cache and the linear state with gradients disabled, so the
differentiable inputs of one hybrid attention are the chunk's queries and the window's keys and
values; the state (L, z), the index lists of the Top-K mask (piecewise constant in Q, K) and the
rotation tables are constants.  Everything below is the chain rule written out on the definitions
(Eq. 5, Eq. 3, Eq. 6), block row by block row, one head at a time; the tests pin it to central
differences of the forward oracle and, in the dense case, to a library autograd.
"""
from __future__ import annotations

import math

import numpy as np

from .hybrid_attention import PHI_ELU1, PHI_RELU, _as2d, phi, rope_rotate

_F = np.float64


def phi_prime(x, kind: int = PHI_RELU) -> np.ndarray:
    """Derivative of the feature map: ReLU -> [x > 0] (0 at the kink), elu(x)+1 -> 1 for x > 0, exp(x) else."""
    x = np.asarray(x, dtype=_F)
    if kind == PHI_RELU:
        return (x > 0.0).astype(_F)
    if kind == PHI_ELU1:
        return np.where(x > 0.0, 1.0, np.exp(np.minimum(x, 0.0)))
    raise ValueError("unknown phi")


def sparse_attention_bwd(Q, K, V, block_idx, b_q: int, b_kv: int, dO, scale=None):
    """Gradients of Eq. 5 for a fixed mask.  Returns (dQ, dK, dV).

    Per query-block row with key set J:  P = softmax(scale Q K_J^T),  O = P V_J
        dV_J += P^T dO            dP = dO V_J^T
        dS    = P * (dP - rowsum(P * dP))
        dQ    = scale dS K_J      dK_J += scale dS^T Q
    Keys that no query block selected get zero gradients.
    """
    Q, K, V, dO = _as2d(Q), _as2d(K), _as2d(V), _as2d(dO)
    n_q, d = Q.shape
    n_kv = K.shape[0]
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    block_idx = np.asarray(block_idx)
    t_m = -(-n_q // b_q)
    dQ = np.zeros((n_q, d), dtype=_F)
    dK = np.zeros((n_kv, d), dtype=_F)
    dV = np.zeros((n_kv, d), dtype=_F)
    for i in range(t_m):
        keys = []
        for j in block_idx[i]:
            keys.extend(range(int(j) * b_kv, min((int(j) + 1) * b_kv, n_kv)))
        keys = np.asarray(keys, dtype=np.int64)
        rows = slice(i * b_q, min((i + 1) * b_q, n_q))
        S = (Q[rows] @ K[keys].T) * scale
        P = np.exp(S - S.max(axis=1, keepdims=True))
        P /= P.sum(axis=1, keepdims=True)
        dP = dO[rows] @ V[keys].T
        dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
        dQ[rows] = (dS @ K[keys]) * scale
        np.add.at(dK, keys, (dS.T @ Q[rows]) * scale)
        np.add.at(dV, keys, P.T @ dO[rows])
    return dQ, dK, dV


def history_readout_bwd(Q, L, z, dO, phi_kind: int = PHI_RELU, cos=None, sin=None,
                        eps: float = 1e-6, z_scale: float = 1.0, W=None) -> np.ndarray:
    """Gradient of Eq. 3 with respect to its queries, the state held constant.

    out = (R(f) L / den) W with f = phi(q), den = z_scale f.z + eps:
        g    = dO W^T                      (back through the Linear map, if any)
        dnum = g / den                     dden = -(g . (R(f) L)) / den^2
        df   = R^T(dnum L^T) + z_scale dden z
        dq   = df * phi'(q)
    R^T is the rotation by the opposite angle.
    """
    Q, dO = _as2d(Q), _as2d(dO)
    L = np.asarray(L, dtype=_F)
    z = np.asarray(z, dtype=_F)
    f = phi(Q, phi_kind)
    num = rope_rotate(f, cos, sin) @ L
    den = z_scale * (f @ z) + eps
    g = dO if W is None else dO @ np.asarray(W, dtype=_F).T
    dnum = g / den[:, None]
    dden = -(g * num).sum(axis=1) / den ** 2
    back = rope_rotate(dnum @ L.T, cos, None if sin is None else -np.asarray(sin, dtype=_F))
    df = back + z_scale * dden[:, None] * z[None, :]
    return df * phi_prime(Q, phi_kind)


def hybrid_attention_bwd(Q, K_win, V_win, state, b_q: int, b_kv: int, block_idx, dO,
                         phi_kind: int = PHI_RELU, cos_q=None, sin_q=None, eps: float = 1e-6,
                         z_scale: float = 1.0, scale=None, W=None, Q_hist=None):
    """Gradients of O = O_local + O_history (Eq. 6) for a fixed mask and a constant state.

    Returns ``(dQ_local, dQ_hist, dK, dV)``: when one tensor feeds both branches its gradient is
    ``dQ_local + dQ_hist``; with split queries the two belong to the two tensors.
    """
    dQ, dK, dV = sparse_attention_bwd(Q, K_win, V_win, block_idx, b_q, b_kv, dO, scale)
    if state is None:
        dQh = np.zeros_like(dQ)
    else:
        dQh = history_readout_bwd(Q if Q_hist is None else Q_hist, state[0], state[1], dO, phi_kind,
                                  cos_q, sin_q, eps, z_scale, W)
    return dQ, dQh, dK, dV
