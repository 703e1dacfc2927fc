"""Gradient oracle: reverse-mode derivative of the Child-Sum Tree-LSTM forest, node by node, fp64.

The paper reports training throughput beside inference (section 5) and runs the backward
pass through the same batched graph; the batched run must again equal the per-sample one.
This module is the per-sample definition for that step: for the scalar

    L = sum_j <gh_j, h_j> + <gc_j, c_j>        (gh, gc: cotangents handed in for every node)

it returns dL/dx [N, D], dL/dW [4H, D], dL/dU [4H, H], dL/db [4H], obtained by applying the
chain rule to the cell equations of treelstm_oracle (same notation), parents before
children:

    dc_j   += dh_j * o * (1 - tanh(c_j)^2)
    dz_o    = dh_j * tanh(c_j) * o (1 - o)
    dz_i    = dc_j * u * i (1 - i)           dz_u = dc_j * i * (1 - u^2)
    dz_f,k  = dc_j * c_k * f_k (1 - f_k)     dc_k += dc_j * f_k               per child k
    dx_j    = W_i^T dz_i + W_o^T dz_o + W_u^T dz_u + W_f^T sum_k dz_f,k
    dhs     = U_i^T dz_i + U_o^T dz_o + U_u^T dz_u
    dh_k   += dhs + U_f^T dz_f,k                                               per child k
    dW_g   += dz_g (x) x_j,  dU_g += dz_g (x) hs,  db_g += dz_g               g in i, o, u
    dW_f   += (sum_k dz_f,k) (x) x_j,  dU_f += sum_k dz_f,k (x) h_k,  db_f += sum_k dz_f,k

Pinned in tests/test_oracle_backward.py.  Test infrastructure only; no code shared with the GPU path.
"""
from __future__ import annotations

import numpy as np

from .treelstm_oracle import _sigmoid, postorder


def _forward_saved(parent, x, W, U, b):
    n = x.shape[0]
    H = U.shape[1]
    Wg = [W[g * H:(g + 1) * H] for g in range(4)]
    Ug = [U[g * H:(g + 1) * H] for g in range(4)]
    bg = [b[g * H:(g + 1) * H] for g in range(4)]
    order, ch = postorder(parent)
    h = np.zeros((n, H)); c = np.zeros((n, H))
    gi = np.zeros((n, H)); go = np.zeros((n, H)); gu = np.zeros((n, H)); hs = np.zeros((n, H))
    f = np.zeros((n, H))          # row k: the forget gate the parent of k applies to k (roots: 0)
    for j in order:
        kids = ch[j]
        for k in kids:
            hs[j] += h[k]
        gi[j] = _sigmoid(Wg[0] @ x[j] + Ug[0] @ hs[j] + bg[0])
        go[j] = _sigmoid(Wg[1] @ x[j] + Ug[1] @ hs[j] + bg[1])
        gu[j] = np.tanh(Wg[2] @ x[j] + Ug[2] @ hs[j] + bg[2])
        c[j] = gi[j] * gu[j]
        fx = Wg[3] @ x[j] + bg[3]
        for k in kids:
            f[k] = _sigmoid(fx + Ug[3] @ h[k])
            c[j] += f[k] * c[k]
        h[j] = go[j] * np.tanh(c[j])
    return order, ch, Wg, Ug, h, c, gi, go, gu, hs, f


def forward_saved(parent, x, W, U, b):
    """(h, c, gates [N, 3H] = i | o | u after their non-linearities, fgate [N, H] with row k =
    the forget gate applied to child k by its parent): what a training forward keeps."""
    x, W, U, b = (np.asarray(a, dtype=np.float64) for a in (x, W, U, b))
    _, _, _, _, h, c, gi, go, gu, _, f = _forward_saved(parent, x, W, U, b)
    return h, c, np.concatenate([gi, go, gu], axis=1), f


def forward_backward(parent, x, W, U, b, gh, gc):
    """Returns (h, c, dx, dW, dU, db), all fp64."""
    x = np.asarray(x, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    gh = np.asarray(gh, dtype=np.float64)
    gc = np.asarray(gc, dtype=np.float64)
    n, D = x.shape
    H = U.shape[1]
    order, ch, Wg, Ug, h, c, gi, go, gu, hs, f = _forward_saved(parent, x, W, U, b)

    dh = gh.copy(); dc = gc.copy()
    dx = np.zeros((n, D)); dW = np.zeros_like(W); dU = np.zeros_like(U); db = np.zeros_like(b)
    for j in reversed(order):
        kids = ch[j]
        t = np.tanh(c[j])
        dcj = dc[j] + dh[j] * go[j] * (1.0 - t * t)
        dz = [dcj * gu[j] * gi[j] * (1.0 - gi[j]),
              dh[j] * t * go[j] * (1.0 - go[j]),
              dcj * gi[j] * (1.0 - gu[j] * gu[j])]
        dzf_sum = np.zeros(H)
        dhs = np.zeros(H)
        for g in range(3):
            dhs += Ug[g].T @ dz[g]
        for k in kids:
            dzf = dcj * c[k] * f[k] * (1.0 - f[k])
            dzf_sum += dzf
            dc[k] += dcj * f[k]
            dh[k] += dhs + Ug[3].T @ dzf
            dU[3 * H:4 * H] += np.outer(dzf, h[k])
        for g in range(3):
            dx[j] += Wg[g].T @ dz[g]
            dW[g * H:(g + 1) * H] += np.outer(dz[g], x[j])
            dU[g * H:(g + 1) * H] += np.outer(dz[g], hs[j])
            db[g * H:(g + 1) * H] += dz[g]
        dx[j] += Wg[3].T @ dzf_sum
        dW[3 * H:4 * H] += np.outer(dzf_sum, x[j])
        db[3 * H:4 * H] += dzf_sum
    return h, c, dx, dW, dU, db
