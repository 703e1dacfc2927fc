"""State oracle of a table that holds cells of different TYPE (TEST INFRASTRUCTURE ONLY, see
oracle/__init__.py).

The paper's look-up key is (depth, operator type, settings, input layouts, result index), sections
4.2 and 4.3: nodes of different operator type never share a slot.  Here a signature names a cell,
and a cell is one of two operator types with its own weights:

  child-sum   the cell of treelstm_oracle.forward (any number of children, their h summed)

  n-ary       the N-ary Tree-LSTM of the model the paper cites, for nodes with at most N ordered
              children k_1..k_m (m <= N, here: ascending node id = position 1, 2, ...); every
              child POSITION has weights of its own, and every forget gate sees all children:

                  hc   = [h_{k_1} ; ... ; h_{k_m} ; 0 ...]           (N blocks of H)
                  i    = sigmoid(W_i x + U_i hc + b_i)     o = sigmoid(W_o x + U_o hc + b_o)
                  u    = tanh   (W_u x + U_u hc + b_u)
                  f_l  = sigmoid(W_{f_l} x + U_{f_l} hc + b_{f_l})   one per position l = 1..N
                  c    = i * u + sum_{l <= m} f_l * c_{k_l}          h = o * tanh(c)

              W [(3+N)H, D], U [(3+N)H, N*H], b [(3+N)H], gate rows i, o, u, f_1, ..., f_N; column
              block l of U multiplies the h of the child in position l.

A node with more children than its cell has positions is an error.  fp64, no intermediate rounding.
"""
from __future__ import annotations

import numpy as np

from .treelstm_oracle import _sigmoid, postorder


class CellError(ValueError):
    pass


def childsum_cell(W, U, b):
    return dict(kind="childsum", W=np.asarray(W, np.float64), U=np.asarray(U, np.float64), b=np.asarray(b, np.float64))


def nary_cell(N, W, U, b):
    W = np.asarray(W, np.float64); U = np.asarray(U, np.float64); b = np.asarray(b, np.float64)
    H = U.shape[1] // N
    if U.shape != ((3 + N) * H, N * H) or W.shape[0] != (3 + N) * H or b.shape != ((3 + N) * H,):
        raise CellError("n-ary cell: W [(3+N)H, D], U [(3+N)H, N*H], b [(3+N)H]")
    return dict(kind="nary", N=int(N), W=W, U=U, b=b)


def forward_cells(parent, sig, x, cells):
    """h, c [n, H] of a forest whose node j is evaluated by cells[sig[j]]."""
    x = np.asarray(x, dtype=np.float64)
    sig = np.asarray(sig)
    n = x.shape[0]
    c0 = cells[0]
    H = c0["U"].shape[1] if c0["kind"] == "childsum" else c0["U"].shape[1] // c0["N"]
    h = np.zeros((n, H))
    c = np.zeros((n, H))
    order, ch = postorder(parent)
    for j in order:
        cell = cells[int(sig[j])]
        W, U, b = cell["W"], cell["U"], cell["b"]
        kids = ch[j]                                  # ascending id
        if cell["kind"] == "childsum":
            hs = np.zeros(H)
            for k in kids:
                hs = hs + h[k]
            pre = W @ x[j] + b
            i = _sigmoid(pre[:H] + U[:H] @ hs)
            o = _sigmoid(pre[H:2 * H] + U[H:2 * H] @ hs)
            u = np.tanh(pre[2 * H:3 * H] + U[2 * H:3 * H] @ hs)
            cj = i * u
            for k in kids:
                cj = cj + _sigmoid(pre[3 * H:] + U[3 * H:] @ h[k]) * c[k]
        else:
            N = cell["N"]
            if len(kids) > N:
                raise CellError(f"node {j} has {len(kids)} children, its cell {N} positions")
            hc = np.zeros(N * H)
            for l, k in enumerate(kids):
                hc[l * H:(l + 1) * H] = h[k]
            pre = W @ x[j] + U @ hc + b
            i = _sigmoid(pre[:H]); o = _sigmoid(pre[H:2 * H]); u = np.tanh(pre[2 * H:3 * H])
            cj = i * u
            for l, k in enumerate(kids):
                cj = cj + _sigmoid(pre[(3 + l) * H:(4 + l) * H]) * c[k]
        c[j] = cj
        h[j] = o * np.tanh(cj)
    return h, c
