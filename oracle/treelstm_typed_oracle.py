"""State oracle of the generic batcher: several cells in one forest (TEST INFRASTRUCTURE ONLY,
see oracle/__init__.py).

The paper's table batches nodes that agree in depth and in operator type, settings and input
layouts (section 4.2); a signature per node stands for the latter.  Each signature names one
Child-Sum Tree-LSTM cell (one weight set); the equations are those of treelstm_oracle.forward.
"""
from __future__ import annotations

import numpy as np

from .treelstm_oracle import _sigmoid, postorder


def forward_typed(parent, sig, x, W, U, b):
    """Several cells in one forest: node j is evaluated by the cell its signature names,
    W[sig[j]], U[sig[j]], b[sig[j]] (W [T, 4H, D], U [T, 4H, H], b [T, 4H]) - including the
    forget gates it applies to its children.  Same equations and order as `forward`."""
    x = np.asarray(x, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    sig = np.asarray(sig)
    n = x.shape[0]
    H = U.shape[2]
    h = np.zeros((n, H))
    c = np.zeros((n, H))
    order, ch = postorder(parent)
    for j in order:
        Wj, Uj, bj = W[sig[j]], U[sig[j]], b[sig[j]]
        hs = np.zeros(H)
        for k in ch[j]:
            hs = hs + h[k]
        pre = Wj @ x[j] + bj                      # all four gates, rows i | o | u | f
        iou = pre[:3 * H] + Uj[:3 * H] @ hs
        i = _sigmoid(iou[:H])
        o = _sigmoid(iou[H:2 * H])
        u = np.tanh(iou[2 * H:])
        cj = i * u
        for k in ch[j]:
            f = _sigmoid(pre[3 * H:] + Uj[3 * H:] @ h[k])
            cj = cj + f * c[k]
        c[j] = cj
        h[j] = o * np.tanh(cj)
    return h, c
