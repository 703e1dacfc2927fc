"""State oracle: Child-Sum Tree-LSTM forward, one node at a time, in fp64.

The paper batches Tree-LSTM cells and requires the batched run to give the
same results as evaluating every sample's graph by itself (section 1, the
isomorphism condition; section 5 compares per-instance and batched runs).  It
cites the cell rather than printing it and describes it as 33 operators of
which 4 depend on the number of children (section 3).  The cell evaluated
here is the Child-Sum form of the cited model, for node j with children C(j):

    hs   = sum_{k in C(j)} h_k                       (zero vector for a leaf)
    i    = sigmoid(W_i x_j + U_i hs + b_i)
    o    = sigmoid(W_o x_j + U_o hs + b_o)
    u    = tanh   (W_u x_j + U_u hs + b_u)
    f_k  = sigmoid(W_f x_j + U_f h_k + b_f)          one per child, from h_k
    c_j  = i * u + sum_k f_k * c_k
    h_j  = o * tanh(c_j)

The four child-dependent operators are the sum of h_k, the per-child forget
gate, its product with c_k and the sum over children.  Rows of W [4H, D],
U [4H, H], b [4H] are grouped by gate in the order i, o, u, f.

Everything is fp64 with no intermediate rounding; inputs are whatever the
caller hands over (fp32 values, or bf16 values widened exactly).

Test infrastructure only; no code shared with the GPU path.
"""
from __future__ import annotations

import numpy as np


def _sigmoid(z: np.ndarray) -> np.ndarray:
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-z[pos]))
    e = np.exp(z[~pos])
    out[~pos] = e / (1.0 + e)
    return out


def postorder(parent) -> list:
    """Node ids ordered so that every child comes before its parent."""
    parent = np.asarray(parent)
    n = parent.shape[0]
    ch = [[] for _ in range(n)]
    roots = []
    for v in range(n):
        p = int(parent[v])
        if p >= 0:
            ch[p].append(v)
        else:
            roots.append(v)
    order = []
    for r in roots:
        stack = [(r, 0)]
        while stack:
            v, i = stack.pop()
            if i < len(ch[v]):
                stack.append((v, i + 1))
                stack.append((ch[v][i], 0))
            else:
                order.append(v)
    if len(order) != n:
        raise ValueError("parent array is not a forest")
    return order, ch


def forward(parent, x, W, U, b):
    """h [N, H], c [N, H] in fp64 for every node of the forest."""
    x = np.asarray(x, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    n = x.shape[0]
    H = U.shape[1]
    assert W.shape[0] == 4 * H and U.shape[0] == 4 * H and b.shape[0] == 4 * H
    Wi, Wo, Wu, Wf = (W[g * H:(g + 1) * H] for g in range(4))
    Ui, Uo, Uu, Uf = (U[g * H:(g + 1) * H] for g in range(4))
    bi, bo, bu, bf = (b[g * H:(g + 1) * H] for g in range(4))
    h = np.zeros((n, H))
    c = np.zeros((n, H))
    order, ch = postorder(parent)
    for j in order:
        hs = np.zeros(H)
        for k in ch[j]:
            hs = hs + h[k]
        i = _sigmoid(Wi @ x[j] + Ui @ hs + bi)
        o = _sigmoid(Wo @ x[j] + Uo @ hs + bo)
        u = np.tanh(Wu @ x[j] + Uu @ hs + bu)
        cj = i * u
        fx = Wf @ x[j] + bf
        for k in ch[j]:
            f = _sigmoid(fx + Uf @ h[k])
            cj = cj + f * c[k]
        c[j] = cj
        h[j] = o * np.tanh(cj)
    return h, c
