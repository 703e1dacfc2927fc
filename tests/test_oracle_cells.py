"""Pins of the oracle for tables with cells of different type (oracle/treelstm_cells_oracle.py)."""
import numpy as np
import pytest

from oracle import treelstm_oracle as T
from oracle import treelstm_typed_oracle as TT
from oracle import treelstm_cells_oracle as C
from workloads import make_forest, make_values, make_values_typed, tree_signatures, chain_forest


def _binary_forest(seed, n_trees=6, max_nodes=15):
    """Trees in which no node has more than two children (ids arbitrary inside a tree)."""
    rng = np.random.default_rng(seed)
    parts, off = [], 0
    for _ in range(n_trees):
        n = int(rng.integers(1, max_nodes + 1))
        par = np.full(n, -1, dtype=np.int64)
        deg = np.zeros(n, dtype=np.int64)
        for v in range(1, n):
            cand = np.flatnonzero(deg[:v] < 2)
            p = int(rng.choice(cand))
            par[v] = p; deg[p] += 1
        parts.append(np.where(par < 0, -1, par + off)); off += n
    return np.concatenate(parts).astype(np.int32)


def _tied_nary(N, W, U, b):
    """The n-ary cell that a child-sum cell (W, U, b) is a special case of: every position's i, o, u
    weights equal U_iou, and forget gate l sees only the child in position l, through U_f."""
    H = U.shape[1]
    Wn = np.concatenate([W[:3 * H]] + [W[3 * H:]] * N)
    bn = np.concatenate([b[:3 * H]] + [b[3 * H:]] * N)
    Un = np.zeros(((3 + N) * H, N * H))
    for l in range(N):
        Un[:3 * H, l * H:(l + 1) * H] = U[:3 * H]
        Un[(3 + l) * H:(4 + l) * H, l * H:(l + 1) * H] = U[3 * H:]
    return C.nary_cell(N, Wn, Un, bn)


def test_childsum_cells_reproduce_the_typed_oracle():
    p = make_forest(2)[:300]
    p = np.where(p >= 300, -1, p).astype(np.int32)
    x, W, U, b = make_values_typed(2, p.shape[0], 2, D=9, H=5)
    sig = tree_signatures(p, 2, 3)
    h0, c0 = TT.forward_typed(p, sig, x, W, U, b)
    h1, c1 = C.forward_cells(p, sig, x, [C.childsum_cell(W[t], U[t], b[t]) for t in range(2)])
    assert np.array_equal(h0, h1) and np.array_equal(c0, c1)


@pytest.mark.parametrize("N", [2, 3])
def test_nary_with_tied_weights_is_the_childsum_cell(N):
    """Position weights all equal and forget gates that see only their own child: the pinned
    child-sum oracle, on forests whose nodes have at most N children."""
    p = _binary_forest(5)
    x, W, U, b = make_values(1, p.shape[0], "random", D=7, H=4)
    h0, c0 = T.forward(p, x, W, U, b)
    h1, c1 = C.forward_cells(p, np.zeros(p.shape[0], np.int32), x, [_tied_nary(N, W.astype(np.float64), U.astype(np.float64), b.astype(np.float64))])
    assert np.abs(h0 - h1).max() <= 1e-13 and np.abs(c0 - c1).max() <= 1e-13


def test_unary_cell_on_chains_is_the_library_lstm():
    """N = 1: one child position, i.e. the LSTM recurrence with recurrent weights U (4 gates i, o, u, f_1)."""
    import torch
    D, H, n = 5, 4, 9
    rng = np.random.default_rng(3)
    W = rng.standard_normal((4 * H, D)); U = rng.standard_normal((4 * H, H)) * 0.5; b = rng.standard_normal(4 * H)
    x = rng.standard_normal((n, D))
    p = chain_forest(n)                                   # node i's parent is i - 1: the leaf is the last node
    h, c = C.forward_cells(p, np.zeros(n, np.int32), x, [C.nary_cell(1, W, U, b)])

    def rows(M):                                           # (i, o, u, f) -> torch's (i, f, g, o)
        i, o, u, f = (M[g * H:(g + 1) * H] for g in range(4))
        return torch.from_numpy(np.concatenate([i, f, u, o]))
    lstm = torch.nn.LSTM(D, H).double()
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(rows(W)); lstm.weight_hh_l0.copy_(rows(U))
        lstm.bias_ih_l0.copy_(rows(b.reshape(-1, 1)).reshape(-1)); lstm.bias_hh_l0.zero_()
        out, (hn, cn) = lstm(torch.from_numpy(x[::-1].copy()).unsqueeze(1))
    assert np.abs(out[:, 0, :].numpy()[::-1] - h).max() <= 1e-12
    assert np.abs(cn[0, 0].numpy() - c[0]).max() <= 1e-12


def test_positions_have_their_own_weights_closed_form():
    """A root with two leaves, H = D = 1, written out: swapping which leaf is first changes the result
    exactly as the position weights say."""
    sg = lambda z: 1.0 / (1.0 + np.exp(-z))
    W = np.array([[0.3], [-0.2], [0.5], [0.1], [-0.4]])          # i, o, u, f_1, f_2
    U = np.array([[0.7, -0.3], [0.2, 0.9], [-0.6, 0.4], [1.1, -0.8], [0.25, 0.65]])
    b = np.array([0.05, -0.1, 0.2, 0.3, -0.15])
    x = np.array([[0.5], [-1.0], [2.0]])
    p = np.array([-1, 0, 0], dtype=np.int32)
    cell = C.nary_cell(2, W, U, b)
    h, c = C.forward_cells(p, np.zeros(3, np.int32), x, [cell])

    def leaf(xv):
        z = W[:, 0] * xv + b
        cc = sg(z[0]) * np.tanh(z[2])
        return sg(z[1]) * np.tanh(cc), cc
    (h1, c1), (h2, c2) = leaf(-1.0), leaf(2.0)
    z = W[:, 0] * 0.5 + U[:, 0] * h1 + U[:, 1] * h2 + b
    c0 = sg(z[0]) * np.tanh(z[2]) + sg(z[3]) * c1 + sg(z[4]) * c2
    h0 = sg(z[1]) * np.tanh(c0)
    assert np.allclose(h[:, 0], [h0, h1, h2], atol=1e-14) and np.allclose(c[:, 0], [c0, c1, c2], atol=1e-14)
    # the leaves' values exchanged: positions matter
    h_sw, c_sw = C.forward_cells(p, np.zeros(3, np.int32), x[[0, 2, 1]], [cell])
    z = W[:, 0] * 0.5 + U[:, 0] * h2 + U[:, 1] * h1 + b
    c0s = sg(z[0]) * np.tanh(z[2]) + sg(z[3]) * c2 + sg(z[4]) * c1
    assert abs(c_sw[0, 0] - c0s) <= 1e-14 and abs(c_sw[0, 0] - c0) > 1e-3
    # a missing second child contributes nothing (zero block, no forget term)
    h1c, c1c = C.forward_cells(np.array([-1, 0], dtype=np.int32), np.zeros(2, np.int32), x[:2], [cell])
    z = W[:, 0] * 0.5 + U[:, 0] * h1 + b
    assert abs(c1c[0, 0] - (sg(z[0]) * np.tanh(z[2]) + sg(z[3]) * c1)) <= 1e-14


def test_mixed_table_each_node_under_its_own_cell_type():
    """Leaves under a child-sum "word" cell, inner nodes under a binary cell: every node equals what
    its own cell computes from its children's states (checked node by node against the two single-cell
    formulas), and too many children under an n-ary cell are refused."""
    p = _binary_forest(11, n_trees=5)
    n = p.shape[0]
    D, H = 6, 3
    rng = np.random.default_rng(8)
    x = rng.standard_normal((n, D))
    cs = C.childsum_cell(rng.standard_normal((4 * H, D)) * 0.4, rng.standard_normal((4 * H, H)) * 0.4, rng.standard_normal(4 * H) * 0.3)
    na = C.nary_cell(2, rng.standard_normal((5 * H, D)) * 0.4, rng.standard_normal((5 * H, 2 * H)) * 0.4, rng.standard_normal(5 * H) * 0.3)
    has_child = np.zeros(n, bool); has_child[p[p >= 0]] = True
    sig = has_child.astype(np.int32)                       # 0: leaves (child-sum), 1: inner nodes (binary)
    h, c = C.forward_cells(p, sig, x, [cs, na])
    sg = lambda z: 1.0 / (1.0 + np.exp(-z))
    for j in range(n):
        kids = [k for k in range(n) if p[k] == j]
        if not kids:
            z = cs["W"] @ x[j] + cs["b"]
            cj = sg(z[:H]) * np.tanh(z[2 * H:3 * H]); hj = sg(z[H:2 * H]) * np.tanh(cj)
        else:
            hc = np.zeros(2 * H)
            for l, k in enumerate(kids): hc[l * H:(l + 1) * H] = h[k]
            z = na["W"] @ x[j] + na["U"] @ hc + na["b"]
            cj = sg(z[:H]) * np.tanh(z[2 * H:3 * H]) + sum(sg(z[(3 + l) * H:(4 + l) * H]) * c[k] for l, k in enumerate(kids))
            hj = sg(z[H:2 * H]) * np.tanh(cj)
        assert np.allclose(h[j], hj, atol=1e-13) and np.allclose(c[j], cj, atol=1e-13)
    star = np.array([-1, 0, 0, 0], dtype=np.int32)
    with pytest.raises(C.CellError):
        C.forward_cells(star, np.ones(4, np.int32), x[:4], [cs, na])
