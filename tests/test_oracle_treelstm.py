"""Pins for the state oracle (numpy and C versions).

None of these retypes the oracle's formula for a general node; each reduces
the recursion to something fixed elsewhere: a library LSTM, a library LSTM
cell, a selection rule under saturated gates, a counting closed form, or an
invariance of the definition.
"""
import math

import numpy as np
import pytest
import torch

from oracle import treelstm_oracle as T
from oracle import schedule_oracle as S
from workloads import (chain_forest, star_forest, make_workload, make_forest, make_values,
                       relabel, tree_ranges, perfect_kary_tree)


def _both(c_oracle):
    return [("numpy", lambda *a: T.forward(*a)), ("c", lambda *a: c_oracle(*a)[:2])]


def _rand(rng, n, D, H, scale=1.0):
    x = rng.standard_normal((n, D))
    W = rng.uniform(-1, 1, (4 * H, D)) * scale / math.sqrt(D)
    U = rng.uniform(-1, 1, (4 * H, H)) * scale / math.sqrt(H)
    b = rng.uniform(-0.5, 0.5, 4 * H)
    return x, W, U, b


def _torch_gate_rows(M, H):
    """our gate order (i, o, u, f) -> torch's documented (i, f, g, o)."""
    i, o, u, f = (M[g * H:(g + 1) * H] for g in range(4))
    return torch.from_numpy(np.concatenate([i, f, u, o], axis=0))


def pin_leaf(fwd, name="oracle"):
    rng = np.random.default_rng(0)
    D, H = 7, 5
    x, W, U, b = _rand(rng, 3, D, H)
    p = np.array([-1, -1, -1], dtype=np.int32)
    sg = lambda z: 1.0 / (1.0 + np.exp(-z))
    h, c = fwd(p, x, W, U, b)
    for j in range(3):
        pre = W @ x[j] + b
        cc = sg(pre[:H]) * np.tanh(pre[2 * H:3 * H])
        hh = sg(pre[H:2 * H]) * np.tanh(cc)
        assert np.allclose(c[j], cc, atol=1e-14), name
        assert np.allclose(h[j], hh, atol=1e-14), name


def test_leaf_closed_form(c_oracle):
    for name, fwd in _both(c_oracle):
        pin_leaf(fwd, name)


def pin_chain(fwd, name="oracle"):
    """A chain is an LSTM over the sequence from the deepest node up to the root."""
    rng = np.random.default_rng(1)
    n, D, H = 9, 6, 4
    x, W, U, b = _rand(rng, n, D, H, scale=2.0)
    p = chain_forest(n)                       # node n-1 is the leaf = first time step
    lstm = torch.nn.LSTM(D, H, batch_first=False).double()
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(_torch_gate_rows(W, H))
        lstm.weight_hh_l0.copy_(_torch_gate_rows(U, H))
        lstm.bias_ih_l0.copy_(_torch_gate_rows(b.reshape(-1, 1), H).reshape(-1))
        lstm.bias_hh_l0.zero_()
        seq = torch.from_numpy(x[::-1].copy()).unsqueeze(1)
        out, (hn, cn) = lstm(seq)
    ref_h = out[:, 0, :].numpy()[::-1]
    h, c = fwd(p, x, W, U, b)
    assert np.allclose(h, ref_h, atol=1e-13), name
    assert np.allclose(c[0], cn[0, 0].numpy(), atol=1e-13), name


def test_chain_equals_library_lstm(c_oracle):
    for name, fwd in _both(c_oracle):
        pin_chain(fwd, name)


def pin_star_cell(fwd, name="oracle"):
    """With U_f = 0 the forget gate is the same for every child, so the parent
    is one LSTM-cell step from (sum of child h, sum of child c)."""
    rng = np.random.default_rng(2)
    m, D, H = 5, 6, 4
    x, W, U, b = _rand(rng, m + 1, D, H, scale=2.0)
    U[3 * H:] = 0.0
    p = star_forest(m + 1)
    cell = torch.nn.LSTMCell(D, H).double()
    with torch.no_grad():
        cell.weight_ih.copy_(_torch_gate_rows(W, H))
        cell.weight_hh.copy_(_torch_gate_rows(U, H))
        cell.bias_ih.copy_(_torch_gate_rows(b.reshape(-1, 1), H).reshape(-1))
        cell.bias_hh.zero_()
    h, c = fwd(p, x, W, U, b)
    with torch.no_grad():
        h0 = torch.from_numpy(h[1:].sum(0, keepdims=True))
        c0 = torch.from_numpy(c[1:].sum(0, keepdims=True))
        h1, c1 = cell(torch.from_numpy(x[:1]), (h0, c0))
    assert np.allclose(h[0], h1[0].numpy(), atol=1e-13), name
    assert np.allclose(c[0], c1[0].numpy(), atol=1e-13), name


def test_star_with_zero_Uf_equals_library_cell_on_summed_children(c_oracle):
    for name, fwd in _both(c_oracle):
        pin_star_cell(fwd, name)


def pin_forget_own_h(fwd, name="oracle"):
    """U_f = 1000 I, W_f = 0, b_f = 0, U_iou = 0: every forget gate saturates to
    exactly 0 or 1 by the sign of that child's own h, so the parent's c is its
    leaf-like term plus the c of the children whose h is positive.  Using the
    summed h instead would keep or drop all children together."""
    rng = np.random.default_rng(3)
    m, D, H = 3, 5, 32
    x, W, U, b = _rand(rng, m + 1, D, H, scale=3.0)
    U[:] = 0.0
    U[3 * H:] = 1000.0 * np.eye(H)
    W[3 * H:] = 0.0
    b[3 * H:] = 0.0
    p = star_forest(m + 1)
    h, c = fwd(p, x, W, U, b)
    hl, cl = fwd(np.array([-1], dtype=np.int32), x[:1], W, U, b)   # root as if it were a leaf
    hk, ck = h[1:], c[1:]
    sat = np.abs(hk) > 0.04                       # |1000 h| > 40: sigmoid is exactly 0 or 1
    ok = sat.all(axis=0)                          # hidden units where every child saturates
    mixed = ok & (hk > 0).any(0) & (hk < 0).any(0)
    assert ok.sum() >= 4 and mixed.any()
    expect = cl[0] + np.where(hk > 0, ck, 0.0).sum(0)
    assert np.allclose(c[0][ok], expect[ok], atol=1e-12), name
    wrong = cl[0] + np.where(hk.sum(0) > 0, 1.0, 0.0) * ck.sum(0)
    assert not np.allclose(c[0][mixed], wrong[mixed], atol=1e-3), name


def test_forget_gate_reads_each_childs_own_h(c_oracle):
    for name, fwd in _both(c_oracle):
        pin_forget_own_h(fwd, name)


def pin_zero_weights(fwd, name="oracle", shape="cfg1"):
    """W = U = 0: gates are constants.  With b_f = 40 the forget gate is exactly
    1.0 in fp64, so c_j = sigmoid(b_i) tanh(b_u) * (size of j's subtree); with a
    general b_f, c_j = s * sum_d n_d(j) sigmoid(b_f)^d over descendant depths."""
    p = {"cfg1": make_forest(1), "kary": perfect_kary_tree(3, 3), "star": star_forest(70)}[shape]
    n, D, H = p.shape[0], 3, 2
    x = np.random.default_rng(4).standard_normal((n, D))
    W = np.zeros((4 * H, D)); U = np.zeros((4 * H, H))
    bi, bo, bu = 0.3, -0.2, 0.7
    sg = lambda z: 1.0 / (1.0 + math.exp(-z))
    s = sg(bi) * math.tanh(bu)
    size = np.ones(n)
    for v in S.schedule_fast(p)["perm"]:          # leaves first
        if p[v] >= 0:
            size[p[v]] += size[v]
    b = np.concatenate([np.full(H, bi), np.full(H, bo), np.full(H, bu), np.full(H, 40.0)])
    h, c = fwd(p, x, W, U, b)
    assert np.allclose(c[:, 0], s * size, rtol=1e-13), name
    assert np.allclose(h[:, 1], sg(bo) * np.tanh(s * size), rtol=1e-13), name
    # general forget bias: polynomial in sigmoid(b_f) over descendant depths
    bf = 0.4
    b2 = np.concatenate([np.full(H, bi), np.full(H, bo), np.full(H, bu), np.full(H, bf)])
    h2, c2 = fwd(p, x, W, U, b2)
    poly = np.zeros(n)
    for v in range(n):
        w, d = v, 0
        while w != -1:
            poly[w] += sg(bf) ** d
            w, d = int(p[w]), d + 1
    assert np.allclose(c2[:, 0], s * poly, rtol=1e-12), name
    b0 = np.zeros(4 * H)
    h0, c0 = fwd(p, x, W, U, b0)
    assert not h0.any() and not c0.any()


@pytest.mark.parametrize("shape", ["cfg1", "kary", "star"])
def test_zero_weights_closed_form_counts_subtrees(c_oracle, shape):
    for name, fwd in _both(c_oracle):
        pin_zero_weights(fwd, name, shape)


def test_relabelling_leaves_states_unchanged(c_oracle):
    cfg, p, x, W, U, b = make_workload(1, bias="random")
    q, new_of_old = relabel(p, 5)
    xq = np.empty_like(x); xq[new_of_old] = x
    for name, fwd in _both(c_oracle):
        h, c = fwd(p, x, W, U, b)
        hq, cq = fwd(q, xq, W, U, b)
        assert np.abs(hq[new_of_old] - h).max() < 1e-12, name
        assert np.abs(cq[new_of_old] - c).max() < 1e-12, name


def test_forest_equals_trees_one_at_a_time(c_oracle):
    cfg, p, x, W, U, b = make_workload(1, bias="random")
    r = tree_ranges(p)
    for name, fwd in _both(c_oracle):
        h, c = fwd(p, x, W, U, b)
        for t in range(len(r) - 1):
            lo, hi = r[t], r[t + 1]
            pt = np.where(p[lo:hi] < 0, -1, p[lo:hi] - lo).astype(np.int32)
            ht, ct = fwd(pt, x[lo:hi], W, U, b)
            assert np.array_equal(ht, h[lo:hi]) and np.array_equal(ct, c[lo:hi]), name


def test_sibling_order_does_not_matter():
    rng = np.random.default_rng(6)
    m, D, H = 7, 5, 4
    x, W, U, b = _rand(rng, m + 1, D, H)
    p = star_forest(m + 1)
    h, c = T.forward(p, x, W, U, b)
    order = np.concatenate(([0], 1 + rng.permutation(m)))
    h2, c2 = T.forward(p, x[order], W, U, b)
    assert np.abs(h2[0] - h[0]).max() < 1e-13 and np.abs(c2[0] - c[0]).max() < 1e-13


@pytest.mark.parametrize("cfg", [1, 2])
def test_numpy_and_c_oracles_agree(c_oracle, cfg):
    cfgo, p, x, W, U, b = make_workload(cfg, bias="random")
    h, c = T.forward(p, x, W, U, b)
    h2, c2, _ = c_oracle(p, x, W, U, b)
    assert np.abs(h - h2).max() < 1e-12 and np.abs(c - c2).max() < 1e-12
    q, new_of_old = relabel(p, 9)                # arbitrary ids through the C postorder
    xq = np.empty_like(x); xq[new_of_old] = x
    h3, c3, _ = c_oracle(q, xq, W, U, b)
    assert np.abs(h3[new_of_old] - h).max() < 1e-12


def test_c_oracle_rejects_non_forests(c_oracle):
    x, W, U, b = make_values(1, 3, D=4, H=2)
    for bad in ([1, 0, -1], [-1, 5, 0], [0, -1, 1]):
        with pytest.raises(ValueError):
            c_oracle(np.array(bad, dtype=np.int32), x, W, U, b)


ALL_PINS = [pin_leaf, pin_chain, pin_star_cell, pin_forget_own_h,
            lambda fwd, name="oracle": pin_zero_weights(fwd, name, "cfg1")]
