"""Pins of the typed (depth x signature) oracles."""
import numpy as np
import pytest

from oracle import schedule_oracle as S
from oracle import treelstm_oracle as T
from oracle import treelstm_typed_oracle as TT
from workloads import (make_forest, make_values, make_values_typed, tree_signatures, node_signatures, mixed_forest,
                       tree_ranges, relabel, chain_forest)


def _sub_forest(parent, keep):
    """Nodes with keep[v], relabelled in ascending id order; parents follow."""
    ids = np.flatnonzero(keep)
    new = -np.ones(parent.shape[0], dtype=np.int64)
    new[ids] = np.arange(ids.shape[0])
    p = parent[ids].astype(np.int64)
    return np.where(p < 0, -1, new[np.maximum(p, 0)]).astype(np.int32), ids


def test_one_signature_is_the_plain_schedule():
    p = make_forest(2)
    a = S.schedule(p)
    b = S.schedule_typed(p, np.zeros(p.shape[0], np.int32), 1)
    for k in ("height", "level_ptr", "perm", "inv_perm", "child_ptr", "child_idx"):
        assert np.array_equal(a[k], b[k]), k
    assert np.array_equal(b["slot_ptr"], a["level_ptr"]) and np.array_equal(b["key"], a["height"])


def test_sub_slots_hold_exactly_their_nodes_in_id_order_with_signatures_per_node():
    p = make_forest(2)
    n_sig = 3
    sig = node_signatures(p, n_sig, 4)
    psig = S.parent_signatures(p, sig)
    assert (psig[p < 0] == sig[p < 0]).all() and (psig[p >= 0] == sig[p[p >= 0]]).all()
    s = S.schedule_typed(p, sig, n_sig)
    h = s["height"]
    seen = 0
    for l in range(s["n_levels"]):
        assert s["slot_ptr"][l * n_sig * n_sig] == s["level_ptr"][l]
        for t in range(n_sig):
            for q in range(n_sig):
                i = (l * n_sig + t) * n_sig + q
                a, b = s["slot_ptr"][i], s["slot_ptr"][i + 1]
                want = [v for v in range(p.shape[0]) if h[v] == l and sig[v] == t and psig[v] == q]   # brute force
                assert list(s["perm"][a:b]) == want
                seen += b - a
    assert seen == p.shape[0]
    f = S.schedule_typed_fast(p, sig, n_sig)
    for k in ("perm", "inv_perm", "key", "slot_ptr", "level_ptr"):
        assert np.array_equal(s[k], f[k]), k


@pytest.mark.parametrize("n_sig", [2, 3])
def test_slots_hold_exactly_their_nodes_in_id_order(n_sig):
    p = make_forest(2)
    sig = tree_signatures(p, n_sig, 11)
    s = S.schedule_typed(p, sig, n_sig)
    h = s["height"]
    L = s["n_levels"]
    assert s["slot_ptr"][0] == 0 and s["slot_ptr"][-1] == p.shape[0]
    for l in range(L):
        assert s["slot_ptr"][l * n_sig * n_sig] == s["level_ptr"][l]
        for t in range(n_sig):        # the cell's batch (l, t): the run of its sub-slots
            a, b = s["slot_ptr"][(l * n_sig + t) * n_sig], s["slot_ptr"][(l * n_sig + t + 1) * n_sig]
            want = [v for v in range(p.shape[0]) if h[v] == l and sig[v] == t]     # brute force
            assert list(s["perm"][a:b]) == want
    assert np.array_equal(s["inv_perm"][s["perm"]], np.arange(p.shape[0]))


def test_restricted_to_one_signature_it_is_that_sub_forests_schedule():
    p, _ = relabel(make_forest(2), 4)
    sig = np.zeros(p.shape[0], np.int32)
    # signatures per tree of the relabelled forest: propagate from the roots down
    s_plain = S.schedule(p)
    rng = np.random.default_rng(2)
    for pos in range(p.shape[0] - 1, -1, -1):                 # parents sit in higher levels: visit them first
        v = s_plain["perm"][pos]
        sig[v] = rng.integers(0, 2) if p[v] < 0 else sig[p[v]]
    s = S.schedule_typed(p, sig, 2)
    for t in range(2):
        sub, ids = _sub_forest(p, sig == t)
        ss = S.schedule(sub)
        order_t = [v for v in s["perm"] if sig[v] == t]       # relative order of the signature's nodes
        assert order_t == list(ids[ss["perm"]])


def test_fast_version_matches():
    p, sig = mixed_forest(2, 40, 30, 3, 40, 5)
    a, b = S.schedule_typed(p, sig, 2), S.schedule_typed_fast(p, sig, 2)
    for k in ("height", "level_ptr", "perm", "inv_perm", "child_ptr", "child_idx", "key", "slot_ptr"):
        assert np.array_equal(a[k], b[k]), k
    with pytest.raises(S.ForestError):
        S.schedule_typed(p, sig + 1, 2)
    with pytest.raises(S.ForestError):
        S.schedule_typed_fast(p, sig - 1, 2)


def test_forward_typed_with_one_cell_is_forward():
    p = make_forest(1)
    x, W, U, b = make_values(1, p.shape[0], "random", D=12, H=7)
    h0, c0 = T.forward(p, x, W, U, b)
    h1, c1 = TT.forward_typed(p, np.zeros(p.shape[0], np.int32), x, W[None], U[None], b[None])
    assert np.allclose(h0, h1, atol=1e-14) and np.allclose(c0, c1, atol=1e-14)
    # two signatures naming equal weights change nothing
    sig = tree_signatures(p, 2, 0)
    h2, c2 = TT.forward_typed(p, sig, x, np.stack([W, W]), np.stack([U, U]), np.stack([b, b]))
    assert np.allclose(h0, h2, atol=1e-14) and np.allclose(c0, c2, atol=1e-14)


def test_forward_typed_is_each_network_on_its_own_trees():
    p, sig = mixed_forest(1, 6, 5, 2, 9, 3)
    n = p.shape[0]
    x, W, U, b = make_values_typed(1, n, 2, D=10, H=6)
    h, c = TT.forward_typed(p, sig, x, W, U, b)
    for t in range(2):
        sub, ids = _sub_forest(p, sig == t)
        ht, ct = T.forward(sub, x[ids], W[t], U[t], b[t])
        assert np.allclose(h[ids], ht, atol=1e-14) and np.allclose(c[ids], ct, atol=1e-14)
    # and the weights matter: swapping the two networks changes the states
    h_sw, _ = TT.forward_typed(p, 1 - sig, x, W, U, b)
    assert np.abs(h_sw - h).max() > 1e-3


def test_forward_typed_parent_cell_owns_the_forget_gate():
    """A two-node chain whose parent and child carry different signatures: the forget gate on the
    child uses the parent's W_f, U_f, b_f (closed form written out here)."""
    p = np.array([-1, 0], dtype=np.int32)
    sig = np.array([1, 0], dtype=np.int32)
    rng = np.random.default_rng(0)
    D, H = 3, 2
    x = rng.standard_normal((2, D)); W = rng.standard_normal((2, 4 * H, D))
    U = rng.standard_normal((2, 4 * H, H)); b = rng.standard_normal((2, 4 * H))
    sg = lambda z: 1 / (1 + np.exp(-z))
    z1 = W[0] @ x[1] + b[0]                                   # leaf, cell 0
    c1 = sg(z1[:H]) * np.tanh(z1[2 * H:3 * H]); h1 = sg(z1[H:2 * H]) * np.tanh(c1)
    z0 = W[1] @ x[0] + b[1]                                   # root, cell 1
    i = sg(z0[:H] + U[1][:H] @ h1); o = sg(z0[H:2 * H] + U[1][H:2 * H] @ h1)
    u = np.tanh(z0[2 * H:3 * H] + U[1][2 * H:3 * H] @ h1); f = sg(z0[3 * H:] + U[1][3 * H:] @ h1)
    c0 = i * u + f * c1; h0 = o * np.tanh(c0)
    h, c = TT.forward_typed(p, sig, x, W, U, b)
    assert np.allclose(h, [h0, h1], atol=1e-13) and np.allclose(c, [c0, c1], atol=1e-13)
