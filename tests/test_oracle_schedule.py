"""Pins for the schedule oracle: brute force, closed forms, invariants.

Each check is independent of the routine it pins: a second algorithm
(ancestor walks), shapes whose schedule is known in closed form, numpy's
stable argsort for the CSR, and structural invariants.
"""
import numpy as np
import pytest

from oracle import schedule_oracle as S
from workloads import (chain_forest, star_forest, perfect_kary_tree, make_forest, relabel)


def _random_forest(rng, n, n_roots):
    """Arbitrary ids: a random recursive forest, then scrambled."""
    p = np.full(n, -1, dtype=np.int32)
    for v in range(n_roots, n):
        p[v] = rng.integers(0, v)
    q, _ = relabel(p, int(rng.integers(1 << 30)))
    return q


@pytest.mark.parametrize("seed", range(20))
def test_heights_match_bruteforce_on_tiny_forests(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 40))
    p = _random_forest(rng, n, int(rng.integers(1, min(n, 4) + 1)))
    s = S.schedule(p)
    assert np.array_equal(s["height"], S.heights_bruteforce(p))
    f = S.schedule_fast(p)
    for k in s:
        assert np.array_equal(np.asarray(s[k]), np.asarray(f[k])), k


def test_chain_closed_form():
    n = 17
    s = S.schedule(chain_forest(n))
    assert s["n_levels"] == n
    assert s["height"].tolist() == list(range(n - 1, -1, -1))
    assert np.diff(s["level_ptr"]).tolist() == [1] * n
    assert s["perm"].tolist() == list(range(n - 1, -1, -1))
    assert s["child_ptr"].tolist() == list(range(n)) + [n - 1]
    assert s["child_idx"].tolist() == list(range(1, n))


def test_star_closed_form():
    n = 23
    s = S.schedule(star_forest(n))
    assert s["n_levels"] == 2
    assert np.diff(s["level_ptr"]).tolist() == [n - 1, 1]
    assert s["perm"].tolist() == list(range(1, n)) + [0]
    assert s["child_idx"].tolist() == list(range(1, n))
    assert s["child_ptr"].tolist() == [0] + [n - 1] * n


@pytest.mark.parametrize("k,d", [(2, 4), (3, 3), (5, 2)])
def test_perfect_kary_closed_form(k, d):
    s = S.schedule(perfect_kary_tree(k, d))
    assert s["n_levels"] == d + 1
    assert np.diff(s["level_ptr"]).tolist() == [k ** (d - l) for l in range(d + 1)]


def test_single_node_and_empty():
    s = S.schedule(np.array([-1], dtype=np.int32))
    assert s["n_levels"] == 1 and s["n_edges"] == 0 and s["level_ptr"].tolist() == [0, 1]
    e = S.schedule(np.zeros(0, dtype=np.int32))
    assert e["n_levels"] == 0 and e["n_edges"] == 0 and e["level_ptr"].tolist() == [0]
    f = S.schedule_fast(np.zeros(0, dtype=np.int32))
    assert f["n_levels"] == 0 and f["level_ptr"].tolist() == [0]


@pytest.mark.parametrize("cfg", [1, 2])
def test_invariants_and_library_csr(cfg):
    p = make_forest(cfg)
    p, _ = relabel(p, 11)
    n = p.shape[0]
    s = S.schedule(p)
    h, perm, inv, lp = s["height"], s["perm"], s["inv_perm"], s["level_ptr"]
    nonroot = np.flatnonzero(p >= 0)
    # every child is strictly lower than its parent, and some child is exactly one lower
    assert (h[p[nonroot]] > h[nonroot]).all()
    best = np.full(n, -1)
    np.maximum.at(best, p[nonroot], h[nonroot])
    internal = best >= 0
    assert np.array_equal(h[internal], best[internal] + 1)
    assert (h[~internal] == 0).all()
    # buckets
    assert lp[0] == 0 and lp[-1] == n and lp[1] == int((~internal).sum())
    assert sorted(perm.tolist()) == list(range(n))
    assert np.array_equal(inv[perm], np.arange(n))
    keys = list(zip(h[perm].tolist(), perm.tolist()))
    assert keys == sorted(keys)
    for lvl in range(s["n_levels"]):
        assert (h[perm[lp[lvl]:lp[lvl + 1]]] == lvl).all()
    # CSR == transpose of the parent relation, via numpy's stable argsort
    assert s["n_edges"] == n - int((p < 0).sum())
    assert np.array_equal(s["child_idx"], nonroot[np.argsort(p[nonroot], kind="stable")])
    assert np.array_equal(np.diff(s["child_ptr"]), np.bincount(p[nonroot], minlength=n))
    owner = np.repeat(np.arange(n), np.diff(s["child_ptr"]))
    assert np.array_equal(p[s["child_idx"]], owner)


def test_relabelling_permutes_the_schedule():
    p = make_forest(1)
    q, new_of_old = relabel(p, 3)
    a, b = S.schedule(p), S.schedule(q)
    assert np.array_equal(b["height"][new_of_old], a["height"])
    assert np.array_equal(a["level_ptr"], b["level_ptr"])


@pytest.mark.parametrize("bad,kind", [
    ([-1, 0, 5], "range"), ([-1, 1], "range"), ([-2, 0], "range"),
    ([1, 0], "cycle"), ([-1, 2, 3, 1], "cycle"), ([1, 2, 0, -1, 3], "cycle"),
])
def test_invalid_forests_are_rejected(bad, kind):
    p = np.array(bad, dtype=np.int32)
    with pytest.raises(S.ForestError) as e:
        S.schedule(p)
    assert e.value.kind == kind
    with pytest.raises(S.ForestError) as e2:
        S.schedule_fast(p)
    assert e2.value.kind == kind


def test_planted_mistake_is_caught():
    """A depth-from-root reading (the wrong one) fails the brute-force pin."""
    p = make_forest(1)
    depth = np.zeros(p.shape[0], dtype=np.int32)
    for v in range(p.shape[0]):
        w, d = int(p[v]), 0
        while w != -1:
            d += 1
            w = int(p[w])
        depth[v] = d
    assert not np.array_equal(depth, S.heights_bruteforce(p))


def test_concat_forests_keeps_each_forest_intact():
    """Appending is concatenation with shifted ids: heights and child lists of each part are
    unchanged, level sizes add up, and inside a level the old nodes come first."""
    a, b = make_forest(2), chain_forest(9, 2)
    j = S.concat_forests(a, b)
    assert j.dtype == np.int32 and len(j) == len(a) + len(b)
    sa, sb, sj = S.schedule(a), S.schedule(b), S.schedule(j)
    assert np.array_equal(sj["height"], np.concatenate([sa["height"], sb["height"]]))
    L = sj["n_levels"]
    size = lambda s, l: (s["level_ptr"][l + 1] - s["level_ptr"][l]) if l < s["n_levels"] else 0
    for l in range(L):
        seg = sj["perm"][sj["level_ptr"][l]:sj["level_ptr"][l + 1]]
        assert len(seg) == size(sa, l) + size(sb, l)
        assert np.all(seg[:size(sa, l)] < len(a)) and np.all(seg[size(sa, l):] >= len(a))
    assert sj["n_edges"] == sa["n_edges"] + sb["n_edges"]
    assert np.array_equal(sj["child_idx"][:sa["n_edges"]], sa["child_idx"])
    assert np.array_equal(sj["child_idx"][sa["n_edges"]:], sb["child_idx"] + len(a))


def test_children_per_level_closed_forms_and_identities():
    """chain: one child per level above the leaf; star: all n - 1 under level 1; perfect k-ary: k times
    the level's size; in general the sum is E, level 0 has none, and a level's count is the sum of its
    nodes' arities from the child lists."""
    assert S.level_kids(chain_forest(9)).tolist() == [0] + [1] * 8
    assert S.level_kids(star_forest(12)).tolist() == [0, 11]
    k, d = 3, 3
    assert S.level_kids(perfect_kary_tree(k, d)).tolist() == [0] + [k * k ** (d - l) for l in range(1, d + 1)]
    assert S.level_kids(np.zeros(0, np.int32)).tolist() == []
    for cfg in (1, 2):
        p = make_forest(cfg)
        s = S.schedule(p)
        kids = S.level_kids(p)
        assert kids[0] == 0 and kids.sum() == s["n_edges"] and len(kids) == s["n_levels"]
        arity = np.diff(s["child_ptr"])
        assert kids.tolist() == [int(arity[s["height"] == l].sum()) for l in range(s["n_levels"])]
        assert (kids[1:] >= np.diff(s["level_ptr"])[1:]).all()      # every node above the leaves has a child
