"""jitdb_schedule_append against the oracle's definition: the schedule of the concatenated
parent array, bit for bit; and the forward over an appended schedule."""
import numpy as np
import pytest
import torch

import paper_1904_07421_amd as J
from oracle import schedule_oracle as so
from workloads import make_forest, make_values, chain_forest, star_forest, tree_ranges

pytestmark = pytest.mark.gpu
KEYS = ("height", "level_ptr", "perm", "inv_perm", "child_ptr", "child_idx")


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def _check(sched, parent_joint, label):
    want = so.schedule_fast(parent_joint)
    got = sched.to_numpy()
    assert got["n_levels"] == want["n_levels"], label
    assert got["n_edges"] == want["n_edges"], label
    for k in KEYS:
        assert np.array_equal(got[k], want[k]), f"{label}: {k}"
    L = got["n_levels"]
    assert np.array_equal(sched.host_level_ptr[:L + 1], want["level_ptr"]), f"{label}: host_level_ptr"
    kids = np.bincount(want["height"], weights=np.diff(want["child_ptr"]), minlength=L).astype(np.int64)
    assert np.array_equal(sched.host_level_kids[:L], kids), f"{label}: host_level_kids"


def _split_at_tree(parent, frac):
    r = tree_ranges(parent)
    cut = int(r[int((len(r) - 1) * frac)])
    a = parent[:cut]
    b = parent[cut:].copy()
    b[b >= 0] -= cut
    return a, b


@pytest.mark.parametrize("cfg,frac", [(1, 0.5), (2, 0.3), (3, 0.5), (3, 0.9), (4, 0.5)])
def test_append_equals_schedule_of_the_joint_forest(cfg, frac):
    parent = make_forest(cfg)
    a, b = _split_at_tree(parent, frac)
    print(f"append cfg={cfg} frac={frac} Na={len(a)} M={len(b)}", flush=True)
    base = J.jitdb_schedule(_dev(a))
    joint = J.jitdb_schedule_append(base, _dev(b))
    torch.cuda.synchronize()
    _check(joint, so.concat_forests(a, b), f"cfg{cfg}")
    _check(base, a, f"cfg{cfg} base unchanged")


def test_append_when_the_new_trees_are_taller_and_when_they_are_flatter():
    tall, flat = chain_forest(40, 3), star_forest(9, 5)
    for a, b, label in ((flat, tall, "tall onto flat"), (tall, flat, "flat onto tall")):
        print(f"append {label}", flush=True)
        joint = J.jitdb_schedule_append(J.jitdb_schedule(_dev(a)), _dev(b))
        torch.cuda.synchronize()
        _check(joint, so.concat_forests(a, b), label)


def test_append_to_an_empty_forest_and_of_nothing():
    parent = make_forest(2)
    empty = np.zeros(0, dtype=np.int32)
    print("append onto empty", flush=True)
    e = J.jitdb_schedule(_dev(empty))
    joint = J.jitdb_schedule_append(e, _dev(parent))
    torch.cuda.synchronize()
    _check(joint, parent, "onto empty")
    print("append nothing", flush=True)
    same = J.jitdb_schedule_append(J.jitdb_schedule(_dev(parent)), _dev(empty))
    torch.cuda.synchronize()
    _check(same, parent, "nothing appended")
    print("empty + empty", flush=True)
    none = J.jitdb_schedule_append(e, _dev(empty))
    assert none.n_levels == 0 and none.n_edges == 0 and none.host_level_ptr[0] == 0


def test_three_batches_arriving_one_after_another():
    parent = make_forest(3)
    r = tree_ranges(parent)
    cuts = [0, int(r[1000]), int(r[2500]), len(parent)]
    parts = []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        p = parent[lo:hi].copy()
        p[p >= 0] -= lo
        parts.append(p)
    print("append three batches", flush=True)
    s = J.jitdb_schedule(_dev(parts[0]))
    s = J.jitdb_schedule_append(s, _dev(parts[1]))
    s = J.jitdb_schedule_append(s, _dev(parts[2]))
    torch.cuda.synchronize()
    _check(s, parent, "three batches")


def test_bad_new_trees_are_reported_and_bad_arguments_refused():
    base = J.jitdb_schedule(_dev(make_forest(1)))
    cyc = np.array([1, 2, 0, -1], dtype=np.int32)
    print("append cycle", flush=True)
    with pytest.raises(J.JitdbError) as e:
        J.jitdb_schedule_append(base, _dev(cyc))
    assert e.value.code == -4
    rng = np.array([-1, 7, 0], dtype=np.int32)
    print("append out-of-range parent", flush=True)
    with pytest.raises(J.JitdbError) as e:
        J.jitdb_schedule_append(base, _dev(rng))
    assert e.value.code == -3
    with pytest.raises(ValueError):
        J.jitdb_schedule_append(base, _dev(cyc), out=J.Schedule(3, "cuda"))


def test_forward_over_an_appended_schedule_matches_the_one_over_a_fresh_schedule():
    parent = make_forest(3)
    x, W, U, b = make_values(3, len(parent))
    a, nb = _split_at_tree(parent, 0.6)
    print("forward on appended schedule", flush=True)
    joint = J.jitdb_schedule_append(J.jitdb_schedule(_dev(a)), _dev(nb))
    fresh = J.jitdb_schedule(_dev(parent))
    xt, Wt, Ut = (torch.from_numpy(t).cuda() for t in (x, W, U))
    bt = torch.from_numpy(b).cuda()
    h1, c1 = J.jitdb_treelstm_forward(xt, Wt, Ut, bt, joint)
    h2, c2 = J.jitdb_treelstm_forward(xt, Wt, Ut, bt, fresh)
    torch.cuda.synchronize()
    assert torch.equal(h1, h2) and torch.equal(c1, c2)
