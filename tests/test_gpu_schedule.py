"""GPU parity: jitdb_schedule against the schedule oracle, bit-exact."""
import numpy as np
import pytest

from oracle import schedule_oracle as S
from workloads import make_forest, relabel, chain_forest, star_forest, perfect_kary_tree
from gpu_util import dev_parent, assert_schedule_equal

pytestmark = pytest.mark.gpu


def _run(parent):
    import paper_1904_07421_amd as J
    return J.jitdb_schedule(dev_parent(parent))


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_configs_bit_exact(cfg):
    p = make_forest(cfg)
    print(f"schedule parity cfg={cfg} N={p.shape[0]}", flush=True)
    got = _run(p).to_numpy()
    want = S.schedule(p) if p.shape[0] < 6000 else S.schedule_fast(p)
    assert_schedule_equal(got, want)
    if p.shape[0] < 6000:                   # children per level against the oracle's own count
        assert np.array_equal(got["level_kids"], S.level_kids(p))


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_relabelled_ids_bit_exact(cfg):
    p, _ = relabel(make_forest(cfg), 100 + cfg)
    print(f"schedule relabelled cfg={cfg} N={p.shape[0]}", flush=True)
    assert_schedule_equal(_run(p).to_numpy(), S.schedule_fast(p))


@pytest.mark.parametrize("name,parent", [
    ("single", np.array([-1], dtype=np.int32)),
    ("two-roots", np.array([-1, -1], dtype=np.int32)),
    ("pair", np.array([1, -1], dtype=np.int32)),
    ("chain-300", chain_forest(300)),             # more than 256 levels: two radix passes
    ("chain-5000", chain_forest(5000)),           # more levels than the LDS histogram holds
    ("star-100000", star_forest(100000)),         # one very wide child list
    ("kary-4-7", perfect_kary_tree(4, 7)),
    ("tile-edge-2048", chain_forest(8, 256)),     # N exactly one sort tile
    ("tile-edge-2049", np.concatenate([chain_forest(8, 256), [-1]]).astype(np.int32)),
    ("tile-edge-4097", star_forest(4097)),
])
def test_shapes_and_edges(name, parent):
    print(f"schedule shape {name} N={parent.shape[0]}", flush=True)
    assert_schedule_equal(_run(parent).to_numpy(), S.schedule_fast(parent))


@pytest.mark.parametrize("n", [8191, 8192, 8193, 16383, 16384, 16385])
@pytest.mark.parametrize("kind", ["chain", "trees"])
def test_sizes_around_the_one_launch_paths(kind, n):
    """Forests of up to 8192 nodes run every pointer-jumping round in one launch, and scans of up to 16384
    entries are one launch: one node below, at and above both limits, as one relabelled chain (as many rounds as
    a forest of that size can need) and as a forest of small trees."""
    if kind == "chain":
        p, _ = relabel(chain_forest(n), n)
    else:
        from workloads import bounded_arity_forest
        p = bounded_arity_forest(n // 8 + 8, 9, 15, 4, n)[:n].copy()      # the last tree may be cut short:
        assert (p < np.arange(n)).all()                                    # parents precede their children
    print(f"schedule one-launch paths {kind} N={p.shape[0]}", flush=True)
    assert p.shape[0] == n
    assert_schedule_equal(_run(p).to_numpy(), S.schedule_fast(p))


def test_small_cycle_is_detected_by_the_one_launch_rounds():
    import paper_1904_07421_amd as J
    p = chain_forest(50, 100).copy()                 # 100 chains of 50, 5000 nodes
    roots = np.flatnonzero(p < 0)
    p[roots[3]] = roots[3] + 49                      # the root of chain 3 under its own leaf
    with pytest.raises(J.JitdbError) as e:
        _run(p)
    assert e.value.code == -4


def test_deep_relabelled_chain():
    p, _ = relabel(chain_forest(70000), 5)       # 70000 levels, three radix passes over heights
    print("schedule deep relabelled chain", flush=True)
    assert_schedule_equal(_run(p).to_numpy(), S.schedule_fast(p))


def test_empty_forest():
    import torch
    import paper_1904_07421_amd as J
    s = J.jitdb_schedule(torch.empty(0, dtype=torch.int32, device="cuda"))
    assert s.n_levels == 0 and s.n_edges == 0 and s.host_level_ptr[0] == 0


@pytest.mark.parametrize("bad,code", [
    ([-1, 0, 5], -3), ([-1, 1], -3), ([-2, 0], -3), ([0], -3),
    ([1, 0], -4), ([-1, 2, 3, 1], -4), ([1, 2, 0, -1, 3], -4),
])
def test_invalid_forests_give_error_codes(bad, code):
    import paper_1904_07421_amd as J
    with pytest.raises(J.JitdbError) as e:
        _run(np.array(bad, dtype=np.int32))
    assert e.value.code == code


def test_large_cycle_is_detected_not_hung():
    import paper_1904_07421_amd as J
    p = make_forest(3).copy()
    n = p.shape[0]
    roots = np.flatnonzero(p < 0)
    p[roots[5]] = n - 1           # hang tree 5 under the last node of the last tree ...
    p[roots[-1]] = roots[5] + 1   # ... and the last tree under a node of tree 5: a cycle
    with pytest.raises(S.ForestError):
        S.schedule_fast(p)
    with pytest.raises(J.JitdbError) as e:
        _run(p)
    assert e.value.code == -4


def test_workspace_too_small_is_rejected():
    import torch
    import paper_1904_07421_amd as J
    p = dev_parent(make_forest(1))
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(J.JitdbError) as e:
        J.jitdb_schedule(p, workspace=ws)
    assert e.value.code == -5


def test_repeatable():
    p = make_forest(4)
    a, b = _run(p).to_numpy(), _run(p).to_numpy()
    assert_schedule_equal(a, b)


@pytest.mark.timeout(600)
def test_largest_forest_the_interface_accepts():
    """N = JITDB_MAX_NODES (2^28): 2^26 chains of four nodes, whose schedule has a closed form
    (height = 3 - v % 4; level l holds the nodes 4t + 3 - l in ascending order; node 4t + k,
    k < 3, has the single child 4t + k + 1).  Checked on the device; int32 offsets must not
    wrap anywhere on the way."""
    import torch
    import paper_1904_07421_amd as J
    n = 1 << 28
    t = 1 << 26
    print(f"schedule N={n}", flush=True)
    v = torch.arange(n, dtype=torch.int32, device="cuda")
    parent = torch.where((v & 3) == 0, torch.full_like(v, -1), v - 1)
    s = J.jitdb_schedule(parent)
    del parent
    torch.cuda.synchronize()
    assert s.n_levels == 4 and s.n_edges == 3 * t
    assert list(s.host_level_ptr[:5]) == [0, t, 2 * t, 3 * t, 4 * t]
    assert torch.equal(s.level_ptr[:5].cpu(), torch.tensor([0, t, 2 * t, 3 * t, 4 * t], dtype=torch.int32))
    assert torch.equal(s.height, 3 - (v & 3))
    lvl = torch.div(v, t, rounding_mode="floor")          # position -> level
    want_perm = 4 * (v - lvl * t) + 3 - lvl
    assert torch.equal(s.perm, want_perm)
    del want_perm, lvl
    assert torch.equal(s.inv_perm, (3 - (v & 3)) * t + torch.div(v, 4, rounding_mode="floor"))
    k = v & 3
    assert torch.equal(s.child_ptr[:n], 3 * torch.div(v, 4, rounding_mode="floor") + k)
    assert int(s.child_ptr[n]) == 3 * t
    e = v[:3 * t]
    assert torch.equal(s.child_idx[:3 * t], 4 * torch.div(e, 3, rounding_mode="floor") + e % 3 + 1)
