"""GPU parity of jitdb_forest_fingerprint (bit-exact against the oracle) and the schedule cache."""
import numpy as np
import pytest

from oracle import cache_oracle as C
from oracle import schedule_oracle as S
from workloads import make_forest, relabel, chain_forest
from gpu_util import dev_parent, assert_schedule_equal

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_fingerprint_bit_exact(cfg):
    import paper_1904_07421_amd as J
    p = make_forest(cfg)
    print(f"fingerprint cfg={cfg} N={p.shape[0]}", flush=True)
    got = J.jitdb_forest_fingerprint(dev_parent(p))
    assert got == C.fingerprint_fast(p)
    if p.shape[0] < 20000:
        assert got == C.fingerprint(p)


@pytest.mark.parametrize("name,parent", [
    ("empty", np.zeros(0, dtype=np.int32)),
    ("one", np.array([-1], dtype=np.int32)),
    ("zero-word", np.array([0], dtype=np.int32)),            # not a forest: the fingerprint does not care
    ("block-edge-1024", chain_forest(4, 256)),
    ("block-edge-1025", np.concatenate([chain_forest(4, 256), [-1]]).astype(np.int32)),
    ("arbitrary-values", np.array([-7, 2**31 - 1, -2**31, 5], dtype=np.int32)),
])
def test_fingerprint_edges(name, parent):
    import paper_1904_07421_amd as J
    print(f"fingerprint {name}", flush=True)
    assert J.jitdb_forest_fingerprint(dev_parent(parent)) == C.fingerprint(parent)


def test_fingerprint_repeatable_and_sensitive():
    import paper_1904_07421_amd as J
    p = make_forest(4)
    a = J.jitdb_forest_fingerprint(dev_parent(p))
    assert a == J.jitdb_forest_fingerprint(dev_parent(p))
    q = p.copy(); q[12345] = q[12345] + 1
    assert J.jitdb_forest_fingerprint(dev_parent(q)) != a
    r, _ = relabel(p, 3)
    assert J.jitdb_forest_fingerprint(dev_parent(r)) != a


@pytest.mark.parametrize("verify", [False, True])
def test_schedule_cache_hits_and_evicts(verify):
    import paper_1904_07421_amd as J
    forests = [make_forest(2), relabel(make_forest(2), 1)[0], make_forest(3)]
    want = [S.schedule_fast(p) for p in forests]
    cache = J.ScheduleCache(capacity=2, verify=verify)
    dev = [dev_parent(p) for p in forests]
    s0, hit = cache.get(dev[0]); assert not hit
    s1, hit = cache.get(dev[1]); assert not hit
    again, hit = cache.get(dev[0]); assert hit and again is s0
    assert_schedule_equal(again.to_numpy(), want[0])
    s2, hit = cache.get(dev[2]); assert not hit                  # evicts forest 1 (least recently used)
    assert_schedule_equal(s2.to_numpy(), want[2])
    _, hit = cache.get(dev[0]); assert hit
    s1b, hit = cache.get(dev[1]); assert not hit                 # was evicted: scheduled again
    assert_schedule_equal(s1b.to_numpy(), want[1])
    st = cache.table.stats()
    assert st["hits"] == 2 and st["misses"] == 4 and st["entries"] == 2


def test_cached_schedule_gives_the_same_forward():
    import torch
    import paper_1904_07421_amd as J
    from workloads import make_values
    p = make_forest(2)
    x, W, U, b = make_values(2, p.shape[0])
    dev = lambda a: torch.from_numpy(a).cuda()
    cache = J.ScheduleCache(4)
    s_a, _ = cache.get(dev_parent(p))
    h_a, c_a = J.jitdb_treelstm_forward(dev(x), dev(W), dev(U), dev(b), s_a)
    s_b, hit = cache.get(dev_parent(p.copy()))
    assert hit
    h_b, c_b = J.jitdb_treelstm_forward(dev(x), dev(W), dev(U), dev(b), s_b)
    assert torch.equal(h_a, h_b) and torch.equal(c_a, c_b)


@pytest.mark.timeout(600)
def test_fingerprint_of_the_largest_forest():
    """N = 2^28: the position enters the hashed word in its upper half; nothing may wrap at 2^31."""
    import torch
    import paper_1904_07421_amd as J
    n = 1 << 28
    v = np.arange(n, dtype=np.int32)
    p = np.where((v & 3) == 0, -1, v - 1).astype(np.int32)
    del v
    print(f"fingerprint N={n}", flush=True)
    got = J.jitdb_forest_fingerprint(torch.from_numpy(p).cuda())
    want = (0, 0)
    step = 1 << 24                                   # the oracle's sums, piecewise to bound host memory
    for lo in range(0, n, step):
        q = p[lo:lo + step]
        with np.errstate(over="ignore"):
            word = ((np.arange(lo, lo + q.shape[0], dtype=np.uint64)) << np.uint64(32)) | q.view(np.uint32).astype(np.uint64)
            f0 = C._mix64_np(word + np.uint64(C.GOLDEN)).sum(dtype=np.uint64)
            f1 = C._mix64_np(word ^ np.uint64(C.KEY1)).sum(dtype=np.uint64)
        want = ((want[0] + int(f0)) & C.MASK, (want[1] + int(f1)) & C.MASK)
    assert got == want
