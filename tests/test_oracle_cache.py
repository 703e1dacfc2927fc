"""Pins of the fingerprint oracle: the published SplitMix64 stream, hand arithmetic, and the
properties a cache key needs."""
import numpy as np

from oracle import cache_oracle as C
from workloads import make_forest, relabel


def test_mix64_is_the_published_splitmix64_output_function():
    # first outputs of SplitMix64 seeded with 0 (state advances by GOLDEN before each output),
    # as listed with the reference implementations of the xoshiro / xoroshiro generators
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F, 0xF88BB8A8724C81EC]
    state = 0
    for w in want:
        state = (state + C.GOLDEN) & C.MASK
        assert C.mix64(state) == w


def test_single_entry_fingerprint_by_hand():
    # one node with parent value 0: word = 0, so fp[0] = mix64(GOLDEN) = first SplitMix64 output
    f0, f1 = C.fingerprint(np.array([0], dtype=np.int32))
    assert f0 == 0xE220A8397B1DCDAF
    assert f1 == C.mix64(C.KEY1)
    # a root (-1) sets the low 32 bits of the word
    g0, _ = C.fingerprint(np.array([-1], dtype=np.int32))
    assert g0 == C.mix64(0xFFFFFFFF + C.GOLDEN)


def test_sum_over_nodes_and_position_dependence():
    a = np.array([-1, 0, 0, 1], dtype=np.int32)
    f = C.fingerprint(a)
    # additivity: the forest's fingerprint is the sum of its entries' terms
    terms = [C.mix64(((i << 32) | (int(p) & 0xFFFFFFFF)) + C.GOLDEN) for i, p in enumerate(a)]
    assert f[0] == sum(terms) & C.MASK
    # swapping two different entries changes both sums
    b = a.copy(); b[[0, 3]] = b[[3, 0]]
    g = C.fingerprint(b)
    assert g[0] != f[0] and g[1] != f[1]
    assert C.fingerprint(np.zeros(0, dtype=np.int32)) == (0, 0)


def test_fast_version_matches_the_loop():
    for cfg in (1, 2):
        p = make_forest(cfg)
        assert C.fingerprint_fast(p) == C.fingerprint(p)
    p = make_forest(3)[:20000]
    assert C.fingerprint_fast(p) == C.fingerprint(p)


def test_distinct_forests_get_distinct_fingerprints():
    seen = set()
    p = make_forest(3)
    rng = np.random.default_rng(0)
    seen.add(C.fingerprint_fast(p))
    for _ in range(200):                       # single-entry edits
        q = p.copy()
        i = int(rng.integers(0, p.shape[0]))
        q[i] = q[i] + 1 if q[i] + 1 < p.shape[0] else -1
        seen.add(C.fingerprint_fast(q))
    q, _ = relabel(p, 7)
    seen.add(C.fingerprint_fast(q))
    seen.add(C.fingerprint_fast(p[:-1]))
    assert len(seen) == 203


def test_lru_model():
    m = C.LruModel(2)
    assert m.lookup("a") == -1
    assert m.insert("a") == (0, False) and m.insert("b") == (1, False)
    assert m.lookup("a") == 0                  # a is now the most recent
    assert m.insert("c") == (1, True)          # b, the least recently used, goes
    assert m.lookup("b") == -1 and m.lookup("c") == 1 and m.lookup("a") == 0
    assert m.insert("a") == (0, False)
