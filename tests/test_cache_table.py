"""Host logic of the schedule cache (no GPU): the library's table against the LRU model."""
import numpy as np

from oracle import cache_oracle as C


def test_table_follows_the_lru_model_on_a_random_trace():
    import paper_1904_07421_amd as J
    rng = np.random.default_rng(3)
    for cap in (1, 2, 5):
        t = J.CacheTable(cap)
        m = C.LruModel(cap)
        hits = misses = 0
        for step in range(600):
            k = int(rng.integers(0, 9))
            fp, n = (k * 0x1234567 + 1, (k << 60) | 5), 100 + (k % 3)
            if rng.random() < 0.6:
                got, want = t.lookup(fp, n), m.lookup((fp, n))
                hits += want >= 0
                misses += want < 0
                assert got == want, (cap, step)
            else:
                assert t.insert(fp, n) == m.insert((fp, n)), (cap, step)
        s = t.stats()
        assert s["hits"] == hits and s["misses"] == misses and s["entries"] == len(m.order)
        t.close()


def test_key_includes_both_words_and_the_size():
    import paper_1904_07421_amd as J
    t = J.CacheTable(8)
    assert t.insert((1, 2), 10) == (0, False)
    assert t.lookup((1, 2), 10) == 0
    assert t.lookup((1, 3), 10) == -1 and t.lookup((2, 2), 10) == -1 and t.lookup((1, 2), 11) == -1
    assert t.insert((1 << 63, (1 << 64) - 1), 10) == (1, False)      # full 64-bit words survive the call
    assert t.lookup((1 << 63, (1 << 64) - 1), 10) == 1


def test_bad_arguments():
    import pytest
    import paper_1904_07421_amd as J
    with pytest.raises(J.JitdbError):
        J.CacheTable(0)
    lib = J.load_library()
    assert lib.jitdb_cache_lookup(None, None, 0) == -1
    assert lib.jitdb_cache_insert(None, None, 0, None) == -1
