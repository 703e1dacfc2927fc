"""Generators: determinism and the shape statistics the configs are quoted with."""
import os

import numpy as np
import pytest

from workloads import (CONFIGS, make_forest, make_values, relabel, to_bf16_bits,
                       bf16_bits_to_f32, tree_ranges)
from oracle import schedule_oracle as S

GOLD = os.path.join(os.path.dirname(__file__), "golden", "workload_stats.txt")


def _gold():
    rows, l5 = {}, None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        t = line.split()
        if t[0] == "L5":
            l5 = [int(v) for v in t[1:]]
        else:
            rows[int(t[0])] = [int(v) for v in t[1:]]
    return rows, l5


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_forest_matches_quoted_shape(cfg):
    rows, l5 = _gold()
    T, N, E, L, amax, leaf_pm = rows[cfg]
    p = make_forest(cfg)
    assert p.dtype == np.int32 and p.shape[0] == N
    assert int((p < 0).sum()) == T and N - T == E
    cnt = np.bincount(p[p >= 0], minlength=N)
    assert int(cnt.max()) == amax
    assert abs(1000.0 * (cnt == 0).mean() - leaf_pm) < 1.0
    s = S.schedule_fast(p)
    assert s["n_levels"] == L
    if cfg == 5:
        assert np.diff(s["level_ptr"]).tolist() == l5


def test_deterministic_and_valid():
    for cfg in (1, 2, 4):
        a, b = make_forest(cfg), make_forest(cfg)
        assert np.array_equal(a, b)
        S.validate(a) if cfg != 4 else S.schedule_fast(a)
    x1, W1, U1, b1 = make_values(1, 74, "random")
    x2, W2, U2, b2 = make_values(1, 74, "random")
    assert np.array_equal(x1, x2) and np.array_equal(W1, W2) and np.array_equal(b1, b2)
    assert x1.dtype == np.float32 and W1.shape == (600, 300) and U1.shape == (600, 150)
    assert np.abs(W1).max() <= 1 / np.sqrt(300) and np.abs(U1).max() <= 1 / np.sqrt(150)
    assert np.abs(b1).max() > 0.1
    assert not make_values(1, 74, "zero")[3].any()


def test_config4_mix_kinds():
    p = make_forest(4)
    r = tree_ranges(p)
    for t in range(9):
        loc = p[r[t]:r[t + 1]] - r[t]
        n = loc.shape[0]
        if t % 3 == 0:
            assert 8 <= n <= 128 and np.array_equal(loc[1:], np.arange(n - 1))
        elif t % 3 == 1:
            assert 17 <= n <= 65 and (loc[1:] == 0).all()
        else:
            assert 8 <= n <= 64


def test_relabel_is_isomorphism():
    p = make_forest(2)
    q, new_of_old = relabel(p, 7)
    nonroot = p >= 0
    assert np.array_equal(q[new_of_old[nonroot]], new_of_old[p[nonroot]])
    assert (q[new_of_old[~nonroot]] == -1).all()


def test_bf16_rounding_is_nearest_even():
    # exactly representable values survive; ties go to the even mantissa
    v = np.array([1.0, -2.5, 0.0, 3.140625], dtype=np.float32)
    assert np.array_equal(bf16_bits_to_f32(to_bf16_bits(v)), v)
    one = np.float32(1.0).view(np.uint32)
    tie_down = np.array([one + 0x8000], dtype=np.uint32).view(np.float32)   # mantissa even -> stays
    tie_up = np.array([one + 0x18000], dtype=np.uint32).view(np.float32)    # odd -> rounds up
    assert to_bf16_bits(tie_down)[0] == (one >> 16)
    assert to_bf16_bits(tie_up)[0] == (one >> 16) + 2
    rng = np.random.default_rng(0)
    a = rng.standard_normal(10000).astype(np.float32)
    r = bf16_bits_to_f32(to_bf16_bits(a))
    assert np.all(np.abs(r - a) <= np.abs(a) * 2.0 ** -8)
    import torch
    t = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(t, r)
