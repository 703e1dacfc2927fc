"""Launch-count bookkeeping of section 3 (CPU): closed forms on forests whose counts are obvious."""
import numpy as np

from paper_1904_07421_amd import granularity as G
from workloads import chain_forest, make_forest, tree_ranges
from oracle import schedule_oracle as S


def test_chains_every_cell_has_arity_one_or_zero():
    # 4 chains of 6 nodes in one batch: 6 heights; arity 0 at height 0, arity 1 above
    c = G.launch_counts(chain_forest(6, 4), batch_trees=256)
    assert c["cells"] == 24 and c["batches"] == 1
    assert c["operator_unbatched"] == 33 * 24 and c["cell_unbatched"] == 24
    assert c["cell_batched"] == 6                       # one (height, arity) pair per height
    assert c["operator_batched"] == 29 * 6 + 4 * 6
    assert c["level_batched"] == 1 + 3 * 6 - 1


def test_stars_of_different_size_split_the_cell_launches_but_not_the_levels():
    # stars with 3, 4 and 5 leaves: roots have arity 3, 4, 5 at height 1
    parent = np.array([-1, 0, 0, 0, -1, 4, 4, 4, 4, -1, 9, 9, 9, 9, 9], dtype=np.int32)
    c = G.launch_counts(parent, batch_trees=256)
    assert c["cell_batched"] == 1 + 3                   # leaves together; three root arities apart
    assert c["operator_batched"] == 29 * 2 + 4 * 4
    assert c["level_batched"] == 1 + 3 * 2 - 1
    # one tree per batch: nothing to share between trees any more
    c1 = G.launch_counts(parent, batch_trees=1)
    assert c1["batches"] == 3 and c1["cell_batched"] == 6 and c1["level_batched"] == 3 * (1 + 3 * 2 - 1)


def test_counts_agree_with_the_schedule_oracle_on_a_config():
    parent = make_forest(2)
    s = S.schedule(parent)
    c = G.launch_counts(parent, batch_trees=10 ** 9)     # the whole forest as one batch
    assert c["batches"] == 1
    assert c["level_batched"] == 1 + 3 * s["n_levels"] - 1
    arity = np.diff(s["child_ptr"])
    pairs = {(int(h), int(a)) for h, a in zip(s["height"], arity)}
    assert c["cell_batched"] == len(pairs)
    assert np.array_equal(G.tree_of(parent),
                          np.searchsorted(tree_ranges(parent), np.arange(len(parent)), side="right") - 1)


def test_empty_forest_and_report_text():
    assert G.launch_counts(np.zeros(0, dtype=np.int32))["cells"] == 0
    txt = G.report(make_forest(1), batch_trees=4)
    assert "zoom ratio" in txt and "level (this library)" in txt
