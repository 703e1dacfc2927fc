"""Launch counts of a Tree-LSTM forest at different batching granularities (CPU only).

The paper's section 3 compares, for batches of 256 samples, how many launches a workload
needs without batching and with depth-matched batching, once counting operators and once
counting whole cells (Table 1), and explains the gap: a cell is 33 operators of which only 4
depend on the number of children, yet cells of different arity cannot share a launch.  This
module repeats that bookkeeping on any forest given as a parent array and adds the
granularity this library uses (one stacked launch set per height level, whatever the arity).

Counting rules (restated from section 3; the constants are the paper's):
  operator, unbatched   every cell launches its 33 operators
  cell, unbatched       one launch per cell
  cell, batched         per batch and height: one launch per distinct arity present
  operator, batched     per batch and height: the 29 arity-independent operators once, the 4
                        arity-dependent ones once per distinct arity present
  level (this library)  per batch: 1 + 3 L - 1 launches (weight packing; per level a stack, a
                        fused gate-GEMM-and-cell and - except for the top level - a projection)
The paper's own table came from its dataset, which is not available here; the figures
this module prints are for the forest it is given.
"""
from __future__ import annotations

import numpy as np

OPS_PER_CELL = 33          # section 3
OPS_ARITY_DEPENDENT = 4    # section 3


def _heights_and_arity(parent: np.ndarray):
    n = parent.shape[0]
    arity = np.bincount(parent[parent >= 0], minlength=n).astype(np.int64)
    height = np.zeros(n, dtype=np.int64)
    # children before parents: repeat "parent height >= child height + 1" until nothing moves
    live = np.flatnonzero(parent >= 0)
    while True:
        cand = height[live] + 1
        new = height.copy()
        np.maximum.at(new, parent[live], cand)
        if np.array_equal(new, height):
            break
        height = new
    return height, arity


def tree_of(parent: np.ndarray) -> np.ndarray:
    """Index of the tree (root order of appearance) every node belongs to."""
    n = parent.shape[0]
    root = np.arange(n)
    p = parent.copy()
    while True:
        up = np.where(p >= 0, p, root)
        if np.array_equal(up, root):
            break
        root = up
        p = np.where(p >= 0, parent[np.maximum(p, 0)], -1)
    roots = np.flatnonzero(parent < 0)
    order = np.full(n, -1, dtype=np.int64)
    order[roots] = np.arange(len(roots))
    return order[root]


def launch_counts(parent, batch_trees: int = 256) -> dict:
    """Launch counts for the forest, cut into batches of `batch_trees` consecutive trees."""
    parent = np.asarray(parent, dtype=np.int64)
    n = parent.shape[0]
    if n == 0:
        return dict(cells=0, batches=0, operator_unbatched=0, cell_unbatched=0, cell_batched=0,
                    operator_batched=0, level_batched=0)
    height, arity = _heights_and_arity(parent)
    batch = tree_of(parent) // int(batch_trees)
    n_batches = int(batch.max()) + 1
    # distinct (batch, height, arity) triples and distinct (batch, height) pairs
    span_h = int(height.max()) + 1
    span_a = int(arity.max()) + 1
    key_bh = batch * span_h + height
    slots_bha = np.unique(key_bh * span_a + arity).shape[0]
    slots_bh = np.unique(key_bh).shape[0]
    return dict(
        cells=n, batches=n_batches,
        operator_unbatched=OPS_PER_CELL * n,
        cell_unbatched=n,
        cell_batched=slots_bha,
        operator_batched=(OPS_PER_CELL - OPS_ARITY_DEPENDENT) * slots_bh + OPS_ARITY_DEPENDENT * slots_bha,
        level_batched=3 * slots_bh,   # per batch: 1 (packing) + 3 L - 1 (no projection on the top level)
    )


def report(parent, batch_trees: int = 256) -> str:
    c = launch_counts(parent, batch_trees)
    rows = [
        ("operator", c["operator_unbatched"], c["operator_batched"]),
        ("cell (subgraph)", c["cell_unbatched"], c["cell_batched"]),
        ("level (this library)", c["operator_unbatched"], c["level_batched"]),
    ]
    out = [f"{c['cells']} cells in {c['batches']} batches of {batch_trees} trees",
           f"{'granularity':22s} {'no-batch':>12s} {'batch':>10s} {'ratio':>9s}"]
    for name, a, b in rows:
        out.append(f"{name:22s} {a:12d} {b:10d} {a / max(b, 1):8.1f}x")
    out.append(f"operators per cell launch (zoom ratio): {c['operator_unbatched'] / max(c['cell_unbatched'], 1):.2f}")
    return "\n".join(out)


if __name__ == "__main__":
    import argparse
    from workloads import make_forest
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--batch-trees", type=int, default=256)
    a = ap.parse_args()
    print(report(make_forest(a.config), a.batch_trees))
