"""Seeded synthetic forests shaped like short-sentence parse trees.

The paper's workload is a Tree-LSTM over parse trees of short sentences whose
nodes have 0-9 children, processed 256 samples at a time (section 5 and the
caption of Table 1).  Neither the dataset nor the parser is available, so these
generators produce forests of the same shape: many small trees (4-128 nodes),
small skewed arity, hundreds to tens of thousands of trees per batch.

A forest is ONE int32 parent array with global node ids; parent == -1 marks a
root.  Trees are laid out one after another (local id + running offset); the
`relabel` helper scrambles ids for tests that need arbitrary numbering.

Randomness: numpy's PCG64 `default_rng(seed)`; structure uses seed = config
index, values use seed = 1000 + config index.  Draw order for the structure:
configs 1, 2, 3, 5 draw all tree sizes first and then one uniform per non-root
node, tree by tree; config 4 draws, per tree, its size and then its uniforms
(also for chains and stars, where they are not used).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np


@dataclass(frozen=True)
class ForestConfig:
    index: int
    name: str
    n_trees: int
    kind: str          # "rrt" | "pa" | "mix"
    size_lo: int
    size_hi: int
    D: int
    H: int
    dtype: str         # "f32" | "bf16"


CONFIGS: Dict[int, ForestConfig] = {
    1: ForestConfig(1, "tiny-rrt-8", 8, "rrt", 5, 12, 300, 150, "f32"),
    2: ForestConfig(2, "sentence-pa-256", 256, "pa", 4, 32, 300, 150, "f32"),
    3: ForestConfig(3, "batch-pa-4096", 4096, "pa", 4, 48, 300, 150, "bf16"),
    4: ForestConfig(4, "adversarial-mix-4096", 4096, "mix", 8, 128, 300, 256, "f32"),
    5: ForestConfig(5, "large-rrt-65536", 65536, "rrt", 8, 64, 300, 512, "bf16"),
}


# --------------------------------------------------------------------------
# single-tree shapes (local ids, root = 0, parent[i] < i)
# --------------------------------------------------------------------------
def _rrt_parents(u: np.ndarray) -> np.ndarray:
    """Random recursive tree: node i >= 1 attaches to a uniform node in [0, i)."""
    n = u.shape[0] + 1
    par = np.empty(n, dtype=np.int64)
    par[0] = -1
    i = np.arange(1, n, dtype=np.float64)
    par[1:] = np.minimum(np.floor(u * i), i - 1).astype(np.int64)
    return par


def _pa_parents(u: np.ndarray) -> np.ndarray:
    """Preferential attachment: node i picks p < i with weight 1 + outdeg(p)."""
    n = u.shape[0] + 1
    par = np.empty(n, dtype=np.int64)
    par[0] = -1
    w = np.zeros(n, dtype=np.float64)
    w[0] = 1.0
    for i in range(1, n):
        r = u[i - 1] * (2 * i - 1)          # total weight of nodes 0..i-1
        cum = np.cumsum(w[:i])
        p = int(np.searchsorted(cum, r, side="right"))
        p = min(p, i - 1)
        par[i] = p
        w[p] += 1.0
        w[i] = 1.0
    return par


def _chain_parents(n: int) -> np.ndarray:
    par = np.arange(-1, n - 1, dtype=np.int64)
    return par


def _star_parents(n: int) -> np.ndarray:
    par = np.zeros(n, dtype=np.int64)
    par[0] = -1
    return par


def _concat(trees) -> np.ndarray:
    total = sum(t.shape[0] for t in trees)
    out = np.empty(total, dtype=np.int32)
    off = 0
    for t in trees:
        n = t.shape[0]
        g = np.where(t < 0, -1, t + off)
        out[off:off + n] = g
        off += n
    return out


# --------------------------------------------------------------------------
# config forests
# --------------------------------------------------------------------------
def make_forest(cfg_index: int, n_trees: int | None = None) -> np.ndarray:
    """Parent array (int32, -1 = root) of config `cfg_index`.

    `n_trees` overrides the tree count (same stream, so a smaller count is NOT
    a prefix of the larger forest for configs that draw all sizes first).
    """
    cfg = CONFIGS[cfg_index]
    T = cfg.n_trees if n_trees is None else int(n_trees)
    rng = np.random.default_rng(cfg.index)
    if cfg.kind in ("rrt", "pa"):
        sizes = rng.integers(cfg.size_lo, cfg.size_hi + 1, size=T)
        if cfg.kind == "rrt":
            # one uniform per non-root node, tree after tree == one long draw
            m = sizes - 1
            u = rng.random(int(m.sum()))
            N = int(sizes.sum())
            start = np.concatenate(([0], np.cumsum(sizes)))[:-1]
            local = np.arange(N, dtype=np.int64) - np.repeat(start, sizes)
            is_root = local == 0
            par = np.empty(N, dtype=np.int64)
            par[is_root] = -1
            li = local[~is_root].astype(np.float64)
            loc_par = np.minimum(np.floor(u * li), li - 1).astype(np.int64)
            par[~is_root] = loc_par + np.repeat(start, sizes)[~is_root]
            return par.astype(np.int32)
        trees = []
        for n in sizes:
            u = rng.random(int(n) - 1)
            trees.append(_pa_parents(u))
        return _concat(trees)
    # mix: tree t has kind t mod 3 (0 chain, 1 star, 2 random recursive tree)
    trees = []
    for t in range(T):
        k = t % 3
        if k == 0:
            n = int(rng.integers(8, 128 + 1))
        elif k == 1:
            n = 1 + int(rng.integers(16, 64 + 1))
        else:
            n = int(rng.integers(8, 64 + 1))
        u = rng.random(n - 1)
        if k == 0:
            trees.append(_chain_parents(n))
        elif k == 1:
            trees.append(_star_parents(n))
        else:
            trees.append(_rrt_parents(u))
    return _concat(trees)


def make_values(cfg_index: int, n_nodes: int, bias: str = "zero",
                D: int | None = None, H: int | None = None):
    """x [N, D], W [4H, D], U [4H, H], b [4H] in fp32.

    x ~ N(0, 1); W, U ~ U(+-1/sqrt(fan_in)) with fan_in = D for W and H for U;
    b = 0 ("zero") or U(-0.5, 0.5) ("random", used by parity tests so that a
    dropped or misplaced bias is seen).  Rows of W, U, b are ordered by gate:
    input i, output o, candidate u, forget f, H rows each.
    """
    cfg = CONFIGS[cfg_index]
    D = cfg.D if D is None else D
    H = cfg.H if H is None else H
    rng = np.random.default_rng(1000 + cfg.index)
    x = rng.standard_normal((n_nodes, D), dtype=np.float32)
    kw = 1.0 / np.sqrt(D)
    ku = 1.0 / np.sqrt(H)
    W = rng.uniform(-kw, kw, size=(4 * H, D)).astype(np.float32)
    U = rng.uniform(-ku, ku, size=(4 * H, H)).astype(np.float32)
    if bias == "zero":
        b = np.zeros(4 * H, dtype=np.float32)
    elif bias == "random":
        b = rng.uniform(-0.5, 0.5, size=4 * H).astype(np.float32)
    else:
        raise ValueError(bias)
    return x, W, U, b


def make_workload(cfg_index: int, bias: str = "zero", n_trees: int | None = None):
    """(cfg, parent, x, W, U, b) of one config."""
    cfg = CONFIGS[cfg_index]
    parent = make_forest(cfg_index, n_trees)
    x, W, U, b = make_values(cfg_index, parent.shape[0], bias)
    return cfg, parent, x, W, U, b


# --------------------------------------------------------------------------
# helpers that move inputs around (no method arithmetic)
# --------------------------------------------------------------------------
def relabel(parent: np.ndarray, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Scramble node ids.  Returns (new_parent, new_id_of_old)."""
    n = parent.shape[0]
    rng = np.random.default_rng(seed)
    new_of_old = rng.permutation(n).astype(np.int64)
    new_parent = np.empty(n, dtype=np.int32)
    p = parent.astype(np.int64)
    mapped = np.where(p < 0, -1, new_of_old[np.maximum(p, 0)])
    new_parent[new_of_old] = mapped.astype(np.int32)
    return new_parent, new_of_old


def tree_ranges(parent: np.ndarray) -> np.ndarray:
    """For forests laid out tree after tree with the root first: [T+1] offsets."""
    roots = np.flatnonzero(parent < 0)
    return np.concatenate((roots, [parent.shape[0]])).astype(np.int64)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns (uint16), round to nearest even.

    This only prepares inputs for the bf16 configs; both the oracle and the
    GPU path receive the very same bf16 values.
    """
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    bits = a32.view(np.uint32)
    rounded = (bits >> 16) & 1
    rounded += 0x7FFF
    rounded += bits                       # wraps only for NaN patterns, fixed below
    out = (rounded >> 16).astype(np.uint16)
    nan = np.isnan(a32)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return b.view(np.float32)


def chain_forest(n: int, n_trees: int = 1) -> np.ndarray:
    return _concat([_chain_parents(n) for _ in range(n_trees)])


def star_forest(n: int, n_trees: int = 1) -> np.ndarray:
    return _concat([_star_parents(n) for _ in range(n_trees)])


def perfect_kary_tree(k: int, depth: int) -> np.ndarray:
    """Heap-numbered perfect k-ary tree with `depth` edges from root to leaves."""
    n = (k ** (depth + 1) - 1) // (k - 1) if k > 1 else depth + 1
    par = (np.arange(n, dtype=np.int64) - 1) // k
    par[0] = -1
    return par.astype(np.int32)


# --------------------------------------------------------------------------
# several networks in one batch (the generic batcher's signatures)
# --------------------------------------------------------------------------
def tree_signatures(parent: np.ndarray, n_sig: int, seed: int) -> np.ndarray:
    """sig [N] int32: every tree draws one of n_sig signatures uniformly; all its nodes carry it."""
    r = tree_ranges(parent)
    rng = np.random.default_rng(seed)
    per_tree = rng.integers(0, n_sig, size=len(r) - 1).astype(np.int32)
    return np.repeat(per_tree, np.diff(r)).astype(np.int32)


def mixed_forest(cfg_index: int, n_trees: int, n_seqs: int, len_lo: int, len_hi: int, seed: int):
    """(parent, sig): n_trees trees of the config (signature 0) followed by n_seqs chains of
    length U[len_lo, len_hi] (signature 1) - a Tree-LSTM batch and a variable-length LSTM
    batch filed in one table.  Trees are laid out one after another, root first."""
    trees = make_forest(cfg_index, n_trees)
    rng = np.random.default_rng(seed)
    lens = rng.integers(len_lo, len_hi + 1, size=n_seqs)
    seqs = _concat([_chain_parents(int(n)) for n in lens]) if n_seqs else np.zeros(0, dtype=np.int32)
    parent = _concat([trees, seqs]) if n_seqs else trees
    sig = np.concatenate([np.zeros(trees.shape[0], np.int32), np.ones(seqs.shape[0], np.int32)])
    return parent.astype(np.int32), sig


def make_values_typed(cfg_index: int, n_nodes: int, n_sig: int, bias: str = "random",
                      D: int | None = None, H: int | None = None):
    """x [N, D], W [n_sig, 4H, D], U [n_sig, 4H, H], b [n_sig, 4H]: one weight set per signature,
    drawn like make_values from different streams."""
    cfg = CONFIGS[cfg_index]
    D = cfg.D if D is None else D
    H = cfg.H if H is None else H
    x = make_values(cfg_index, n_nodes, bias, D, H)[0]
    Ws, Us, bs = [], [], []
    for t in range(n_sig):
        rng = np.random.default_rng(5000 + 17 * cfg.index + t)
        kw, ku = 1.0 / np.sqrt(D), 1.0 / np.sqrt(H)
        Ws.append(rng.uniform(-kw, kw, size=(4 * H, D)).astype(np.float32))
        Us.append(rng.uniform(-ku, ku, size=(4 * H, H)).astype(np.float32))
        bs.append(rng.uniform(-0.5, 0.5, size=4 * H).astype(np.float32) if bias == "random"
                  else np.zeros(4 * H, np.float32))
    return x, np.stack(Ws), np.stack(Us), np.stack(bs)


def node_signatures(parent: np.ndarray, n_sig: int, seed: int) -> np.ndarray:
    """sig [N] int32 drawn per NODE: leaves get signature 0 (a "word" cell), every other node one
    of the remaining n_sig - 1 uniformly (n_sig >= 2), so parents and children differ freely."""
    rng = np.random.default_rng(seed)
    n = parent.shape[0]
    has_child = np.zeros(n, dtype=bool)
    has_child[parent[parent >= 0]] = True
    sig = np.zeros(n, dtype=np.int32)
    k = int(has_child.sum())
    sig[has_child] = 1 + rng.integers(0, n_sig - 1, size=k).astype(np.int32)
    return sig


# --------------------------------------------------------------------------
# cells of different type in one table (child-sum next to N-ary cells)
# --------------------------------------------------------------------------
def bounded_arity_forest(n_trees: int, nodes_lo: int, nodes_hi: int, max_children: int, seed: int) -> np.ndarray:
    """Trees of U[nodes_lo, nodes_hi] nodes in which no node has more than max_children children
    (binarised constituency trees for max_children = 2): node v > 0 of a tree attaches to a uniformly
    drawn earlier node that still has a free position.  Root first, trees one after another."""
    rng = np.random.default_rng(seed)
    parts = []
    for _ in range(n_trees):
        n = int(rng.integers(nodes_lo, nodes_hi + 1))
        par = np.full(n, -1, dtype=np.int64)
        free = [0]                               # nodes with a free position
        deg = np.zeros(n, dtype=np.int64)
        for v in range(1, n):
            i = int(rng.integers(0, len(free)))
            p = free[i]
            par[v] = p
            deg[p] += 1
            if deg[p] == max_children:
                free[i] = free[-1]
                free.pop()
            free.append(v)
        parts.append(par.astype(np.int32))
    return _concat(parts)


def arity_signatures(parent: np.ndarray, positions, seed: int) -> np.ndarray:
    """sig [N] int32 for a table of len(positions) cells; positions[t] = the number of child positions
    of cell t (0: any number, a child-sum cell).  Every node draws uniformly among the cells that can
    take its number of children, so parents and children differ freely."""
    rng = np.random.default_rng(seed)
    n = parent.shape[0]
    arity = np.bincount(parent[parent >= 0], minlength=n)
    positions = np.asarray(positions)
    u = rng.random(n)
    sig = np.empty(n, dtype=np.int32)
    for a in np.unique(arity):
        ok = np.flatnonzero((positions == 0) | (positions >= a))
        if ok.size == 0:
            raise ValueError(f"no cell can take a node with {a} children")
        m = arity == a
        sig[m] = ok[np.minimum((u[m] * ok.size).astype(np.int64), ok.size - 1)]
    return sig


def make_cell_values(positions, D: int, H: int, seed: int):
    """One (W, U, b) per cell: [4H, D], [4H, H], [4H] for positions[t] = 0 (child-sum), else
    [(3+N)H, D], [(3+N)H, N*H], [(3+N)H] with N = positions[t].  Uniform like make_values_typed; U of
    an N-ary cell is scaled by its fan-in N*H."""
    out = []
    for t, N in enumerate(positions):
        rng = np.random.default_rng(seed + 31 * t)
        rows = 4 * H if N == 0 else (3 + N) * H
        cols = H if N == 0 else N * H
        kw, ku = 1.0 / np.sqrt(D), 1.0 / np.sqrt(cols)
        out.append((rng.uniform(-kw, kw, size=(rows, D)).astype(np.float32),
                    rng.uniform(-ku, ku, size=(rows, cols)).astype(np.float32),
                    rng.uniform(-0.5, 0.5, size=rows).astype(np.float32)))
    return out
