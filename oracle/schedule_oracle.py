"""Schedule oracle: what the batching analysis must produce for a forest.

The paper files every computation node in a table keyed by its depth in the
computation graph; nodes of one depth are independent and run as one batch, and
slots are visited in depth order (section 4.2, section 4.3).  For a tree
evaluated bottom-up that depth is the node's HEIGHT: 0 for a leaf, otherwise
1 + the largest height among its children.

The paper does not fix an order inside a slot or among children.  The reading
used here, needed for a bit-exact contract: ascending node id in both.

Test infrastructure only; plain Python/numpy, no code shared with the GPU path.
"""
from __future__ import annotations

import numpy as np


class ForestError(ValueError):
    def __init__(self, kind: str, msg: str):
        super().__init__(msg)
        self.kind = kind   # "range" | "cycle"


def validate(parent) -> None:
    """Every parent is -1 or a node id other than the node itself, and walking
    parents from any node reaches -1 within N steps."""
    parent = np.asarray(parent)
    n = parent.shape[0]
    for v in range(n):
        p = int(parent[v])
        if p < -1 or p >= n or p == v:
            raise ForestError("range", f"parent[{v}] = {p} is not a valid parent")
    # state: 0 unknown, 1 on current walk, 2 known to reach a root
    state = np.zeros(n, dtype=np.int8)
    for v in range(n):
        path = []
        w = v
        while w != -1 and state[w] == 0:
            state[w] = 1
            path.append(w)
            w = int(parent[w])
        if w != -1 and state[w] == 1:
            raise ForestError("cycle", f"node {w} is its own ancestor")
        for q in path:
            state[q] = 2


def children_lists(parent):
    """children[j] = ids v with parent[v] == j, ascending."""
    parent = np.asarray(parent)
    n = parent.shape[0]
    ch = [[] for _ in range(n)]
    for v in range(n):          # ascending v => ascending lists
        p = int(parent[v])
        if p >= 0:
            ch[p].append(v)
    return ch


def heights(parent) -> np.ndarray:
    """height[v] = 0 for a leaf, else 1 + max over children (iterative postorder)."""
    parent = np.asarray(parent)
    n = parent.shape[0]
    ch = children_lists(parent)
    h = np.zeros(n, dtype=np.int32)
    for r in range(n):
        if parent[r] != -1:
            continue
        stack = [(r, 0)]
        while stack:
            v, i = stack.pop()
            if i < len(ch[v]):
                stack.append((v, i + 1))
                stack.append((ch[v][i], 0))
            else:
                h[v] = 0 if not ch[v] else 1 + max(int(h[k]) for k in ch[v])
    return h


def heights_bruteforce(parent) -> np.ndarray:
    """Independent twin: height[j] = the largest number of parent steps that
    lead from some node v up to j.  O(N * depth); for tiny forests."""
    parent = np.asarray(parent)
    n = parent.shape[0]
    h = np.zeros(n, dtype=np.int32)
    for v in range(n):
        steps = 0
        w = int(parent[v])
        while w != -1:
            steps += 1
            if steps > h[w]:
                h[w] = steps
            w = int(parent[w])
    return h


def schedule(parent) -> dict:
    """Full schedule of a forest.

    Returns a dict of int32 arrays:
      height[N], level_ptr[L+1], perm[N] (position -> id, sorted by (height, id)),
      inv_perm[N] (id -> position), child_ptr[N+1], child_idx[E]
    and ints n_levels (L), n_edges (E = N - number of roots).
    """
    parent = np.asarray(parent)
    n = parent.shape[0]
    validate(parent)
    ch = children_lists(parent)
    child_ptr = np.zeros(n + 1, dtype=np.int32)
    for j in range(n):
        child_ptr[j + 1] = child_ptr[j] + len(ch[j])
    child_idx = np.array([k for j in range(n) for k in ch[j]], dtype=np.int32)
    h = heights(parent)
    L = int(h.max()) + 1 if n else 0
    order = sorted(range(n), key=lambda v: (int(h[v]), v))
    perm = np.array(order, dtype=np.int32)
    inv_perm = np.zeros(n, dtype=np.int32)
    for pos, v in enumerate(order):
        inv_perm[v] = pos
    level_ptr = np.zeros(L + 1, dtype=np.int32)
    for lvl in range(L + 1):
        level_ptr[lvl] = int(np.count_nonzero(h < lvl))
    return dict(height=h, level_ptr=level_ptr, perm=perm, inv_perm=inv_perm,
                child_ptr=child_ptr, child_idx=child_idx,
                n_levels=L, n_edges=int(child_ptr[n]))


def level_kids(parent) -> np.ndarray:
    """kids[l] = number of children of the nodes of level l (0 for the leaves), l < L: every non-root
    node counts once, for the level of its parent.  Derived data of the schedule (the sum of the
    arities over a level); the forward only uses it to pick kernels."""
    parent = np.asarray(parent)
    validate(parent)
    h = heights(parent)
    L = int(h.max()) + 1 if parent.shape[0] else 0
    kids = np.zeros(L, dtype=np.int64)
    for v in range(parent.shape[0]):
        if parent[v] >= 0:
            kids[int(h[int(parent[v])])] += 1
    return kids


def schedule_fast(parent) -> dict:
    """Same outputs as `schedule` for large forests, using numpy routines
    (stable argsort, bincount) and a level-by-level height sweep.  Checked
    against `schedule` in the CPU tests; used where `schedule` is too slow."""
    parent = np.asarray(parent).astype(np.int64)
    n = parent.shape[0]
    if n == 0:
        z = np.zeros(0, dtype=np.int32)
        return dict(height=z, level_ptr=np.zeros(1, np.int32), perm=z, inv_perm=z,
                    child_ptr=np.zeros(1, np.int32), child_idx=z, n_levels=0, n_edges=0)
    if ((parent < -1) | (parent >= n) | (parent == np.arange(n))).any():
        raise ForestError("range", "invalid parent")
    nonroot = np.flatnonzero(parent >= 0)
    cnt = np.bincount(parent[nonroot], minlength=n)
    child_ptr = np.concatenate(([0], np.cumsum(cnt))).astype(np.int32)
    child_idx = nonroot[np.argsort(parent[nonroot], kind="stable")].astype(np.int32)
    # peel leaves upward: a node's height is final once all children reported
    h = np.zeros(n, dtype=np.int64)
    remaining = cnt.copy()
    frontier = np.flatnonzero(cnt == 0)
    done = 0
    while frontier.size:
        done += frontier.size
        p = parent[frontier]
        ok = p >= 0
        p = p[ok]
        np.maximum.at(h, p, h[frontier[ok]] + 1)
        np.subtract.at(remaining, p, 1)
        up = np.unique(p)
        frontier = up[remaining[up] == 0]
    if done != n:
        raise ForestError("cycle", "some node never becomes ready: cycle")
    L = int(h.max()) + 1
    perm = np.lexsort((np.arange(n), h)).astype(np.int32)
    inv_perm = np.empty(n, dtype=np.int32)
    inv_perm[perm] = np.arange(n, dtype=np.int32)
    level_ptr = np.concatenate(([0], np.cumsum(np.bincount(h, minlength=L)))).astype(np.int32)
    return dict(height=h.astype(np.int32), level_ptr=level_ptr, perm=perm,
                inv_perm=inv_perm, child_ptr=child_ptr, child_idx=child_idx,
                n_levels=L, n_edges=int(child_ptr[n]))


def concat_forests(parent_a, parent_b) -> np.ndarray:
    """Parent array of forest A followed by forest B: B's node v becomes node len(A) + v
    (roots stay -1).  This is what "appending trees" means; the schedule of an appended
    forest is by definition `schedule(concat_forests(a, b))` (section 2: new work joins
    while earlier work is in flight; sections 4.2-4.3 define the table it joins)."""
    a = np.asarray(parent_a, dtype=np.int64)
    b = np.asarray(parent_b, dtype=np.int64)
    shifted = np.where(b >= 0, b + a.shape[0], b)
    return np.concatenate([a, shifted]).astype(np.int32)


def parent_signatures(parent, sig) -> np.ndarray:
    """psig[v] = signature of v's parent; a root carries its own."""
    parent = np.asarray(parent).astype(np.int64)
    sig = np.asarray(sig)
    return np.where(parent >= 0, sig[np.maximum(parent, 0)], sig).astype(np.int32)


def schedule_typed(parent, sig, n_sig: int) -> dict:
    """The look-up table of the generic batcher (section 4.2): nodes are filed by depth and by
    a signature that stands for (operator type, settings, input layouts).  A node takes part in
    two batched operations with different partners: its own cell, shared with the nodes of its
    (height, sig), and the forget projection its PARENT's cell applies to it, shared with the
    nodes of its (height, parent's sig).  The table therefore files by (height, sig, psig):
    Same outputs as `schedule`, with positions sorted by (height, sig, psig, id), plus
      key[N] = (height * n_sig + sig) * n_sig + psig,
      slot_ptr[L * n_sig^2 + 1]: sub-slot (l, t, p) holds positions
      [slot_ptr[(l*n_sig + t)*n_sig + p], slot_ptr[(l*n_sig + t)*n_sig + p + 1]);
      slot (l, t), the cell's batch, is the run of its n_sig sub-slots.
    Plain Python: sorted() on tuples and counting."""
    parent = np.asarray(parent)
    sig = np.asarray(sig)
    n = parent.shape[0]
    if sig.shape[0] != n or ((sig < 0) | (sig >= n_sig)).any():
        raise ForestError("range", "signature outside [0, n_sig)")
    out = schedule(parent)
    h = out["height"]
    L = out["n_levels"]
    psig = parent_signatures(parent, sig)
    order = sorted(range(n), key=lambda v: (int(h[v]), int(sig[v]), int(psig[v]), v))
    perm = np.array(order, dtype=np.int32)
    inv_perm = np.zeros(n, dtype=np.int32)
    for pos, v in enumerate(order):
        inv_perm[v] = pos
    key = ((h.astype(np.int64) * n_sig + sig) * n_sig + psig).astype(np.int32)
    S = L * n_sig * n_sig
    slot_ptr = np.zeros(S + 1, dtype=np.int32)
    for q in range(S + 1):
        slot_ptr[q] = int(np.count_nonzero(key < q))
    out.update(perm=perm, inv_perm=inv_perm, key=key, slot_ptr=slot_ptr, n_sig=n_sig)
    return out


def schedule_typed_fast(parent, sig, n_sig: int) -> dict:
    """schedule_typed with numpy routines (lexsort, bincount), for large forests; checked
    against schedule_typed in the CPU tests."""
    sig = np.asarray(sig).astype(np.int64)
    out = schedule_fast(parent)
    n = sig.shape[0]
    if ((sig < 0) | (sig >= n_sig)).any():
        raise ForestError("range", "signature outside [0, n_sig)")
    h = out["height"].astype(np.int64)
    L = out["n_levels"]
    key = (h * n_sig + sig) * n_sig + parent_signatures(parent, sig)
    perm = np.lexsort((np.arange(n), key)).astype(np.int32)
    inv_perm = np.empty(n, dtype=np.int32)
    inv_perm[perm] = np.arange(n, dtype=np.int32)
    slot_ptr = np.concatenate(([0], np.cumsum(np.bincount(key, minlength=L * n_sig * n_sig)))).astype(np.int32)
    out.update(perm=perm, inv_perm=inv_perm, key=key.astype(np.int32), slot_ptr=slot_ptr, n_sig=n_sig)
    return out
