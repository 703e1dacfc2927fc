"""GPU parity of the depth x signature batcher: jitdb_schedule_typed (bit-exact against the
typed schedule oracle) and jitdb_treelstm_forward_typed (states within the forward's tolerances).

The expected states at sizes the numpy oracle is too slow for come from the C oracle run on each
signature's sub-forest with that signature's weights; tests/test_oracle_typed.py pins that this is
what the typed oracle computes when signatures are constant inside trees."""
import numpy as np
import pytest

from oracle import schedule_oracle as S
from oracle import treelstm_oracle as T
from oracle import treelstm_typed_oracle as TT
from workloads import (make_forest, make_values_typed, tree_signatures, node_signatures, mixed_forest, tree_ranges,
                       relabel, chain_forest)
from gpu_util import dev_parent, bf16_tensor, assert_schedule_equal

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _typed_equal(got, want):
    assert_schedule_equal(got, want)
    assert np.array_equal(got["key"], want["key"])
    assert np.array_equal(got["slot_ptr"], want["slot_ptr"])
    assert np.array_equal(got["host_slot_ptr"], want["slot_ptr"])


def _sched(p, sig, n_sig, **kw):
    import paper_1904_07421_amd as J
    return J.jitdb_schedule_typed(dev_parent(p), dev_parent(sig), n_sig, **kw)


@pytest.mark.parametrize("cfg,n_sig", [(1, 2), (2, 2), (2, 3), (3, 2), (3, 16), (4, 4), (5, 2)])
def test_typed_schedule_bit_exact(cfg, n_sig):
    p = make_forest(cfg)
    sig = tree_signatures(p, n_sig, 10 + cfg)
    print(f"typed schedule cfg={cfg} n_sig={n_sig} N={p.shape[0]}", flush=True)
    got = _sched(p, sig, n_sig).to_numpy()
    want = S.schedule_typed(p, sig, n_sig) if p.shape[0] < 6000 else S.schedule_typed_fast(p, sig, n_sig)
    _typed_equal(got, want)


@pytest.mark.parametrize("cfg,n_sig", [(1, 2), (2, 3), (3, 2), (4, 3), (5, 2)])
def test_typed_schedule_signatures_per_node(cfg, n_sig):
    """Leaves under one cell, inner nodes under others: parents and children differ, every sub-slot is used."""
    p = make_forest(cfg)
    sig = node_signatures(p, n_sig, 30 + cfg)
    print(f"typed schedule per-node cfg={cfg} n_sig={n_sig} N={p.shape[0]}", flush=True)
    got = _sched(p, sig, n_sig).to_numpy()
    want = S.schedule_typed(p, sig, n_sig) if p.shape[0] < 6000 else S.schedule_typed_fast(p, sig, n_sig)
    _typed_equal(got, want)


def test_typed_schedule_mixed_and_relabelled():
    p, sig = mixed_forest(3, 500, 700, 2, 90, 1)
    print(f"typed schedule mixed N={p.shape[0]}", flush=True)
    _typed_equal(_sched(p, sig, 2).to_numpy(), S.schedule_typed_fast(p, sig, 2))
    q, new_of_old = relabel(p, 9)
    sig_q = np.empty_like(sig)
    sig_q[new_of_old] = sig
    _typed_equal(_sched(q, sig_q, 2).to_numpy(), S.schedule_typed_fast(q, sig_q, 2))


def test_one_signature_equals_plain_schedule_and_unused_signatures_give_empty_slots():
    import paper_1904_07421_amd as J
    p = make_forest(3)
    plain = J.jitdb_schedule(dev_parent(p)).to_numpy()
    one = _sched(p, np.zeros_like(p), 1).to_numpy()
    assert_schedule_equal(one, plain)
    assert np.array_equal(one["slot_ptr"], plain["level_ptr"])
    sig = 2 * tree_signatures(p, 2, 3)                       # signatures 0 and 2 of 4: 1 and 3 never occur
    got = _sched(p, sig, 4).to_numpy()
    _typed_equal(got, S.schedule_typed_fast(p, sig, 4))
    sp = got["slot_ptr"]
    assert (sp[4::16][:got["n_levels"]] == sp[8::16][:got["n_levels"]]).all()    # slot (l, 1) is empty


def test_deep_chain_many_slots():
    p = chain_forest(3000, 2)
    sig = np.concatenate([np.zeros(3000, np.int32), np.full(3000, 2, np.int32)])
    _typed_equal(_sched(p, sig, 3).to_numpy(), S.schedule_typed_fast(p, sig, 3))


def test_typed_schedule_errors():
    import torch
    import paper_1904_07421_amd as J
    p = make_forest(1)
    sig = tree_signatures(p, 2, 0)
    bad = sig.copy(); bad[3] = 2
    with pytest.raises(J.JitdbError) as e:
        _sched(p, bad, 2)
    assert e.value.code == -8
    bad = sig.copy(); bad[0] = -1
    with pytest.raises(J.JitdbError) as e:
        _sched(p, bad, 2)
    assert e.value.code == -8
    with pytest.raises(J.JitdbError) as e:
        _sched(p, sig, 0)
    assert e.value.code == -2
    with pytest.raises(J.JitdbError) as e:
        _sched(p, sig, 2, slot_capacity=3)
    assert e.value.code == -5
    with pytest.raises(J.JitdbError) as e:                      # forest errors are still reported
        _sched(np.array([1, 0], np.int32), np.zeros(2, np.int32), 1)
    assert e.value.code == -4
    s = J.jitdb_schedule_typed(torch.empty(0, dtype=torch.int32, device="cuda"),
                               torch.empty(0, dtype=torch.int32, device="cuda"), 2)
    assert s.n_levels == 0 and s.host_slot_ptr[0] == 0


# ---- forward ---------------------------------------------------------------------------
def _gpu_forward_typed(p, sig, n_sig, x, W, U, b, dtype):
    import torch
    import paper_1904_07421_amd as J
    s = _sched(p, sig, n_sig)
    bt = torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).cuda()
    if dtype == "bf16":
        xt, xo = bf16_tensor(x)
        Wt, Wo = bf16_tensor(W)
        Ut, Uo = bf16_tensor(U)
    else:
        xt, Wt, Ut = (torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda() for a in (x, W, U))
        xo, Wo, Uo = x, W, U
    h, c = J.jitdb_treelstm_forward_typed(xt, Wt, Ut, bt, s)
    torch.cuda.synchronize()
    return s, h.float().cpu().numpy(), c.cpu().numpy(), (xo, Wo, Uo, b)


def _per_signature_oracle(c_oracle, p, sig, n_sig, seen, trees=None):
    """Expected (rows, h, c): the C oracle on each signature's trees (all of them, or the listed ones)."""
    xo, Wo, Uo, bo = seen
    r = tree_ranges(p)
    trees = np.arange(len(r) - 1) if trees is None else np.asarray(trees)
    rows_all, h_all, c_all = [], [], []
    for t in range(n_sig):
        mine = [k for k in trees if sig[r[k]] == t]
        if not mine:
            continue
        rows = np.concatenate([np.arange(r[k], r[k + 1]) for k in mine])
        sub, off = [], 0
        for k in mine:
            sp = p[r[k]:r[k + 1]].astype(np.int64)
            sub.append(np.where(sp < 0, -1, sp - r[k] + off))
            off += r[k + 1] - r[k]
        ho, co, _ = c_oracle(np.concatenate(sub).astype(np.int32), xo[rows], Wo[t], Uo[t], bo[t])
        rows_all.append(rows); h_all.append(ho); c_all.append(co)
    return np.concatenate(rows_all), np.concatenate(h_all), np.concatenate(c_all)


@pytest.mark.parametrize("cfg,n_sig,dtype", [(1, 2, "f32"), (2, 2, "f32"), (2, 3, "bf16")])
def test_typed_forward_small_against_the_typed_oracle(cfg, n_sig, dtype):
    p = make_forest(cfg)
    sig = tree_signatures(p, n_sig, 5)
    x, W, U, b = make_values_typed(cfg, p.shape[0], n_sig)
    print(f"typed forward cfg={cfg} n_sig={n_sig} {dtype} N={p.shape[0]}", flush=True)
    _, h, c, (xo, Wo, Uo, bo) = _gpu_forward_typed(p, sig, n_sig, x, W, U, b, dtype)
    ho, co = TT.forward_typed(p, sig, xo, Wo, Uo, bo)
    eh, ec = float(np.abs(h - ho).max()), float(np.abs(c - co).max())
    print(f"  max|dh|={eh:.3e} max|dc|={ec:.3e}", flush=True)
    assert eh <= TOL[dtype] and ec <= TOL[dtype]


@pytest.mark.timeout(300)
@pytest.mark.parametrize("cfg,n_sig,dtype", [(1, 2, "f32"), (2, 3, "f32"), (2, 2, "bf16"), (3, 3, "bf16"), (4, 2, "f32")])
def test_typed_forward_signatures_per_node(cfg, n_sig, dtype):
    """Cells differ along edges: the forget gate on a child uses the parent cell's W_f, U_f, b_f.
    Every node against the typed oracle (config 3 reaches the grouped launch, config 4 the per-sub-slot
    projections of 128 thin levels)."""
    p = make_forest(cfg)
    if cfg == 4:
        p = p[:tree_ranges(p)[600]]             # keeps the numpy oracle to seconds
    sig = node_signatures(p, n_sig, 40 + cfg)
    x, W, U, b = make_values_typed(cfg, p.shape[0], n_sig)
    print(f"typed forward per-node cfg={cfg} n_sig={n_sig} {dtype} N={p.shape[0]}", flush=True)
    _, h, c, (xo, Wo, Uo, bo) = _gpu_forward_typed(p, sig, n_sig, x, W, U, b, dtype)
    ho, co = TT.forward_typed(p, sig, xo, Wo, Uo, bo)
    eh, ec = float(np.abs(h - ho).max()), float(np.abs(c - co).max())
    print(f"  max|dh|={eh:.3e} max|dc|={ec:.3e}", flush=True)
    tol_c = TOL[dtype] * max(1.0, float(np.abs(co).max()) / 8.0)      # |c| grows with the arity (stars of config 4)
    assert eh <= TOL[dtype] and ec <= tol_c


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_typed_forward_trees_and_sequences_in_one_table(c_oracle, dtype):
    """A Tree-LSTM batch (signature 0) and a variable-length LSTM batch written as chains
    (signature 1, its own weights), every node checked."""
    p, sig = mixed_forest(3, 600, 900, 2, 120, 4)
    x, W, U, b = make_values_typed(3, p.shape[0], 2)
    print(f"typed forward mixed {dtype} N={p.shape[0]}", flush=True)
    _, h, c, seen = _gpu_forward_typed(p, sig, 2, x, W, U, b, dtype)
    rows, ho, co = _per_signature_oracle(c_oracle, p, sig, 2, seen)
    assert rows.shape[0] == p.shape[0]
    eh, ec = float(np.abs(h[rows] - ho).max()), float(np.abs(c[rows] - co).max())
    print(f"  max|dh|={eh:.3e} max|dc|={ec:.3e}", flush=True)
    assert eh <= TOL[dtype] and ec <= TOL[dtype]


@pytest.mark.timeout(400)
@pytest.mark.parametrize("cfg,n_sig", [(3, 16), (4, 3), (5, 2)])
def test_typed_forward_full_size_sampled_trees(c_oracle, cfg, n_sig):
    from workloads import CONFIGS
    dtype = CONFIGS[cfg].dtype
    p = make_forest(cfg)
    sig = tree_signatures(p, n_sig, 21)
    x, W, U, b = make_values_typed(cfg, p.shape[0], n_sig, bias="zero")
    print(f"typed forward cfg={cfg} n_sig={n_sig} {dtype} N={p.shape[0]} (oracle on sampled trees)", flush=True)
    _, h, c, seen = _gpu_forward_typed(p, sig, n_sig, x, W, U, b, dtype)
    assert np.isfinite(h).all() and np.isfinite(c).all()
    r = tree_ranges(p)
    rng = np.random.default_rng(3)
    pick = np.unique(np.concatenate([rng.choice(len(r) - 1, size=120, replace=False),
                                     [int(np.argmax(np.diff(r)))], np.arange(6)]))
    rows, ho, co = _per_signature_oracle(c_oracle, p, sig, n_sig, seen, trees=pick)
    eh, ec = float(np.abs(h[rows] - ho).max()), float(np.abs(c[rows] - co).max())
    print(f"  max|dh|={eh:.3e} max|dc|={ec:.3e}", flush=True)
    assert eh <= TOL[dtype] and ec <= TOL[dtype]


def test_one_signature_matches_the_plain_forward():
    import torch
    import paper_1904_07421_amd as J
    p = make_forest(3)
    x, W, U, b = make_values_typed(3, p.shape[0], 1)
    _, h, c, _ = _gpu_forward_typed(p, np.zeros_like(p), 1, x, W, U, b, "f32")
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    s = J.jitdb_schedule(dev_parent(p))
    # the plain forward over the same launches as the table's: without the children-per-level counts it
    # does not take the single-launch kernels for thin levels, which the typed forward does not have
    s.host_level_kids[:] = -1
    h0, c0 = J.jitdb_treelstm_forward(dev(x), dev(W[0]), dev(U[0]), dev(b[0]), s)
    assert np.array_equal(h, h0.cpu().numpy()) and np.array_equal(c, c0.cpu().numpy())


def test_typed_forward_rejects_mismatched_tables():
    import torch
    import paper_1904_07421_amd as J
    p = make_forest(1)
    sig = tree_signatures(p, 2, 0)
    x, W, U, b = make_values_typed(1, p.shape[0], 2)
    s = _sched(p, sig, 2)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    with pytest.raises(ValueError):
        J.jitdb_treelstm_forward_typed(dev(x), dev(W[:1]), dev(U[:1]), dev(b[:1]), s)
    s.host_slot_ptr[1] = s.host_slot_ptr[2] + 1                  # a corrupted table is refused, not run
    with pytest.raises(J.JitdbError) as e:
        J.jitdb_treelstm_forward_typed(dev(x), dev(W), dev(U), dev(b), s)
    assert e.value.code == -7


def test_packed_weights_on_a_typed_table():
    import torch
    import paper_1904_07421_amd as J
    p = make_forest(3)
    sig = node_signatures(p, 3, 8)
    x, W, U, b = make_values_typed(3, p.shape[0], 3)
    s = _sched(p, sig, 3)
    xt, Wt, Ut = bf16_tensor(x)[0], bf16_tensor(W)[0], bf16_tensor(U)[0]
    bt = torch.from_numpy(b).cuda()
    h0, c0 = J.jitdb_treelstm_forward_typed(xt, Wt, Ut, bt, s)
    pk = J.jitdb_treelstm_pack(Wt, Ut, bt)
    h1, c1 = J.jitdb_treelstm_forward_packed(xt, pk, s)
    assert torch.equal(h0, h1) and torch.equal(c0, c1)
