"""Training entry points against the gradient oracle (GPU)."""
import numpy as np
import pytest
import torch

import paper_1904_07421_amd as J
from oracle import treelstm_backward_oracle as B
from workloads import make_forest, make_values, to_bf16_bits, bf16_bits_to_f32, chain_forest, star_forest

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


def _upload(x, W, U, b, dtype):
    if dtype == "bf16":
        bits = [to_bf16_bits(a) for a in (x, W, U)]
        dev = [torch.from_numpy(t.view(np.int16)).view(torch.bfloat16).cuda() for t in bits]
        seen = [bf16_bits_to_f32(t) for t in bits]
    else:
        dev = [torch.from_numpy(a).cuda() for a in (x, W, U)]
        seen = [x, W, U]
    return dev + [torch.from_numpy(b).cuda()], seen + [b]


def _forest(kind):
    if kind == "cfg1":
        return make_forest(1)
    if kind == "cfg2":
        return make_forest(2)
    if kind == "mix":
        a, c, s = make_forest(1), chain_forest(9, 2), star_forest(20, 2)
        parts, off = [], 0
        for p in (a, c, s):
            parts.append(np.where(p < 0, -1, p + off)); off += len(p)
        return np.concatenate(parts).astype(np.int32)
    raise ValueError(kind)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kind,D,H", [("cfg1", 300, 150), ("cfg2", 300, 150), ("mix", 20, 36), ("cfg2", 64, 64)])
def test_training_forward_keeps_the_gate_activations(kind, D, H, dtype):
    parent = _forest(kind)
    x, W, U, b = make_values(1, len(parent), "random", D=D, H=H)
    print(f"forward_train {kind} D={D} H={H} dtype={dtype} N={len(parent)}", flush=True)
    dev, seen = _upload(x, W, U, b, dtype)
    s = J.jitdb_schedule(torch.from_numpy(parent).cuda())
    h, c, gates, fgate = J.jitdb_treelstm_forward_train(*dev, s)
    # the plain forward over the same launches: without the children-per-level counts it cannot pick
    # the single-launch kernel for levels of one-child nodes, which the training forward does not have
    kids = s.host_level_kids.copy()
    s.host_level_kids[:] = -1
    h2, c2 = J.jitdb_treelstm_forward(*dev, s)
    torch.cuda.synchronize()
    s.host_level_kids[:] = kids
    assert torch.equal(h, h2) and torch.equal(c, c2)
    ho, co, go, fo = B.forward_saved(parent, *seen)
    tol = TOL[dtype]
    assert np.abs(h.float().cpu().numpy() - ho).max() <= tol
    assert np.abs(gates.float().cpu().numpy() - go).max() <= tol
    has_parent = parent >= 0
    assert np.abs(fgate.float().cpu().numpy()[has_parent] - fo[has_parent]).max() <= tol
    assert not fgate.float().cpu().numpy()[~has_parent].any()          # rows of roots stay as handed in (zeros)


def _rel(got, want):
    return float(np.abs(got - want).max() / max(1.0, np.abs(want).max()))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("kind,D,H", [("cfg1", 300, 150), ("cfg2", 300, 150), ("mix", 20, 36), ("cfg2", 64, 64),
                                      ("mix", 7, 33)])
def test_backward_against_the_gradient_oracle(kind, D, H, dtype):
    parent = _forest(kind)
    n = len(parent)
    x, W, U, b = make_values(1, n, "random", D=D, H=H)
    rng = np.random.default_rng(11)
    gh = rng.standard_normal((n, H)).astype(np.float32)
    gc = rng.standard_normal((n, H)).astype(np.float32)
    print(f"backward {kind} D={D} H={H} dtype={dtype} N={n}", flush=True)
    dev, seen = _upload(x, W, U, b, dtype)
    s = J.jitdb_schedule(torch.from_numpy(parent).cuda())
    h, c, gates, fgate = J.jitdb_treelstm_forward_train(*dev, s)
    dx, dW, dU, db = J.jitdb_treelstm_backward(dev[0], dev[1], dev[2], s, h, c, gates, fgate,
                                               torch.from_numpy(gh).cuda(), torch.from_numpy(gc).cuda())
    torch.cuda.synchronize()
    _, _, rx, rW, rU, rb = B.forward_backward(parent, *seen, gh, gc)
    tol = {"f32": 1e-4, "bf16": 2e-2}[dtype]
    errs = {k: _rel(g.cpu().numpy(), r) for k, g, r in (("dx", dx, rx), ("dW", dW, rW), ("dU", dU, rU), ("db", db, rb))}
    print("   relative-to-max errors:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert v <= tol, (k, v)


def _sampled_backward_check(cfg, n_sample, dtype, D=None, H=None):
    """Full-size forest on the GPU; cotangents are non-zero only on sampled trees, so that the
    oracle, run on those trees alone, predicts every output: dx on their rows (zero elsewhere)
    and dW, dU, db in full.  Saved activations are checked on the same rows."""
    from workloads import CONFIGS, tree_ranges
    cfgo = CONFIGS[cfg]
    parent = make_forest(cfg)
    n = len(parent)
    x, W, U, b = make_values(cfg, n, "random", D=D, H=H)
    H_ = U.shape[1]
    r = tree_ranges(parent)
    T_ = len(r) - 1
    rng = np.random.default_rng(123)
    pick = np.unique(np.concatenate([rng.choice(T_, size=min(n_sample, T_), replace=False),
                                     [int(np.argmax(np.diff(r)))], np.arange(min(4, T_))]))
    rows = np.concatenate([np.arange(r[t], r[t + 1]) for t in pick])
    gh = np.zeros((n, H_), dtype=np.float32); gc = np.zeros((n, H_), dtype=np.float32)
    gh[rows] = rng.standard_normal((len(rows), H_)).astype(np.float32)
    gc[rows] = rng.standard_normal((len(rows), H_)).astype(np.float32)
    print(f"backward cfg={cfg} dtype={dtype} D={x.shape[1]} H={H_} N={n}, cotangents on {len(pick)} trees "
          f"({len(rows)} nodes)", flush=True)
    dev, seen = _upload(x, W, U, b, dtype)
    s = J.jitdb_schedule(torch.from_numpy(parent).cuda())
    h, c, gates, fgate = J.jitdb_treelstm_forward_train(*dev, s)
    dx, dW, dU, db = J.jitdb_treelstm_backward(dev[0], dev[1], dev[2], s, h, c, gates, fgate,
                                               torch.from_numpy(gh).cuda(), torch.from_numpy(gc).cuda())
    torch.cuda.synchronize()
    # oracle on the sampled trees, re-based to a forest of their own
    sub, off = [], 0
    for t in pick:
        p = parent[r[t]:r[t + 1]].astype(np.int64)
        sub.append(np.where(p < 0, -1, p - r[t] + off)); off += r[t + 1] - r[t]
    sub = np.concatenate(sub).astype(np.int32)
    xo, Wo, Uo, bo = seen
    ho, co, rx, rW, rU, rb = B.forward_backward(sub, xo[rows], Wo, Uo, bo, gh[rows], gc[rows])
    _, _, go, fo = B.forward_saved(sub, xo[rows], Wo, Uo, bo)
    tol = TOL[dtype]
    dxn = dx.cpu().numpy()
    errs = {"dx": _rel(dxn[rows], rx), "dW": _rel(dW.cpu().numpy(), rW), "dU": _rel(dU.cpu().numpy(), rU),
            "db": _rel(db.cpu().numpy(), rb), "gates": float(np.abs(gates.float().cpu().numpy()[rows] - go).max())}
    hp = sub >= 0
    errs["fgate"] = float(np.abs(fgate.float().cpu().numpy()[rows][hp] - fo[hp]).max())
    print("   errors:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    mask = np.ones(n, dtype=bool); mask[rows] = False
    assert not dxn[mask].any()                      # no cotangent reaches the other trees
    for k, v in errs.items():
        assert v <= tol, (k, v)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("cfg,dtype,n_sample", [(3, "bf16", 200), (3, "f32", 200), (4, "f32", 120), (5, "bf16", 24)])
def test_backward_at_full_size_with_cotangents_on_sampled_trees(cfg, dtype, n_sample):
    _sampled_backward_check(cfg, n_sample, dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_odd_sizes_on_large_levels(dtype):
    _sampled_backward_check(3, 100, dtype, D=52, H=100)


def test_backward_without_cotangents_and_on_an_empty_forest():
    parent = make_forest(1)
    n = len(parent)
    x, W, U, b = make_values(1, n, "random")
    dev, _ = _upload(x, W, U, b, "f32")
    s = J.jitdb_schedule(torch.from_numpy(parent).cuda())
    h, c, gates, fgate = J.jitdb_treelstm_forward_train(*dev, s)
    print("backward with gh = gc = None", flush=True)
    dx, dW, dU, db = J.jitdb_treelstm_backward(dev[0], dev[1], dev[2], s, h, c, gates, fgate)
    torch.cuda.synchronize()
    assert not dx.any() and not dW.any() and not dU.any() and not db.any()
    print("backward on an empty forest", flush=True)
    e = J.jitdb_schedule(torch.zeros(0, dtype=torch.int32, device="cuda"))
    z = lambda *shape: torch.zeros(shape, device="cuda")
    dx, dW, dU, db = J.jitdb_treelstm_backward(z(0, 300), dev[1], dev[2], e, z(0, 150), z(0, 150), z(0, 450), z(0, 150),
                                               out=(z(0, 300), torch.ones(600, 300, device="cuda"),
                                                    torch.ones(600, 150, device="cuda"), torch.ones(600, device="cuda")))
    torch.cuda.synchronize()
    assert not dW.any() and not dU.any() and not db.any()


def test_backward_on_sequences_against_the_library_lstm_autograd():
    """Chains through the HIP training step, the same sequences through torch.nn.LSTM and its own
    autograd on the CPU (fp64): gradients of L = sum <gh_t, h_t> compared directly, no oracle between."""
    rng = np.random.default_rng(21)
    D, H = 24, 32
    lens = rng.integers(1, 40, size=60)
    W = (rng.uniform(-1, 1, (4 * H, D)) / np.sqrt(D)).astype(np.float32)
    U = (rng.uniform(-1, 1, (4 * H, H)) / np.sqrt(H)).astype(np.float32)
    b = rng.uniform(-0.5, 0.5, 4 * H).astype(np.float32)
    parts, off = [], 0
    for n in lens:
        parts.append(np.where(np.arange(n) == 0, -1, np.arange(n) - 1 + off)); off += n
    parent = np.concatenate(parts).astype(np.int32)
    N = parent.shape[0]
    x = rng.standard_normal((N, D)).astype(np.float32)
    gh = rng.standard_normal((N, H)).astype(np.float32)
    dev = [torch.from_numpy(a).cuda() for a in (x, W, U, b)]
    s = J.jitdb_schedule(torch.from_numpy(parent).cuda())
    h, c, gates, fgate = J.jitdb_treelstm_forward_train(*dev, s)
    dx, dW, dU, db = J.jitdb_treelstm_backward(dev[0], dev[1], dev[2], s, h, c, gates, fgate,
                                               torch.from_numpy(gh).cuda(), None)
    torch.cuda.synchronize()

    def torch_rows(M):            # our gate order (i, o, u, f) -> torch's (i, f, g, o)
        i, o, u, f = (M[g * H:(g + 1) * H] for g in range(4))
        return torch.from_numpy(np.concatenate([i, f, u, o]).astype(np.float64))

    def our_rows(M):              # and back, for the gradients
        i, f, g, o = (M[k * H:(k + 1) * H] for k in range(4))
        return np.concatenate([i, o, g, f])
    lstm = torch.nn.LSTM(D, H).double()
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch_rows(W)); lstm.weight_hh_l0.copy_(torch_rows(U))
        lstm.bias_ih_l0.copy_(torch_rows(b.reshape(-1, 1)).reshape(-1)); lstm.bias_hh_l0.zero_()
    xt = torch.from_numpy(x.astype(np.float64)).requires_grad_(True)
    loss, off = 0.0, 0
    for n in lens:
        seq = xt[off:off + n].flip(0).unsqueeze(1)                         # leaf (last node) first
        out, _ = lstm(seq)
        loss = loss + (out[:, 0, :].flip(0) * torch.from_numpy(gh[off:off + n].astype(np.float64))).sum()
        off += n
    loss.backward()
    want = {"dx": xt.grad.numpy(), "dW": our_rows(lstm.weight_ih_l0.grad.numpy()),
            "dU": our_rows(lstm.weight_hh_l0.grad.numpy()), "db": our_rows(lstm.bias_ih_l0.grad.numpy().reshape(-1, 1)).reshape(-1)}
    got = {"dx": dx, "dW": dW, "dU": dU, "db": db}
    errs = {k: _rel(got[k].cpu().numpy(), want[k]) for k in want}
    print("   sequences vs torch autograd, relative-to-max errors:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert v <= 1e-4, (k, v)
