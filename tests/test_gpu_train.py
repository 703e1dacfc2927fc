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
    h2, c2 = J.jitdb_treelstm_forward(*dev, s)
    torch.cuda.synchronize()
    assert torch.equal(h, h2) and torch.equal(c, c2)
    ho, co, go, fo = B.forward_saved(parent, *seen)
    tol = TOL[dtype]
    assert np.abs(h.float().cpu().numpy() - ho).max() <= tol
    assert np.abs(gates.cpu().numpy() - go).max() <= tol
    has_parent = parent >= 0
    assert np.abs(fgate.cpu().numpy()[has_parent] - fo[has_parent]).max() <= tol
    assert not fgate.cpu().numpy()[~has_parent].any()          # rows of roots stay as handed in (zeros)


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
