"""Pins for the gradient oracle (CPU): reverse-mode autograd of an independently written torch
forward, a library LSTM differentiated by the library, central differences of the forward
oracle, and closed forms."""
import numpy as np
import pytest
import torch

from oracle import treelstm_oracle as T
from oracle import treelstm_backward_oracle as B
from workloads import chain_forest, star_forest, make_forest


def _rand(rng, n, D, H, scale=1.0):
    x = rng.standard_normal((n, D))
    W = rng.uniform(-1, 1, (4 * H, D)) * scale / np.sqrt(D)
    U = rng.uniform(-1, 1, (4 * H, H)) * scale / np.sqrt(H)
    b = rng.uniform(-0.5, 0.5, 4 * H)
    return x, W, U, b


def _torch_forest(parent, x, W, U, b, gh, gc):
    """The forest written with torch ops and differentiated by autograd (fp64)."""
    n = len(parent)
    H = U.shape[1]
    xt, Wt, Ut, bt = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (x, W, U, b))
    kids = [[] for _ in range(n)]
    for v, p in enumerate(parent):
        if p >= 0:
            kids[p].append(v)
    h, c = [None] * n, [None] * n

    def visit(j):
        for k in kids[j]:
            if h[k] is None:
                visit(k)
        hs = sum((h[k] for k in kids[j]), torch.zeros(H, dtype=torch.float64))
        z = Wt @ xt[j] + bt
        zi, zo, zu, zf = z[:H], z[H:2 * H], z[2 * H:3 * H], z[3 * H:]
        i = torch.sigmoid(zi + Ut[:H] @ hs)
        o = torch.sigmoid(zo + Ut[H:2 * H] @ hs)
        u = torch.tanh(zu + Ut[2 * H:3 * H] @ hs)
        cj = i * u
        for k in kids[j]:
            cj = cj + torch.sigmoid(zf + Ut[3 * H:] @ h[k]) * c[k]
        c[j] = cj
        h[j] = o * torch.tanh(cj)

    import sys
    sys.setrecursionlimit(10000)
    for j in range(n):
        if h[j] is None:
            visit(j)
    loss = sum((torch.tensor(gh[j]) * h[j]).sum() + (torch.tensor(gc[j]) * c[j]).sum() for j in range(n))
    loss.backward()
    return xt.grad.numpy(), Wt.grad.numpy(), Ut.grad.numpy(), bt.grad.numpy()


@pytest.mark.parametrize("shape", ["cfg1", "stars", "chain", "mixed"])
def test_matches_autograd_of_an_independent_torch_forward(shape):
    rng = np.random.default_rng(5)
    parent = {"cfg1": make_forest(1), "stars": star_forest(6, 3), "chain": chain_forest(7, 2),
              "mixed": np.array([-1, 0, 0, 1, 1, 1, 2, -1, 7, 8, 8], dtype=np.int32)}[shape]
    n, D, H = len(parent), 5, 4
    x, W, U, b = _rand(rng, n, D, H, scale=2.0)
    gh, gc = rng.standard_normal((n, H)), rng.standard_normal((n, H))
    h, c, dx, dW, dU, db = B.forward_backward(parent, x, W, U, b, gh, gc)
    ho, co = T.forward(parent, x, W, U, b)
    assert np.array_equal(h, ho) and np.array_equal(c, co)       # same forward as the state oracle
    rx, rW, rU, rb = _torch_forest(parent, x, W, U, b, gh, gc)
    for got, want, name in ((dx, rx, "dx"), (dW, rW, "dW"), (dU, rU, "dU"), (db, rb, "db")):
        assert np.allclose(got, want, rtol=1e-10, atol=1e-12), name


def test_chain_gradients_equal_the_library_lstm_differentiated_by_the_library():
    rng = np.random.default_rng(9)
    n, D, H = 8, 6, 5
    x, W, U, b = _rand(rng, n, D, H, scale=2.0)
    parent = chain_forest(n)                  # node n-1 is the first time step, node 0 the last
    gh = rng.standard_normal((n, H)); gc = np.zeros((n, H)); gc[0] = rng.standard_normal(H)
    _, _, dx, dW, dU, db = B.forward_backward(parent, x, W, U, b, gh, gc)
    perm = lambda M: np.concatenate([M[0:H], M[3 * H:4 * H], M[2 * H:3 * H], M[H:2 * H]])   # (i,o,u,f) -> torch's (i,f,g,o)
    lstm = torch.nn.LSTM(D, H).double()
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch.from_numpy(perm(W)))
        lstm.weight_hh_l0.copy_(torch.from_numpy(perm(U)))
        lstm.bias_ih_l0.copy_(torch.from_numpy(perm(b.reshape(-1, 1)).reshape(-1)))
        lstm.bias_hh_l0.zero_()
    seq = torch.tensor(x[::-1].copy(), dtype=torch.float64, requires_grad=True)
    out, (hn, cn) = lstm(seq.unsqueeze(1))
    loss = (out[:, 0, :] * torch.from_numpy(gh[::-1].copy())).sum() + (cn[0, 0] * torch.from_numpy(gc[0])).sum()
    loss.backward()
    unperm = lambda M: np.concatenate([M[0:H], M[3 * H:4 * H], M[2 * H:3 * H], M[H:2 * H]])  # its own inverse
    assert np.allclose(dx, seq.grad.numpy()[::-1], rtol=1e-10, atol=1e-12)
    assert np.allclose(dW, unperm(lstm.weight_ih_l0.grad.numpy()), rtol=1e-10, atol=1e-12)
    assert np.allclose(dU, unperm(lstm.weight_hh_l0.grad.numpy()), rtol=1e-10, atol=1e-12)
    assert np.allclose(db, unperm(lstm.bias_ih_l0.grad.numpy().reshape(-1, 1)).reshape(-1), rtol=1e-10, atol=1e-12)


def test_central_differences_of_the_forward_oracle():
    rng = np.random.default_rng(3)
    parent = np.array([-1, 0, 0, 1, 1, 2, -1, 6], dtype=np.int32)
    n, D, H = len(parent), 3, 3
    x, W, U, b = _rand(rng, n, D, H)
    gh, gc = rng.standard_normal((n, H)), rng.standard_normal((n, H))
    _, _, dx, dW, dU, db = B.forward_backward(parent, x, W, U, b, gh, gc)

    def loss(x_, W_, U_, b_):
        h, c = T.forward(parent, x_, W_, U_, b_)
        return float((gh * h).sum() + (gc * c).sum())

    eps = 1e-6
    for arr, grad, idx in ((x, dx, (3, 1)), (x, dx, (0, 2)), (W, dW, (2, 0)), (W, dW, (10, 1)),
                           (U, dU, (4, 2)), (U, dU, (11, 0)), (b, db, (1,)), (b, db, (9,))):
        hi = [a.copy() for a in (x, W, U, b)]
        lo = [a.copy() for a in (x, W, U, b)]
        which = [a is arr for a in (x, W, U, b)].index(True)
        hi[which][idx] += eps
        lo[which][idx] -= eps
        num = (loss(*hi) - loss(*lo)) / (2 * eps)
        assert abs(num - grad[idx]) <= 1e-7 * max(1.0, abs(num)), (which, idx, num, grad[idx])


def test_leaves_only_closed_form():
    """A single leaf with W = 0: h = sigmoid(b_o) tanh(sigmoid(b_i) tanh(b_u)); its b_f gradient is 0
    and dx = 0; d/db_o is gh * tanh(c) * o (1 - o)."""
    H, D = 3, 2
    b = np.array([0.3, -0.2, 0.1, 0.5, 0.4, -0.6, 0.2, 0.0, -0.1, 9.0, 9.0, 9.0])
    x = np.ones((1, D)); W = np.zeros((4 * H, D)); U = np.zeros((4 * H, H))
    gh = np.array([[1.0, 2.0, -1.0]]); gc = np.zeros((1, H))
    h, c, dx, dW, dU, db = B.forward_backward(np.array([-1]), x, W, U, b, gh, gc)
    sig = lambda z: 1 / (1 + np.exp(-z))
    i, o, u = sig(b[:3]), sig(b[3:6]), np.tanh(b[6:9])
    cc = i * u
    assert np.allclose(db[3:6], gh[0] * np.tanh(cc) * o * (1 - o), atol=1e-15)
    assert np.allclose(db[0:3], gh[0] * o * (1 - np.tanh(cc) ** 2) * u * i * (1 - i), atol=1e-15)
    assert not dx.any() and not db[9:].any() and not dU.any()
    assert np.allclose(dW[3:6], np.outer(db[3:6], x[0]), atol=1e-15)
