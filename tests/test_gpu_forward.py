"""GPU parity: jitdb_treelstm_forward against the CPU oracle.

Tolerances (max abs error over every element of h and c):
  fp32 path  1e-4      bf16 MFMA / fp32 accumulate path  2e-2
"""
import numpy as np
import pytest

from oracle import treelstm_oracle as T
from workloads import (CONFIGS, make_forest, make_values, make_workload, relabel, tree_ranges,
                       chain_forest, star_forest)
from gpu_util import run_gpu_forward

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _oracle(c_oracle, parent, inputs):
    x, W, U, b = inputs
    h, c, _ = c_oracle(parent, x, W, U, b)
    return h, c


def _c_scale(dtype, co):
    """Bound on c in the cases outside the five configs, where |c| is not O(1): c = i u + sum f_k c_k grows
    with the arity, and an absolute bound on a value of magnitude M cannot be tighter than M times the
    arithmetic's relative error.  The flat bound holds up to max|c| = 8 (bf16) / 50 (fp32) and grows
    in proportion beyond; h (|h| < 1) always keeps the flat bound."""
    return max(1.0, float(np.abs(co).max()) / (8.0 if dtype == "bf16" else 50.0))


def _report(tag, h, c, ho, co):
    eh, ec = float(np.abs(h - ho).max()), float(np.abs(c - co).max())
    print(f"{tag}: max|dh|={eh:.3e} max|dc|={ec:.3e} max|c|={float(np.abs(co).max()):.2f}", flush=True)
    return eh, ec


@pytest.mark.parametrize("cfg,bias", [(1, "zero"), (1, "random"), (2, "zero"), (2, "random"),
                                      (3, "zero"), (3, "random")])
def test_small_configs_every_node(c_oracle, cfg, bias):
    cfgo, p, x, W, U, b = make_workload(cfg, bias=bias)
    print(f"forward parity cfg={cfg} bias={bias} dtype={cfgo.dtype} N={p.shape[0]}", flush=True)
    s, h, c, seen = run_gpu_forward(p, x, W, U, b, cfgo.dtype)
    ho, co = _oracle(c_oracle, p, seen)
    eh, ec = _report(f"cfg{cfg}/{bias}", h, c, ho, co)
    assert eh <= TOL[cfgo.dtype] and ec <= TOL[cfgo.dtype]


def _sampled_tree_check(c_oracle, cfg, n_sample, dtype=None, bias="zero", D=None, H=None, scale_tol=False):
    cfgo, p, x, W, U, b = make_workload(cfg, bias=bias)
    if D is not None or H is not None:
        x, W, U, b = make_values(cfg, p.shape[0], bias, D=D, H=H)
    dtype = dtype or cfgo.dtype
    print(f"forward parity cfg={cfg} dtype={dtype} D={x.shape[1]} H={U.shape[1]} N={p.shape[0]} "
          f"(oracle on {n_sample} sampled trees)", flush=True)
    s, h, c, seen = run_gpu_forward(p, x, W, U, b, dtype)
    xo, Wo, Uo, bo = seen
    r = tree_ranges(p)
    T_ = len(r) - 1
    rng = np.random.default_rng(77)
    pick = np.sort(rng.choice(T_, size=min(n_sample, T_), replace=False))
    # always include the largest and the deepest-looking trees
    sizes = np.diff(r)
    pick = np.unique(np.concatenate([pick, [int(np.argmax(sizes))], np.arange(min(6, T_))]))
    rows = np.concatenate([np.arange(r[t], r[t + 1]) for t in pick])
    sub_parent = []
    off = 0
    for t in pick:
        lo, hi = r[t], r[t + 1]
        sp = p[lo:hi].astype(np.int64)
        sub_parent.append(np.where(sp < 0, -1, sp - lo + off))
        off += hi - lo
    sub_parent = np.concatenate(sub_parent).astype(np.int32)
    ho, co, _ = c_oracle(sub_parent, xo[rows], Wo, Uo, bo)
    eh, ec = _report(f"cfg{cfg}/{dtype}", h[rows], c[rows], ho, co)
    assert np.isfinite(h).all() and np.isfinite(c).all()
    # |c| grows with the arity; the bf16 bound is stated for |c| of a few units
    tol_c = TOL[dtype] * (max(1.0, float(np.abs(co).max()) / 8.0) if scale_tol else 1.0)
    assert eh <= TOL[dtype] and ec <= tol_c


def _progress(line):
    """Long tests say where they are: a line on stdout and, if JITDB_PROGRESS_DIR names a directory,
    one in a file there (for a runner that watches files rather than captured output)."""
    import os
    print(line, flush=True)
    d = os.environ.get("JITDB_PROGRESS_DIR")
    if not d:
        return
    try:
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "parity_progress.txt"), "a") as f:
            f.write(line + "\n")
    except OSError:
        pass


def _every_node_check(c_oracle, cfg, bias, trees_per_chunk):
    """Full-size parity: EVERY node of the forest against the C oracle (fp64), the forest cut into
    runs of whole trees so that the oracle's fp64 copies stay small.  Trees are independent, so
    the oracle on a run of trees alone gives exactly the states it gives inside the forest
    (pinned bitwise in the CPU suite)."""
    cfgo, p, x, W, U, b = make_workload(cfg, bias=bias)
    dtype = cfgo.dtype
    _progress(f"forward parity cfg={cfg} bias={bias} dtype={dtype} N={p.shape[0]}: every node")
    s, h, c, seen = run_gpu_forward(p, x, W, U, b, dtype)
    xo, Wo, Uo, bo = seen
    assert np.isfinite(h).all() and np.isfinite(c).all()
    r = tree_ranges(p)
    T_ = len(r) - 1
    eh = ec = 0.0
    worst = (0, 0)
    nodes = 0
    for t0 in range(0, T_, trees_per_chunk):
        t1 = min(t0 + trees_per_chunk, T_)
        lo, hi = int(r[t0]), int(r[t1])
        sp = p[lo:hi].astype(np.int64)
        sub = np.where(sp < 0, -1, sp - lo).astype(np.int32)
        ho, co, _ = c_oracle(sub, xo[lo:hi], Wo, Uo, bo)
        dh = np.abs(h[lo:hi] - ho).max(axis=1)
        dc = np.abs(c[lo:hi] - co).max(axis=1)
        if dh.max() > eh:
            eh = float(dh.max()); worst = (lo + int(dh.argmax()), worst[1])
        if dc.max() > ec:
            ec = float(dc.max()); worst = (worst[0], lo + int(dc.argmax()))
        nodes += hi - lo
        _progress(f"  cfg{cfg}: trees [{t0}, {t1}) nodes {nodes}/{p.shape[0]} max|dh|={eh:.3e} max|dc|={ec:.3e}")
    assert nodes == p.shape[0]
    _progress(f"cfg{cfg}/{bias}: every node compared; worst h at node {worst[0]}, worst c at node {worst[1]}")
    assert eh <= TOL[dtype] and ec <= TOL[dtype]


@pytest.mark.timeout(600)
@pytest.mark.parametrize("bias", ["zero", "random"])
def test_config4_full_size_every_node(c_oracle, bias):
    _every_node_check(c_oracle, 4, bias, 1024)


@pytest.mark.timeout(900)
def test_config5_full_size_every_node(c_oracle):
    """2.36 M nodes, about 100 s of oracle time on 16 cores."""
    _every_node_check(c_oracle, 5, "zero", 4096)


def test_config3_in_fp32_too(c_oracle):
    _sampled_tree_check(c_oracle, 3, 300, dtype="f32", bias="random")


@pytest.mark.timeout(600)
def test_config5_in_fp32_too(c_oracle):
    """The fp32 MFMA path on the largest forest (million-row levels, H = 512), with a bias."""
    _sampled_tree_check(c_oracle, 5, 48, dtype="f32", bias="random")


@pytest.mark.timeout(400)
def test_config4_in_bf16_too(c_oracle):
    """The bf16 path on the deep / wide shapes (128 levels, 64-child stars)."""
    _sampled_tree_check(c_oracle, 4, 240, dtype="bf16", bias="random", scale_tol=True)


def test_relabelled_ids_give_the_same_states(c_oracle):
    cfgo, p, x, W, U, b = make_workload(2, bias="random")
    q, new_of_old = relabel(p, 21)
    xq = np.empty_like(x); xq[new_of_old] = x
    _, h, c, _ = run_gpu_forward(p, x, W, U, b, "f32")
    _, hq, cq, seen = run_gpu_forward(q, xq, W, U, b, "f32")
    assert np.abs(hq[new_of_old] - h).max() <= 2e-5 and np.abs(cq[new_of_old] - c).max() <= 2e-5
    ho, co = _oracle(c_oracle, q, seen)
    assert np.abs(hq - ho).max() <= 1e-4 and np.abs(cq - co).max() <= 1e-4


def test_forest_equals_trees_run_alone(c_oracle):
    cfgo, p, x, W, U, b = make_workload(1, bias="random")
    _, h, c, _ = run_gpu_forward(p, x, W, U, b, "f32")
    r = tree_ranges(p)
    for t in range(len(r) - 1):
        lo, hi = r[t], r[t + 1]
        pt = np.where(p[lo:hi] < 0, -1, p[lo:hi] - lo).astype(np.int32)
        _, ht, ct, _ = run_gpu_forward(pt, x[lo:hi], W, U, b, "f32")
        assert np.abs(ht - h[lo:hi]).max() <= 2e-5 and np.abs(ct - c[lo:hi]).max() <= 2e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name,H,D", [("H32", 32, 4), ("H33", 33, 8), ("H64", 64, 300),
                                      ("H100", 100, 52), ("H257", 257, 300),
                                      ("H36-D7", 36, 7), ("H150-D302", 150, 302)])
def test_odd_dimensions(c_oracle, name, H, D, dtype):
    """Hidden sizes on and off every padding boundary; forests with leaves only,
    one chain, one wide star and a ragged last row tile."""
    parent = np.concatenate([
        np.full(3, -1), chain_forest(37) + 3, star_forest(150) + 40,
        np.where(make_forest(1) < 0, -1, make_forest(1) + 190)]).astype(np.int32)
    parent[3] = -1; parent[40] = -1
    x, W, U, b = make_values(1, parent.shape[0], "random", D=D, H=H)
    print(f"forward odd dims {name} D={D} dtype={dtype} N={parent.shape[0]}", flush=True)
    _, h, c, seen = run_gpu_forward(parent, x, W, U, b, dtype)
    ho, co = _oracle(c_oracle, parent, seen)
    eh, ec = _report(f"{name}/{dtype}", h, c, ho, co)
    # the 149-child star reaches |c| ~ 50: scale the bf16 bound with the magnitude there
    scale = _c_scale(dtype, co)
    assert eh <= TOL[dtype] and ec <= TOL[dtype] * scale


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name,H,D", [("H33-D8", 33, 8), ("H64-D4", 64, 4), ("H100-D52", 100, 52),
                                      ("H257-D300", 257, 300), ("H36-D7", 36, 7), ("H150-D302", 150, 302),
                                      ("H520-D64", 520, 64)])
def test_odd_dimensions_on_levels_large_enough_for_the_tiled_kernel(c_oracle, name, H, D, dtype):
    """Config 3's forest (leaf level 68 k rows, two more levels above the thin-kernel limit) with
    hidden and input sizes on and off every padding boundary: partial unit tiles, partial column
    tiles, a two-stage K loop (D = 4), more than eight column tiles (H = 520)."""
    _sampled_tree_check(c_oracle, 3, 150, dtype=dtype, bias="random", D=D, H=H, scale_tol=True)


def test_leaves_only_and_single_node(c_oracle):
    for n in (1, 2, 129):
        parent = np.full(n, -1, dtype=np.int32)
        x, W, U, b = make_values(1, n, "random", D=300, H=150)
        _, h, c, seen = run_gpu_forward(parent, x, W, U, b, "f32")
        ho, co = _oracle(c_oracle, parent, seen)
        assert np.abs(h - ho).max() <= 1e-4 and np.abs(c - co).max() <= 1e-4


@pytest.mark.parametrize("name,n_stars,size,dtype", [("three-wide", 3, 5000, "f32"), ("many-tiled", 9000, 41, "f32"),
                                                    ("many-tiled", 9000, 41, "bf16")])
def test_stars_with_long_child_lists(c_oracle, name, n_stars, size, dtype):
    """Child lists far beyond the four ids a row record carries, on the thin kernel (three roots with
    4999 children each) and on the tiled kernel (9000 roots with 40 children: a level of more than 8192
    rows).  The cell state of a root grows with its arity, and so does the bound on its error."""
    parent = star_forest(size, n_stars)
    x, W, U, b = make_values(2, parent.shape[0], "random", D=64, H=96)
    print(f"forward stars {name} {n_stars} x {size} {dtype}", flush=True)
    _, h, c, seen = run_gpu_forward(parent, x, W, U, b, dtype)
    ho, co = _oracle(c_oracle, parent, seen)
    eh, ec = _report(f"stars/{name}/{dtype}", h, c, ho, co)
    assert np.isfinite(h).all() and np.isfinite(c).all()
    assert eh <= TOL[dtype] and ec <= TOL[dtype] * _c_scale(dtype, co)


def test_deep_chain_fp32(c_oracle):
    parent = chain_forest(128, 3)
    x, W, U, b = make_values(4, parent.shape[0], "random", D=300, H=256)
    _, h, c, seen = run_gpu_forward(parent, x, W, U, b, "f32")
    ho, co = _oracle(c_oracle, parent, seen)
    eh, ec = _report("chain128/f32", h, c, ho, co)
    assert eh <= 1e-4 and ec <= 1e-4


def test_empty_forest_forward():
    import torch
    import paper_1904_07421_amd as J
    s = J.jitdb_schedule(torch.empty(0, dtype=torch.int32, device="cuda"))
    x = torch.empty((0, 300), device="cuda"); W = torch.zeros((600, 300), device="cuda")
    U = torch.zeros((600, 150), device="cuda"); b = torch.zeros(600, device="cuda")
    h, c = J.jitdb_treelstm_forward(x, W, U, b, s)
    assert h.shape == (0, 150) and c.shape == (0, 150)


def test_bitwise_repeatable():
    cfgo, p, x, W, U, b = make_workload(3)
    _, h1, c1, _ = run_gpu_forward(p, x, W, U, b, "bf16")
    _, h2, c2, _ = run_gpu_forward(p, x, W, U, b, "bf16")
    assert np.array_equal(h1, h2) and np.array_equal(c1, c2)


def test_bad_arguments_are_rejected():
    import torch
    import paper_1904_07421_amd as J
    from gpu_util import dev_parent
    s = J.jitdb_schedule(dev_parent(make_forest(1)))
    n = s.n_nodes
    x = torch.zeros((n, 300), device="cuda"); W = torch.zeros((600, 300), device="cuda")
    U = torch.zeros((600, 150), device="cuda"); b = torch.zeros(600, device="cuda")
    h_misaligned = torch.zeros(n * 150 + 1, device="cuda")[1:].view(n, 150)   # 4 bytes off
    with pytest.raises(J.JitdbError) as e:
        J.jitdb_treelstm_forward(x, W, U, b, s, out=(h_misaligned, torch.zeros((n, 150), device="cuda")))
    assert e.value.code == -2
    with pytest.raises(J.JitdbError) as e:          # workspace too small
        J.jitdb_treelstm_forward(x, W, U, b, s, workspace=torch.empty(512, dtype=torch.uint8, device="cuda"))
    assert e.value.code == -5


def test_schedule_is_reusable_and_streams_are_honoured(c_oracle):
    """One schedule, several forwards with different values, on a non-default stream."""
    import torch
    import paper_1904_07421_amd as J
    from gpu_util import dev_parent
    cfgo, p, x, W, U, b = make_workload(2, bias="random")
    s = J.jitdb_schedule(dev_parent(p))
    st = torch.cuda.Stream()
    Wt, Ut, bt = (torch.from_numpy(a).cuda() for a in (W, U, b))
    for scale in (1.0, -0.5):
        xs = (x * scale).astype(np.float32)
        xt = torch.from_numpy(xs).cuda()
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            h, c = J.jitdb_treelstm_forward(xt, Wt, Ut, bt, s, stream=st)
        st.synchronize()
        ho, co, _ = c_oracle(p, xs, W, U, b)
        assert np.abs(h.cpu().numpy() - ho).max() <= 1e-4 and np.abs(c.cpu().numpy() - co).max() <= 1e-4


def test_forward_can_be_captured_in_a_graph(c_oracle):
    """The forward is asynchronous and allocates nothing, so it can be recorded into a HIP
    graph; every replay (with new x in the same buffer, eager work in between) must match."""
    import torch
    import paper_1904_07421_amd as J
    from gpu_util import dev_parent
    cfgo, p, x, W, U, b = make_workload(2, bias="random")
    s = J.jitdb_schedule(dev_parent(p))
    n, D, H = p.shape[0], cfgo.D, cfgo.H
    Wt, Ut, bt = (torch.from_numpy(a).cuda() for a in (W, U, b))
    xt = torch.from_numpy(x).cuda()
    h = torch.empty((n, H), device="cuda"); c = torch.empty((n, H), device="cuda")
    ws = torch.empty(J.jitdb_treelstm_workspace_bytes(n, s.n_edges, D, H, J.JITDB_F32),
                     dtype=torch.uint8, device="cuda")
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):                      # warm-up on the capture stream
        J.jitdb_treelstm_forward(xt, Wt, Ut, bt, s, stream=st, workspace=ws, out=(h, c))
    st.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st):
        J.jitdb_treelstm_forward(xt, Wt, Ut, bt, s, stream=st, workspace=ws, out=(h, c))
    for scale in (1.0, 0.25, -2.0):
        xs = (x * scale).astype(np.float32)
        xt.copy_(torch.from_numpy(xs).cuda())        # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ho, co, _ = c_oracle(p, xs, W, U, b)
        assert np.abs(h.cpu().numpy() - ho).max() <= 1e-4 and np.abs(c.cpu().numpy() - co).max() <= 1e-4


@pytest.mark.timeout(900)
def test_largest_forest_the_interface_accepts():
    """N = JITDB_MAX_NODES (2^28) with D = H = 1: 2^26 chains of four nodes that all carry the same
    inputs, so every chain must reproduce the oracle's states for one chain.  What is tested is the
    addressing: node ids, row offsets and workspace offsets beyond 2^31 bytes in every kernel."""
    import torch
    import paper_1904_07421_amd as J
    n, t = 1 << 28, 1 << 26
    print(f"forward N={n} D=H=1 bf16", flush=True)
    v = torch.arange(n, dtype=torch.int32, device="cuda")
    parent = torch.where((v & 3) == 0, torch.full_like(v, -1), v - 1)
    xs = np.array([0.5, -1.0, 0.25, 2.0], dtype=np.float32)          # exact in bf16
    W = np.array([[0.75], [-0.5], [1.25], [0.375]], dtype=np.float32)
    U = np.array([[0.5], [0.25], [-0.75], [1.5]], dtype=np.float32)
    b = np.array([0.125, -0.25, 0.5, 0.0625], dtype=np.float32)
    x = torch.from_numpy(xs).cuda().to(torch.bfloat16)[(v & 3).long()].reshape(n, 1).contiguous()
    del v
    s = J.jitdb_schedule(parent)
    del parent
    dev = lambda a: torch.from_numpy(a).cuda().to(torch.bfloat16)
    h, c = J.jitdb_treelstm_forward(x, dev(W), dev(U), torch.from_numpy(b).cuda(), s)
    torch.cuda.synchronize()
    ho, co = T.forward(np.array([-1, 0, 1, 2], dtype=np.int32), xs.reshape(4, 1), W, U, b)
    h4, c4 = h.view(t, 4), c.view(t, 4)
    assert np.abs(h4[0].float().cpu().numpy() - ho[:, 0]).max() <= TOL["bf16"]
    assert np.abs(c4[0].cpu().numpy() - co[:, 0]).max() <= TOL["bf16"]
    assert bool((h4 == h4[0]).all()) and bool((c4 == c4[0]).all())


@pytest.mark.parametrize("cfg", [2, 3])
def test_packed_weights_give_the_same_forward(cfg):
    """Weights packed once, forward called twice with them: bit-identical to the call that packs."""
    import torch
    import paper_1904_07421_amd as J
    from gpu_util import bf16_tensor, dev_parent
    cfgo, p, x, W, U, b = make_workload(cfg, bias="random")
    dev = (lambda a: bf16_tensor(a)[0]) if cfgo.dtype == "bf16" else (lambda a: torch.from_numpy(a).cuda())
    xt, Wt, Ut, bt = dev(x), dev(W), dev(U), torch.from_numpy(b).cuda()
    s = J.jitdb_schedule(dev_parent(p))
    h0, c0 = J.jitdb_treelstm_forward(xt, Wt, Ut, bt, s)
    pk = J.jitdb_treelstm_pack(Wt, Ut, bt)
    for _ in range(2):
        h1, c1 = J.jitdb_treelstm_forward_packed(xt, pk, s)
        assert torch.equal(h0, h1) and torch.equal(c0, c1)
    with pytest.raises(ValueError):
        J.jitdb_treelstm_forward_packed(xt, J.jitdb_treelstm_pack(torch.stack([Wt, Wt]), torch.stack([Ut, Ut]),
                                                                  torch.stack([bt, bt])), s)


def test_variable_length_sequences_against_the_library_lstm():
    """A batch of sequences of different lengths, written as chains, through the HIP path and through
    torch.nn.LSTM on the CPU (fp64, each sequence on its own): the "variable-length LSTM batch" workload,
    checked against the library directly rather than through the oracle."""
    import torch
    rng = np.random.default_rng(12)
    D, H = 48, 64
    lens = rng.integers(1, 60, size=200)
    W = (rng.uniform(-1, 1, (4 * H, D)) / np.sqrt(D)).astype(np.float32)
    U = (rng.uniform(-1, 1, (4 * H, H)) / np.sqrt(H)).astype(np.float32)
    b = rng.uniform(-0.5, 0.5, 4 * H).astype(np.float32)
    parts, off = [], 0
    for n in lens:                                         # chain: node i's parent is i - 1, the last node is the leaf
        parts.append(np.where(np.arange(n) == 0, -1, np.arange(n) - 1 + off)); off += n
    parent = np.concatenate(parts).astype(np.int32)
    x = rng.standard_normal((parent.shape[0], D)).astype(np.float32)
    _, h, c, _ = run_gpu_forward(parent, x, W, U, b, "f32")

    def torch_rows(M):                                     # our gate order (i, o, u, f) -> torch's (i, f, g, o)
        i, o, u, f = (M[g * H:(g + 1) * H] for g in range(4))
        return torch.from_numpy(np.concatenate([i, f, u, o]).astype(np.float64))
    lstm = torch.nn.LSTM(D, H).double()
    with torch.no_grad():
        lstm.weight_ih_l0.copy_(torch_rows(W)); lstm.weight_hh_l0.copy_(torch_rows(U))
        lstm.bias_ih_l0.copy_(torch_rows(b.reshape(-1, 1)).reshape(-1)); lstm.bias_hh_l0.zero_()
        off, worst = 0, 0.0
        for n in lens:
            seq = torch.from_numpy(x[off:off + n][::-1].astype(np.float64).copy()).unsqueeze(1)   # leaf first
            out, (hn, cn) = lstm(seq)
            worst = max(worst, float(np.abs(out[:, 0, :].numpy()[::-1] - h[off:off + n]).max()),
                        float(np.abs(cn[0, 0].numpy() - c[off]).max()))
            off += n
    print(f"sequences vs torch.nn.LSTM: max error {worst:.3e}", flush=True)
    assert worst <= 1e-4


def test_default_buffers_follow_the_launch_stream(c_oracle):
    """stream=st WITHOUT making st current: the buffers the binding allocates by default must belong to
    st, so that other work on the current stream cannot be handed them while the forward still runs."""
    import torch
    import paper_1904_07421_amd as J
    from gpu_util import dev_parent
    cfgo, p, x, W, U, b = make_workload(2, bias="random")
    s = J.jitdb_schedule(dev_parent(p))
    xt, Wt, Ut, bt = (torch.from_numpy(a).cuda() for a in (x, W, U, b))
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    outs = []
    for _ in range(4):
        h, c = J.jitdb_treelstm_forward(xt, Wt, Ut, bt, s, stream=st)      # current stream stays the default one
        # work on the current stream that would love to reuse freed blocks
        junk = [torch.full((p.shape[0], cfgo.H), float("nan"), device="cuda") for _ in range(8)]
        del junk
        outs.append((h, c))
    st.synchronize()
    torch.cuda.synchronize()
    ho, co, _ = c_oracle(p, x, W, U, b)
    for h, c in outs:
        assert np.abs(h.cpu().numpy() - ho).max() <= 1e-4 and np.abs(c.cpu().numpy() - co).max() <= 1e-4


# ---- levels of one-child nodes (one launch per level) ------------------------------------------
def _profile_classes(fn):
    """Run fn() under the library's per-kernel timers; returns launches per class."""
    import torch
    import paper_1904_07421_amd as J
    J.jitdb_profile_start(4096)
    try:
        out = fn()
        torch.cuda.synchronize()
    finally:
        prof = J.jitdb_profile_stop()
    return out, {k: v["launches"] for k, v in prof.items() if isinstance(v, dict)}


def _trees_and_sequences(n_trees, n_seqs, len_hi, seed):
    from workloads import mixed_forest
    return mixed_forest(2, n_trees, n_seqs, 2, len_hi, seed)[0]


@pytest.mark.parametrize("dtype,D,H", [("f32", 300, 256), ("bf16", 300, 512), ("f32", 44, 50), ("bf16", 44, 50),
                                       ("bf16", 64, 72), ("f32", 300, 512), ("f32", 512, 512), ("f32", 4, 1)])
def test_chain_levels_run_as_one_launch_each(c_oracle, dtype, D, H):
    """Parse trees plus sequences up to 90 long: above the trees' heights every level holds only nodes
    with one child and takes the single-launch kernel (x and the child's h read in place, all four
    gates full K); below, the usual stack / level / projection launches.  Padded widths included.
    fp32 splits K over two waves per gate where the LDS beside the A tile allows: (300, 256), (300, 512) and the
    small widths do, (512, 512) does not."""
    parent = _trees_and_sequences(300, 700, 90, 5)
    x, W, U, b = make_values(2, parent.shape[0], "random", D=D, H=H)
    (res, launches) = _profile_classes(lambda: run_gpu_forward(parent, x, W, U, b, dtype))
    sched, h, c, seen = res
    L = sched.n_levels
    lp, kids = sched.host_level_ptr[:L + 1], sched.host_level_kids[:L]
    rows = np.diff(lp)
    chain_from = L
    for l in range(L - 1, 0, -1):
        if kids[l] != rows[l]:
            break
        chain_from = l
    print(f"chain levels {dtype} D={D} H={H}: N={parent.shape[0]} L={L} chain_from={chain_from} launches={launches}",
          flush=True)
    assert 1 < chain_from < L - 20
    assert launches["chain"] == L - chain_from
    ho, co = _oracle(c_oracle, parent, seen)
    eh, ec = _report(f"chain-levels/{dtype}", h, c, ho, co)
    assert eh <= TOL[dtype] and ec <= TOL[dtype] * _c_scale(dtype, co)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chain_levels_need_the_child_counts_and_whole_x_pieces(c_oracle, dtype):
    """Without the schedule's children-per-level, or with D not a multiple of 4, the same forest takes
    the general launches and gives the same states within the tolerance."""
    import torch
    import paper_1904_07421_amd as J
    parent = _trees_and_sequences(100, 300, 40, 6)
    for D in (48, 46):
        x, W, U, b = make_values(2, parent.shape[0], "random", D=D, H=40)
        (res, launches) = _profile_classes(lambda: run_gpu_forward(parent, x, W, U, b, dtype))
        sched, h, c, seen = res
        assert (launches["chain"] > 0) == (D % 4 == 0), (D, launches)
        ho, co = _oracle(c_oracle, parent, seen)
        eh, ec = _report(f"chain D={D}/{dtype}", h, c, ho, co)
        assert eh <= TOL[dtype] and ec <= TOL[dtype] * _c_scale(dtype, co)
        if D % 4 == 0:
            # the same schedule with the counts withheld
            sched.host_level_kids[:] = -1
            to = (lambda a: torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda()) if dtype == "f32" else \
                (lambda a: __import__("gpu_util").bf16_tensor(a)[0])
            args = (to(x), to(W), to(U), torch.from_numpy(b).cuda(), sched)
            (res2, launches2) = _profile_classes(lambda: J.jitdb_treelstm_forward(*args))
            assert launches2["chain"] == 0 and launches2["thin_proj"] > launches["thin_proj"]
            h2, c2 = res2[0].float().cpu().numpy(), res2[1].cpu().numpy()
            assert np.abs(h2 - h).max() <= TOL[dtype] and np.abs(c2 - c).max() <= TOL[dtype] * _c_scale(dtype, co)


def test_chain_levels_inside_a_captured_graph(c_oracle):
    """The single-launch kernel of chain levels asks for more dynamic LDS than the default; the attribute is
    set outside the stream's work, so the forward still records into a HIP graph and every replay matches."""
    import torch
    import paper_1904_07421_amd as J
    from gpu_util import dev_parent
    parent = _trees_and_sequences(60, 200, 50, 8)
    D, H = 300, 256
    x, W, U, b = make_values(2, parent.shape[0], "random", D=D, H=H)
    s = J.jitdb_schedule(dev_parent(parent))
    n = parent.shape[0]
    assert (s.host_level_kids[s.n_levels - 10:s.n_levels] == np.diff(s.host_level_ptr[s.n_levels - 10:s.n_levels + 1])).all()
    Wt, Ut, bt = (torch.from_numpy(a).cuda() for a in (W, U, b))
    xt = torch.from_numpy(x).cuda()
    h = torch.empty((n, H), device="cuda"); c = torch.empty((n, H), device="cuda")
    ws = torch.empty(J.jitdb_treelstm_workspace_bytes(n, s.n_edges, D, H, J.JITDB_F32), dtype=torch.uint8, device="cuda")
    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):                      # warm-up on the capture stream
        J.jitdb_treelstm_forward(xt, Wt, Ut, bt, s, stream=st, workspace=ws, out=(h, c))
    st.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=st):
        J.jitdb_treelstm_forward(xt, Wt, Ut, bt, s, stream=st, workspace=ws, out=(h, c))
    for scale in (1.0, -0.5, 2.0):
        xs = (x * scale).astype(np.float32)
        xt.copy_(torch.from_numpy(xs).cuda())        # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        ho, co, _ = c_oracle(parent, xs, W, U, b)
        assert np.abs(h.cpu().numpy() - ho).max() <= 1e-4 and np.abs(c.cpu().numpy() - co).max() <= 1e-4


def test_chain_levels_too_wide_for_lds_take_the_general_launches(c_oracle):
    """K = D + H so large that 32 rows of A do not fit the LDS the kernel may use: same result, other launches."""
    parent = chain_forest(12, 40)
    D, H = 1024, 1280                                  # 32 x (9216 + 16) bytes: more than a compute unit's LDS
    x, W, U, b = make_values(2, parent.shape[0], "random", D=D, H=H)
    (res, launches) = _profile_classes(lambda: run_gpu_forward(parent, x, W, U, b, "f32"))
    _, h, c, seen = res
    assert launches["chain"] == 0 and launches["thin_internal"] == 11
    ho, co = _oracle(c_oracle, parent, seen)
    eh, ec = _report("wide chain/f32", h, c, ho, co)
    assert eh <= 1e-4 and ec <= 1e-4 * _c_scale("f32", co)


def test_children_per_level_are_optional_in_the_c_struct(c_oracle):
    """A caller of the C ABI that leaves host_level_kids NULL gets the same schedule and a forward over the
    general launches; one that sets it gets the counts filled in by jitdb_schedule."""
    import torch
    import paper_1904_07421_amd as J
    from gpu_util import dev_parent
    parent = _trees_and_sequences(40, 120, 30, 9)
    x, W, U, b = make_values(2, parent.shape[0], "random", D=32, H=32)
    dp = dev_parent(parent)
    with_counts = J.jitdb_schedule(dp)
    without = J.Schedule(parent.shape[0], dp.device)
    without.struct.host_level_kids = None                    # NULL in the C struct
    J.jitdb_schedule(dp, out=without)
    a, bb = with_counts.to_numpy(), without.to_numpy()
    for k in ("height", "level_ptr", "perm", "inv_perm", "child_ptr", "child_idx"):
        assert np.array_equal(a[k], bb[k]), k
    assert (without.host_level_kids == -1).all() and (with_counts.host_level_kids[:with_counts.n_levels] >= 0).all()
    dev = lambda v: torch.from_numpy(np.ascontiguousarray(v, np.float32)).cuda()
    (res, launches) = _profile_classes(lambda: J.jitdb_treelstm_forward(dev(x), dev(W), dev(U), dev(b), without))
    assert launches["chain"] == 0
    h, c = res[0].cpu().numpy(), res[1].cpu().numpy()
    ho, co = _oracle(c_oracle, parent, (x, W, U, b))
    assert np.abs(h - ho).max() <= 1e-4 and np.abs(c - co).max() <= 1e-4


@pytest.mark.parametrize("seed", list(range(8)))
def test_chain_levels_random_shapes(c_oracle, seed):
    """Random widths (H from 1 up, D any multiple of 4), tree / sequence mixes and row counts around the
    tile edges, both types: the single-launch levels against the oracle."""
    rng = np.random.default_rng(100 + seed)
    D = int(rng.choice([4, 8, 12, 36, 100, 132, 300]))
    H = int(rng.integers(1, 200))
    dtype = "bf16" if seed % 2 else "f32"
    n_seqs = int(rng.choice([1, 31, 32, 33, 97, 260]))
    parent = _trees_and_sequences(int(rng.integers(0, 20)), n_seqs, int(rng.integers(3, 40)), 200 + seed)
    x, W, U, b = make_values(2, parent.shape[0], "random", D=D, H=H)
    (res, launches) = _profile_classes(lambda: run_gpu_forward(parent, x, W, U, b, dtype))
    sched, h, c, seen = res
    L = sched.n_levels
    rows, kids = np.diff(sched.host_level_ptr[:L + 1]), sched.host_level_kids[:L]
    expect = 0
    for l in range(L - 1, 0, -1):
        if kids[l] != rows[l]:
            break
        expect += 1
    print(f"chain random seed={seed} D={D} H={H} {dtype} N={parent.shape[0]} L={L} chain levels={expect}", flush=True)
    assert launches["chain"] == expect
    ho, co = _oracle(c_oracle, parent, seen)
    eh, ec = _report(f"chain-random/{seed}", h, c, ho, co)
    assert eh <= TOL[dtype] and ec <= TOL[dtype] * _c_scale(dtype, co)
