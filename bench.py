#!/usr/bin/env python3
"""Benchmark of the level-batched Tree-LSTM forward on one MI355X.

One "step" = the whole hot path over one batch: jitdb_schedule (heights, level
buckets, permutation, child CSR) followed by jitdb_treelstm_forward (all levels),
on the large synthetic forest (config 5: 65536 random recursive trees, 8-64
nodes each, D=300, H=512, bf16 operands with fp32 accumulate).  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

  value        nodes/s of the whole step (schedule + forward)
  roofline     the dominant kernel against its bound; duration from HIP events
               recorded on the launch stream inside the timed region
  cpu_baseline the fp64 C oracle timed on the host cores on the first trees of
               the same forest (a reported baseline, not a target)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_F32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def measured_traffic(cfg, key):
    """A figure from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE scaled by a copy kernel
    of known size), or None: key = "traffic_bytes_per_launch[<kernel class>]" or "traffic_bytes_per_forward"."""
    path = os.path.join(ROOT, "profiles", f"level_kernel_{cfg.dtype}_config{cfg.index}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith(key + ":"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def train_bench(args, J, torch, cfg, dev, N, D, H, esz, peak_tflops, xt, Wt, Ut, bt, pt, sched, ws_s,
                n_leaf, n_int, E, L):
    """Training step = jitdb_schedule + jitdb_treelstm_forward_train + jitdb_treelstm_backward, one stream."""
    dt = J.JITDB_BF16 if esz == 2 else J.JITDB_F32
    f32 = dict(dtype=torch.float32, device=dev)
    ws_f = torch.empty(J.jitdb_treelstm_workspace_bytes(N, E, D, H, dt), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(J.jitdb_treelstm_backward_workspace_bytes(sched, D, H, dt), dtype=torch.uint8, device=dev)
    h = torch.empty((N, H), dtype=xt.dtype, device=dev)
    c = torch.empty((N, H), **f32)
    gates = torch.empty((N, 3 * H), dtype=xt.dtype, device=dev)
    fgate = torch.zeros((N, H), dtype=xt.dtype, device=dev)
    gh = torch.randn((N, H), **f32)
    gc = torch.randn((N, H), **f32)
    grads = (torch.empty((N, D), **f32), torch.empty((4 * H, D), **f32), torch.empty((4 * H, H), **f32),
             torch.empty(4 * H, **f32))
    stream = torch.cuda.current_stream()

    def fwd():
        J.jitdb_treelstm_forward_train(xt, Wt, Ut, bt, sched, stream=stream, workspace=ws_f, out=(h, c, gates, fgate))

    def bwd():
        J.jitdb_treelstm_backward(xt, Wt, Ut, sched, h, c, gates, fgate, gh, gc, stream=stream, workspace=ws_b,
                                  out=grads)

    def step():
        J.jitdb_schedule(pt, stream=stream, workspace=ws_s, out=sched)
        fwd()
        bwd()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps

    def timed(fn, reps):
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / reps
    reps = max(2, min(args.steps, 5))
    ms_f, ms_b = timed(fwd, reps), timed(bwd, reps)
    # every multiply-add of the forward has two in the backward (data and weight gradient)
    f_min = n_leaf * 2.0 * D * 3 * H + n_int * (2.0 * D * 4 * H + 2.0 * H * 3 * H) + E * 2.0 * H * H
    out = {
        "metric": "Tree-LSTM training step nodes/sec on 1 MI355X", "value": N / (ms_step * 1e-3), "unit": "nodes/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype if cfg.dtype == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"config {cfg.index}: {cfg.name}", "n_trees": cfg.n_trees, "n_nodes": N, "n_edges": E,
                   "n_levels": L, "D": D, "H": H,
                   "step": "jitdb_schedule + jitdb_treelstm_forward_train + jitdb_treelstm_backward "
                           "(cotangents on h and c of every node), one stream"},
        "ms_forward_train": ms_f, "ms_backward": ms_b,
        "roofline": {"kernel": "backward pass as a whole (its GEMMs: gemm_kb_kernel)",
                     "bound": "mfma", "achieved": 2.0 * f_min / (ms_b * 1e-3) / 1e12, "peak": peak_tflops,
                     "unit": "TFLOP/s", "frac": 2.0 * f_min / (ms_b * 1e-3) / 1e12 / peak_tflops, "traffic": None,
                     "flops_per_step": 2.0 * f_min},
    }
    print(json.dumps(out), flush=True)


def typed_bench(args, J, torch, cfg, dev, N, D, H, esz, peak_tflops, xt, parent, n_leaf, n_int, E):
    """Several cells in one table: step = jitdb_schedule_typed + jitdb_treelstm_forward_typed, one stream.
    Every tree draws one of --signatures networks; the work per node is that of the headline step."""
    from workloads import tree_signatures, node_signatures, make_values_typed, to_bf16_bits
    T = args.signatures
    sig = node_signatures(parent, T, 99) if args.signatures_per_node else tree_signatures(parent, T, 99)
    _, W, U, b = make_values_typed(cfg.index, 1, T, bias="zero")
    if esz == 2:
        up = lambda a: torch.from_numpy(to_bf16_bits(a).view(np.int16)).view(torch.bfloat16).to(dev)
    else:
        up = lambda a: torch.from_numpy(a).to(dev)
    Wt, Ut, bt = up(W), up(U), torch.from_numpy(b).to(dev)
    pt, st_ = torch.from_numpy(parent).to(dev), torch.from_numpy(sig).to(dev)
    dt = J.JITDB_BF16 if esz == 2 else J.JITDB_F32
    sched = J.jitdb_schedule_typed(pt, st_, T)
    ws_s = torch.empty(J.jitdb_schedule_typed_workspace_bytes(N, T), dtype=torch.uint8, device=dev)
    ws_f = torch.empty(J.jitdb_treelstm_typed_workspace_bytes(N, E, D, H, dt, T), dtype=torch.uint8, device=dev)
    h = torch.empty((N, H), dtype=xt.dtype, device=dev)
    c = torch.empty((N, H), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def sch():
        J.jitdb_schedule_typed(pt, st_, T, stream=stream, workspace=ws_s, out=sched)

    def fwd():
        J.jitdb_treelstm_forward_typed(xt, Wt, Ut, bt, sched, stream=stream, workspace=ws_f, out=(h, c))

    def step():
        sch()
        fwd()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps

    def timed(fn, reps):
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / reps
    reps = max(3, min(args.steps, 10))
    ms_s, ms_f = timed(sch, reps), timed(fwd, reps)
    f_min = n_leaf * 2.0 * D * 3 * H + n_int * (2.0 * D * 4 * H + 2.0 * H * 3 * H) + E * 2.0 * H * H
    S = sched.n_levels * T * T
    nonempty = int(np.count_nonzero(np.diff(sched.host_slot_ptr[:S + 1])))
    out = {
        "metric": f"Tree-LSTM forward nodes/sec on 1 MI355X, {T} cells in one table", "value": N / (ms_step * 1e-3),
        "unit": "nodes/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg.index}: {cfg.name}, " + (f"leaves under cell 0, every other node under one of {T - 1} cells"
                                                                   if args.signatures_per_node else f"each tree under one of {T} networks"),
                   "n_trees": cfg.n_trees, "n_nodes": N, "n_edges": E, "n_levels": sched.n_levels, "n_sig": T,
                   "slots": S, "non_empty_slots": nonempty, "D": D, "H": H,
                   "step": "jitdb_schedule_typed + jitdb_treelstm_forward_typed, one stream"},
        "ms_schedule": ms_s, "ms_forward": ms_f,
        "roofline": {"kernel": "typed forward as a whole (level_kernel / thin_kernel per slot)", "bound": "mfma",
                     "achieved": f_min / (ms_f * 1e-3) / 1e12, "peak": peak_tflops, "unit": "TFLOP/s",
                     "frac": f_min / (ms_f * 1e-3) / 1e12 / peak_tflops, "traffic": None, "flops_per_step": f_min},
    }
    print(json.dumps(out), flush=True)


def nary_bench(args, J, torch, cfg, dev, D, H, esz, peak_tflops):
    """A second operator type in the table: trees with at most --nary children per node (binarised parse
    trees for 2), as many trees and nodes per tree as the config, every node under ONE N-ary Tree-LSTM
    cell.  step = jitdb_schedule_typed + jitdb_treelstm_forward_cells, one stream; the states of a sample
    of trees are checked against the cells oracle (fp64, numpy)."""
    from workloads import bounded_arity_forest, make_cell_values, make_values, to_bf16_bits, bf16_bits_to_f32, tree_ranges
    Nc = args.nary
    t0 = time.time()
    parent = bounded_arity_forest(cfg.n_trees, cfg.size_lo, cfg.size_hi, Nc, 700 + cfg.index)
    N = int(parent.shape[0])
    x = make_values(cfg.index, N, "zero", D=D, H=H)[0]
    (W, U, b), = make_cell_values([Nc], D, H, 800 + cfg.index)
    log(f"{cfg.n_trees} trees with at most {Nc} children per node: N={N} generated in {time.time() - t0:.1f}s")
    if esz == 2:
        def up(a):
            bits = to_bf16_bits(a)
            return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev), bf16_bits_to_f32(bits)
    else:
        def up(a):
            return torch.from_numpy(a).to(dev), a
    (xt, xs), (Wt, Ws), (Ut, Us) = up(x), up(W), up(U)
    bt = torch.from_numpy(b).to(dev)
    pt = torch.from_numpy(parent).to(dev)
    st_ = torch.zeros(N, dtype=torch.int32, device=dev)
    dt = J.JITDB_BF16 if esz == 2 else J.JITDB_F32
    sched = J.jitdb_schedule_typed(pt, st_, 1)
    E = sched.n_edges
    cells = [(J.JITDB_CELL_NARY, Nc, Wt, Ut, bt)]
    ws_s = torch.empty(J.jitdb_schedule_typed_workspace_bytes(N, 1), dtype=torch.uint8, device=dev)
    ws_f = torch.empty(J.jitdb_treelstm_cells_workspace_bytes(N, E, D, H, dt, [(J.JITDB_CELL_NARY, Nc)]),
                       dtype=torch.uint8, device=dev)
    h = torch.empty((N, H), dtype=xt.dtype, device=dev)
    c = torch.empty((N, H), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def sch():
        J.jitdb_schedule_typed(pt, st_, 1, stream=stream, workspace=ws_s, out=sched)

    def fwd():
        J.jitdb_treelstm_forward_cells(xt, cells, sched, stream=stream, workspace=ws_f, out=(h, c))

    for _ in range(args.warmup):
        sch(); fwd()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sch(); fwd()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fwd()
    torch.cuda.synchronize()
    ms_f = (time.perf_counter() - t0) * 1e3 / args.steps
    # algorithmic work: a leaf needs i, o, u from x; an internal node all 3 + N gates from x and from each child's h
    n_leaf = int(sched.host_level_ptr[1])
    f_alg = n_leaf * 2.0 * D * 3 * H + (N - n_leaf) * 2.0 * D * (3 + Nc) * H + E * 2.0 * H * (3 + Nc) * H
    # parity of the timed output on the first trees
    from oracle import treelstm_cells_oracle as C
    r = tree_ranges(parent)
    k = int(np.searchsorted(r, 4000))
    n_s = int(r[max(k, 1)])
    ho, co = C.forward_cells(parent[:n_s], np.zeros(n_s, np.int32), xs[:n_s], [C.nary_cell(Nc, Ws, Us, b)])
    hg, cg = h[:n_s].float().cpu().numpy(), c[:n_s].cpu().numpy()
    tol = 2e-2 if esz == 2 else 1e-4
    dh, dc = float(np.abs(hg - ho).max()), float(np.abs(cg - co).max())
    ok = bool(dh <= tol and dc <= tol * max(1.0, float(np.abs(co).max()) / (8.0 if esz == 2 else 50.0)))
    out = {
        "metric": f"Tree-LSTM forward nodes/sec on 1 MI355X, {Nc}-ary cell", "value": N / (ms_step * 1e-3),
        "unit": "nodes/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.n_trees} trees of {cfg.size_lo}-{cfg.size_hi} nodes, at most {Nc} children per node, "
                               f"one {Nc}-ary Tree-LSTM cell", "n_nodes": N, "n_edges": E, "n_levels": sched.n_levels,
                   "D": D, "H": H, "step": "jitdb_schedule_typed + jitdb_treelstm_forward_cells, one stream"},
        "ms_forward": ms_f,
        "roofline": {"kernel": "N-ary forward as a whole (nary_stack_kernel, gemm_kb_kernel, nary_cell_kernel per slot)",
                     "bound": "mfma", "achieved": f_alg / (ms_f * 1e-3) / 1e12, "peak": peak_tflops, "unit": "TFLOP/s",
                     "frac": f_alg / (ms_f * 1e-3) / 1e12 / peak_tflops, "traffic": None, "flops_per_step": f_alg},
        "parity": {"nodes": n_s, "max_abs_dh": dh, "max_abs_dc": dc, "tolerance": tol, "ok": ok},
    }
    print(json.dumps(out), flush=True)
    if not ok:
        sys.exit(1)


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload config index (1-5)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket kernels with events inside the timed region")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 1 GiB device copy (reference for HBM counters)")
    ap.add_argument("--cpu-trees", type=int, default=0, help="trees in the oracle sample (0 = auto)")
    ap.add_argument("--no-peaks", action="store_true", help="skip the copy / MFMA peak probes")
    ap.add_argument("--train", action="store_true",
                    help="time the training step instead (schedule + forward that keeps the gates + backward); "
                         "not the headline metric")
    ap.add_argument("--signatures", type=int, default=0,
                    help="time the typed table instead: every tree under one of this many networks "
                         "(jitdb_schedule_typed + jitdb_treelstm_forward_typed); not the headline metric")
    ap.add_argument("--signatures-per-node", action="store_true",
                    help="with --signatures >= 2: draw the signature per node (leaves cell 0, others 1..n-1) instead of per tree")
    ap.add_argument("--nary", type=int, default=0,
                    help="time a table with one N-ary Tree-LSTM cell (N = this, 1..4) over trees of bounded arity "
                         "(jitdb_schedule_typed + jitdb_treelstm_forward_cells); not the headline metric")
    ap.add_argument("--serial", action="store_true",
                    help="schedule and forward of a batch strictly one after the other on one stream "
                         "(default: the schedule of the next batch overlaps the forward of this one)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the forest shards by tree with no "
              "exchange). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1904_07421_amd as J
    from workloads import CONFIGS, make_forest, make_values, to_bf16_bits, bf16_bits_to_f32, tree_ranges

    cfg = CONFIGS[args.config]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.nary > 0:
        bf = cfg.dtype == "bf16"
        return nary_bench(args, J, torch, cfg, dev, cfg.D, cfg.H, 2 if bf else 4,
                          PEAK_BF16_TFLOPS if bf else PEAK_F32_MFMA_TFLOPS)

    t0 = time.time()
    parent = make_forest(cfg.index)
    N = int(parent.shape[0])
    x, W, U, b = make_values(cfg.index, N)
    log(f"config {cfg.index} ({cfg.name}): N={N} generated in {time.time() - t0:.1f}s")
    D, H = cfg.D, cfg.H
    if cfg.dtype == "bf16":
        def up(a):
            bits = to_bf16_bits(a)
            return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(dev), bits
        xt, xbits = up(x)
        Wt, Wbits = up(W)
        Ut, Ubits = up(U)
        esz = 2
        peak_tflops = PEAK_BF16_TFLOPS
    else:
        xt, Wt, Ut = (torch.from_numpy(a).to(dev) for a in (x, W, U))
        esz = 4
        peak_tflops = PEAK_F32_MFMA_TFLOPS
    bt = torch.from_numpy(b).to(dev)
    pt = torch.from_numpy(parent).to(dev)
    log(f"inputs resident on {torch.cuda.get_device_name(0)} after {time.time() - t0:.1f}s")

    # one untimed call sizes the buffers; they are then reused by every step
    sched = J.jitdb_schedule(pt)
    E, L = sched.n_edges, sched.n_levels
    lp = sched.host_level_ptr[:L + 1].astype(np.int64)
    n_leaf = int(lp[1])
    n_int = N - n_leaf
    ws_s = torch.empty(J.jitdb_schedule_workspace_bytes(N), dtype=torch.uint8, device=dev)
    if args.signatures > 0:
        return typed_bench(args, J, torch, cfg, dev, N, D, H, esz, peak_tflops, xt, parent, n_leaf, n_int, E)
    if args.train:
        return train_bench(args, J, torch, cfg, dev, N, D, H, esz, peak_tflops, xt, Wt, Ut, bt, pt, sched, ws_s,
                           n_leaf, n_int, E, L)
    ws_f = torch.empty(J.jitdb_treelstm_workspace_bytes(N, E, D, H, J.JITDB_BF16 if esz == 2 else J.JITDB_F32),
                       dtype=torch.uint8, device=dev)
    h = torch.empty((N, H), dtype=xt.dtype, device=dev)
    c = torch.empty((N, H), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def step_serial():     # every buffer is reused; the schedule is recomputed from the parent array
        s = J.jitdb_schedule(pt, stream=stream, workspace=ws_s, out=sched)
        J.jitdb_treelstm_forward(xt, Wt, Ut, bt, s, stream=stream, workspace=ws_f, out=(h, c))

    # Batches arrive one after another: the analysis of batch i+1 runs on a second stream while
    # batch i executes (the call blocks the host, not the GPU).  Two schedule objects take turns;
    # an event keeps the analysis from overwriting one that a forward still reads.  Every step is
    # still one jitdb_schedule (from the parent array) and one jitdb_treelstm_forward.
    s_fwd, s_sch = torch.cuda.Stream(), torch.cuda.Stream()
    scheds = [sched, J.jitdb_schedule(pt)]
    ws_ss = [ws_s, torch.empty_like(ws_s)]
    last_use = [None, None]
    turn = [0]

    def step_pipelined():
        k = turn[0] & 1
        J.jitdb_treelstm_forward(xt, Wt, Ut, bt, scheds[k], stream=s_fwd, workspace=ws_f, out=(h, c))
        last_use[k] = torch.cuda.Event()
        last_use[k].record(s_fwd)
        if last_use[k ^ 1] is not None:
            s_sch.wait_event(last_use[k ^ 1])
        J.jitdb_schedule(pt, stream=s_sch, workspace=ws_ss[k ^ 1], out=scheds[k ^ 1])
        turn[0] += 1

    def rate(fn, n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / n

    # Forests with many thin levels are a chain of short dependent kernels; there a second stream
    # only gets in the way.  Unless --serial forces it, a short trial picks the faster mode.
    pipelined = not args.serial
    if pipelined:
        torch.cuda.synchronize()
        J.jitdb_schedule(pt, stream=s_sch, workspace=ws_ss[0], out=scheds[0])
        rate(step_pipelined, 2); rate(step_serial, 2)
        t_pipe, t_ser = rate(step_pipelined, 3), rate(step_serial, 3)
        pipelined = t_pipe <= t_ser
        log(f"trial: pipelined {t_pipe * 1e3:.3f} ms/step, serial {t_ser * 1e3:.3f} ms/step -> "
            f"{'pipelined' if pipelined else 'serial'}")
        if pipelined:       # leave the pipeline primed: scheds[turn & 1] holds a finished analysis
            torch.cuda.synchronize()
    step = step_pipelined if pipelined else step_serial

    if args.calibration_copy:
        # a plain copy of known size (1 GiB read + 1 GiB written, more than the 256 MB last-level
        # cache holds), for scaling the
        # FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command
        src = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # The timed region: exactly K steps, nothing but the library's own launches on the streams.
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    ms_per_step = (t_end - t_begin) * 1e3 / args.steps
    value = N / (ms_per_step * 1e-3)

    # The same K steps once more with a HIP event pair around every kernel launch, on the launch
    # stream (jitdb_profile_start/stop): the per-kernel durations behind `roofline` and `kernels`.
    # Kept out of the region above because the event records themselves keep consecutive kernels
    # from overlapping (about 3 % of a step at config 5, a third for a forest of many thin levels).
    launches_per_step = 1 + 3 * L
    prof = None
    ms_with_events = None
    if not args.no_kernel_events:
        J.jitdb_profile_start(launches_per_step * args.steps + 8)
        ms_with_events = rate(step, args.steps) * 1e3
        prof = J.jitdb_profile_stop()

    # schedule and forward separately (same buffers), HIP events on the launch stream
    def timed(fn, reps):
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) / reps
    reps = max(3, min(args.steps, 10))
    ms_sched = timed(lambda: J.jitdb_schedule(pt, stream=stream, workspace=ws_s, out=sched), reps)
    ms_fwd = timed(lambda: J.jitdb_treelstm_forward(xt, Wt, Ut, bt, sched, stream=stream,
                                                     workspace=ws_f, out=(h, c)), reps)

    # the forward with weights packed beforehand (a serving loop whose weights do not change)
    packed = J.jitdb_treelstm_pack(Wt, Ut, bt, stream=stream)
    ms_fwd_packed = timed(lambda: J.jitdb_treelstm_forward_packed(xt, packed, sched, stream=stream,
                                                                   workspace=ws_f, out=(h, c)), reps)
    del packed

    # a cache hit instead of the analysis: fingerprint of the parent array + table lookup (host clock:
    # the call synchronises to hand the fingerprint to the host)
    cache = J.ScheduleCache(2)
    cache.get(pt, stream=stream)
    torch.cuda.synchronize()
    t_c = time.perf_counter()
    for _ in range(reps):
        _, hit = cache.get(pt, stream=stream)
        assert hit
    ms_cache_hit = (time.perf_counter() - t_c) * 1e3 / reps
    del cache

    # algorithmic work per step and per kernel class (padding and unused rows do not count);
    # the library reports how many level rows each class of launches covered
    flops_row = {"leaf": 2.0 * D * 3 * H, "internal": 2.0 * D * 4 * H + 2.0 * H * 3 * H, "proj": 2.0 * H * H,
                 # a level of one-child nodes in one launch: the internal row's work plus its child's projection
                 "chain": 2.0 * D * 4 * H + 2.0 * H * 4 * H}
    flops_total = {"leaf": n_leaf * flops_row["leaf"], "internal": n_int * flops_row["internal"],
                   "proj": E * flops_row["proj"]}
    # Algorithmic bytes per row of each kernel class as this design moves them (padding does not count):
    #   leaf      reads its stacked x row, writes h and c (fp32)
    #   internal  reads its stacked [x | sum h] row, per child P_k and c_k (fp32), writes h and c
    #   proj      reads h, writes P
    #   chain     reads its x row, its child's h and c, writes h and c
    bytes_row = {"leaf": D * esz + H * esz + 4.0 * H,
                 "internal": (D + H) * esz + H * esz + 4.0 * H,
                 "proj": 2.0 * H * esz,
                 "chain": D * esz + H * esz + 4.0 * H + H * esz + 4.0 * H}
    bytes_edge_internal = H * esz + 4.0 * H
    # the gather ("stack" step): the child sum reads every child's h row once and writes one row per
    # internal node; the copy of x into the stacked matrix (read + written) is overhead of this design
    bytes_gather = (E * H + n_int * H) * esz
    bytes_xcopy = 2.0 * N * D * esz
    # the fully fused minimum of the whole forward: x, h, c once, h_k and c_k once per edge, weights once
    bytes_min = N * (D * esz + H * esz + 4.0 * H) + E * (H * esz + 4.0 * H) + (D + H) * 4.0 * H * esz
    ridge = peak_tflops * 1e12 / (PEAK_HBM_GBS * 1e9)      # flop per byte at which the two roofs meet
    kernels = {}
    roof = None
    if prof is not None:
        proj_rows = (prof["proj"]["rows"] + prof["thin_proj"]["rows"]) / args.steps   # includes roots, whose P nobody reads
        chain_rows = prof["chain"]["edges"] / args.steps     # edges projected inside the chain launches (one per row)
        for name in ("leaf", "internal", "proj", "thin_leaf", "thin_internal", "thin_proj", "chain"):
            job = name.replace("thin_", "")
            ms = prof[name]["ms"] / args.steps
            n_l = prof[name]["launches"] / args.steps
            rows = prof[name]["rows"] / args.steps
            fl = rows * flops_row[job]
            if job == "proj" and proj_rows > 0:
                fl *= (E - chain_rows) / proj_rows
            if ms > 0:
                by = rows * bytes_row[job]
                if job == "internal":      # its share of the edges, by rows (exact when one class holds all of them)
                    by += (E - chain_rows) * bytes_edge_internal * rows / max(n_int - chain_rows, 1)
                gbs = by / (ms * 1e-3) / 1e9
                kernels[name] = {"ms_per_step": ms, "launches_per_step": n_l, "rows_per_step": rows,
                                 "flops_per_step": fl, "tflops": fl / (ms * 1e-3) / 1e12,
                                 "frac_mfma_peak": fl / (ms * 1e-3) / 1e12 / peak_tflops,
                                 "bytes_per_step": by, "gbs": gbs, "frac_hbm_peak": gbs / PEAK_HBM_GBS,
                                 "flop_per_byte": fl / by,
                                 # the roof that binds a kernel of this intensity
                                 "bound": "mfma" if fl / by >= ridge else "hbm"}
        ms = prof["stack"]["ms"] / args.steps
        if ms > 0:
            kernels["stack"] = {"ms_per_step": ms,
                                "launches_per_step": prof["stack"]["launches"] / args.steps,
                                "bound": "hbm",
                                # the gather proper (child sums): what the metric's "HBM GB/s of the gather" means
                                "gather_bytes_per_step": bytes_gather,
                                "gbs": bytes_gather / (ms * 1e-3) / 1e9,
                                "frac_hbm_peak": bytes_gather / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                # with the copy of x (this design's overhead) counted as moved bytes too
                                "xcopy_bytes_per_step": bytes_xcopy,
                                "gbs_with_xcopy": (bytes_gather + bytes_xcopy) / (ms * 1e-3) / 1e9}
        kernels["pack"] = {"ms_per_step": prof["pack"]["ms"] / args.steps}
        mfma_names = [n for n in ("leaf", "internal", "proj", "thin_leaf", "thin_internal", "thin_proj", "chain") if n in kernels]
        dom = max(mfma_names, key=lambda k: kernels[k]["ms_per_step"])
        k = kernels[dom]
        kname = (f"thin_kernel<{cfg.dtype},{dom[5:]}>" if dom.startswith("thin_") else
                 f"chain_kernel<{cfg.dtype}>" if dom == "chain" else f"level_kernel<{cfg.dtype},{dom}>")
        # the dominant kernel against the roof that binds a kernel of its own intensity; the other
        # roof's fraction is given beside it
        launches = max(k["launches_per_step"], 1)
        if k["bound"] == "mfma":
            roof = {"kernel": kname, "bound": "mfma", "achieved": k["tflops"], "peak": peak_tflops,
                    "unit": "TFLOP/s", "frac": k["frac_mfma_peak"]}
        else:
            roof = {"kernel": kname, "bound": "hbm", "achieved": k["gbs"], "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": k["frac_hbm_peak"]}
        roof.update({"traffic": measured_traffic(cfg, f"traffic_bytes_per_launch[{dom}]"),
                     "avg_launch_ms": k["ms_per_step"] / launches,
                     "flop_per_byte": k["flop_per_byte"], "ridge_flop_per_byte": ridge,
                     "frac_mfma_peak": k["frac_mfma_peak"], "frac_hbm_peak": k["frac_hbm_peak"],
                     "tflops": k["tflops"], "gbs": k["gbs"],
                     "flops_per_launch": k["flops_per_step"] / launches, "bytes_per_launch": k["bytes_per_step"] / launches,
                     "flops_per_step": k["flops_per_step"], "dropped_events": prof["dropped"]})
        tt = measured_traffic(cfg, "traffic_bytes_per_forward")
        roof["traffic_total"] = tt
        roof["traffic_total_over_bytes_min"] = None if tt is None else tt / bytes_min
        mfma_ms = sum(kernels[n]["ms_per_step"] for n in mfma_names)
        roof["all_mfma_kernels_frac"] = sum(flops_total.values()) / (mfma_ms * 1e-3) / 1e12 / peak_tflops

    # what this machine sustains: a plain device copy (1 GiB each way) and a loop of independent MFMAs
    measured = None
    if not args.no_peaks:
        src = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev).fill_(1.0)
        dst = torch.empty_like(src)
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        measured = {"copy_gbs": J.jitdb_probe_copy(src, dst, stream=stream),
                    "mfma_tflops": J.jitdb_probe_mfma(J.JITDB_BF16 if esz == 2 else J.JITDB_F32, sink, stream=stream),
                    "what": "plain 1 GiB device copy, read + written; loop of independent 32x32 MFMAs on all CUs"}
        # other shapes of stream: the best of them is the ceiling the HBM-bound pieces are quoted against
        for kind, name in ((1, "read_gbs"), (2, "write_gbs"), (3, "copy_nt_gbs"), (4, "copy_chunk_gbs")):
            measured[name] = J.jitdb_probe_stream(kind, src, dst, stream=stream)
        measured["best_copy_gbs"] = max(measured["copy_gbs"], measured["copy_nt_gbs"], measured["copy_chunk_gbs"])
        measured["what"] += ("; read-only, write-only, non-temporal and per-block-chunk copies of the same 1 GiB "
                             "(best_copy_gbs = the fastest copy)")
        if roof is not None:
            roof["measured_peak"] = measured["mfma_tflops"] if roof["bound"] == "mfma" else measured["best_copy_gbs"]
            roof["frac_of_measured_peak"] = roof["achieved"] / roof["measured_peak"]
        if "stack" in kernels:
            kernels["stack"]["frac_of_measured_copy"] = kernels["stack"]["gbs_with_xcopy"] / measured["best_copy_gbs"]
        del src, dst

    out = {
        "metric": "Tree-LSTM forward nodes/sec on 1 MI355X; MFMA util % + HBM GB/s vs peak",
        "value": value, "unit": "nodes/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"config {cfg.index}: {cfg.name}", "n_trees": cfg.n_trees, "n_nodes": N,
                   "n_edges": E, "n_levels": L, "D": D, "H": H,
                   "step": "jitdb_schedule + jitdb_treelstm_forward per batch" +
                           ("; schedule of batch i+1 on a second stream beside the forward of batch i" if pipelined else "; one stream")},
        "ms_schedule": ms_sched, "ms_forward": ms_fwd, "ms_per_step_one_stream": ms_sched + ms_fwd,
        "ms_schedule_cache_hit": ms_cache_hit, "ms_forward_packed_weights": ms_fwd_packed,
        "ms_per_step_with_kernel_events": ms_with_events,
        "forward_only_nodes_per_s": N / (ms_fwd * 1e-3),
        # the whole forward against its own roofline: max(F_min / MFMA peak, bytes_min / HBM peak) / ms_forward
        "forward_roofline": {"f_min_flops": sum(flops_total.values()), "bytes_min": bytes_min,
                             "ms_at_mfma_peak": sum(flops_total.values()) / (peak_tflops * 1e12) * 1e3,
                             "ms_at_hbm_peak": bytes_min / (PEAK_HBM_GBS * 1e9) * 1e3},
        "forward_frac_of_roofline": max(sum(flops_total.values()) / (peak_tflops * 1e12),
                                        bytes_min / (PEAK_HBM_GBS * 1e9)) * 1e3 / ms_fwd,
        "roofline": roof, "kernels": kernels, "measured_peaks": measured,
        # the metric's other two figures: useful flops of all MFMA kernels / their summed time, as % of the bf16
        # (fp32) MFMA peak; algorithmic bytes of the gather ("stack") kernels / their time, and as % of 8 TB/s
        "mfma_util_pct": None if roof is None else 100.0 * roof["all_mfma_kernels_frac"],
        "hbm_gbs_gather": kernels.get("stack", {}).get("gbs"),
        "hbm_pct_gather": None if "stack" not in kernels or "gbs" not in kernels["stack"]
        else 100.0 * kernels["stack"]["frac_hbm_peak"],
    }

    if not args.no_cpu_baseline:
        from oracle.build import forward_c
        r = tree_ranges(parent)
        n_trees = args.cpu_trees or min(len(r) - 1, max(64, int(8192 * (812 * 2048) / ((D + H) * 4.0 * H))))
        n_trees = min(n_trees, len(r) - 1)
        hi = int(r[n_trees])
        sub = parent[:hi]
        if esz == 2:
            xo, Wo, Uo = (bf16_bits_to_f32(a) for a in (xbits[:hi], Wbits, Ubits))
        else:
            xo, Wo, Uo = x[:hi], W, U
        forward_c(sub[:r[1]], xo[:r[1]], Wo, Uo, b)          # build + first-touch outside the clock
        forward_c(sub[:r[1]], xo[:r[1]], Wo, Uo, b, precision="f32")
        # the oracle as it is used for parity: fp64, every host core
        t1 = time.perf_counter()
        ho, co, used = forward_c(sub, xo, Wo, Uo, b)
        dt = time.perf_counter() - t1
        # ... and what it just computed is compared with what the GPU computed in the timed steps
        # (h, c of the last forward; the forest's first trees are the same nodes in both)
        hg = h[:hi].float().cpu().numpy()
        cg = c[:hi].cpu().numpy()
        tol = 2e-2 if esz == 2 else 1e-4
        parity = {"nodes": hi, "max_abs_dh": float(np.abs(hg - ho).max()), "max_abs_dc": float(np.abs(cg - co).max()),
                  "tolerance": tol}
        parity["ok"] = bool(parity["max_abs_dh"] <= tol and parity["max_abs_dc"] <= tol)
        del ho, co, hg, cg
        # the same source compiled with fp32 arithmetic: the timing build (never compared with anything)
        t1 = time.perf_counter()
        _, _, used32 = forward_c(sub, xo, Wo, Uo, b, precision="f32")
        dt32 = time.perf_counter() - t1
        # the fp64 oracle on one thread, on a sixteenth of the sample
        n1 = max(1, n_trees // 16)
        hi1 = int(r[n1])
        t1 = time.perf_counter()
        forward_c(sub[:hi1], xo[:hi1], Wo, Uo, b, n_threads=1)
        dt1 = time.perf_counter() - t1
        out["cpu_baseline"] = {"value": hi / dt, "unit": "nodes/s", "cores": int(used), "kind": "oracle",
                               "sample": f"first {n_trees} trees ({hi} nodes) of the same forest, "
                                         f"fp64 C oracle (-O3 -march=native) with OpenMP over trees, {dt:.1f}s",
                               "fp32_build": {"value": hi / dt32, "unit": "nodes/s", "cores": int(used32),
                                              "sample": f"same trees, the oracle's source compiled with float, {dt32:.1f}s"},
                               "one_thread": {"value": hi1 / dt1, "unit": "nodes/s", "cores": 1,
                                              "sample": f"first {n1} trees ({hi1} nodes), fp64, {dt1:.1f}s"}}
        out["parity"] = parity
        if not parity["ok"]:
            log(f"PARITY FAILED against the oracle: {parity}")
    print(json.dumps(out), flush=True)
    if out.get("parity") is not None and not out["parity"]["ok"]:
        sys.exit(1)


if __name__ == "__main__":
    main()
