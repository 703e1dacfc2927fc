"""Helpers shared by the GPU parity tests: move seeded inputs to the device,
call the library through its binding, bring results back as numpy."""
from __future__ import annotations

import numpy as np

from workloads import to_bf16_bits, bf16_bits_to_f32


def dev_parent(parent):
    import torch
    return torch.from_numpy(np.ascontiguousarray(parent, dtype=np.int32)).cuda()


def bf16_tensor(a32: np.ndarray):
    """fp32 array -> (bf16 CUDA tensor, the same values widened to fp32 numpy)."""
    import torch
    bits = to_bf16_bits(a32)
    t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    return t, bf16_bits_to_f32(bits)


def run_gpu_forward(parent, x, W, U, b, dtype: str):
    """Schedule + forward on the GPU.  Returns (schedule, h, c, inputs_as_seen_by_gpu)
    where h, c are fp32 numpy arrays and inputs are what the oracle must be fed."""
    import torch
    import paper_1904_07421_amd as J
    dp = dev_parent(parent)
    sched = J.jitdb_schedule(dp)
    bt = torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).cuda()
    if dtype == "bf16":
        xt, xo = bf16_tensor(x)
        Wt, Wo = bf16_tensor(W)
        Ut, Uo = bf16_tensor(U)
    else:
        xt = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
        Wt = torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32)).cuda()
        Ut = torch.from_numpy(np.ascontiguousarray(U, dtype=np.float32)).cuda()
        xo, Wo, Uo = x, W, U
    h, c = J.jitdb_treelstm_forward(xt, Wt, Ut, bt, sched)
    torch.cuda.synchronize()
    return sched, h.float().cpu().numpy(), c.cpu().numpy(), (xo, Wo, Uo, b)


def assert_schedule_equal(got: dict, want: dict):
    assert got["n_levels"] == want["n_levels"], (got["n_levels"], want["n_levels"])
    assert got["n_edges"] == want["n_edges"]
    if "level_kids" in got:     # children per level: the sum of the oracle's arities over each level
        arity = np.diff(np.asarray(want["child_ptr"]))
        kids = np.bincount(np.asarray(want["height"]), weights=arity, minlength=want["n_levels"]).astype(np.int64)
        assert np.array_equal(np.asarray(got["level_kids"]), kids), ("level_kids", got["level_kids"][:8], kids[:8])
    for k in ("height", "level_ptr", "perm", "inv_perm", "child_ptr", "child_idx"):
        g, w = np.asarray(got[k]), np.asarray(want[k])
        assert g.shape == w.shape, (k, g.shape, w.shape)
        if not np.array_equal(g, w):
            bad = np.flatnonzero(g != w)
            raise AssertionError(f"{k}: {bad.size} mismatches, first at {bad[0]}: "
                                 f"got {g[bad[0]]} want {w[bad[0]]}")
