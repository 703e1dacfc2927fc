"""The forward for callers that cannot allocate (jitdb_treelstm_forward_static): through the C ABI,
against jitdb_treelstm_forward with a caller workspace, on two calls in a row, the second smaller."""
import ctypes

import numpy as np
import pytest

from workloads import make_workload
from gpu_util import dev_parent, bf16_tensor

pytestmark = pytest.mark.gpu


def _device_inputs(cfg, dtype):
    import torch
    cfgo, p, x, W, U, b = make_workload(cfg, bias="random")
    if dtype == "bf16":
        xt, Wt, Ut = bf16_tensor(x)[0], bf16_tensor(W)[0], bf16_tensor(U)[0]
    else:
        xt, Wt, Ut = (torch.from_numpy(a).cuda() for a in (x, W, U))
    return p, xt, Wt, Ut, torch.from_numpy(b).cuda()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_static_scratch_forward_equals_the_workspace_forward(dtype):
    import torch
    import paper_1904_07421_amd as J
    from paper_1904_07421_amd import binding
    lib = binding.load_library()
    dt = J.JITDB_F32 if dtype == "f32" else J.JITDB_BF16
    for cfg in (2, 1):                       # the second forest is the smaller one: stale scratch must not matter
        p, xt, Wt, Ut, bt = _device_inputs(cfg, dtype)
        s = J.jitdb_schedule(dev_parent(p))
        n, D, H = p.shape[0], Wt.shape[1], Ut.shape[1]
        print(f"static-scratch forward cfg={cfg} dtype={dtype} N={n}", flush=True)
        h_ref, c_ref = J.jitdb_treelstm_forward(xt, Wt, Ut, bt, s)
        h = torch.full((n, H), float("nan"), dtype=xt.dtype, device="cuda")
        c = torch.full((n, H), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        # raw C ABI call: pointers and sizes only
        code = lib.jitdb_treelstm_forward_static(
            xt.data_ptr(), Wt.data_ptr(), Ut.data_ptr(), bt.data_ptr(), D, H, dt,
            ctypes.byref(s.struct), h.data_ptr(), c.data_ptr(), int(torch.cuda.current_stream().cuda_stream))
        assert code == 0, J.jitdb_strerror(code)
        torch.cuda.synchronize()
        # same kernels, same order of arithmetic: the results are the same bits
        assert torch.equal(h, h_ref) and torch.equal(c, c_ref)
        # and the Python binding of the same name marshals the same call
        h2 = torch.empty_like(h); c2 = torch.empty_like(c)
        J.jitdb_treelstm_forward_static(xt, Wt, Ut, bt, s, out=(h2, c2))
        torch.cuda.synchronize()
        assert torch.equal(h2, h_ref) and torch.equal(c2, c_ref)


def test_static_scratch_forward_refuses_what_does_not_fit():
    import torch
    import paper_1904_07421_amd as J
    p, xt, Wt, Ut, bt = _device_inputs(3, "bf16")     # 105 k nodes: needs more than the fixed array holds
    s = J.jitdb_schedule(dev_parent(p))
    n, D, H = p.shape[0], Wt.shape[1], Ut.shape[1]
    assert J.jitdb_treelstm_workspace_bytes(n, s.n_edges, D, H, J.JITDB_BF16) > 64 * 1024 * 1024
    h = torch.zeros((n, H), dtype=xt.dtype, device="cuda"); c = torch.zeros((n, H), device="cuda")
    with pytest.raises(J.JitdbError) as e:
        J.jitdb_treelstm_forward_static(xt, Wt, Ut, bt, s, out=(h, c))
    assert e.value.code == -5
    torch.cuda.synchronize()
    assert not bool(h.any()) and not bool(c.any())     # nothing ran
