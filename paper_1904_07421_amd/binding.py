"""ctypes binding of the C ABI in include/jitdb.h.

PyTorch supplies device memory and the HIP stream; nothing is computed here.
The shared library must have been built (paper_1904_07421_amd/build.py); if it
is missing the binding builds it once, and if that fails every call raises.
There is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libjitdb.so")

JITDB_F32 = 0
JITDB_CELL_CHILDSUM = 0
JITDB_CELL_NARY = 1
JITDB_MAX_NARY = 4
JITDB_BF16 = 1

_c_i32p = ctypes.POINTER(ctypes.c_int32)


class JitdbError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"jitdb error {code}: {msg}")
        self.code = code


class _ScheduleStruct(ctypes.Structure):
    _fields_ = [
        ("n_nodes", ctypes.c_int64),
        ("height", ctypes.c_void_p),
        ("level_ptr", ctypes.c_void_p),
        ("perm", ctypes.c_void_p),
        ("inv_perm", ctypes.c_void_p),
        ("child_ptr", ctypes.c_void_p),
        ("child_idx", ctypes.c_void_p),
        ("host_level_ptr", ctypes.c_void_p),
        ("n_levels", ctypes.c_int32),
        ("n_edges", ctypes.c_int64),
        ("host_level_kids", ctypes.c_void_p),
    ]


class _SlotsStruct(ctypes.Structure):
    _fields_ = [
        ("n_sig", ctypes.c_int32),
        ("slot_capacity", ctypes.c_int64),
        ("key", ctypes.c_void_p),
        ("slot_ptr", ctypes.c_void_p),
        ("host_slot_ptr", ctypes.c_void_p),
    ]


K_CLASSES = ("pack", "stack", "leaf", "internal", "proj", "thin_leaf", "thin_internal", "thin_proj", "chain")


class _CellStruct(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("arity", ctypes.c_int32),
                ("W", ctypes.c_void_p), ("U", ctypes.c_void_p), ("b", ctypes.c_void_p)]


class _ProfileStruct(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_double * 9), ("launches", ctypes.c_int64 * 9),
                ("rows", ctypes.c_int64 * 9), ("edges", ctypes.c_int64 * 9), ("dropped", ctypes.c_int64)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libjitdb.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    lib.jitdb_schedule_workspace_bytes.restype = ctypes.c_size_t
    lib.jitdb_schedule_workspace_bytes.argtypes = [ctypes.c_int64]
    lib.jitdb_schedule.restype = ctypes.c_int
    lib.jitdb_schedule.argtypes = [ctypes.c_void_p, ctypes.POINTER(_ScheduleStruct),
                                   ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.jitdb_schedule_append_workspace_bytes.restype = ctypes.c_size_t
    lib.jitdb_schedule_append_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64]
    lib.jitdb_schedule_append.restype = ctypes.c_int
    lib.jitdb_schedule_append.argtypes = [ctypes.POINTER(_ScheduleStruct), ctypes.c_void_p, ctypes.c_int64,
                                          ctypes.POINTER(_ScheduleStruct), ctypes.c_void_p, ctypes.c_size_t,
                                          ctypes.c_void_p]
    lib.jitdb_treelstm_workspace_bytes.restype = ctypes.c_size_t
    lib.jitdb_treelstm_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                                   ctypes.c_int32, ctypes.c_int]
    lib.jitdb_treelstm_forward.restype = ctypes.c_int
    lib.jitdb_treelstm_forward.argtypes = [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_int32, ctypes.c_int32, ctypes.c_int,
        ctypes.POINTER(_ScheduleStruct), ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.jitdb_treelstm_forward_static.restype = ctypes.c_int
    lib.jitdb_treelstm_forward_static.argtypes = [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_int32, ctypes.c_int32, ctypes.c_int,
        ctypes.POINTER(_ScheduleStruct), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.jitdb_treelstm_forward_train.restype = ctypes.c_int
    lib.jitdb_treelstm_forward_train.argtypes = [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_int32, ctypes.c_int32, ctypes.c_int,
        ctypes.POINTER(_ScheduleStruct), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.jitdb_treelstm_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.jitdb_treelstm_backward_workspace_bytes.argtypes = [ctypes.POINTER(_ScheduleStruct), ctypes.c_int32,
                                                            ctypes.c_int32, ctypes.c_int]
    lib.jitdb_treelstm_backward.restype = ctypes.c_int
    lib.jitdb_treelstm_backward.argtypes = [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int,
        ctypes.POINTER(_ScheduleStruct), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.jitdb_profile_start.restype = ctypes.c_int
    lib.jitdb_profile_start.argtypes = [ctypes.c_int32]
    lib.jitdb_profile_stop.restype = ctypes.c_int
    lib.jitdb_profile_stop.argtypes = [ctypes.POINTER(_ProfileStruct)]
    lib.jitdb_probe_stream.restype = ctypes.c_int
    lib.jitdb_probe_stream.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                       ctypes.c_void_p, ctypes.POINTER(ctypes.c_double)]
    lib.jitdb_probe_copy.restype = ctypes.c_int
    lib.jitdb_probe_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                     ctypes.POINTER(ctypes.c_double)]
    lib.jitdb_probe_mfma.restype = ctypes.c_int
    lib.jitdb_probe_mfma.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                     ctypes.POINTER(ctypes.c_double)]
    lib.jitdb_schedule_typed_workspace_bytes.restype = ctypes.c_size_t
    lib.jitdb_schedule_typed_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int32]
    lib.jitdb_schedule_typed.restype = ctypes.c_int
    lib.jitdb_schedule_typed.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(_ScheduleStruct),
                                         ctypes.POINTER(_SlotsStruct), ctypes.c_void_p, ctypes.c_size_t,
                                         ctypes.c_void_p]
    lib.jitdb_treelstm_typed_workspace_bytes.restype = ctypes.c_size_t
    lib.jitdb_treelstm_typed_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                                         ctypes.c_int32, ctypes.c_int, ctypes.c_int32]
    lib.jitdb_treelstm_forward_typed.restype = ctypes.c_int
    lib.jitdb_treelstm_forward_typed.argtypes = [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_int32, ctypes.c_int32, ctypes.c_int,
        ctypes.POINTER(_ScheduleStruct), ctypes.POINTER(_SlotsStruct), ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.jitdb_treelstm_packed_bytes.restype = ctypes.c_size_t
    lib.jitdb_treelstm_cells_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                                         ctypes.c_int32, ctypes.c_int, ctypes.POINTER(_CellStruct),
                                                         ctypes.c_int32]
    lib.jitdb_treelstm_cells_workspace_bytes.restype = ctypes.c_size_t
    lib.jitdb_treelstm_forward_cells.argtypes = [
        ctypes.c_void_p, ctypes.POINTER(_CellStruct), ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int,
        ctypes.POINTER(_ScheduleStruct), ctypes.POINTER(_SlotsStruct), ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.jitdb_treelstm_forward_cells.restype = ctypes.c_int
    lib.jitdb_treelstm_packed_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int, ctypes.c_int32]
    lib.jitdb_treelstm_pack.restype = ctypes.c_int
    lib.jitdb_treelstm_pack.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.c_int, ctypes.c_int32, ctypes.c_void_p,
                                        ctypes.c_size_t, ctypes.c_void_p]
    lib.jitdb_treelstm_forward_packed.restype = ctypes.c_int
    lib.jitdb_treelstm_forward_packed.argtypes = [
        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_int,
        ctypes.POINTER(_ScheduleStruct), ctypes.POINTER(_SlotsStruct), ctypes.c_void_p, ctypes.c_void_p,
        ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.jitdb_forest_fingerprint.restype = ctypes.c_int
    lib.jitdb_forest_fingerprint.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                             ctypes.POINTER(ctypes.c_uint64), ctypes.c_void_p]
    lib.jitdb_cache_create.restype = ctypes.c_int
    lib.jitdb_cache_create.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_void_p)]
    lib.jitdb_cache_destroy.restype = None
    lib.jitdb_cache_destroy.argtypes = [ctypes.c_void_p]
    lib.jitdb_cache_lookup.restype = ctypes.c_int32
    lib.jitdb_cache_lookup.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_uint64), ctypes.c_int64]
    lib.jitdb_cache_insert.restype = ctypes.c_int32
    lib.jitdb_cache_insert.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_uint64), ctypes.c_int64,
                                       ctypes.POINTER(ctypes.c_int32)]
    lib.jitdb_cache_stats.restype = None
    lib.jitdb_cache_stats.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64),
                                      ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32)]
    lib.jitdb_strerror.restype = ctypes.c_char_p
    lib.jitdb_strerror.argtypes = [ctypes.c_int]
    lib.jitdb_last_hip_error.restype = ctypes.c_char_p
    lib.jitdb_last_hip_error.argtypes = []
    lib.jitdb_version.restype = ctypes.c_char_p
    lib.jitdb_version.argtypes = []
    _lib = lib
    return lib


def jitdb_strerror(code: int) -> str:
    return load_library().jitdb_strerror(int(code)).decode()


def jitdb_version() -> str:
    return load_library().jitdb_version().decode()


def jitdb_profile_start(capacity: int) -> None:
    _check(load_library().jitdb_profile_start(int(capacity)))


def jitdb_profile_stop() -> dict:
    """{class: {"ms": total milliseconds, "launches": count, "rows": level rows covered}} plus "dropped"."""
    p = _ProfileStruct()
    _check(load_library().jitdb_profile_stop(ctypes.byref(p)))
    out = {name: {"ms": float(p.ms[i]), "launches": int(p.launches[i]), "rows": int(p.rows[i]), "edges": int(p.edges[i])}
           for i, name in enumerate(K_CLASSES)}
    out["dropped"] = int(p.dropped)
    return out


def jitdb_probe_copy(src, dst, stream=None) -> float:
    """(read + written) GB/s of a plain device copy of src into dst (equal-sized device tensors)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst differ in size")
    out = ctypes.c_double(0.0)
    _check(load_library().jitdb_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream_ptr(stream),
                                           ctypes.byref(out)))
    return float(out.value)


def jitdb_probe_stream(kind: int, src, dst, stream=None) -> float:
    """GB/s of one shape of memory stream over two equally sized CUDA tensors (kinds: 0 copy, 1 read,
    2 write, 3 copy with non-temporal accesses, 4 copy in per-block chunks)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst must have the same size")
    out = ctypes.c_double(0.0)
    _check(load_library().jitdb_probe_stream(int(kind), src.data_ptr(), dst.data_ptr(), nbytes, _stream_ptr(stream),
                                             ctypes.byref(out)))
    return float(out.value)


def jitdb_probe_mfma(dtype: int, sink, stream=None) -> float:
    """TFLOP/s of a loop of independent MFMAs of the dtype's kind; sink = device tensor of one float."""
    out = ctypes.c_double(0.0)
    _check(load_library().jitdb_probe_mfma(int(dtype), sink.data_ptr(), _stream_ptr(stream), ctypes.byref(out)))
    return float(out.value)


def jitdb_schedule_workspace_bytes(n_nodes: int) -> int:
    return int(load_library().jitdb_schedule_workspace_bytes(int(n_nodes)))


def jitdb_treelstm_workspace_bytes(n_nodes: int, n_edges: int, D: int, H: int, dtype: int) -> int:
    return int(load_library().jitdb_treelstm_workspace_bytes(int(n_nodes), int(n_edges),
                                                             int(D), int(H), int(dtype)))


def _check(code: int):
    if code != 0:
        msg = jitdb_strerror(code)
        if code == -6:
            msg += ": " + load_library().jitdb_last_hip_error().decode()
        raise JitdbError(code, msg)


def _stream_ptr(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _empty(stream, *args, **kw):
    import torch
    with _on_stream(stream):
        return torch.empty(*args, **kw)


def _zeros(stream, *args, **kw):
    import torch
    with _on_stream(stream):
        return torch.zeros(*args, **kw)


def _on_stream(stream):
    """Context in which default buffers are allocated: the stream the launches go to.  Memory the
    caching allocator hands out belongs to the stream that is current at that moment; allocated under
    another stream it could be given to other work while these kernels still use it."""
    import contextlib
    import torch
    return contextlib.nullcontext() if stream is None else torch.cuda.stream(stream)


class Schedule:
    """Device arrays of one forest's schedule plus the C struct that points at them."""

    def __init__(self, n_nodes: int, device):
        import torch
        n = int(n_nodes)
        i32 = dict(dtype=torch.int32, device=device)
        self.n_nodes = n
        self.height = torch.empty(max(n, 1), **i32)
        self.level_ptr = torch.empty(n + 1, **i32)
        self.perm = torch.empty(max(n, 1), **i32)
        self.inv_perm = torch.empty(max(n, 1), **i32)
        self.child_ptr = torch.empty(n + 1, **i32)
        self.child_idx = torch.empty(max(n, 1), **i32)
        self.host_level_ptr = np.zeros(n + 1, dtype=np.int32)
        self.host_level_kids = np.full(n + 1, -1, dtype=np.int32)    # children per level; -1 = not known
        self.n_levels = 0
        self.n_edges = 0
        self.struct = _ScheduleStruct(
            n, self.height.data_ptr(), self.level_ptr.data_ptr(), self.perm.data_ptr(),
            self.inv_perm.data_ptr(), self.child_ptr.data_ptr(), self.child_idx.data_ptr(),
            self.host_level_ptr.ctypes.data, 0, 0, self.host_level_kids.ctypes.data)

    def to_numpy(self) -> dict:
        """Host copies trimmed to their valid lengths (for comparison in tests)."""
        n, L, E = self.n_nodes, self.n_levels, self.n_edges
        return dict(
            height=self.height[:n].cpu().numpy(),
            level_ptr=self.level_ptr[:L + 1].cpu().numpy(),
            perm=self.perm[:n].cpu().numpy(),
            inv_perm=self.inv_perm[:n].cpu().numpy(),
            child_ptr=self.child_ptr[:n + 1].cpu().numpy(),
            child_idx=self.child_idx[:E].cpu().numpy(),
            level_kids=self.host_level_kids[:L].copy(),
            n_levels=L, n_edges=E)


def jitdb_schedule(parent, stream=None, workspace=None, out: Optional[Schedule] = None) -> Schedule:
    """parent: int32 CUDA tensor [N], -1 = root.  Returns the forest's Schedule.
    `out` reuses the buffers of an earlier Schedule of the same size."""
    import torch
    lib = load_library()
    if parent.dtype != torch.int32 or not parent.is_cuda or not parent.is_contiguous():
        raise TypeError("parent must be a contiguous int32 CUDA tensor")
    n = parent.numel()
    if out is not None and out.n_nodes != n:
        raise ValueError("out was made for a forest of another size")
    sched = out if out is not None else Schedule(n, parent.device)
    need = jitdb_schedule_workspace_bytes(n)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=parent.device)
    with torch.cuda.device(parent.device):
        code = lib.jitdb_schedule(parent.data_ptr() if n else None, ctypes.byref(sched.struct),
                                  workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(code)
    sched.n_levels = int(sched.struct.n_levels)
    sched.n_edges = int(sched.struct.n_edges)
    return sched


def jitdb_schedule_append_workspace_bytes(n_base: int, n_new: int) -> int:
    return int(load_library().jitdb_schedule_append_workspace_bytes(int(n_base), int(n_new)))


def jitdb_schedule_append(base: Schedule, parent_new, stream=None, workspace=None,
                          out: Optional[Schedule] = None) -> Schedule:
    """Schedule of the forest `base` describes followed by the trees in parent_new (int32 CUDA
    tensor, ids local to the new trees); new node v gets id base.n_nodes + v."""
    import torch
    lib = load_library()
    if parent_new.dtype != torch.int32 or not parent_new.is_cuda or not parent_new.is_contiguous():
        raise TypeError("parent_new must be a contiguous int32 CUDA tensor")
    m = parent_new.numel()
    n = base.n_nodes + m
    if out is not None and (out.n_nodes != n or out is base):
        raise ValueError("out must be another Schedule, made for the joint forest's size")
    sched = out if out is not None else Schedule(n, parent_new.device)
    base.struct.n_levels = base.n_levels
    base.struct.n_edges = base.n_edges
    need = jitdb_schedule_append_workspace_bytes(base.n_nodes, m)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=parent_new.device)
    with torch.cuda.device(parent_new.device):
        code = lib.jitdb_schedule_append(ctypes.byref(base.struct), parent_new.data_ptr() if m else None, m,
                                         ctypes.byref(sched.struct), workspace.data_ptr(), workspace.numel(),
                                         _stream_ptr(stream))
    _check(code)
    sched.n_levels = int(sched.struct.n_levels)
    sched.n_edges = int(sched.struct.n_edges)
    return sched


def jitdb_treelstm_forward(x, W, U, b, schedule: Schedule, stream=None, workspace=None,
                           out: Optional[Tuple] = None):
    """x [N, D], W [4H, D], U [4H, H] (all fp32 or all bf16), b [4H] fp32, on the GPU.
    Returns (h [N, H] in x's dtype, c [N, H] fp32), rows indexed by node id."""
    return _forward(x, W, U, b, schedule, stream, workspace, out, train=False)


def jitdb_treelstm_forward_static(x, W, U, b, schedule: Schedule, out: Tuple, stream=None):
    """jitdb_treelstm_forward on the library's own fixed scratch array: no workspace, nothing allocated
    (the caller passes the outputs h [N, H] in x's dtype and c [N, H] fp32).  Returns (h, c)."""
    import torch
    lib = load_library()
    dt = JITDB_F32 if x.dtype == torch.float32 else JITDB_BF16
    if x.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("x must be float32 or bfloat16")
    h, c = out
    n, H, D = schedule.n_nodes, U.shape[1], W.shape[1]
    for t, name in ((x, "x"), (W, "W"), (U, "U"), (b, "b"), (h, "h"), (c, "c")):
        if not t.is_cuda or not t.is_contiguous():
            raise TypeError(f"{name} must be a contiguous CUDA tensor")
    if W.dtype != x.dtype or U.dtype != x.dtype or h.dtype != x.dtype or b.dtype != torch.float32 or c.dtype != torch.float32:
        raise TypeError("W, U, h must have x's dtype; b, c must be float32")
    if (x.shape != (n, D) or W.shape[0] != 4 * H or U.shape[0] != 4 * H or b.numel() != 4 * H
            or h.shape != (n, H) or c.shape != (n, H)):
        raise ValueError("shape mismatch between x, W, U, b, out and the schedule")
    with torch.cuda.device(x.device):
        code = lib.jitdb_treelstm_forward_static(
            x.data_ptr() if n else None, W.data_ptr(), U.data_ptr(), b.data_ptr(), D, H, dt,
            ctypes.byref(schedule.struct), h.data_ptr() if n else None, c.data_ptr() if n else None,
            _stream_ptr(stream))
    _check(code)
    return h, c


def jitdb_treelstm_forward_train(x, W, U, b, schedule: Schedule, stream=None, workspace=None,
                                 out: Optional[Tuple] = None):
    """As jitdb_treelstm_forward; returns (h, c, gates [N, 3H], fgate [N, H]), the last two in x's dtype.
    `out` = (h, c, gates, fgate) reuses buffers.  fgate rows of roots are left as they are."""
    return _forward(x, W, U, b, schedule, stream, workspace, out, train=True)


def jitdb_treelstm_backward_workspace_bytes(schedule: Schedule, D: int, H: int, dtype: int) -> int:
    schedule.struct.n_levels = schedule.n_levels
    schedule.struct.n_edges = schedule.n_edges
    return int(load_library().jitdb_treelstm_backward_workspace_bytes(ctypes.byref(schedule.struct), int(D),
                                                                      int(H), int(dtype)))


def jitdb_treelstm_backward(x, W, U, schedule: Schedule, h, c, gates, fgate, gh=None, gc=None,
                            stream=None, workspace=None, out: Optional[Tuple] = None):
    """Gradients of L = sum <gh, h> + <gc, c> (gh, gc: fp32 [N, H] CUDA tensors or None = zeros)
    from what jitdb_treelstm_forward_train returned.  Returns fp32 (dx [N, D], dW [4H, D],
    dU [4H, H], db [4H])."""
    import torch
    lib = load_library()
    dt = JITDB_F32 if x.dtype == torch.float32 else JITDB_BF16
    if x.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("x must be float32 or bfloat16")
    n = schedule.n_nodes
    H = U.shape[1]
    D = W.shape[1]
    for t, name in ((x, "x"), (W, "W"), (U, "U"), (h, "h"), (c, "c"), (gates, "gates"), (fgate, "fgate")):
        if not t.is_cuda or not t.is_contiguous():
            raise TypeError(f"{name} must be a contiguous CUDA tensor")
    if any(t.dtype != x.dtype for t in (W, U, h, gates, fgate)):
        raise TypeError("W, U, h, gates, fgate must have x's dtype")
    for t, name in ((c, "c"), (gh, "gh"), (gc, "gc")):
        if t is not None and (t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous()):
            raise TypeError(f"{name} must be a contiguous float32 CUDA tensor")
    if (x.shape != (n, D) or h.shape != (n, H) or c.shape != (n, H) or gates.shape != (n, 3 * H)
            or fgate.shape != (n, H) or W.shape[0] != 4 * H or U.shape[0] != 4 * H):
        raise ValueError("shape mismatch")
    for t in (gh, gc):
        if t is not None and t.shape != (n, H):
            raise ValueError("gh, gc must be [N, H]")
    if out is None:
        f32 = dict(dtype=torch.float32, device=x.device)
        dx = _empty(stream, (n, D), **f32); dW = _empty(stream, (4 * H, D), **f32)
        dU = _empty(stream, (4 * H, H), **f32); db = _empty(stream, 4 * H, **f32)
    else:
        dx, dW, dU, db = out
    need = jitdb_treelstm_backward_workspace_bytes(schedule, D, H, dt)
    if workspace is None:
        workspace = _empty(stream, max(need, 256), dtype=torch.uint8, device=x.device)
    ptr = lambda t: t.data_ptr() if (t is not None and t.numel()) else None
    with torch.cuda.device(x.device):
        code = lib.jitdb_treelstm_backward(
            ptr(x), W.data_ptr(), U.data_ptr(), D, H, dt, ctypes.byref(schedule.struct),
            ptr(h), ptr(c), ptr(gates), ptr(fgate), ptr(gh), ptr(gc),
            ptr(dx), dW.data_ptr(), dU.data_ptr(), db.data_ptr(),
            workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(code)
    return dx, dW, dU, db


def _forward(x, W, U, b, schedule, stream, workspace, out, train):
    import torch
    lib = load_library()
    if x.dtype == torch.float32:
        dt = JITDB_F32
    elif x.dtype == torch.bfloat16:
        dt = JITDB_BF16
    else:
        raise TypeError("x must be float32 or bfloat16")
    for t, name in ((x, "x"), (W, "W"), (U, "U"), (b, "b")):
        if not t.is_cuda or not t.is_contiguous():
            raise TypeError(f"{name} must be a contiguous CUDA tensor")
    if W.dtype != x.dtype or U.dtype != x.dtype or b.dtype != torch.float32:
        raise TypeError("W, U must have x's dtype and b must be float32")
    n = schedule.n_nodes
    H = U.shape[1]
    D = W.shape[1]
    if x.shape != (n, D) or W.shape[0] != 4 * H or U.shape[0] != 4 * H or b.numel() != 4 * H:
        raise ValueError("shape mismatch between x, W, U, b and the schedule")
    gates = fgate = None
    if out is None:
        h = _empty(stream, (n, H), dtype=x.dtype, device=x.device)
        c = _empty(stream, (n, H), dtype=torch.float32, device=x.device)
        if train:
            gates = _empty(stream, (n, 3 * H), dtype=x.dtype, device=x.device)
            fgate = _zeros(stream, (n, H), dtype=x.dtype, device=x.device)
    elif train:
        h, c, gates, fgate = out
    else:
        h, c = out
    need = jitdb_treelstm_workspace_bytes(n, schedule.n_edges, D, H, dt)
    if workspace is None:
        workspace = _empty(stream, max(need, 256), dtype=torch.uint8, device=x.device)
    with torch.cuda.device(x.device):
        if train:
            code = lib.jitdb_treelstm_forward_train(
                x.data_ptr() if n else None, W.data_ptr(), U.data_ptr(), b.data_ptr(), D, H, dt,
                ctypes.byref(schedule.struct), h.data_ptr() if n else None, c.data_ptr() if n else None,
                gates.data_ptr() if n else None, fgate.data_ptr() if n else None,
                workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
        else:
            code = lib.jitdb_treelstm_forward(
                x.data_ptr() if n else None, W.data_ptr(), U.data_ptr(), b.data_ptr(), D, H, dt,
                ctypes.byref(schedule.struct), h.data_ptr() if n else None, c.data_ptr() if n else None,
                workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(code)
    return (h, c, gates, fgate) if train else (h, c)


def jitdb_forest_fingerprint(parent, stream=None, fp_dev=None) -> Tuple[int, int]:
    """(fp[0], fp[1]) of an int32 CUDA parent tensor; synchronises the stream."""
    import torch
    if parent.dtype != torch.int32 or not parent.is_cuda or not parent.is_contiguous():
        raise TypeError("parent must be a contiguous int32 CUDA tensor")
    if fp_dev is None:
        fp_dev = torch.empty(2, dtype=torch.int64, device=parent.device)
    host = (ctypes.c_uint64 * 2)()
    n = parent.numel()
    with torch.cuda.device(parent.device):
        _check(load_library().jitdb_forest_fingerprint(parent.data_ptr() if n else None, n, fp_dev.data_ptr(),
                                                       host, _stream_ptr(stream)))
    return int(host[0]), int(host[1])


class CacheTable:
    """The library's key -> slot table (host only; usable without a GPU)."""

    def __init__(self, capacity: int):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        _check(self._lib.jitdb_cache_create(int(capacity), ctypes.byref(self._h)))
        self.capacity = int(capacity)

    def close(self):
        if self._h:
            self._lib.jitdb_cache_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def lookup(self, fp: Tuple[int, int], n_nodes: int) -> int:
        return int(self._lib.jitdb_cache_lookup(self._h, (ctypes.c_uint64 * 2)(*fp), int(n_nodes)))

    def insert(self, fp: Tuple[int, int], n_nodes: int) -> Tuple[int, bool]:
        ev = ctypes.c_int32(0)
        slot = int(self._lib.jitdb_cache_insert(self._h, (ctypes.c_uint64 * 2)(*fp), int(n_nodes), ctypes.byref(ev)))
        return slot, bool(ev.value)

    def stats(self) -> dict:
        h, m, e = ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_int32(0)
        self._lib.jitdb_cache_stats(self._h, ctypes.byref(h), ctypes.byref(m), ctypes.byref(e))
        return {"hits": int(h.value), "misses": int(m.value), "entries": int(e.value)}


class ScheduleCache:
    """Schedules kept by fingerprint of their parent array: get(parent) returns the cached
    Schedule when this forest was scheduled before, else schedules it and keeps the result
    (dropping the least recently used one when full).  verify=True also keeps the parent
    arrays and compares them on a hit."""

    def __init__(self, capacity: int = 16, verify: bool = False):
        self.table = CacheTable(capacity)
        self._slots = [None] * int(capacity)
        self._parents = [None] * int(capacity) if verify else None
        self._fp_dev = None

    def get(self, parent, stream=None) -> Tuple[Schedule, bool]:
        import torch
        if self._fp_dev is None or self._fp_dev.device != parent.device:
            self._fp_dev = torch.empty(2, dtype=torch.int64, device=parent.device)
        fp = jitdb_forest_fingerprint(parent, stream=stream, fp_dev=self._fp_dev)
        n = parent.numel()
        slot = self.table.lookup(fp, n)
        if slot >= 0 and (self._parents is None or torch.equal(self._parents[slot], parent)):
            return self._slots[slot], True
        sched = jitdb_schedule(parent, stream=stream)
        slot, _ = self.table.insert(fp, n)
        self._slots[slot] = sched
        if self._parents is not None:
            self._parents[slot] = parent.clone()
        return sched, False


class TypedSchedule(Schedule):
    """A Schedule whose positions are filed by (height, signature, parent's signature), plus the
    table of sub-slot boundaries (n_sig * n_sig per level)."""

    def __init__(self, n_nodes: int, n_sig: int, device, slot_capacity: Optional[int] = None):
        import torch
        super().__init__(n_nodes, device)
        self.n_sig = int(n_sig)
        cap = int(n_nodes) * self.n_sig * self.n_sig + 1 if slot_capacity is None else int(slot_capacity)
        self.key = torch.empty(max(int(n_nodes), 1), dtype=torch.int32, device=device)
        self.slot_ptr = torch.empty(cap, dtype=torch.int32, device=device)
        self.host_slot_ptr = np.zeros(cap, dtype=np.int32)
        self.slots = _SlotsStruct(self.n_sig, cap, self.key.data_ptr(), self.slot_ptr.data_ptr(),
                                  self.host_slot_ptr.ctypes.data)

    def to_numpy(self) -> dict:
        out = super().to_numpy()
        S = self.n_levels * self.n_sig * self.n_sig
        out.update(key=self.key[:self.n_nodes].cpu().numpy(), slot_ptr=self.slot_ptr[:S + 1].cpu().numpy(),
                   host_slot_ptr=self.host_slot_ptr[:S + 1].copy(), n_sig=self.n_sig)
        return out


def jitdb_schedule_typed_workspace_bytes(n_nodes: int, n_sig: int) -> int:
    return int(load_library().jitdb_schedule_typed_workspace_bytes(int(n_nodes), int(n_sig)))


def jitdb_schedule_typed(parent, sig, n_sig: int, stream=None, workspace=None,
                         out: Optional[TypedSchedule] = None, slot_capacity: Optional[int] = None) -> TypedSchedule:
    """parent, sig: int32 CUDA tensors [N]; sig[v] in [0, n_sig) names the cell that evaluates node v."""
    import torch
    lib = load_library()
    for t, name in ((parent, "parent"), (sig, "sig")):
        if t.dtype != torch.int32 or not t.is_cuda or not t.is_contiguous():
            raise TypeError(f"{name} must be a contiguous int32 CUDA tensor")
    n = parent.numel()
    if sig.numel() != n:
        raise ValueError("sig and parent differ in length")
    if out is not None and (out.n_nodes != n or out.n_sig != n_sig):
        raise ValueError("out was made for another size or signature count")
    sched = out if out is not None else TypedSchedule(n, n_sig, parent.device, slot_capacity)
    need = jitdb_schedule_typed_workspace_bytes(n, n_sig)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=parent.device)
    with torch.cuda.device(parent.device):
        code = lib.jitdb_schedule_typed(parent.data_ptr() if n else None, sig.data_ptr() if n else None,
                                        ctypes.byref(sched.struct), ctypes.byref(sched.slots),
                                        workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(code)
    sched.n_levels = int(sched.struct.n_levels)
    sched.n_edges = int(sched.struct.n_edges)
    return sched


def jitdb_treelstm_typed_workspace_bytes(n_nodes: int, n_edges: int, D: int, H: int, dtype: int, n_sig: int) -> int:
    return int(load_library().jitdb_treelstm_typed_workspace_bytes(int(n_nodes), int(n_edges), int(D), int(H),
                                                                   int(dtype), int(n_sig)))


def jitdb_treelstm_forward_typed(x, W, U, b, schedule: TypedSchedule, stream=None, workspace=None,
                                 out: Optional[Tuple] = None):
    """x [N, D]; W [n_sig, 4H, D], U [n_sig, 4H, H] in x's dtype, b [n_sig, 4H] fp32: node j is
    evaluated by cell sig[j].  Returns (h, c) as jitdb_treelstm_forward."""
    import torch
    lib = load_library()
    if x.dtype == torch.float32:
        dt = JITDB_F32
    elif x.dtype == torch.bfloat16:
        dt = JITDB_BF16
    else:
        raise TypeError("x must be float32 or bfloat16")
    for t, name in ((x, "x"), (W, "W"), (U, "U"), (b, "b")):
        if not t.is_cuda or not t.is_contiguous():
            raise TypeError(f"{name} must be a contiguous CUDA tensor")
    if W.dtype != x.dtype or U.dtype != x.dtype or b.dtype != torch.float32:
        raise TypeError("W, U must have x's dtype and b must be float32")
    n, T = schedule.n_nodes, schedule.n_sig
    if W.dim() != 3 or U.dim() != 3 or b.dim() != 2:
        raise ValueError("W, U, b need a leading signature axis")
    H, D = U.shape[2], W.shape[2]
    if x.shape != (n, D) or W.shape != (T, 4 * H, D) or U.shape != (T, 4 * H, H) or b.shape != (T, 4 * H):
        raise ValueError("shape mismatch between x, W, U, b and the schedule")
    if out is None:
        h = _empty(stream, (n, H), dtype=x.dtype, device=x.device)
        c = _empty(stream, (n, H), dtype=torch.float32, device=x.device)
    else:
        h, c = out
    need = jitdb_treelstm_typed_workspace_bytes(n, schedule.n_edges, D, H, dt, T)
    if workspace is None:
        workspace = _empty(stream, max(need, 256), dtype=torch.uint8, device=x.device)
    with torch.cuda.device(x.device):
        code = lib.jitdb_treelstm_forward_typed(
            x.data_ptr() if n else None, W.data_ptr(), U.data_ptr(), b.data_ptr(), D, H, dt,
            ctypes.byref(schedule.struct), ctypes.byref(schedule.slots),
            h.data_ptr() if n else None, c.data_ptr() if n else None,
            workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(code)
    return h, c


def _cell_array(cells, x, D: int, H: int):
    """cells: a sequence of (kind, arity, W, U, b).  Returns the ctypes array for the library."""
    import torch
    arr = (_CellStruct * len(cells))()
    for t, (kind, arity, W, U, b) in enumerate(cells):
        if kind not in (JITDB_CELL_CHILDSUM, JITDB_CELL_NARY):
            raise ValueError(f"cell {t}: unknown kind {kind}")
        rows = 4 * H if kind == JITDB_CELL_CHILDSUM else (3 + arity) * H
        cols = H if kind == JITDB_CELL_CHILDSUM else arity * H
        for v, name in ((W, "W"), (U, "U"), (b, "b")):
            if not v.is_cuda or not v.is_contiguous():
                raise TypeError(f"cell {t}: {name} must be a contiguous CUDA tensor")
        if W.dtype != x.dtype or U.dtype != x.dtype or b.dtype != torch.float32:
            raise TypeError(f"cell {t}: W, U must have x's dtype and b must be float32")
        if tuple(W.shape) != (rows, D) or tuple(U.shape) != (rows, cols) or tuple(b.shape) != (rows,):
            raise ValueError(f"cell {t}: W, U, b must be [{rows}, {D}], [{rows}, {cols}], [{rows}]")
        arr[t].kind, arr[t].arity = kind, arity if kind == JITDB_CELL_NARY else 0
        arr[t].W, arr[t].U, arr[t].b = W.data_ptr(), U.data_ptr(), b.data_ptr()
    return arr


def jitdb_treelstm_cells_workspace_bytes(n_nodes: int, n_edges: int, D: int, H: int, dtype: int, cells) -> int:
    """cells: a sequence of (kind, arity) pairs (weights are not needed to size the workspace)."""
    arr = (_CellStruct * len(cells))()
    for t, c in enumerate(cells):
        arr[t].kind, arr[t].arity = c[0], c[1]
    return int(load_library().jitdb_treelstm_cells_workspace_bytes(n_nodes, n_edges, D, H, dtype, arr, len(cells)))


def jitdb_treelstm_forward_cells(x, cells, schedule: TypedSchedule, stream=None, workspace=None,
                                 out: Optional[Tuple] = None):
    """x [N, D]; cells: one (kind, arity, W, U, b) per signature of the schedule, kind JITDB_CELL_CHILDSUM
    (W [4H, D], U [4H, H], b [4H]) or JITDB_CELL_NARY (W [(3+N)H, D], U [(3+N)H, N*H], b [(3+N)H]).
    H is taken from the first cell's U.  Returns (h, c) as jitdb_treelstm_forward."""
    import torch
    lib = load_library()
    if x.dtype == torch.float32:
        dt = JITDB_F32
    elif x.dtype == torch.bfloat16:
        dt = JITDB_BF16
    else:
        raise TypeError("x must be float32 or bfloat16")
    if not x.is_cuda or not x.is_contiguous():
        raise TypeError("x must be a contiguous CUDA tensor")
    n, T = schedule.n_nodes, schedule.n_sig
    if len(cells) != T:
        raise ValueError("one cell per signature of the schedule")
    kind0, arity0, _, U0, _ = cells[0]
    H = U0.shape[0] // (4 if kind0 == JITDB_CELL_CHILDSUM else 3 + arity0)
    D = cells[0][2].shape[1]
    if x.shape != (n, D):
        raise ValueError("shape mismatch between x and the schedule")
    arr = _cell_array(cells, x, D, H)
    if out is None:
        h = _empty(stream, (n, H), dtype=x.dtype, device=x.device)
        c = _empty(stream, (n, H), dtype=torch.float32, device=x.device)
    else:
        h, c = out
    need = int(lib.jitdb_treelstm_cells_workspace_bytes(n, schedule.n_edges, D, H, dt, arr, T))
    if workspace is None:
        workspace = _empty(stream, max(need, 256), dtype=torch.uint8, device=x.device)
    with torch.cuda.device(x.device):
        code = lib.jitdb_treelstm_forward_cells(
            x.data_ptr() if n else None, arr, T, D, H, dt,
            ctypes.byref(schedule.struct), ctypes.byref(schedule.slots),
            h.data_ptr() if n else None, c.data_ptr() if n else None,
            workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(code)
    return h, c


class PackedWeights:
    """W, U, b of one or several cells in the library's operand layout (jitdb_treelstm_pack)."""

    def __init__(self, buffer, D: int, H: int, dtype: int, n_sig: int, torch_dtype):
        self.buffer, self.D, self.H, self.dtype, self.n_sig, self.torch_dtype = buffer, D, H, dtype, n_sig, torch_dtype


def jitdb_treelstm_pack(W, U, b, stream=None) -> PackedWeights:
    """W [4H, D] (or [n_sig, 4H, D]), U, b likewise: pack once, reuse in jitdb_treelstm_forward_packed."""
    import torch
    lib = load_library()
    if W.dim() == 2:
        W, U, b = W[None], U[None], b[None]
    for t, name in ((W, "W"), (U, "U"), (b, "b")):
        if not t.is_cuda or not t.is_contiguous():
            raise TypeError(f"{name} must be a contiguous CUDA tensor")
    if W.dtype not in (torch.float32, torch.bfloat16) or U.dtype != W.dtype or b.dtype != torch.float32:
        raise TypeError("W, U float32 or bfloat16 alike, b float32")
    dt = JITDB_F32 if W.dtype == torch.float32 else JITDB_BF16
    T, H, D = U.shape[0], U.shape[2], W.shape[2]
    if W.shape != (T, 4 * H, D) or U.shape != (T, 4 * H, H) or b.shape != (T, 4 * H):
        raise ValueError("shape mismatch between W, U, b")
    need = int(lib.jitdb_treelstm_packed_bytes(D, H, dt, T))
    buf = _empty(stream, max(need, 256), dtype=torch.uint8, device=W.device)
    with torch.cuda.device(W.device):
        _check(lib.jitdb_treelstm_pack(W.data_ptr(), U.data_ptr(), b.data_ptr(), D, H, dt, T, buf.data_ptr(),
                                       buf.numel(), _stream_ptr(stream)))
    return PackedWeights(buf, D, H, dt, T, W.dtype)


def jitdb_treelstm_forward_packed(x, packed: PackedWeights, schedule: Schedule, stream=None, workspace=None,
                                  out: Optional[Tuple] = None):
    """jitdb_treelstm_forward / _typed with weights packed beforehand.  A TypedSchedule selects the
    typed path (its n_sig must match the packed weights'); a plain Schedule needs one packed cell."""
    import torch
    lib = load_library()
    typed = isinstance(schedule, TypedSchedule)
    if (schedule.n_sig if typed else 1) != packed.n_sig:
        raise ValueError("the schedule and the packed weights differ in the number of signatures")
    if x.dtype != packed.torch_dtype or not x.is_cuda or not x.is_contiguous():
        raise TypeError("x must be a contiguous CUDA tensor of the packed weights' dtype")
    n, D, H = schedule.n_nodes, packed.D, packed.H
    if x.shape != (n, D):
        raise ValueError("x must be [N, D]")
    if out is None:
        h = _empty(stream, (n, H), dtype=x.dtype, device=x.device)
        c = _empty(stream, (n, H), dtype=torch.float32, device=x.device)
    else:
        h, c = out
    need = jitdb_treelstm_typed_workspace_bytes(n, schedule.n_edges, D, H, packed.dtype, packed.n_sig)
    if workspace is None:
        workspace = _empty(stream, max(need, 256), dtype=torch.uint8, device=x.device)
    with torch.cuda.device(x.device):
        code = lib.jitdb_treelstm_forward_packed(
            x.data_ptr() if n else None, packed.buffer.data_ptr(), D, H, packed.dtype,
            ctypes.byref(schedule.struct), ctypes.byref(schedule.slots) if typed else None,
            h.data_ptr() if n else None, c.data_ptr() if n else None,
            workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(code)
    return h, c
