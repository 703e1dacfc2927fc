"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol the header declares, and its pure-host entry points behave."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "jitdb.h")


@pytest.fixture(scope="module")
def lib():
    import paper_1904_07421_amd as J
    return J.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(jitdb_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"jitdb_schedule", "jitdb_treelstm_forward", "jitdb_schedule_workspace_bytes",
            "jitdb_treelstm_workspace_bytes", "jitdb_strerror", "jitdb_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_strerror_and_version(lib):
    import paper_1904_07421_amd as J
    assert J.jitdb_strerror(0) == "ok"
    seen = {J.jitdb_strerror(c) for c in range(-10, 1)}
    assert len(seen) == 11
    assert "unknown" in J.jitdb_strerror(-99)
    assert re.fullmatch(r"\d+\.\d+", J.jitdb_version())


def test_workspace_queries(lib):
    import paper_1904_07421_amd as J
    assert J.jitdb_schedule_workspace_bytes(-1) == 0
    assert J.jitdb_schedule_workspace_bytes((1 << 28) + 1) == 0
    a, b = J.jitdb_schedule_workspace_bytes(1000), J.jitdb_schedule_workspace_bytes(100000)
    assert 0 < a < b and a % 256 == 0
    assert J.jitdb_schedule_workspace_bytes(0) > 0
    assert J.jitdb_treelstm_workspace_bytes(100, 90, 300, 150, J.JITDB_F32) > 0
    assert J.jitdb_treelstm_workspace_bytes(100, 90, 300, 150, J.JITDB_BF16) > 0
    assert J.jitdb_treelstm_workspace_bytes(100, 90, 0, 150, J.JITDB_F32) == 0
    assert J.jitdb_treelstm_workspace_bytes(100, 90, 300, 0, J.JITDB_F32) == 0
    assert J.jitdb_treelstm_workspace_bytes(100, 90, 300, 150, 7) == 0
    assert J.jitdb_treelstm_workspace_bytes(-1, 0, 300, 150, 0) == 0
    # typed table: more weight sets and the tile tables; signature count and N * n_sig^2 are bounded
    one = J.jitdb_treelstm_workspace_bytes(1000, 900, 300, 150, J.JITDB_BF16)
    assert J.jitdb_treelstm_typed_workspace_bytes(1000, 900, 300, 150, J.JITDB_BF16, 1) == one
    assert J.jitdb_treelstm_typed_workspace_bytes(1000, 900, 300, 150, J.JITDB_BF16, 3) > one
    assert J.jitdb_treelstm_typed_workspace_bytes(1000, 900, 300, 150, J.JITDB_BF16, 0) == 0
    assert J.jitdb_treelstm_typed_workspace_bytes(1000, 900, 300, 150, J.JITDB_BF16, 65) == 0
    assert J.jitdb_schedule_typed_workspace_bytes(1000, 1) == J.jitdb_schedule_workspace_bytes(1000)
    assert J.jitdb_schedule_typed_workspace_bytes(1000, 4) >= J.jitdb_schedule_workspace_bytes(1000)
    assert J.jitdb_schedule_typed_workspace_bytes(1 << 28, 3) == 0          # 2^28 * 9 does not fit int32 keys
    assert J.jitdb_schedule_typed_workspace_bytes(1000, 0) == 0
    assert J.jitdb_schedule_append_workspace_bytes(1000, 10) > 0
    assert J.jitdb_schedule_append_workspace_bytes(-1, 10) == 0


def test_argument_errors_before_any_gpu_work(lib):
    """NULL / out-of-range arguments are rejected on the host."""
    import paper_1904_07421_amd as J
    from paper_1904_07421_amd.binding import _ScheduleStruct
    assert lib.jitdb_schedule(None, None, None, 0, None) == -1
    s = _ScheduleStruct()
    s.n_nodes = -5
    assert lib.jitdb_schedule(None, ctypes.byref(s), None, 0, None) == -2
    s.n_nodes = 10
    assert lib.jitdb_schedule(None, ctypes.byref(s), None, 0, None) == -1
    assert lib.jitdb_treelstm_forward(None, None, None, None, 300, 150, 0, None, None, None,
                                      None, 0, None) == -1
