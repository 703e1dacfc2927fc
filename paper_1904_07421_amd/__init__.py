"""Thin Python binding of libjitdb: level-batched Child-Sum Tree-LSTM forward
on MI355X.  Argument marshalling only - every step runs in the HIP library."""
from .binding import (  # noqa: F401
    JITDB_F32,
    JITDB_BF16,
    JitdbError,
    Schedule,
    jitdb_schedule,
    jitdb_schedule_workspace_bytes,
    jitdb_schedule_append,
    jitdb_schedule_append_workspace_bytes,
    jitdb_treelstm_forward,
    jitdb_treelstm_workspace_bytes,
    jitdb_strerror,
    jitdb_profile_start,
    jitdb_profile_stop,
    jitdb_probe_copy,
    jitdb_probe_mfma,
    jitdb_version,
    library_path,
    load_library,
)
