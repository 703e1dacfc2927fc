// Entry points of the C ABI that need no kernels.
#include "common.h"

#include <stdio.h>

extern "C" const char *jitdb_strerror(int code) {
    switch (code) {
        case JITDB_OK: return "ok";
        case JITDB_E_NULL: return "a required pointer is NULL";
        case JITDB_E_BADARG: return "argument out of range (size, dimension, dtype or alignment)";
        case JITDB_E_PARENT_RANGE: return "parent array holds an id outside [-1, N) or a self loop";
        case JITDB_E_CYCLE: return "parent array is not a forest: some node never reaches a root";
        case JITDB_E_WORKSPACE: return "workspace is smaller than required";
        case JITDB_E_HIP: return "a HIP runtime call failed";
        case JITDB_E_SCHEDULE: return "schedule is incomplete or does not match the call";
        case JITDB_E_SIGNATURE: return "a signature is outside [0, n_sig)";
        case JITDB_E_NOMEM: return "a host-side allocation failed";
        case JITDB_E_ARITY: return "a node has more children than its cell has child positions";
        default: return "unknown jitdb status";
    }
}

namespace jitdb {
static char g_hip_detail[256] = "no HIP failure recorded";
void note_hip_failure(hipError_t e, const char *file, int line) {
    const char *slash = file;
    for (const char *p = file; *p; ++p)
        if (*p == '/') slash = p + 1;
    snprintf(g_hip_detail, sizeof(g_hip_detail), "%s (%d) at %s:%d", hipGetErrorString(e), (int)e, slash, line);
}
}  // namespace jitdb

extern "C" const char *jitdb_last_hip_error(void) { return jitdb::g_hip_detail; }

extern "C" const char *jitdb_version(void) { return "0.1"; }
