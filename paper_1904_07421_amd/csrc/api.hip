// Entry points of the C ABI that need no kernels.
#include "common.h"

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
        default: return "unknown jitdb status";
    }
}

extern "C" const char *jitdb_version(void) { return "0.1"; }
