// Shared host-side helpers of the jitdb library (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "jitdb.h"

namespace jitdb {

// Carves 256-byte aligned pieces out of a caller-supplied workspace.  With a
// null base it only measures, which is how the *_workspace_bytes queries work.
struct Carver {
    char *base;
    size_t off;
    explicit Carver(void *b) : base(static_cast<char *>(b)), off(0) {}
    template <typename T>
    T *take(size_t count) {
        size_t bytes = (count * sizeof(T) + 255) & ~size_t(255);
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += bytes;
        return p;
    }
};

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

// Where and why the last JITDB_E_HIP happened (process-wide, for diagnostics only).
void note_hip_failure(hipError_t e, const char *file, int line);

#define JITDB_HIP_CHECK(expr)                                   \
    do {                                                        \
        hipError_t e_ = (expr);                                 \
        if (e_ != hipSuccess) {                                 \
            ::jitdb::note_hip_failure(e_, __FILE__, __LINE__);  \
            return JITDB_E_HIP;                                 \
        }                                                       \
    } while (0)

// Launch check: kernels are launched with <<<>>>; a bad configuration surfaces here.
#define JITDB_LAUNCH_CHECK() JITDB_HIP_CHECK(hipGetLastError())

// The HIP "last error" is per thread and sticky across unrelated runtime calls
// made by the host program; every entry point drops whatever it inherits so
// that the launch checks only see this library's own launches.
inline void drop_stale_hip_error() { (void)hipGetLastError(); }

}  // namespace jitdb
