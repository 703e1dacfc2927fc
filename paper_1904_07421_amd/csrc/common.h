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

#define JITDB_HIP_CHECK(expr)                      \
    do {                                           \
        hipError_t e_ = (expr);                    \
        if (e_ != hipSuccess) return JITDB_E_HIP;  \
    } while (0)

// Launch check: kernels are launched with <<<>>>; a bad configuration surfaces here.
#define JITDB_LAUNCH_CHECK()                       \
    do {                                           \
        hipError_t e_ = hipGetLastError();         \
        if (e_ != hipSuccess) return JITDB_E_HIP;  \
    } while (0)

}  // namespace jitdb
