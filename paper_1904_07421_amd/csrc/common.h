// Shared host-side helpers of the jitdb library (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <new>

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

// Nothing may throw across the C ABI: host-side containers and `new` can (std::bad_alloc).
// Every extern "C" entry point that reaches such code wraps its body in these.
#define JITDB_ABI_TRY try {
#define JITDB_ABI_CATCH                                         \
    }                                                           \
    catch (const std::bad_alloc &) { return JITDB_E_NOMEM; }    \
    catch (...) { return JITDB_E_NOMEM; }

// ---- bfloat16 as stored (uint16_t bit patterns); shared by the forward and backward kernels
typedef uint16_t bf16_t;
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest even
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ T from_f32(float f);
template <> __device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) { return f32_to_bf16(f); }
template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }

// K-blocked operand layout of the tiled GEMM core: bytes [64 s, 64 s + 64) of every row form
// slab s, rows consecutive inside a slab (n_rows_alloc rows per slab).  Byte offset of byte
// `kbyte` of row `row`.
__host__ __device__ __forceinline__ int64_t operand_offset(int64_t row, int64_t kbyte, int64_t n_rows_alloc) {
    return ((kbyte >> 6) * n_rows_alloc + row) * 64 + (kbyte & 63);
}

// Fragment-major layout of the packed weights for the 256 x 256 tile kernel: the 32 packed rows of
// one gate of one unit tile (packed row = unit_tile * 128 + gate * 32 + u) times one K group of 32
// bytes form 1 KB in MFMA operand order, lane (u, half) holding bytes [16 half, 16 half + 16) of the
// group; the four gates of a K group are consecutive, then the K groups (n_kg per packed row), then
// the unit tiles.  Byte offset of byte `kbyte` of packed row `row`.
__host__ __device__ __forceinline__ int64_t fragment_offset(int64_t row, int64_t kbyte, int64_t n_kg) {
    const int64_t ut = row >> 7, gate = (row >> 5) & 3, u = row & 31;
    const int64_t kg = kbyte >> 5, half = (kbyte >> 4) & 1;
    return ((((ut * n_kg + kg) * 4 + gate) * 64) + half * 32 + u) * 16 + (kbyte & 15);
}

// C = A B^T on the tiled GEMM core of the level kernel (128 x 256 tiles, stages straight into
// LDS), for operands in the K-blocked layout above.  A has M rows (a_rows_alloc >= M rounded up
// to 128 per slab), B has N rows (b_rows_alloc >= N rounded up to 256); K is k_bytes / element
// size, k_bytes a multiple of 128.  k_splits > 1 deals ranges of K to different blocks.
enum KbEpilogue : int {
    KB_EPI_DX_DHS = 0,       // col < D: out0[node[row] * D + col] = v (fp32), else out1[node[row] * H + col - D] = v
                             // (in the operands' element type)
    KB_EPI_ATOMIC_ACC = 1,   // atomicAdd(out0[row * ldc + col], v), fp32
    KB_EPI_STORE = 2,        // out0[row * ldc + col] = v, in the operands' element type
    KB_EPI_STORE_F32 = 3     // out0[row * ldc + col] = v, fp32 whatever the operands are
};
struct KbGemm {
    const void *A; int64_t a_rows_alloc; int M;
    const void *B; int64_t b_rows_alloc; int N;
    int64_t k_bytes; int k_splits;
    int epilogue;
    void *out0; void *out1; const int32_t *node; int D; int H; int ldc;
};
int launch_kb_gemm(jitdb_dtype dtype, const KbGemm &g, hipStream_t st);

}  // namespace jitdb
