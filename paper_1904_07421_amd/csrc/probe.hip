// Machine peaks measured on the spot, so that kernel rates can be quoted against what this
// box sustains as well as against the data sheet: a plain device copy and a loop of
// independent MFMAs.  Used by the benchmark only; nothing on the forward path calls them.
#include "common.h"

namespace jitdb {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(256)
probe_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n16) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256)
        dst[i] = src[i];
}

// Other shapes of the same streams, to find what the memory system gives at best: read only
// (folded into a value nobody stores), write only, a copy with four non-temporal 16-byte loads and
// stores in flight per thread, and a copy in which every block owns one contiguous chunk.
__global__ void __launch_bounds__(256)
probe_read_kernel(const u32x4 *__restrict__ src, int64_t n16, uint32_t *sink) {
    uint32_t acc = 0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) {
        const u32x4 v = src[i];
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    if (acc == 0x12345679u) sink[0] = acc;   // keeps the loads alive; never true for the probe's data
}
__global__ void __launch_bounds__(256)
probe_write_kernel(u32x4 *__restrict__ dst, int64_t n16) {
    const u32x4 v = {1u, 2u, 3u, (uint32_t)threadIdx.x};
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) dst[i] = v;
}
__global__ void __launch_bounds__(256)
probe_copy_nt4_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n16) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}
__global__ void __launch_bounds__(256)
probe_copy_chunk_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, int64_t n16) {
    const int64_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const int64_t b0 = per * blockIdx.x, b1 = b0 + per < n16 ? b0 + per : n16;
    int64_t i = b0 + threadIdx.x;
    for (; i + 3 * 256 < b1; i += 4 * 256) {
        u32x4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = src[i + u * 256];
#pragma unroll
        for (int u = 0; u < 4; ++u) dst[i + u * 256] = v[u];
    }
    for (; i < b1; i += 256) dst[i] = src[i];
}

// Eight independent accumulators per wave: consecutive MFMAs never wait for each other.
template <bool BF16>
__global__ void __launch_bounds__(256)
probe_mfma_kernel(int iters, float *sink) {
    floatx16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    const uint32_t seed = 0x3f803f80u + (threadIdx.x & 3);   // small finite bf16 / fp32 values
    const u32x4 a = {seed, seed, seed, seed}, b = {seed, seed, seed, seed};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if constexpr (BF16)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                                 __builtin_bit_cast(bf16x8, b), acc[j], 0, 0, 0);
            else
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[0]), __uint_as_float(b[0]), acc[j], 0, 0, 0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[j][0];
    if (s == 12345.678f) sink[0] = s;   // keeps the loop alive; never true
}

int time_launches(hipStream_t st, int reps, double *ms_out, int (*launch)(hipStream_t, void *), void *ctx) {
    hipEvent_t e0, e1;
    JITDB_HIP_CHECK(hipEventCreate(&e0));
    JITDB_HIP_CHECK(hipEventCreate(&e1));
    int rc = launch(st, ctx);                                // warm-up
    if (rc == JITDB_OK) {
        (void)hipEventRecord(e0, st);
        for (int r = 0; r < reps && rc == JITDB_OK; ++r) rc = launch(st, ctx);
        (void)hipEventRecord(e1, st);
        float ms = 0.0f;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = JITDB_E_HIP;
        *ms_out = ms / reps;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return rc;
}

struct CopyCtx { const void *src; void *dst; int64_t n16; int kind; };
int launch_copy(hipStream_t st, void *p) {
    CopyCtx *c = static_cast<CopyCtx *>(p);
    const u32x4 *src = static_cast<const u32x4 *>(c->src);
    u32x4 *dst = static_cast<u32x4 *>(c->dst);
    switch (c->kind) {
        case JITDB_STREAM_READ: probe_read_kernel<<<256 * 4, 256, 0, st>>>(src, c->n16, reinterpret_cast<uint32_t *>(dst)); break;
        case JITDB_STREAM_WRITE: probe_write_kernel<<<256 * 2, 256, 0, st>>>(dst, c->n16); break;
        case JITDB_STREAM_COPY_NT: probe_copy_nt4_kernel<<<256 * 2, 256, 0, st>>>(src, dst, c->n16); break;
        case JITDB_STREAM_COPY_CHUNK: probe_copy_chunk_kernel<<<256 * 16, 256, 0, st>>>(src, dst, c->n16); break;
        default: probe_copy_kernel<<<256 * 16, 256, 0, st>>>(src, dst, c->n16); break;
    }
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

struct MfmaCtx { int dtype; int iters; float *sink; };
constexpr int kMfmaBlocks = 256 * 8;   // 8 blocks of 4 waves per CU's worth of work
int launch_mfma(hipStream_t st, void *p) {
    MfmaCtx *c = static_cast<MfmaCtx *>(p);
    if (c->dtype == JITDB_BF16) probe_mfma_kernel<true><<<kMfmaBlocks, 256, 0, st>>>(c->iters, c->sink);
    else probe_mfma_kernel<false><<<kMfmaBlocks, 256, 0, st>>>(c->iters, c->sink);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

}  // namespace
}  // namespace jitdb

using namespace jitdb;

extern "C" int jitdb_probe_copy(const void *src, void *dst, size_t bytes, void *hip_stream, double *gb_per_s) {
    if (!src || !dst || !gb_per_s) return JITDB_E_NULL;
    if (bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return JITDB_E_BADARG;
    drop_stale_hip_error();
    CopyCtx c{src, dst, (int64_t)(bytes / 16), JITDB_STREAM_COPY};
    double ms = 0.0;
    const int rc = time_launches((hipStream_t)hip_stream, 5, &ms, launch_copy, &c);
    if (rc != JITDB_OK) return rc;
    *gb_per_s = 2.0 * (double)bytes / (ms * 1e-3) / 1e9;    // read + written
    return JITDB_OK;
}

extern "C" int jitdb_probe_stream(int kind, const void *src, void *dst, size_t bytes, void *hip_stream, double *gb_per_s) {
    if (!src || !dst || !gb_per_s) return JITDB_E_NULL;
    if (kind < JITDB_STREAM_COPY || kind > JITDB_STREAM_COPY_CHUNK) return JITDB_E_BADARG;
    if (bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return JITDB_E_BADARG;
    drop_stale_hip_error();
    CopyCtx c{src, dst, (int64_t)(bytes / 16), kind};
    double ms = 0.0;
    const int rc = time_launches((hipStream_t)hip_stream, 5, &ms, launch_copy, &c);
    if (rc != JITDB_OK) return rc;
    const double moved = (kind == JITDB_STREAM_READ || kind == JITDB_STREAM_WRITE) ? (double)bytes : 2.0 * (double)bytes;
    *gb_per_s = moved / (ms * 1e-3) / 1e9;
    return JITDB_OK;
}

extern "C" int jitdb_probe_mfma(jitdb_dtype dtype, float *sink, void *hip_stream, double *tflop_per_s) {
    if (!sink || !tflop_per_s) return JITDB_E_NULL;
    if (dtype != JITDB_F32 && dtype != JITDB_BF16) return JITDB_E_BADARG;
    drop_stale_hip_error();
    MfmaCtx c{(int)dtype, dtype == JITDB_BF16 ? 4000 : 1000, sink};
    double ms = 0.0;
    const int rc = time_launches((hipStream_t)hip_stream, 3, &ms, launch_mfma, &c);
    if (rc != JITDB_OK) return rc;
    const double flops_per_mfma = dtype == JITDB_BF16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 2;
    const double flops = (double)kMfmaBlocks * 4 * c.iters * 8 * flops_per_mfma;
    *tflop_per_s = flops / (ms * 1e-3) / 1e12;
    return JITDB_OK;
}
