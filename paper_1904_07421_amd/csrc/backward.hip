// jitdb_treelstm_backward: reverse-mode gradients of the level-batched Tree-LSTM forward.
//
// The paper trains through the same batched graph it infers with (section 5).  Here the
// levels of the schedule are visited from the roots down; per level
//
//   (nodes that have parents)  dh_k += U_f^T dz_f,k              one GEMM over the level's rows
//                              dU_f += sum_k dz_f,k (x) h_k      one GEMM, reduction over rows
//   bwd_cell_kernel            the cell's elementwise derivative: dz_i, dz_o, dz_u and the
//                              per-child dz_f,k, dc_k from dh_j, dc_j and the saved gates
//   [dx_j | dhs_j] = dZ_j [W | U]                                one GEMM over the level's rows
//   bwd_scatter_kernel         dh_k += dhs_parent(k)             over the child CSR
//   dW, dU_iou, db += dZ^T [x | hs]                              one GEMM, reduction over rows
//
// This first version keeps every step separate and simple: the GEMMs are one generic
// MFMA kernel (C = A B^T, both operands K-contiguous, fragments straight from global
// memory / L2), reductions over rows go through explicit transposes.  Gradients are fp32;
// with JITDB_BF16 the GEMM operands (dz, x, h, hs, weights) are bfloat16, sums fp32.

#include "common.h"

namespace jitdb {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t bf16_t;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kT = 256;

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

template <typename T>
__device__ __forceinline__ void mfma_step(const u32x4 &a, const u32x4 &b, floatx16 &acc) {
    if constexpr (sizeof(T) == 2) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                      __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[0]), __uint_as_float(b[0]), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[1]), __uint_as_float(b[1]), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[2]), __uint_as_float(b[2]), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[3]), __uint_as_float(b[3]), acc, 0, 0, 0);
    }
}

// ---- small helpers -----------------------------------------------------------------
__global__ void __launch_bounds__(kT)
fill_f32_kernel(float *p, int64_t n, float v) {
    for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += (int64_t)gridDim.x * kT) p[i] = v;
}
__global__ void __launch_bounds__(kT)
copy_or_zero_kernel(const float *src, float *dst, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += (int64_t)gridDim.x * kT)
        dst[i] = src ? src[i] : 0.0f;
}
__global__ void __launch_bounds__(kT)
fill_bytes16_kernel(u32x4 *p, int64_t n16) {
    const u32x4 z = {0, 0, 0, 0};
    for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n16; i += (int64_t)gridDim.x * kT) p[i] = z;
}

// ---- weights for the data-gradient GEMMs ---------------------------------------------
// Mt [D + H rows, 4 Hk] (K-blocked, for the tiled GEMM): row n < D is column n of W, row D + n' column n' of U, the four gates
// side by side at stride Hk (H rounded up, pad zero); the forget gate has no h-sum part, so
// its block is zero in the rows of U.  Uft [H rows, Hk]: row n = column n of U_f.
template <typename T>
__global__ void __launch_bounds__(kT)
pack_bwd_weights_kernel(const T *__restrict__ W, const T *__restrict__ U, int D, int H, int Hk,
                        T *__restrict__ Mt, int64_t mt_rows_alloc, T *__restrict__ Uft) {
    const int64_t total = (int64_t)(D + H) * 4 * Hk;
    for (int64_t idx = (int64_t)blockIdx.x * kT + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * kT) {
        const int n = (int)(idx / (4 * Hk)), k = (int)(idx % (4 * Hk));
        const int g = k / Hk, m = k % Hk;
        T v = T(0);
        if (m < H) {
            if (n < D) v = W[((int64_t)g * H + m) * D + n];
            else if (g < 3) v = U[((int64_t)g * H + m) * H + (n - D)];
        }
        *reinterpret_cast<T *>(reinterpret_cast<char *>(Mt) + operand_offset(n, (int64_t)k * sizeof(T), mt_rows_alloc)) = v;
    }
    const int64_t total_f = (int64_t)H * Hk;
    for (int64_t idx = (int64_t)blockIdx.x * kT + threadIdx.x; idx < total_f; idx += (int64_t)gridDim.x * kT) {
        const int n = (int)(idx / Hk), m = (int)(idx % Hk);
        Uft[idx] = m < H ? U[((int64_t)3 * H + m) * H + n] : T(0);
    }
}

// ---- the cell's elementwise derivative ---------------------------------------------
// One thread per (level row, hidden unit).  dh_j and dc_j are complete when the level is
// reached (all parents are in higher levels).  Writes dZ row r = [dz_i | dz_o | dz_u |
// sum_k dz_f,k] (gate stride Hk), and for every child k: G[k] = dz_f,k and dc_k += dc_j f_k
// (a node has one parent, so nobody else writes those rows).
template <typename T>
__global__ void __launch_bounds__(kT)
bwd_cell_kernel(const int32_t *__restrict__ nodes, int n_rows, int H, int Hk,
                const int32_t *__restrict__ child_ptr, const int32_t *__restrict__ child_idx,
                const float *__restrict__ c, const float *__restrict__ gates, const float *__restrict__ fgate,
                const float *__restrict__ dh, float *__restrict__ dc,
                T *__restrict__ dZ, int64_t dz_rows_alloc, T *__restrict__ G) {
    const int64_t id = (int64_t)blockIdx.x * kT + threadIdx.x;
    if (id >= (int64_t)n_rows * Hk) return;
    const int r = (int)(id / Hk), m = (int)(id % Hk);
    char *zb = reinterpret_cast<char *>(dZ);
    if (m >= H) {       // pad columns of the K-blocked operand
#pragma unroll
        for (int g = 0; g < 4; ++g)
            *reinterpret_cast<T *>(zb + operand_offset(r, (int64_t)(g * Hk + m) * sizeof(T), dz_rows_alloc)) = T(0);
        return;
    }
    const int64_t j = nodes[r];
    const float gi = gates[j * 3 * H + m], go = gates[j * 3 * H + H + m], gu = gates[j * 3 * H + 2 * H + m];
    const float t = tanhf(c[j * H + m]);
    const float dhj = dh[j * H + m];
    const float dcj = dc[j * H + m] + dhj * go * (1.0f - t * t);
    const float dzi = dcj * gu * gi * (1.0f - gi);
    const float dzo = dhj * t * go * (1.0f - go);
    const float dzu = dcj * gi * (1.0f - gu * gu);
    float dzf_sum = 0.0f;
    const int e0 = child_ptr[j], e1 = child_ptr[j + 1];
    for (int e = e0; e < e1; ++e) {
        const int64_t k = child_idx[e];
        const float fk = fgate[k * H + m];
        const float dzf = dcj * c[k * H + m] * fk * (1.0f - fk);
        dzf_sum += dzf;
        G[k * Hk + m] = from_f32<T>(dzf);
        dc[k * H + m] += dcj * fk;
    }
    const float dz[4] = {dzi, dzo, dzu, dzf_sum};
#pragma unroll
    for (int g = 0; g < 4; ++g)
        *reinterpret_cast<T *>(zb + operand_offset(r, (int64_t)(g * Hk + m) * sizeof(T), dz_rows_alloc)) = from_f32<T>(dz[g]);
}

// dh_k += dhs_r for every child k of the node in level row r
__global__ void __launch_bounds__(kT)
bwd_scatter_kernel(const int32_t *__restrict__ nodes, int n_rows, int H,
                   const int32_t *__restrict__ child_ptr, const int32_t *__restrict__ child_idx,
                   const float *__restrict__ dhs, float *__restrict__ dh) {
    const int64_t id = (int64_t)blockIdx.x * kT + threadIdx.x;
    if (id >= (int64_t)n_rows * H) return;
    const int r = (int)(id / H), m = (int)(id % H);
    const int64_t j = nodes[r];
    const float v = dhs[(int64_t)r * H + m];
    for (int e = child_ptr[j]; e < child_ptr[j + 1]; ++e) dh[(int64_t)child_idx[e] * H + m] += v;
}

// hs_r = sum over children of h_k (fp32 sum, rounded once), level order
template <typename T>
__global__ void __launch_bounds__(kT)
bwd_hsum_kernel(const int32_t *__restrict__ nodes, int n_rows, int H,
                const int32_t *__restrict__ child_ptr, const int32_t *__restrict__ child_idx,
                const T *__restrict__ h, T *__restrict__ hs) {
    const int64_t id = (int64_t)blockIdx.x * kT + threadIdx.x;
    if (id >= (int64_t)n_rows * H) return;
    const int r = (int)(id / H), m = (int)(id % H);
    const int64_t j = nodes[r];
    float s = 0.0f;
    for (int e = child_ptr[j]; e < child_ptr[j + 1]; ++e) s += to_f32<T>(h[(int64_t)child_idx[e] * H + m]);
    hs[(int64_t)r * H + m] = from_f32<T>(s);
}

// ---- transpose with an optional row gather -------------------------------------------
// dst[c][r] = src[row(r)][c] for r < n_rows, 0 for n_rows <= r < ld_dst (the reduction axis
// of the weight-gradient GEMMs is padded with zeros).  row(r) = index[r] or r.
// The destination is a K-blocked operand (dst_rows_alloc rows per slab) whose K axis is r, padded
// with zeros up to k_pad; the source is row-major with stride ld_src, or K-blocked itself when
// src_rows_alloc > 0.
template <typename T>
__global__ void __launch_bounds__(kT)
transpose_rows_kernel(const T *__restrict__ src, const int32_t *__restrict__ index, int64_t ld_src,
                      int64_t src_rows_alloc, int n_rows, int n_cols, T *__restrict__ dst,
                      int64_t dst_rows_alloc, int k_pad) {
    __shared__ T tile[32][33];
    const int r0 = blockIdx.x * 32, c0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = r0 + ty + 8 * i, cc = c0 + tx;
        T v = T(0);
        if (r < n_rows && cc < n_cols) {
            const int64_t row = index ? index[r] : r;
            if (src_rows_alloc > 0)
                v = *reinterpret_cast<const T *>(reinterpret_cast<const char *>(src) +
                                                 operand_offset(row, (int64_t)cc * sizeof(T), src_rows_alloc));
            else
                v = src[row * ld_src + cc];
        }
        tile[ty + 8 * i][tx] = v;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int cc = c0 + ty + 8 * i, r = r0 + tx;
        if (cc < n_cols && r < k_pad)
            *reinterpret_cast<T *>(reinterpret_cast<char *>(dst) +
                                   operand_offset(cc, (int64_t)r * sizeof(T), dst_rows_alloc)) = tile[tx][ty + 8 * i];
    }
}

// db_p += sum over the row of dZt (fp32 sum of the operand values)
template <typename T>
__global__ void __launch_bounds__(kT)
rowsum_kernel(const T *__restrict__ src, int64_t rows_alloc, int n, float *__restrict__ out) {
    __shared__ float part[kT];
    float s = 0.0f;
    for (int i = threadIdx.x; i < n; i += kT)
        s += to_f32<T>(*reinterpret_cast<const T *>(reinterpret_cast<const char *>(src) +
                                                    operand_offset(blockIdx.x, (int64_t)i * sizeof(T), rows_alloc)));
    part[threadIdx.x] = s;
    __syncthreads();
    for (int d = kT / 2; d > 0; d >>= 1) {
        if (threadIdx.x < d) part[threadIdx.x] += part[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[blockIdx.x] += part[0];
}

// ---- generic GEMM: C = A B^T, A [M, K] and B [N, K] with K contiguous -------------------
// Block = 4 waves; wave w owns rows m0 + 32 w .. + 31 and 128 columns (four MFMA tiles that
// share the A fragment).  Fragments come straight from global memory (16 bytes per lane
// and K group of 32 bytes), kAhead groups requested ahead; no LDS, no barriers.  Rows of A
// may be gathered through an index.  K (in bytes) must be a multiple of 32 and every row
// 16-byte aligned.  What happens to an output element is the epilogue functor's business.
constexpr int kAhead = 4;

struct EpiDxDhs {          // columns < D are dx of the row's node, the rest dhs in level order
    float *dx; const int32_t *node; int D; float *dhs; int H;
    __device__ __forceinline__ void operator()(int row, int col, float v) const {
        if (col < D) dx[(int64_t)node[row] * D + col] = v;
        else dhs[(int64_t)row * H + (col - D)] = v;
    }
};
struct EpiAddRows {        // dst[node[row]] += v
    float *dst; const int32_t *node; int ld;
    __device__ __forceinline__ void operator()(int row, int col, float v) const {
        dst[(int64_t)node[row] * ld + col] += v;
    }
};
struct EpiAtomicAcc {      // C += v, from several blocks that split the reduction axis
    float *C; int ldc;
    __device__ __forceinline__ void operator()(int row, int col, float v) const {
        atomicAdd(&C[(int64_t)row * ldc + col], v);
    }
};

template <typename T, typename Epi>
__global__ void __launch_bounds__(kT, 2)
gemm_nt_kernel(const T *__restrict__ A, const int32_t *__restrict__ a_index, int64_t lda, int M,
               const T *__restrict__ B, int64_t ldb, int N, int K, int k_chunk, Epi epi) {
    constexpr int ESZ = (int)sizeof(T);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    const int m0 = (blockIdx.x * 4 + wave) * 32;
    const int n0 = blockIdx.y * 128;
    if (m0 >= M) return;
    int ar = m0 + l32;
    if (ar >= M) ar = M - 1;
    const int64_t arow = a_index ? a_index[ar] : ar;
    // blockIdx.z takes the K range [z * k_chunk, min(K, (z + 1) * k_chunk))
    const int64_t k_begin = (int64_t)blockIdx.z * k_chunk;
    const int k_len = (int)((K - k_begin) < k_chunk ? (K - k_begin) : k_chunk);
    const char *ap = reinterpret_cast<const char *>(A) + (arow * lda + k_begin) * ESZ + hf * 16;
    const char *bp[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        int br = n0 + q * 32 + l32;
        if (br >= N) br = N - 1;
        bp[q] = reinterpret_cast<const char *>(B) + ((int64_t)br * ldb + k_begin) * ESZ + hf * 16;
    }
    const int n_groups = k_len * ESZ / 32;
    floatx16 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[q][v] = 0.0f;
    u32x4 fa[kAhead], fb[kAhead][4];
    auto request = [&](int g, int slot) __attribute__((always_inline)) {
        fa[slot] = *reinterpret_cast<const u32x4 *>(ap + (int64_t)g * 32);
#pragma unroll
        for (int q = 0; q < 4; ++q) fb[slot][q] = *reinterpret_cast<const u32x4 *>(bp[q] + (int64_t)g * 32);
    };
#pragma unroll
    for (int s = 0; s < kAhead; ++s)
        if (s < n_groups) request(s, s);
    for (int g0 = 0; g0 < n_groups; g0 += kAhead) {
#pragma unroll
        for (int s = 0; s < kAhead; ++s) {
            const int g = g0 + s;
            if (g < n_groups) {
#pragma unroll
                for (int q = 0; q < 4; ++q) mfma_step<T>(fa[s], fb[s][q], acc[q]);
                if (g + kAhead < n_groups) request(g + kAhead, s);
            }
        }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int col = n0 + q * 32 + l32;
        if (col >= N) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = m0 + (v >> 2) * 8 + hf * 4 + (v & 3);
            if (row < M) epi(row, col, acc[q][v]);
        }
    }
}

// k_splits > 1 cuts the reduction axis into that many ranges (multiples of 64 elements) handled
// by different blocks; the epilogue must then add atomically.
template <typename T, typename Epi>
int launch_gemm_nt(const T *A, const int32_t *a_index, int64_t lda, int M, const T *B, int64_t ldb, int N, int K,
                   Epi epi, hipStream_t st, int k_splits = 1) {
    if (M <= 0 || N <= 0 || K <= 0) return JITDB_OK;
    int k_chunk = K;
    if (k_splits > 1) k_chunk = (int)round_up(ceil_div(K, k_splits), 64);
    dim3 grid((unsigned)ceil_div(M, 128), (unsigned)ceil_div(N, 128), (unsigned)ceil_div(K, k_chunk));
    gemm_nt_kernel<T, Epi><<<grid, kT, 0, st>>>(A, a_index, lda, M, B, ldb, N, K, k_chunk, epi);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

// enough ranges of the reduction axis to give every SIMD several waves, none shorter than 512
inline int splits_for(int M, int N, int K) {
    const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 128);
    int64_t want = ceil_div(4096, tiles);
    const int64_t most = K / 512 > 0 ? K / 512 : 1;
    if (want > most) want = most;
    return (int)(want < 1 ? 1 : want);
}

// dW [4H, D], dU [4H, H], db [4H] from the packed accumulators (gate stride Hk)
__global__ void __launch_bounds__(kT)
unpack_grads_kernel(const float *__restrict__ dMp, const float *__restrict__ dUfp, const float *__restrict__ dbp,
                    int D, int H, int Hk, float *__restrict__ dW, float *__restrict__ dU, float *__restrict__ db) {
    const int64_t total = (int64_t)4 * H * (D + H);
    for (int64_t idx = (int64_t)blockIdx.x * kT + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * kT) {
        const int row = (int)(idx / (D + H)), col = (int)(idx % (D + H));
        const int g = row / H, m = row % H;
        const float v = dMp[((int64_t)g * Hk + m) * (D + H) + col];
        if (col < D) dW[(int64_t)row * D + col] = v;
        else dU[(int64_t)row * H + (col - D)] = g < 3 ? v : dUfp[(int64_t)m * H + (col - D)];
        if (col == 0) db[row] = dbp[g * Hk + m];
    }
}

// ---- workspace ---------------------------------------------------------------------
struct BwdDims {
    int D, H, Hk;         // Hk: H rounded up to 16 elements (K groups of the GEMMs)
    int n_max, n_pad;     // largest level; rounded up to 64 (reduction axis of the weight GEMMs)
    size_t esz;
};
struct BwdWs {
    float *dh, *dc, *dhs, *dMp, *dUfp, *dbp;
    void *Mt, *Uft, *dZ, *G, *hs, *dZt, *At, *Gt, *Hkt;
    size_t bytes;
};

BwdWs carve_bwd_ws(int64_t n, const BwdDims &d, void *base) {
    Carver c(base);
    BwdWs w;
    w.dh = c.take<float>((size_t)n * d.H);
    w.dc = c.take<float>((size_t)n * d.H);
    w.dhs = c.take<float>((size_t)d.n_max * d.H);
    w.dMp = c.take<float>((size_t)4 * d.Hk * (d.D + d.H));
    w.dUfp = c.take<float>((size_t)d.Hk * d.H);
    w.dbp = c.take<float>((size_t)4 * d.Hk);
    w.Mt = c.take<char>((size_t)round_up(d.D + d.H, 256) * 4 * d.Hk * d.esz);
    w.Uft = c.take<char>((size_t)d.H * d.Hk * d.esz);
    w.dZ = c.take<char>((size_t)round_up(d.n_max, 128) * 4 * d.Hk * d.esz);
    w.G = c.take<char>((size_t)n * d.Hk * d.esz);
    w.hs = c.take<char>((size_t)d.n_max * d.H * d.esz);
    w.dZt = c.take<char>((size_t)round_up(4 * d.Hk, 128) * d.n_pad * d.esz);
    w.At = c.take<char>((size_t)round_up(d.D + d.H, 256) * d.n_pad * d.esz);
    w.Gt = c.take<char>((size_t)round_up(d.Hk, 128) * d.n_pad * d.esz);
    w.Hkt = c.take<char>((size_t)round_up(d.H, 256) * d.n_pad * d.esz);
    w.bytes = c.off;
    return w;
}

int zero_bytes(void *p, size_t bytes, hipStream_t st) {    // bytes is a multiple of 16 (256-byte pieces)
    const int64_t n16 = (int64_t)((bytes + 15) / 16);
    const unsigned grid = (unsigned)(ceil_div(n16, kT) < 8192 ? ceil_div(n16, kT) : 8192);
    fill_bytes16_kernel<<<grid ? grid : 1, kT, 0, st>>>(static_cast<u32x4 *>(p), n16);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

template <typename T>
int run_backward(const T *x, const T *W, const T *U, const BwdDims &d, const jitdb_schedule_t *s,
                 const T *h, const float *c, const float *gates, const float *fgate,
                 const float *gh, const float *gc, float *dx, float *dW, float *dU, float *db,
                 const BwdWs &w, hipStream_t st) {
    const int64_t n = s->n_nodes;
    const int L = s->n_levels;
    const int32_t *lp = s->host_level_ptr;
    const int D = d.D, H = d.H, Hk = d.Hk;
    int rc;
    {
        const unsigned grid = (unsigned)(ceil_div(n * H, kT) < 16384 ? ceil_div(n * H, kT) : 16384);
        copy_or_zero_kernel<<<grid, kT, 0, st>>>(gh, w.dh, n * H);
        JITDB_LAUNCH_CHECK();
        copy_or_zero_kernel<<<grid, kT, 0, st>>>(gc, w.dc, n * H);
        JITDB_LAUNCH_CHECK();
    }
    // pad columns and the rows of roots must read as zero
    if ((rc = zero_bytes(w.G, round_up((size_t)n * Hk * d.esz, 256), st)) != JITDB_OK) return rc;
    if ((rc = zero_bytes(w.dMp, round_up((size_t)4 * Hk * (D + H) * 4, 256), st)) != JITDB_OK) return rc;
    if ((rc = zero_bytes(w.dUfp, round_up((size_t)Hk * H * 4, 256), st)) != JITDB_OK) return rc;
    if ((rc = zero_bytes(w.dbp, round_up((size_t)4 * Hk * 4, 256), st)) != JITDB_OK) return rc;
    const int64_t mt_alloc = round_up(D + H, 256), zt_alloc = round_up(4 * Hk, 128), at_alloc = round_up(D + H, 256);
    const int64_t gt_alloc = round_up(Hk, 128), ht_alloc = round_up(H, 256);
    const jitdb_dtype dtype = sizeof(T) == 4 ? JITDB_F32 : JITDB_BF16;
    pack_bwd_weights_kernel<T><<<1024, kT, 0, st>>>(W, U, D, H, Hk, static_cast<T *>(w.Mt), mt_alloc, static_cast<T *>(w.Uft));
    JITDB_LAUNCH_CHECK();

    T *dZ = static_cast<T *>(w.dZ), *G = static_cast<T *>(w.G), *hs = static_cast<T *>(w.hs);
    T *dZt = static_cast<T *>(w.dZt), *At = static_cast<T *>(w.At), *Gt = static_cast<T *>(w.Gt), *Hkt = static_cast<T *>(w.Hkt);
    for (int l = L - 1; l >= 0; --l) {
        const int rows = lp[l + 1] - lp[l];
        if (rows <= 0) return JITDB_E_SCHEDULE;
        const int32_t *nodes = s->perm + lp[l];
        const int kpad = (int)round_up(rows, 64);           // reduction length of the weight GEMMs
        const int64_t dz_alloc = round_up(rows, 128);
        const unsigned g_elem = (unsigned)ceil_div((int64_t)rows * H, kT);
        const unsigned g_elem_k = (unsigned)ceil_div((int64_t)rows * Hk, kT);
        const unsigned tr = (unsigned)ceil_div(kpad, 32);
        auto weight_gemm = [&](const T *A, int64_t a_alloc, int M, const T *B, int64_t b_alloc, int N, float *C, int ldc) {
            KbGemm g = {};
            g.A = A; g.a_rows_alloc = a_alloc; g.M = M; g.B = B; g.b_rows_alloc = b_alloc; g.N = N;
            g.k_bytes = (int64_t)kpad * sizeof(T);
            const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 256);
            int64_t want = ceil_div(2048, tiles);
            const int64_t most = kpad / 512 > 0 ? kpad / 512 : 1;
            g.k_splits = (int)(want < most ? want : most);
            g.epilogue = KB_EPI_ATOMIC_ACC; g.out0 = C; g.ldc = ldc;
            return launch_kb_gemm(dtype, g, st);
        };
        if (l < L - 1) {
            // these nodes may have parents: dh_k += G_k U_f, and dU_f += sum_k G_k (x) h_k
            if ((rc = launch_gemm_nt<T>(G, nodes, Hk, rows, static_cast<const T *>(w.Uft), Hk, H, Hk,
                                        EpiAddRows{w.dh, nodes, H}, st)) != JITDB_OK) return rc;
            transpose_rows_kernel<T><<<dim3(tr, (unsigned)ceil_div(Hk, 32)), kT, 0, st>>>(
                G, nodes, Hk, 0, rows, Hk, Gt, gt_alloc, kpad);
            JITDB_LAUNCH_CHECK();
            transpose_rows_kernel<T><<<dim3(tr, (unsigned)ceil_div(H, 32)), kT, 0, st>>>(
                h, nodes, H, 0, rows, H, Hkt, ht_alloc, kpad);
            JITDB_LAUNCH_CHECK();
            if ((rc = weight_gemm(Gt, gt_alloc, Hk, Hkt, ht_alloc, H, w.dUfp, H)) != JITDB_OK) return rc;
        }
        bwd_cell_kernel<T><<<g_elem_k, kT, 0, st>>>(nodes, rows, H, Hk, s->child_ptr, s->child_idx, c, gates, fgate,
                                                    w.dh, w.dc, dZ, dz_alloc, G);
        JITDB_LAUNCH_CHECK();
        {   // [dx | dhs] = dZ [W | U]
            KbGemm g = {};
            g.A = dZ; g.a_rows_alloc = dz_alloc; g.M = rows;
            g.B = w.Mt; g.b_rows_alloc = mt_alloc; g.N = D + H;
            g.k_bytes = (int64_t)4 * Hk * sizeof(T); g.k_splits = 1;
            g.epilogue = KB_EPI_DX_DHS; g.out0 = dx; g.out1 = w.dhs; g.node = nodes; g.D = D; g.H = H;
            if ((rc = launch_kb_gemm(dtype, g, st)) != JITDB_OK) return rc;
        }
        if (l > 0) {
            bwd_scatter_kernel<<<g_elem, kT, 0, st>>>(nodes, rows, H, s->child_ptr, s->child_idx, w.dhs, w.dh);
            JITDB_LAUNCH_CHECK();
            bwd_hsum_kernel<T><<<g_elem, kT, 0, st>>>(nodes, rows, H, s->child_ptr, s->child_idx, h, hs);
            JITDB_LAUNCH_CHECK();
        }
        // weight gradients: dMp += dZ^T [x | hs] (leaves have hs = 0: the x columns only)
        transpose_rows_kernel<T><<<dim3(tr, (unsigned)ceil_div(4 * Hk, 32)), kT, 0, st>>>(
            dZ, nullptr, 0, dz_alloc, rows, 4 * Hk, dZt, zt_alloc, kpad);
        JITDB_LAUNCH_CHECK();
        transpose_rows_kernel<T><<<dim3(tr, (unsigned)ceil_div(D, 32)), kT, 0, st>>>(
            x, nodes, D, 0, rows, D, At, at_alloc, kpad);
        JITDB_LAUNCH_CHECK();
        int q_cols = D;
        if (l > 0) {
            transpose_rows_kernel<T><<<dim3(tr, (unsigned)ceil_div(H, 32)), kT, 0, st>>>(
                hs, nullptr, H, 0, rows, H,
                reinterpret_cast<T *>(reinterpret_cast<char *>(At) + (int64_t)D * 64), at_alloc, kpad);
            JITDB_LAUNCH_CHECK();
            q_cols = D + H;
        }
        if ((rc = weight_gemm(dZt, zt_alloc, 4 * Hk, At, at_alloc, q_cols, w.dMp, D + H)) != JITDB_OK) return rc;
        rowsum_kernel<T><<<4 * Hk, kT, 0, st>>>(dZt, zt_alloc, rows, w.dbp);
        JITDB_LAUNCH_CHECK();
    }
    unpack_grads_kernel<<<1024, kT, 0, st>>>(w.dMp, w.dUfp, w.dbp, D, H, Hk, dW, dU, db);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

bool bwd_dims(const jitdb_schedule_t *s, int32_t D, int32_t H, jitdb_dtype dtype, BwdDims &d) {
    if (!s || s->n_nodes < 0 || s->n_nodes > JITDB_MAX_NODES) return false;
    if (D < 1 || D > (1 << 16) || H < 1 || H > (1 << 14)) return false;
    if (dtype != JITDB_F32 && dtype != JITDB_BF16) return false;
    d.D = D; d.H = H; d.Hk = (int)round_up(H, 16);
    d.esz = dtype == JITDB_F32 ? 4 : 2;
    int n_max = 1;
    if (s->host_level_ptr)
        for (int l = 0; l < s->n_levels; ++l) {
            const int r = s->host_level_ptr[l + 1] - s->host_level_ptr[l];
            if (r > n_max) n_max = r;
        }
    d.n_max = n_max;
    d.n_pad = (int)round_up(n_max, 64);
    return true;
}

}  // namespace
}  // namespace jitdb

using namespace jitdb;

extern "C" size_t jitdb_treelstm_backward_workspace_bytes(const jitdb_schedule_t *s, int32_t D, int32_t H,
                                                          jitdb_dtype dtype) {
    BwdDims d;
    if (!bwd_dims(s, D, H, dtype, d)) return 0;
    return carve_bwd_ws(s->n_nodes, d, nullptr).bytes;
}

extern "C" int jitdb_treelstm_backward(const void *x, const void *W, const void *U,
                                       int32_t D, int32_t H, jitdb_dtype dtype, const jitdb_schedule_t *s,
                                       const void *h, const float *c, const float *gates, const float *fgate,
                                       const float *gh, const float *gc,
                                       float *dx, float *dW, float *dU, float *db,
                                       void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!s) return JITDB_E_NULL;
    drop_stale_hip_error();
    BwdDims d;
    if (!bwd_dims(s, D, H, dtype, d)) return JITDB_E_BADARG;
    if (!W || !U || !dW || !dU || !db) return JITDB_E_NULL;
    const int64_t n = s->n_nodes;
    hipStream_t st = (hipStream_t)hip_stream;
    if (n == 0) {
        fill_f32_kernel<<<256, kT, 0, st>>>(dW, (int64_t)4 * H * D, 0.0f);
        JITDB_LAUNCH_CHECK();
        fill_f32_kernel<<<256, kT, 0, st>>>(dU, (int64_t)4 * H * H, 0.0f);
        JITDB_LAUNCH_CHECK();
        fill_f32_kernel<<<1, kT, 0, st>>>(db, (int64_t)4 * H, 0.0f);
        JITDB_LAUNCH_CHECK();
        return JITDB_OK;
    }
    if (!x || !h || !c || !gates || !fgate || !dx || !workspace) return JITDB_E_NULL;
    if (!s->perm || !s->child_ptr || !s->child_idx || !s->host_level_ptr) return JITDB_E_NULL;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return JITDB_E_BADARG;
    // operand rows are read in 16-byte pieces
    if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(h) & 15)) return JITDB_E_BADARG;
    const int L = s->n_levels;
    if (L < 1 || L > n || s->host_level_ptr[0] != 0 || s->host_level_ptr[L] != n) return JITDB_E_SCHEDULE;
    const BwdWs w = carve_bwd_ws(n, d, workspace);
    if (workspace_bytes < w.bytes) return JITDB_E_WORKSPACE;
    if (dtype == JITDB_F32)
        return run_backward<float>(static_cast<const float *>(x), static_cast<const float *>(W),
                                   static_cast<const float *>(U), d, s, static_cast<const float *>(h), c, gates,
                                   fgate, gh, gc, dx, dW, dU, db, w, st);
    return run_backward<bf16_t>(static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(W),
                                static_cast<const bf16_t *>(U), d, s, static_cast<const bf16_t *>(h), c, gates,
                                fgate, gh, gc, dx, dW, dU, db, w, st);
}
