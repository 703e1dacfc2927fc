// jitdb_treelstm_backward: reverse-mode gradients of the level-batched Tree-LSTM forward.
//
// The paper trains through the same batched graph it infers with (section 5).  Here the
// levels of the schedule are visited from the roots down.  A node's parent lies in a higher
// level, so when a level is reached every parent has already left its total dc and its dhs =
// U_iou^T dz_iou (by node id); per level
//
//   (rows of G for this level: dz_f,k = dc_p c_k f_k (1 - f_k), written by the parents' cell kernels)
//   ufg = G U_f                                      GEMM over the level's rows
//   dU_f += G^T h                                    GEMM, reduction over the level's rows
//   bwd_cell_kernel      dh_j = gh_j + dhs_p + ufg_j, dc_j = gc_j + dc_p f_j + ..., then dz_i, dz_o,
//                        dz_u, sum_k dz_f,k from them and the saved gates; each child's dz_f,k -> G
//   [dx_j | dhs_j] = dZ_j [W | U]                    GEMM over the level's rows
//   [dW | db | dU_iou]^T += [x | 1 | hs]^T dZ        GEMM, reduction over the level's rows
//
// All four GEMMs run on the forward's tiled MFMA core (launch_kb_gemm: both operands
// K-blocked).  A reduction over rows needs operands whose K axis is the level's rows: the cell
// kernel writes dZ a second time, transposed through LDS; G, x and h are transposed by
// transpose_kb_kernel, the child sums hs are formed inside hsum_transpose_kernel.  Gradients
// are fp32; with JITDB_BF16 the GEMM operands (dz, x, h, hs, weights) and the values handed
// from level to level through dhs and ufg are bfloat16, every sum and dc fp32.

#include "common.h"

namespace jitdb {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kT = 256;

// ---- small helpers -----------------------------------------------------------------
__global__ void __launch_bounds__(kT)
fill_f32_kernel(float *p, int64_t n, float v) {
    for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += (int64_t)gridDim.x * kT) p[i] = v;
}
__global__ void __launch_bounds__(kT)
fill_bytes16_kernel(u32x4 *p, int64_t n16) {
    const u32x4 z = {0, 0, 0, 0};
    for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n16; i += (int64_t)gridDim.x * kT) p[i] = z;
}

// ---- weights for the data-gradient GEMMs ---------------------------------------------
// Both K-blocked, for the tiled GEMM.  Mt [D + H rows, 4 Hk]: row n < D is column n of W, row
// D + n' column n' of U, the four gates side by side at stride Hk (H rounded up, pad zero);
// the forget gate has no h-sum part, so its block is zero in the rows of U.  Uft [H rows, Hk]:
// row n = column n of U_f.
template <typename T>
__global__ void __launch_bounds__(kT)
pack_bwd_weights_kernel(const T *__restrict__ W, const T *__restrict__ U, int D, int H, int Hk,
                        T *__restrict__ Mt, int64_t mt_rows_alloc, T *__restrict__ Uft, int64_t uft_rows_alloc) {
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
        const T v = m < H ? U[((int64_t)3 * H + m) * H + n] : T(0);
        *reinterpret_cast<T *>(reinterpret_cast<char *>(Uft) + operand_offset(n, (int64_t)m * sizeof(T), uft_rows_alloc)) = v;
    }
}

// parent_of[k] for every node with a parent (the array is filled with -1 first)
__global__ void __launch_bounds__(kT)
parent_of_kernel(const int32_t *__restrict__ child_ptr, const int32_t *__restrict__ child_idx, int n,
                 int32_t *__restrict__ parent_of) {
    const int64_t j = (int64_t)blockIdx.x * kT + threadIdx.x;
    if (j >= n) return;
    for (int e = child_ptr[j]; e < child_ptr[j + 1]; ++e) parent_of[child_idx[e]] = (int32_t)j;
}
__global__ void __launch_bounds__(kT)
fill_i32_kernel(int32_t *p, int64_t n, int32_t v) {
    for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += (int64_t)gridDim.x * kT) p[i] = v;
}

// ---- elementwise kernels on (RT rows) x (64 units) tiles ------------------------------
// RT = 32 (bf16) / 16 (fp32) level rows fill one 64-byte slab of a K-blocked operand whose K
// axis is the level's rows.  Wave w of a block takes the rows w, w + 4, ... of the tile, a
// lane one unit; what a kernel produces goes out twice: row-wise into the K-blocked operand
// of the data-gradient GEMM, and, through an LDS tile, transposed into the operand of the
// weight-gradient GEMM (a thread stores 16 bytes, a wave 1 KB of consecutive memory).  Rows
// past the level's end and units past H are written as zeros in the transposed operand (they
// are part of the reduction); grid = (padded rows / RT, Hk / 64).
template <typename T, int NG>
__device__ __forceinline__ void store_transposed_tile(const T (*tile)[64 / sizeof(T)][64 + 2], int t, int Hk, int m0,
                                                      T *__restrict__ dst, int64_t dst_rows_alloc, int n_gates = NG) {
    constexpr int PER = 16 / (int)sizeof(T);
    const int cc = t >> 2, piece = t & 3;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        if (g >= n_gates) break;
        T out[PER];
#pragma unroll
        for (int e = 0; e < PER; ++e) out[e] = tile[g][piece * PER + e][cc];
        char *d = reinterpret_cast<char *>(dst) +
                  ((int64_t)blockIdx.x * dst_rows_alloc + (g * Hk + m0 + cc)) * 64 + piece * 16;
        *reinterpret_cast<u32x4 *>(d) = *reinterpret_cast<const u32x4 *>(out);
    }
}

// G holds dz_f,k = dc_p c_k f_k (1 - f_k) for every node k, K-blocked, rows in the order of the
// schedule's positions (all levels in one operand: a level is a range of rows).  The rows of
// nodes with a parent are written by the parent's cell kernel; this kernel zeroes the rows of
// the level's roots.  One thread per (level row, 16 bytes of the row).
template <typename T>
__global__ void __launch_bounds__(kT)
zero_root_rows_kernel(const int32_t *__restrict__ nodes, int n_rows, int Hk, const int32_t *__restrict__ parent_of,
                      T *__restrict__ G, int64_t g_rows_alloc) {
    constexpr int PER = 16 / (int)sizeof(T);
    const int pieces = Hk / PER;
    const int64_t id = (int64_t)blockIdx.x * kT + threadIdx.x;
    if (id >= (int64_t)n_rows * pieces) return;
    const int r = (int)(id / pieces), q = (int)(id % pieces);
    if (parent_of[nodes[r]] >= 0) return;
    const u32x4 z = {0, 0, 0, 0};
    *reinterpret_cast<u32x4 *>(reinterpret_cast<char *>(G) + operand_offset(r, (int64_t)q * 16, g_rows_alloc)) = z;
}

// The cell's elementwise derivative.  What node j receives is fetched here, by node id, from
// what its parent p left in a higher level (total dc_p, dhs_p = U_iou^T dz_iou,p):
//     dh_j = gh_j + dhs_p + ufg_r      ufg (level order, may be null) = U_f^T dz_f,j, the product
//                                      the GEMM before this kernel left
//     dc_j = gc_j + dc_p f_j + dh_j o_j (1 - tanh^2 c_j)
// Every child k of j gets its dz_f,k = dc_j c_k f_k (1 - f_k) written to row inv_perm[k] of G (the
// operand of the child level's GEMMs; pad units as zeros).
// Writes dZ row r = [dz_i | dz_o | dz_u | sum_k dz_f,k] (K-blocked, gate stride Hk), the same
// transposed into dZt, and leaves the total dc_j in dc[j] for the children's level.  Only the
// first n_gates blocks are written (3 at the leaf level, whose forget block is zero and unused).
template <typename T>
__global__ void __launch_bounds__(kT)
bwd_cell_kernel(const int32_t *__restrict__ nodes, int n_rows, int H, int Hk,
                const int32_t *__restrict__ child_ptr, const int32_t *__restrict__ child_idx,
                const int32_t *__restrict__ parent_of,
                const float *__restrict__ c, const T *__restrict__ gates, const T *__restrict__ fgate,
                const float *__restrict__ gh, const float *__restrict__ gc, const T *__restrict__ dhs,
                const T *__restrict__ ufg, float *__restrict__ dc,
                const int32_t *__restrict__ inv_perm, T *__restrict__ G, int64_t g_rows_alloc,
                T *__restrict__ dZ, int64_t dz_rows_alloc, T *__restrict__ dZt, int64_t zt_rows_alloc, int n_gates) {
    constexpr int RT = 64 / (int)sizeof(T);
    __shared__ T tile[4][RT][64 + 2];
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    const int r0 = blockIdx.x * RT, m0 = blockIdx.y * 64, m = m0 + lane;
    char *zb = reinterpret_cast<char *>(dZ);
#pragma unroll
    for (int i = 0; i < RT / 4; ++i) {
        const int rr = w + 4 * i, r = r0 + rr;
        float dz[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (r < n_rows && m < H) {
            const int64_t j = nodes[r];
            const float gi = to_f32<T>(gates[j * 3 * H + m]), go = to_f32<T>(gates[j * 3 * H + H + m]),
                        gu = to_f32<T>(gates[j * 3 * H + 2 * H + m]);
            const float th = tanhf(c[j * H + m]);
            const int64_t p = parent_of[j];
            float dhj = (gh ? gh[j * H + m] : 0.0f) + (ufg ? to_f32<T>(ufg[(int64_t)r * H + m]) : 0.0f);
            float dcj = gc ? gc[j * H + m] : 0.0f;
            if (p >= 0) {
                dhj += to_f32<T>(dhs[p * H + m]);
                dcj += dc[p * H + m] * to_f32<T>(fgate[j * H + m]);
            }
            dcj += dhj * go * (1.0f - th * th);
            dc[j * H + m] = dcj;
            float dzf_sum = 0.0f;
            for (int e = child_ptr[j]; e < child_ptr[j + 1]; ++e) {
                const int64_t k = child_idx[e];
                const float fk = to_f32<T>(fgate[k * H + m]);
                const float dzf = dcj * c[k * H + m] * fk * (1.0f - fk);
                dzf_sum += dzf;
                *reinterpret_cast<T *>(reinterpret_cast<char *>(G) +
                                       operand_offset(inv_perm[k], (int64_t)m * sizeof(T), g_rows_alloc)) = from_f32<T>(dzf);
            }
            dz[0] = dcj * gu * gi * (1.0f - gi);
            dz[1] = dhj * th * go * (1.0f - go);
            dz[2] = dcj * gi * (1.0f - gu * gu);
            dz[3] = dzf_sum;
        } else if (r < n_rows) {    // pad units of the children's rows
            const int64_t j = nodes[r];
            for (int e = child_ptr[j]; e < child_ptr[j + 1]; ++e)
                *reinterpret_cast<T *>(reinterpret_cast<char *>(G) +
                                       operand_offset(inv_perm[child_idx[e]], (int64_t)m * sizeof(T), g_rows_alloc)) = T(0);
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (g >= n_gates) break;
            const T v = from_f32<T>(dz[g]);
            tile[g][rr][lane] = v;
            if (r < n_rows)
                *reinterpret_cast<T *>(zb + operand_offset(r, (int64_t)(g * Hk + m) * sizeof(T), dz_rows_alloc)) = v;
        }
    }
    __syncthreads();
    store_transposed_tile<T, 4>(tile, t, Hk, m0, dZt, zt_rows_alloc, n_gates);
}

// ---- transposes into K-blocked operands ---------------------------------------------
// dst row c, K position r  =  src[row(r)][c]  for r < n_rows, 0 for n_rows <= r < k_pad: the rows
// of a level become the reduction axis of the weight-gradient GEMMs.  row(r) = index[r] or r;
// the source is row-major with stride ld_src, or K-blocked itself when src_rows_alloc > 0.  A
// block moves one 64-byte slab of the destination's K axis (RT = 32 bf16 / 16 fp32 source rows)
// times 64 columns; a thread stores 16 bytes, and since consecutive destination rows are
// consecutive inside a slab a wave stores 1 KB of consecutive memory.
// SRC selects how the tile is read: SRC_SCALAR one element per thread and step (any row
// stride), SRC_VEC LW bytes per thread and step (row-major rows that start on LW-byte
// boundaries; LW = 16 or 8), SRC_KB 16 bytes per thread from a K-blocked source whose width is
// a multiple of 64.
enum { SRC_SCALAR = 0, SRC_VEC = 1, SRC_KB = 2 };
template <typename T, int SRC, int LW = 16>
__global__ void __launch_bounds__(kT)
transpose_kb_kernel(const T *__restrict__ src, const int32_t *__restrict__ index, int64_t ld_src,
                    int64_t src_rows_alloc, int n_rows, int n_cols, T *__restrict__ dst, int64_t dst_rows_alloc) {
    constexpr int RT = 64 / (int)sizeof(T);
    constexpr int PER = 16 / (int)sizeof(T);        // elements in 16 bytes
    __shared__ T tile[RT][64 + 2];
    const int r0 = blockIdx.x * RT, c0 = blockIdx.y * 64;
    const int t = threadIdx.x;
    if (SRC == SRC_SCALAR) {
        const int tx = t & 63, ty = t >> 6;          // 64 columns x 4 rows per sweep
#pragma unroll
        for (int i = 0; i < RT / 4; ++i) {
            const int r = r0 + ty + 4 * i, cc = c0 + tx;
            T v = T(0);
            if (r < n_rows && cc < n_cols) v = src[(int64_t)(index ? index[r] : r) * ld_src + cc];
            tile[ty + 4 * i][tx] = v;
        }
    } else if (SRC == SRC_VEC) {
        // a row's 64 columns are 64 / PL pieces of LW bytes; 256 threads sweep the tile
        constexpr int PL = LW / (int)sizeof(T);
        constexpr int PPR = 64 / PL;
#pragma unroll
        for (int it = 0; it < RT * PPR / kT; ++it) {
            const int idx = t + kT * it;
            const int row = idx / PPR, col = (idx % PPR) * PL;
            T v[PL];
#pragma unroll
            for (int e = 0; e < PL; ++e) v[e] = T(0);
            if (r0 + row < n_rows && c0 + col < n_cols) {
                const T *a = src + (int64_t)(index ? index[r0 + row] : r0 + row) * ld_src + c0 + col;
                if (c0 + col + PL <= n_cols) {
                    if constexpr (LW == 16) *reinterpret_cast<u32x4 *>(v) = *reinterpret_cast<const u32x4 *>(a);
                    else *reinterpret_cast<uint2 *>(v) = *reinterpret_cast<const uint2 *>(a);
                } else {
#pragma unroll
                    for (int e = 0; e < PL; ++e)
                        if (c0 + col + e < n_cols) v[e] = a[e];
                }
            }
#pragma unroll
            for (int e = 0; e < PL; ++e) tile[row][col + e] = v[e];
        }
    } else {
        // the tile is 64 / RT slabs of RT rows x 64 bytes: 256 threads x 16 bytes
        const int piece = t & 3, sl = (t >> 2) / RT;
        const int row = (t >> 2) % RT, col = sl * RT + piece * PER;
        T v[PER];
#pragma unroll
        for (int e = 0; e < PER; ++e) v[e] = T(0);
        if (r0 + row < n_rows)
            *reinterpret_cast<u32x4 *>(v) = *reinterpret_cast<const u32x4 *>(
                reinterpret_cast<const char *>(src) + ((int64_t)((c0 + col) / RT) * src_rows_alloc + r0 + row) * 64 + piece * 16);
#pragma unroll
        for (int e = 0; e < PER; ++e) tile[row][col + e] = v[e];
    }
    __syncthreads();
    const int cc = t >> 2, piece = t & 3;
    if (c0 + cc >= n_cols) return;
    T out[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) out[e] = tile[piece * PER + e][cc];
    char *d = reinterpret_cast<char *>(dst) + ((int64_t)blockIdx.x * dst_rows_alloc + (c0 + cc)) * 64 + piece * 16;
    *reinterpret_cast<u32x4 *>(d) = *reinterpret_cast<const u32x4 *>(out);
}

// picks the widest read the source allows
template <typename T>
int launch_transpose(const T *src, const int32_t *index, int64_t ld_src, int64_t src_rows_alloc, int n_rows, int n_cols,
                     int k_pad, T *dst, int64_t dst_rows_alloc, hipStream_t st) {
    constexpr int RT = 64 / (int)sizeof(T);
    const dim3 grid((unsigned)(k_pad / RT), (unsigned)ceil_div(n_cols, 64));
    const uintptr_t base = reinterpret_cast<uintptr_t>(src);
    const int64_t row_bytes = ld_src * (int64_t)sizeof(T);
    if (src_rows_alloc > 0) {
        if (n_cols % 64 != 0) return JITDB_E_BADARG;
        transpose_kb_kernel<T, SRC_KB><<<grid, kT, 0, st>>>(src, index, ld_src, src_rows_alloc, n_rows, n_cols, dst, dst_rows_alloc);
    } else if (row_bytes % 16 == 0 && base % 16 == 0) {
        transpose_kb_kernel<T, SRC_VEC, 16><<<grid, kT, 0, st>>>(src, index, ld_src, 0, n_rows, n_cols, dst, dst_rows_alloc);
    } else if (row_bytes % 8 == 0 && base % 8 == 0) {
        transpose_kb_kernel<T, SRC_VEC, 8><<<grid, kT, 0, st>>>(src, index, ld_src, 0, n_rows, n_cols, dst, dst_rows_alloc);
    } else {
        transpose_kb_kernel<T, SRC_SCALAR><<<grid, kT, 0, st>>>(src, index, ld_src, 0, n_rows, n_cols, dst, dst_rows_alloc);
    }
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

// The child sums of a level, transposed: dst row c, K position r = sum over the children k of
// node nodes[r] of h_k[c], summed in fp32 and rounded once as the forward does.  Same tiles
// and stores as transpose_kb_kernel; VEC reads 16 bytes of a child's row per thread.
template <typename T, bool VEC>
__global__ void __launch_bounds__(kT)
hsum_transpose_kernel(const T *__restrict__ h, const int32_t *__restrict__ nodes, int n_rows, int H,
                      const int32_t *__restrict__ child_ptr, const int32_t *__restrict__ child_idx,
                      T *__restrict__ dst, int64_t dst_rows_alloc) {
    constexpr int RT = 64 / (int)sizeof(T);
    constexpr int PER = 16 / (int)sizeof(T);
    __shared__ T tile[RT][64 + 2];
    const int r0 = blockIdx.x * RT, c0 = blockIdx.y * 64;
    const int t = threadIdx.x;
    const int row = t / (64 / PER), col = (t % (64 / PER)) * PER;
    float sum[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) sum[e] = 0.0f;
    if (r0 + row < n_rows && c0 + col < H) {
        const int64_t j = nodes[r0 + row];
        for (int ce = child_ptr[j]; ce < child_ptr[j + 1]; ++ce) {
            const T *a = h + (int64_t)child_idx[ce] * H + c0 + col;
            if (VEC && c0 + col + PER <= H) {
                T v[PER];
                *reinterpret_cast<u32x4 *>(v) = *reinterpret_cast<const u32x4 *>(a);
#pragma unroll
                for (int e = 0; e < PER; ++e) sum[e] += to_f32<T>(v[e]);
            } else {
#pragma unroll
                for (int e = 0; e < PER; ++e)
                    if (c0 + col + e < H) sum[e] += to_f32<T>(a[e]);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < PER; ++e) tile[row][col + e] = from_f32<T>(sum[e]);
    __syncthreads();
    const int cc = t >> 2, piece = t & 3;
    if (c0 + cc >= H) return;
    T out[PER];
#pragma unroll
    for (int e = 0; e < PER; ++e) out[e] = tile[piece * PER + e][cc];
    char *d = reinterpret_cast<char *>(dst) + ((int64_t)blockIdx.x * dst_rows_alloc + (c0 + cc)) * 64 + piece * 16;
    *reinterpret_cast<u32x4 *>(d) = *reinterpret_cast<const u32x4 *>(out);
}

// one K-blocked row of ones (r < n_rows) and zeros (up to k_pad): the column of the weight
// GEMM's right operand that turns its result into the bias gradient
template <typename T>
__global__ void __launch_bounds__(kT)
ones_row_kernel(T *__restrict__ dst, int64_t dst_rows_alloc, int row, int n_rows, int k_pad) {
    const int r = blockIdx.x * kT + threadIdx.x;
    if (r >= k_pad) return;
    *reinterpret_cast<T *>(reinterpret_cast<char *>(dst) + operand_offset(row, (int64_t)r * sizeof(T), dst_rows_alloc)) =
        from_f32<T>(r < n_rows ? 1.0f : 0.0f);
}

// dW [4H, D], dU [4H, H], db [4H] from the packed accumulators: dMp [D + 1 + H, 4 Hk] (transposed:
// row n < D belongs to x_n, row D to the bias, row D + 1 + n' to hs_n'), dUfp [Hk, H]
__global__ void __launch_bounds__(kT)
unpack_grads_kernel(const float *__restrict__ dMp, const float *__restrict__ dUfp,
                    int D, int H, int Hk, float *__restrict__ dW, float *__restrict__ dU, float *__restrict__ db) {
    const int ld = D + 1 + H;
    const int64_t total = (int64_t)4 * H * ld;
    for (int64_t idx = (int64_t)blockIdx.x * kT + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * kT) {
        const int row = (int)(idx / ld), col = (int)(idx % ld);
        const int g = row / H, m = row % H;
        const float v = dMp[(int64_t)col * 4 * Hk + g * Hk + m];
        if (col < D) dW[(int64_t)row * D + col] = v;
        else if (col == D) db[row] = v;
        else dU[(int64_t)row * H + (col - D - 1)] = g < 3 ? v : dUfp[(int64_t)m * H + (col - D - 1)];
    }
}

// ---- workspace ---------------------------------------------------------------------
struct BwdDims {
    int D, H, Hk;         // Hk: H rounded up to 64 elements (whole stages of the tiled GEMM)
    int n_max, n_pad;     // largest level; rounded up to 64 (reduction axis of the weight GEMMs)
    size_t esz;
};
struct BwdWs {
    float *dc, *dMp, *dUfp;
    void *dhs, *ufg;      // in the operands' element type
    int32_t *parent_of;
    void *Mt, *Uft, *dZ, *G, *dZt, *At, *Gt, *Hkt;
    size_t bytes;
};

BwdWs carve_bwd_ws(int64_t n, const BwdDims &d, void *base) {
    Carver c(base);
    BwdWs w;
    w.dc = c.take<float>((size_t)n * d.H);
    w.dhs = c.take<char>((size_t)n * d.H * d.esz);
    w.ufg = c.take<char>((size_t)d.n_max * d.H * d.esz);
    w.dMp = c.take<float>((size_t)4 * d.Hk * (d.D + 1 + d.H));
    w.dUfp = c.take<float>((size_t)d.Hk * d.H);
    w.parent_of = c.take<int32_t>((size_t)n);
    w.Mt = c.take<char>((size_t)round_up(d.D + d.H, 256) * 4 * d.Hk * d.esz);
    w.Uft = c.take<char>((size_t)round_up(d.H, 256) * d.Hk * d.esz);
    w.dZ = c.take<char>((size_t)round_up(d.n_max, 128) * 4 * d.Hk * d.esz);
    w.G = c.take<char>((size_t)(round_up(n, 128) + 128) * d.Hk * d.esz);   // all levels; whole row tiles are read
    w.dZt = c.take<char>((size_t)round_up(4 * d.Hk, 128) * d.n_pad * d.esz);
    w.At = c.take<char>((size_t)round_up(d.D + 1 + d.H, 256) * d.n_pad * d.esz);
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
                 const T *h, const float *c, const T *gates, const T *fgate,
                 const float *gh, const float *gc, float *dx, float *dW, float *dU, float *db,
                 const BwdWs &w, hipStream_t st) {
    const int64_t n = s->n_nodes;
    const int L = s->n_levels;
    const int32_t *lp = s->host_level_ptr;
    const int D = d.D, H = d.H, Hk = d.Hk;
    const jitdb_dtype dtype = sizeof(T) == 4 ? JITDB_F32 : JITDB_BF16;
    int rc;
    if ((rc = zero_bytes(w.dMp, round_up((size_t)4 * Hk * (D + 1 + H) * 4, 256), st)) != JITDB_OK) return rc;
    if ((rc = zero_bytes(w.dUfp, round_up((size_t)Hk * H * 4, 256), st)) != JITDB_OK) return rc;
    const int64_t mt_alloc = round_up(D + H, 256), uft_alloc = round_up(H, 256);
    const int64_t zt_alloc = round_up(4 * Hk, 128), at_alloc = round_up(D + 1 + H, 256);
    const int64_t gt_alloc = round_up(Hk, 128), ht_alloc = round_up(H, 256);
    pack_bwd_weights_kernel<T><<<1024, kT, 0, st>>>(W, U, D, H, Hk, static_cast<T *>(w.Mt), mt_alloc,
                                                    static_cast<T *>(w.Uft), uft_alloc);
    JITDB_LAUNCH_CHECK();
    {
        const unsigned g = (unsigned)ceil_div(n, kT);
        fill_i32_kernel<<<g < 8192 ? g : 8192, kT, 0, st>>>(w.parent_of, n, -1);
        JITDB_LAUNCH_CHECK();
        parent_of_kernel<<<g, kT, 0, st>>>(s->child_ptr, s->child_idx, (int)n, w.parent_of);
        JITDB_LAUNCH_CHECK();
    }

    T *dZ = static_cast<T *>(w.dZ), *G_all = static_cast<T *>(w.G);
    const int64_t g_alloc = round_up(n, 128) + 128;
    T *dZt = static_cast<T *>(w.dZt), *At = static_cast<T *>(w.At), *Gt = static_cast<T *>(w.Gt), *Hkt = static_cast<T *>(w.Hkt);
    for (int l = L - 1; l >= 0; --l) {
        const int rows = lp[l + 1] - lp[l];
        if (rows <= 0) return JITDB_E_SCHEDULE;
        const int32_t *nodes = s->perm + lp[l];
        const int kpad = (int)round_up(rows, 64);           // reduction length of the weight GEMMs
        const int64_t lvl_alloc = round_up(rows, 128);
        const dim3 tile_grid((unsigned)(kpad / (64 / (int)sizeof(T))), (unsigned)(Hk / 64));
        auto weight_gemm = [&](const T *A, int64_t a_alloc, int M, const T *B, int64_t b_alloc, int N, float *C, int ldc) {
            KbGemm g = {};
            g.A = A; g.a_rows_alloc = a_alloc; g.M = M; g.B = B; g.b_rows_alloc = b_alloc; g.N = N;
            g.k_bytes = (int64_t)kpad * sizeof(T);
            const int64_t tiles = ceil_div(M, 128) * ceil_div(N, 256);
            // one round of blocks (two per CU), in multiples of eight splits: a split's XCD is split % 8
            int64_t want = 8 * (512 / (8 * tiles));
            if (want < 8) want = tiles >= 512 ? 1 : 8;
            const int64_t most = kpad / 512 > 0 ? kpad / 512 : 1;
            g.k_splits = (int)(want < most ? want : most);
            g.epilogue = KB_EPI_ATOMIC_ACC; g.out0 = C; g.ldc = ldc;
            return launch_kb_gemm(dtype, g, st);
        };
        // leaves have no children: their forget-gate block of dZ is zero and is left out of both GEMMs
        const int n_gates = l > 0 ? 4 : 3;
        // what the level receives from above
        if (l < L - 1) {
            // the level's rows of G: written by the parents' cell kernels, zero for roots
            T *G = reinterpret_cast<T *>(reinterpret_cast<char *>(G_all) + (int64_t)lp[l] * 64);
            const int pieces = Hk / (16 / (int)sizeof(T));
            zero_root_rows_kernel<T><<<(unsigned)ceil_div((int64_t)rows * pieces, kT), kT, 0, st>>>(
                nodes, rows, Hk, w.parent_of, G, g_alloc);
            JITDB_LAUNCH_CHECK();
            if ((rc = launch_transpose<T>(G, nullptr, 0, g_alloc, rows, Hk, kpad, Gt, gt_alloc, st)) != JITDB_OK) return rc;
            // ufg_r = U_f^T dz_f,k (level order), and dU_f += sum_k dz_f,k (x) h_k
            KbGemm g = {};
            g.A = G; g.a_rows_alloc = g_alloc; g.M = rows;
            g.B = w.Uft; g.b_rows_alloc = uft_alloc; g.N = H;
            g.k_bytes = (int64_t)Hk * sizeof(T); g.k_splits = 1;
            g.epilogue = KB_EPI_STORE; g.out0 = w.ufg; g.ldc = H;
            if ((rc = launch_kb_gemm(dtype, g, st)) != JITDB_OK) return rc;
            if ((rc = launch_transpose<T>(h, nodes, H, 0, rows, H, kpad, Hkt, ht_alloc, st)) != JITDB_OK) return rc;
            if ((rc = weight_gemm(Gt, gt_alloc, Hk, Hkt, ht_alloc, H, w.dUfp, H)) != JITDB_OK) return rc;
        }
        bwd_cell_kernel<T><<<tile_grid, kT, 0, st>>>(nodes, rows, H, Hk, s->child_ptr, s->child_idx, w.parent_of, c,
                                                     gates, fgate, gh, gc, static_cast<const T *>(w.dhs),
                                                     l < L - 1 ? static_cast<const T *>(w.ufg) : nullptr, w.dc,
                                                     s->inv_perm, G_all, g_alloc, dZ, lvl_alloc, dZt, zt_alloc, n_gates);
        JITDB_LAUNCH_CHECK();
        {   // [dx | dhs] = dZ [W | U]; leaves have nobody to pass dhs to
            KbGemm g = {};
            g.A = dZ; g.a_rows_alloc = lvl_alloc; g.M = rows;
            g.B = w.Mt; g.b_rows_alloc = mt_alloc; g.N = l > 0 ? D + H : D;
            g.k_bytes = (int64_t)n_gates * Hk * sizeof(T); g.k_splits = 1;
            g.epilogue = KB_EPI_DX_DHS; g.out0 = dx; g.out1 = w.dhs; g.node = nodes; g.D = D; g.H = H;
            if ((rc = launch_kb_gemm(dtype, g, st)) != JITDB_OK) return rc;
        }
        // weight gradients: dMp += [x | 1 | hs]^T dZ (leaves have hs = 0: the x and bias rows only)
        if ((rc = launch_transpose<T>(x, nodes, D, 0, rows, D, kpad, At, at_alloc, st)) != JITDB_OK) return rc;
        ones_row_kernel<T><<<(unsigned)ceil_div(kpad, kT), kT, 0, st>>>(At, at_alloc, D, rows, kpad);
        JITDB_LAUNCH_CHECK();
        int q_cols = D + 1;
        if (l > 0) {
            T *hs_rows = reinterpret_cast<T *>(reinterpret_cast<char *>(At) + (int64_t)(D + 1) * 64);
            const dim3 grid((unsigned)(kpad / (64 / (int)sizeof(T))), (unsigned)ceil_div(H, 64));
            if ((H * sizeof(T)) % 16 == 0)
                hsum_transpose_kernel<T, true><<<grid, kT, 0, st>>>(h, nodes, rows, H, s->child_ptr, s->child_idx, hs_rows, at_alloc);
            else
                hsum_transpose_kernel<T, false><<<grid, kT, 0, st>>>(h, nodes, rows, H, s->child_ptr, s->child_idx, hs_rows, at_alloc);
            JITDB_LAUNCH_CHECK();
            q_cols = D + 1 + H;
        }
        // [x | 1 | hs]^T dZ rather than its transpose: the narrow side (813 or 301) then pads to
        // 128-row tiles instead of 256-column tiles
        if ((rc = weight_gemm(At, at_alloc, q_cols, dZt, zt_alloc, n_gates * Hk, w.dMp, 4 * Hk)) != JITDB_OK) return rc;
    }
    unpack_grads_kernel<<<1024, kT, 0, st>>>(w.dMp, w.dUfp, D, H, Hk, dW, dU, db);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

bool bwd_dims(const jitdb_schedule_t *s, int32_t D, int32_t H, jitdb_dtype dtype, BwdDims &d) {
    if (!s || s->n_nodes < 0 || s->n_nodes > JITDB_MAX_NODES) return false;
    if (D < 1 || D > (1 << 16) || H < 1 || H > (1 << 14)) return false;
    if (dtype != JITDB_F32 && dtype != JITDB_BF16) return false;
    d.D = D; d.H = H; d.Hk = (int)round_up(H, 64);
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
                                       const void *h, const float *c, const void *gates, const void *fgate,
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
    if (!s->perm || !s->inv_perm || !s->child_ptr || !s->child_idx || !s->host_level_ptr) return JITDB_E_NULL;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return JITDB_E_BADARG;
    // operand rows are read in 16-byte pieces
    if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(h) & 15) ||
        (reinterpret_cast<uintptr_t>(dx) & 15))
        return JITDB_E_BADARG;
    const int L = s->n_levels;
    if (L < 1 || L > n || s->host_level_ptr[0] != 0 || s->host_level_ptr[L] != n) return JITDB_E_SCHEDULE;
    const BwdWs w = carve_bwd_ws(n, d, workspace);
    if (workspace_bytes < w.bytes) return JITDB_E_WORKSPACE;
    if (dtype == JITDB_F32)
        return run_backward<float>(static_cast<const float *>(x), static_cast<const float *>(W),
                                   static_cast<const float *>(U), d, s, static_cast<const float *>(h), c,
                                   static_cast<const float *>(gates), static_cast<const float *>(fgate), gh, gc, dx, dW, dU, db, w, st);
    return run_backward<bf16_t>(static_cast<const bf16_t *>(x), static_cast<const bf16_t *>(W),
                                static_cast<const bf16_t *>(U), d, s, static_cast<const bf16_t *>(h), c,
                                static_cast<const bf16_t *>(gates), static_cast<const bf16_t *>(fgate), gh, gc, dx, dW, dU, db, w, st);
}
