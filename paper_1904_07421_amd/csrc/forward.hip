// jitdb_treelstm_forward: the execution half of the method for gfx950.
//
// The paper runs the look-up table slot by slot in depth order; per slot it
// stacks the samples, runs the shared subgraph once and slices the results
// (section 4.3).  Here a slot is one height level of the forest and the
// subgraph is the Child-Sum Tree-LSTM cell (section 3).  Per level:
//
//   stack_kernel       row r of the level's input matrix = [x_j | sum_k h_k] over the
//                      child CSR (the arity-dependent operator; HBM-bound, 16-byte
//                      coalesced row pieces)
//   level_kernel<LEAF|INTERNAL>   [x_j ; hs_j] x [W ; U]^T on MFMA with the whole cell
//                      fused into the epilogue: per-child forget gates from the
//                      precomputed P_k = U_f h_k, c_j and h_j written once
//   level_kernel<PROJ> P_k = U_f h_k for the nodes just produced, so that their
//                      parent reads one row per child (every non-root node is a
//                      child exactly once)
//   thin_kernel        the same three jobs for levels too small to fill the chip with
//                      128 x 256 tiles: one 32 x 32-unit tile per wave, operands straight
//                      from L2; a thin level's projection and the next level's stack
//                      step share one launch (thin_proj_stack_kernel)
//   chain_kernel       a thin level whose nodes all have exactly one child (sequences, the long
//                      tail of a deep forest) as ONE launch: x and the child's h read in place,
//                      all four gates over the full K, no stack step and no projection
//   tile256_kernel     (level256.hip) the level kernel on 256 x 256 tiles, bf16; switched off
//
// With cells of different type in the table (jitdb_treelstm_forward_cells) a slot of N-ary cells
// runs nary_level_kernel below: the same GEMM core with the N-ary cell update as its epilogue.
// With a typed table (jitdb_treelstm_forward_typed) a slot is (level, signature): each
// signature has its own packed weights, the projection of a sub-slot uses the parent
// cell's, and the slots of a large level run in one grouped launch through a tile table.
// gemm_kb_kernel is the same GEMM core as a plain C = A B^T for the backward pass.
//
// "Stack" is the row gather through perm (level-major order) done by
// stack_kernel, "slice" is the scatter of rows back to node-id order in the
// epilogue.
//
// Weights are re-packed once per call: gate rows of 32 hidden units are
// interleaved (i|o|u|f blocks of 32 rows), so that one wave holds all four
// gates of a hidden unit in its own accumulators and the cell update needs no
// exchange between lanes; rows and K are zero padded to tile multiples.

#include "level_common.h"

#include <mutex>
#include <vector>

namespace jitdb {
namespace {

// ---- weight packing ----------------------------------------------------------------
// Packed row r = tile*128 + gate*32 + uu holds gate `gate` of hidden unit tile*32 + uu as
// [ W row (D values, zero padded to Dp) | U row (H values, zero padded to Hp) ].  There are
// NPU >= NP rows; rows of units >= H are zero.
struct PackArgs {
    const void *W, *U; const float *b;
    int D, H, Dp, Hp, NP, NPU;
    void *Bp; float *bp;
    void *Bf;       // the same rows fragment-major for the 256 x 256 tile kernel (bf16, one cell), or null
};

// block `block` of `n_blocks` (NT threads each, stride loop)
template <typename T, int NT = kThreads>
__device__ __forceinline__ void pack_weights_body(const T *__restrict__ W, const T *__restrict__ U,
                                                  const float *__restrict__ b, int D, int H, int Dp, int Hp,
                                                  int NP, int NPU, T *__restrict__ Bp, float *__restrict__ bp,
                                                  T *__restrict__ Bf, int64_t block, int64_t n_blocks) {
    const int Kp = Dp + Hp;
    const int64_t total = (int64_t)NPU * Kp;
    for (int64_t idx = block * NT + threadIdx.x; idx < total; idx += n_blocks * NT) {
        const int r = (int)(idx / Kp), k = (int)(idx % Kp);
        const int tile = r / kGateTile, gate = (r % kGateTile) / kUnit, uu = r % kUnit;
        const int unit = tile * kUnit + uu;
        const bool row_ok = unit < H;
        const int64_t src = (int64_t)gate * H + unit;
        T v = T(0);
        if (row_ok) {
            if (k < D) v = W[src * D + k];
            else if (k >= Dp && k - Dp < H) v = U[src * H + (k - Dp)];
        }
        *reinterpret_cast<T *>(reinterpret_cast<char *>(Bp) +
                               operand_offset(r, (int64_t)k * sizeof(T), NPU)) = v;
        if (Bf)
            *reinterpret_cast<T *>(reinterpret_cast<char *>(Bf) + fragment_offset(r, (int64_t)k * sizeof(T), Kp * (int)sizeof(T) / 32)) = v;
        if (k == 0 && r < NP) bp[r] = row_ok ? b[src] : 0.0f;
    }
}

template <typename T>
__global__ void __launch_bounds__(kThreads)
pack_weights_kernel(const PackArgs p) {
    pack_weights_body<T>(static_cast<const T *>(p.W), static_cast<const T *>(p.U), p.b, p.D, p.H, p.Dp, p.Hp, p.NP,
                         p.NPU, static_cast<T *>(p.Bp), p.bp, static_cast<T *>(p.Bf), blockIdx.x, gridDim.x);
}

// ---- row records -------------------------------------------------------------------
// What the stack step and the cell update need to know about the node in row r of a
// level, in one 32-byte record: { node, arity, CSR start, - } { first four child ids (-1
// where there is none) }.  Written once per forward for all levels, so that the per-level
// kernels start from one load instead of the chain perm -> child_ptr -> child_idx.
//
// The rows of a level are independent, so their order inside the level is free.  The
// cell update walks the child lists of 32 rows in lock step and takes as many rounds as
// the longest of them; with rows in node-id order that is about twice the average need.
// The records are therefore ordered by falling arity inside windows of kRecWindow level
// positions (a counting sort in LDS; positions are already ordered by level, and the
// level is the major key so every row stays inside its level).  A window that spans 16 or
// more levels is left in position order: its levels are too small for the order to matter.
// The longer the runs of equal arity, the fewer passes of the cell update mix child lists of different length: a
// large forest takes windows of 16384 positions (blocks of 1024 threads, a launch of their own); measured on
// 2.36 M nodes, windows of 4096 -> 8192 -> 16384 rows take the internal levels from 5.26 to 5.17 to 5.10 ms
// (32768: 5.13) for 0.04 / 0.085 ms more in this step.
constexpr int kRecPerThread = 16;
constexpr int kRecWindow = kRecPerThread * kThreads;          // 4096
constexpr int kRecThreadsLarge = 1024;
constexpr int kRecWindowLarge = kRecPerThread * kRecThreadsLarge;   // 16384
constexpr int64_t kRecLargeMinNodes = 262144;      // forests of at least this many nodes take the large windows

// window `window` of the records (NT threads, kRecPerThread records each)
template <int NT>
__device__ __forceinline__ void row_record_body(const int32_t *__restrict__ perm, const int32_t *__restrict__ height,
                                                const int32_t *__restrict__ child_ptr,
                                                const int32_t *__restrict__ child_idx,
                                                int4 *__restrict__ row_rec, int n, int window) {
    constexpr int kWin = kRecPerThread * NT;
    __shared__ int s_count[256];   // per key: count, then the next free slot
    __shared__ int s_scan[256];
    const int t = threadIdx.x;
    const int w0 = window * kWin;
    const int wn = (n - w0) < kWin ? (n - w0) : kWin;
    const int lvl0 = height[perm[w0]];
    const int lvl1 = height[perm[w0 + wn - 1]];
    const bool sorted = (lvl1 - lvl0) < 16;
    if (t < 256) s_count[t] = 0;
    __syncthreads();
    // A thread's sixteen records are fetched side by side, not one after the other: every load of a step is
    // unconditional (a position past the window reads the window's last one and is dropped afterwards), so the
    // chain perm -> child_ptr / height costs its two trips to memory once per thread, not once per record.
    int node[kRecPerThread], ar[kRecPerThread], cb[kRecPerThread], key[kRecPerThread];
    bool live[kRecPerThread];
#pragma unroll
    for (int i = 0; i < kRecPerThread; ++i) {
        const int p = w0 + i * NT + t;
        live[i] = p < w0 + wn;
        node[i] = perm[live[i] ? p : w0 + wn - 1];
    }
    int hgt[kRecPerThread];
#pragma unroll
    for (int i = 0; i < kRecPerThread; ++i) {
        cb[i] = child_ptr[node[i]];
        ar[i] = child_ptr[node[i] + 1] - cb[i];
        hgt[i] = sorted ? height[node[i]] : 0;
    }
#pragma unroll
    for (int i = 0; i < kRecPerThread; ++i) {
        key[i] = 0;
        if (!live[i]) {
            node[i] = -1; ar[i] = 0; cb[i] = 0;
        } else if (sorted) {
            key[i] = (hgt[i] - lvl0) * 16 + (15 - (ar[i] < 15 ? ar[i] : 15));
            atomicAdd(&s_count[key[i]], 1);
        }
    }
    __syncthreads();
    // exclusive scan of the 256 counts (by the first 256 threads; every thread meets the barriers)
    const int v = t < 256 ? s_count[t] : 0;
    if (t < 256) s_scan[t] = v;
    __syncthreads();
    for (int d = 1; d < 256; d <<= 1) {
        const int add = (t < 256 && t >= d) ? s_scan[t - d] : 0;
        __syncthreads();
        if (t < 256) s_scan[t] += add;
        __syncthreads();
    }
    if (t < 256) s_count[t] = s_scan[t] - v;
    __syncthreads();
    // the first four child ids of every record, again all loads of the thread side by side (a child position the
    // node does not have reads the node's first position, or, for a leaf, whatever stands at its CSR start, which
    // lies inside the array: child_ptr <= E < N; the value is replaced by -1)
    // (in two halves: eight records' ids are in flight at a time, which keeps the large-window form in its registers)
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        constexpr int HB = kRecPerThread / 2;
        int kid[HB][4];
#pragma unroll
        for (int i = 0; i < HB; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) kid[i][j] = child_idx[cb[half * HB + i] + (j < ar[half * HB + i] ? j : 0)];
#pragma unroll
        for (int k = 0; k < HB; ++k) {
            const int i = half * HB + k;
            if (node[i] < 0) continue;
            const int64_t q = sorted ? (int64_t)w0 + atomicAdd(&s_count[key[i]], 1) : (int64_t)w0 + i * NT + t;
            row_rec[2 * q] = make_int4(node[i], ar[i], cb[i], 0);
            row_rec[2 * q + 1] = make_int4(0 < ar[i] ? kid[k][0] : -1, 1 < ar[i] ? kid[k][1] : -1,
                                           2 < ar[i] ? kid[k][2] : -1, 3 < ar[i] ? kid[k][3] : -1);
        }
    }
}

// Once per forward, in one launch: the row records of every level position (blocks
// [0, n_windows)) and the first cell's packed weights (the remaining blocks); neither needs
// the other.
template <typename T>
__global__ void __launch_bounds__(kThreads)
prepare_kernel(const int32_t *__restrict__ perm, const int32_t *__restrict__ key,
               const int32_t *__restrict__ child_ptr, const int32_t *__restrict__ child_idx,
               int4 *__restrict__ row_rec, int n, int n_windows, const PackArgs p) {
    if ((int)blockIdx.x < n_windows)
        row_record_body<kThreads>(perm, key, child_ptr, child_idx, row_rec, n, blockIdx.x);
    else
        pack_weights_body<T>(static_cast<const T *>(p.W), static_cast<const T *>(p.U), p.b, p.D, p.H, p.Dp, p.Hp,
                             p.NP, p.NPU, static_cast<T *>(p.Bp), p.bp, static_cast<T *>(p.Bf),
                             (int64_t)blockIdx.x - n_windows, (int64_t)gridDim.x - n_windows);
}

// The same launch for large forests: row records in windows of kRecWindowLarge positions, blocks of 1024 threads.
template <typename T>
__global__ void __launch_bounds__(kRecThreadsLarge)
prepare_large_kernel(const int32_t *__restrict__ perm, const int32_t *__restrict__ key,
                     const int32_t *__restrict__ child_ptr, const int32_t *__restrict__ child_idx,
                     int4 *__restrict__ row_rec, int n, int n_windows, const PackArgs p) {
    if ((int)blockIdx.x < n_windows)
        row_record_body<kRecThreadsLarge>(perm, key, child_ptr, child_idx, row_rec, n, blockIdx.x);
    else
        pack_weights_body<T, kRecThreadsLarge>(static_cast<const T *>(p.W), static_cast<const T *>(p.U), p.b, p.D, p.H,
                                               p.Dp, p.Hp, p.NP, p.NPU, static_cast<T *>(p.Bp), p.bp,
                                               static_cast<T *>(p.Bf), (int64_t)blockIdx.x - n_windows,
                                               (int64_t)gridDim.x - n_windows);
}

// ---- stack -------------------------------------------------------------------------
// The paper's "stack" step (section 4.3): the samples of one slot are laid side by
// side on the batch axis.  Row r of the level's dense input matrix A is
//     [ x_j (D values, zero padded to Dp) | hsum_j = sum over children of h_k (Hp values) ]
// for the r-th node j of the level; leaves have the x part only.  One thread
// per 16-byte piece of a row; child rows come from hs (stride Hp, pad columns zero,
// rows by node id) in 16-byte pieces, up to four children in flight.
template <typename T>
__device__ __forceinline__ void add_piece(float (&acc)[Traits<T>::VEC], const uint4 &v) {
    if constexpr (sizeof(T) == 4) {
        acc[0] += __uint_as_float(v.x); acc[1] += __uint_as_float(v.y);
        acc[2] += __uint_as_float(v.z); acc[3] += __uint_as_float(v.w);
    } else {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[2 * j] += __uint_as_float(w[j] << 16);
            acc[2 * j + 1] += __uint_as_float(w[j] & 0xFFFF0000u);
        }
    }
}

struct StackArgs {
    const void *x; int D, Dp; const void *hs; int Hp;
    const int4 *row_rec; const int32_t *child_idx;
    void *A; int n_rows, n_rows_alloc;
};

// block `block` of the stack step (kThreads threads)
template <typename T, bool WITH_H>
__device__ __forceinline__ void stack_body(const T *__restrict__ x, int D, int Dp, const T *__restrict__ hs, int Hp,
                                           const int4 *__restrict__ row_rec, const int32_t *__restrict__ child_idx,
                                           T *__restrict__ A, int n_rows, int n_rows_alloc, int64_t block) {
    constexpr int VEC = Traits<T>::VEC;
    const int Kp = Dp + (WITH_H ? Hp : 0);
    const int cpr = Kp / VEC;
    const int64_t gid = block * kThreads + threadIdx.x;
    const int64_t row = gid / cpr;
    const int ch = (int)(gid % cpr);
    if (row >= n_rows) return;
    const int4 r0 = row_rec[2 * row];
    const int node = r0.x;
    const int k0 = ch * VEC;
    uint4 o = make_uint4(0u, 0u, 0u, 0u);
    if (k0 < Dp) {
        const T *src = x + (int64_t)node * D + k0;
        if ((D & 3) == 0) {
            // rows of x are 4-element aligned: move 4-element halves, zero past D
            if constexpr (sizeof(T) == 4) {
                if (k0 < D) o = *reinterpret_cast<const uint4 *>(src);
            } else {
                if (k0 < D) { const uint2 q = *reinterpret_cast<const uint2 *>(src); o.x = q.x; o.y = q.y; }
                if (k0 + 4 < D) { const uint2 q = *reinterpret_cast<const uint2 *>(src + 4); o.z = q.x; o.w = q.y; }
            }
        } else {
            // any other D: element by element
            T e[VEC];
#pragma unroll
            for (int j = 0; j < VEC; ++j) e[j] = (k0 + j < D) ? src[j] : T(0);
            if constexpr (sizeof(T) == 4) {
                o.x = __float_as_uint(e[0]); o.y = __float_as_uint(e[1]);
                o.z = __float_as_uint(e[2]); o.w = __float_as_uint(e[3]);
            } else {
                o.x = (uint32_t)e[0] | ((uint32_t)e[1] << 16); o.y = (uint32_t)e[2] | ((uint32_t)e[3] << 16);
                o.z = (uint32_t)e[4] | ((uint32_t)e[5] << 16); o.w = (uint32_t)e[6] | ((uint32_t)e[7] << 16);
            }
        }
    } else if constexpr (WITH_H) {
        const int kh = k0 - Dp;
        const int ar = r0.y;
        const int4 kids = row_rec[2 * row + 1];
        const int kid[4] = {kids.x, kids.y, kids.z, kids.w};
        float acc[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) acc[j] = 0.0f;
        uint4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v[j] = make_uint4(0u, 0u, 0u, 0u);
            if (j < ar) v[j] = *reinterpret_cast<const uint4 *>(hs + (int64_t)kid[j] * Hp + kh);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) add_piece<T>(acc, v[j]);   // ascending child id; zeros add nothing
        for (int c = 4; c < ar; ++c) {
            const int k = child_idx[r0.z + c];
            add_piece<T>(acc, *reinterpret_cast<const uint4 *>(hs + (int64_t)k * Hp + kh));
        }
        if constexpr (sizeof(T) == 4) {
            o.x = __float_as_uint(acc[0]); o.y = __float_as_uint(acc[1]);
            o.z = __float_as_uint(acc[2]); o.w = __float_as_uint(acc[3]);
        } else {
            uint32_t w[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                w[j] = (uint32_t)f32_to_bf16(acc[2 * j]) | ((uint32_t)f32_to_bf16(acc[2 * j + 1]) << 16);
            o.x = w[0]; o.y = w[1]; o.z = w[2]; o.w = w[3];
        }
    }
    *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(A) +
                               operand_offset(row, (int64_t)k0 * sizeof(T), n_rows_alloc)) = o;
}

template <typename T, bool WITH_H>
__global__ void __launch_bounds__(kThreads)
stack_kernel(const T *__restrict__ x, int D, int Dp, const T *__restrict__ hs, int Hp,
             const int4 *__restrict__ row_rec, const int32_t *__restrict__ child_idx,
             T *__restrict__ A, int n_rows, int n_rows_alloc) {
    stack_body<T, WITH_H>(x, D, Dp, hs, Hp, row_rec, child_idx, A, n_rows, n_rows_alloc, blockIdx.x);
}

// Block id -> tile of the level kernel.  The hardware deals consecutive block ids
// round-robin to the 8 XCDs, each with its own L2.  Row tile r belongs to XCD r % 8, so
// that the blocks of all its column tiles read the same A rows through one L2.  Inside an
// XCD the column tiles are taken in groups of kColGroup: the XCD sweeps all its row tiles
// with one group of columns, then with the next, which bounds the B rows in use at a
// time; A is fetched once per group.  (With 8 column tiles, H = 512, one group measured
// faster than two: re-reading A costs more than the B rows that fall out of L2.)  The
// grid holds 8 * ceil(R / 8) * C blocks; blocks past an XCD's share return at once.
constexpr int kColGroup = 8;
__device__ __forceinline__ bool block_to_tile(int b, int n_row_tiles, int n_col_tiles, int &row_tile, int &col_tile) {
    const int xcd = b & 7, idx = b >> 3;
    const int rows_x = (n_row_tiles - xcd + 7) >> 3;        // row tiles of this XCD
    if (idx >= rows_x * n_col_tiles) return false;
    const int g = idx / (rows_x * kColGroup);
    const int rem = idx - g * rows_x * kColGroup;
    const int left = n_col_tiles - g * kColGroup;
    const int cg = left < kColGroup ? left : kColGroup;    // columns in this group
    row_tile = xcd + 8 * (rem / cg);
    col_tile = g * kColGroup + rem % cg;
    return true;
}

// ---- the level GEMM ------------------------------------------------------------------
// One block of four waves computes 128 rows x 256 packed columns (2 unit tiles x 4 gates x
// 32 units); each wave a 64 x 128 sub-tile, i.e. 2 x 4 MFMA tiles of 32 x 32, so that all
// four gates of a hidden unit end up in one wave's accumulators.  Two blocks share a CU
// (half the LDS and at most 256 registers each): the start-up and the memory-bound cell
// update of one leave the matrix cores to the other.
//
// A is the level's stacked input [x | hsum], B the packed [W | U]; K runs over stages of
// 64 bytes per row, n_x stages of the x part, then n_h of the h part, in which the forget
// gate is skipped (U_f applies to each child's own h, not to the sum).  The projection
// instead reads A rows from h by node id and uses only the U part of the forget rows.
// Stages travel from global memory straight into LDS (global_load_lds, 16 bytes per lane)
// without passing through registers.  Three stage buffers: while stage g is multiplied,
// g+1 and g+2 (and for half the time g+3) are in flight; one barrier per stage.
//
// In each 16-wide (bf16) or 8-wide (fp32) K group, lanes 0-31 take the first 16 bytes and
// lanes 32-63 the next 16 for A and B alike; since the same assignment is used on both
// operands any such split of K is a valid MFMA schedule.
//
// A direct load writes the 64 lanes' pieces to 1024 consecutive LDS bytes, i.e. 16 rows of
// 64 bytes with no room for padding, so bank conflicts are avoided by permuting the four
// 16-byte pieces of a row instead: piece p of row r is kept in slot p ^ ((r >> 2) & 3).
// The lane that fills slot s of row r therefore fetches piece s ^ ((r >> 2) & 3), and a
// fragment read of 16 consecutive rows touches 16 distinct 16-byte columns.
constexpr int kDmaThreads = 256;
constexpr int kDmaBM = 128;        // rows per block
constexpr int kDmaStage = 64;      // bytes of K per row and stage
constexpr int kDmaBuf = (kDmaBM + kBN) * kDmaStage;
constexpr int kDmaBufs = 3;
constexpr int kWarmMaxStages = 256; // longest K loop whose A tile is requested up front (2 MB)


// Waits until at most N of this wave's loads are outstanding and all its LDS operations
// are done, then meets the block at a barrier.  Written as one asm statement with a memory
// clobber so that nothing moves across it, and without the fence of __syncthreads(), which
// would wait for every direct-to-LDS load in flight.
template <int N>
__device__ __forceinline__ void dma_wait_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

template <typename T, int MODE, int NBUF = kDmaBufs, typename Hook>
__device__ __forceinline__ void dma_gemm(const LevelArgs &a, char *lds, const int *row_node,
                                         int tile_row0, int col_tile, floatx16 (&acc)[2][4],
                                         char *sink, Hook &&after_first_requests) {
    constexpr int ESZ = (int)sizeof(T);
    constexpr int NG_X = (MODE == MODE_LEAF) ? 3 : 4;      // gate tiles multiplied in the x part
    constexpr int NG_H = (MODE == MODE_INTERNAL) ? 3 : 4;  // ... in the h part
    constexpr int NB = (MODE == MODE_LEAF) ? 3 : 4;        // 16-row B units a wave moves per stage
    constexpr int NLOAD = 2 + NB;                          // loads per wave and stage

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int hf = lane >> 5, l32 = lane & 31;

    const int n_x = (MODE == MODE_PROJ) ? 0 : a.Dp * ESZ / kDmaStage;
    const int n_h = (MODE == MODE_LEAF) ? 0 : a.Hp * ESZ / kDmaStage;
    const int n_stages = n_x + n_h;   // even and >= 2: K is padded to 128 bytes

    // ---- mover: lane l fills slot l&3 of row l>>2 of each 16-row unit it is given
    const int lrow = lane >> 2;
    const int piece16 = ((lane & 3) ^ ((lane >> 4) & 3)) * 16;
    const char *pa[2];
    int a_lds[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = (wave + 4 * i) * 16 + lrow;      // row of the tile
        a_lds[i] = (wave + 4 * i) * 16 * kDmaStage;
        if constexpr (MODE == MODE_PROJ) {
            int g = tile_row0 + r;
            if (g >= a.n_rows) g = a.n_rows - 1;
            pa[i] = static_cast<const char *>(a.hs) + (int64_t)row_node[g - tile_row0] * a.Hp * ESZ + piece16;
        } else {
            pa[i] = static_cast<const char *>(a.stack) + (int64_t)(tile_row0 + r) * kDmaStage + piece16;
        }
    }
    // bytes from one stage to the next: a slab of A / of B; the projection's A rows are
    // rows of h in node order, K contiguous
    const int64_t a_stage = (MODE == MODE_PROJ) ? kDmaStage : (int64_t)a.n_rows_alloc * kDmaStage;
    const int64_t b_stage = (int64_t)a.NPU * kDmaStage;
    const char *pb[NB];
    int b_lds[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int idx = wave * NB + i;
        int lds_row;
        int64_t src_row;
        if constexpr (MODE == MODE_PROJ) {
            // LDS row q*32 + u holds the forget row of unit u of unit tile col_tile*8 + q
            const int q = idx >> 1;
            lds_row = q * kUnit + (idx & 1) * 16;
            src_row = (int64_t)(col_tile * 8 + q) * kGateTile + 3 * kUnit + (idx & 1) * 16 + lrow;
        } else {
            // LDS row = packed row within the block's 256; the leaf level skips the forget rows
            const int ut = idx / (2 * NB), gate = (idx % (2 * NB)) >> 1;
            lds_row = ut * kGateTile + gate * kUnit + (idx & 1) * 16;
            src_row = (int64_t)col_tile * kBN + lds_row + lrow;
        }
        b_lds[i] = (kDmaBM + lds_row) * kDmaStage;
        pb[i] = static_cast<const char *>(a.Bp) +
                operand_offset(src_row, MODE == MODE_PROJ ? (int64_t)a.Dp * ESZ : 0, a.NPU) + piece16;
    }
    // load i (0 .. NLOAD-1) of stage s
    auto issue_one = [&](int s, int buf, int i) __attribute__((always_inline)) {
        char *dst = lds + buf * kDmaBuf;
        if (i < 2)
            __builtin_amdgcn_global_load_lds(JITDB_GLOBAL_PTR(pa[i] + s * a_stage), JITDB_LDS_PTR(dst + a_lds[i]), 16, 0, 0);
        else
            __builtin_amdgcn_global_load_lds(JITDB_GLOBAL_PTR(pb[i - 2] + s * b_stage), JITDB_LDS_PTR(dst + b_lds[i - 2]), 16, 0, 0);
    };
    auto issue = [&](int s, int buf) __attribute__((always_inline)) {
        char *dst = lds + buf * kDmaBuf;
#pragma unroll
        for (int i = 0; i < 2; ++i)
            __builtin_amdgcn_global_load_lds(JITDB_GLOBAL_PTR(pa[i] + s * a_stage), JITDB_LDS_PTR(dst + a_lds[i]), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < NB; ++i)
            __builtin_amdgcn_global_load_lds(JITDB_GLOBAL_PTR(pb[i] + s * b_stage), JITDB_LDS_PTR(dst + b_lds[i]), 16, 0, 0);
    };

    // ---- fragments: K group h (0, 1) of a stage is pieces 2h (lanes 0-31) and 2h+1 (lanes 32-63)
    const int sw = (l32 >> 2) & 3;
    int a_rd[2], b_rd[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int slot16 = ((2 * h + hf) ^ sw) * 16;
        a_rd[h] = (wm * 64 + l32) * kDmaStage + slot16;
        b_rd[h] = (kDmaBM + wn * 128 + l32) * kDmaStage + slot16;
    }
    // Fragment reads are written as asm: the compiler would otherwise make every LDS read
    // wait for all direct-to-LDS loads in flight, which it cannot tell apart from the
    // buffer being read.  The waits for the reads are therefore placed by hand as well
    // (LDS operations of a wave complete in order).  A K group's fragments: two of A, NG of B.
    const uint32_t lds_base = (uint32_t)(uintptr_t)JITDB_LDS_PTR(lds);
    struct Frags {
        u32x4 a[2], b[4];
    };
    auto read_group = [&](int buf, int h, auto ng_tag, Frags &f) __attribute__((always_inline)) {
        constexpr int NG = decltype(ng_tag)::value;
        const uint32_t aa = lds_base + buf * kDmaBuf + a_rd[h];
        const uint32_t bb = lds_base + buf * kDmaBuf + b_rd[h];
        asm volatile("ds_read_b128 %0, %1" : "=v"(f.a[0]) : "v"(aa) : "memory");
        asm volatile("ds_read_b128 %0, %1" : "=v"(f.b[0]) : "v"(bb) : "memory");
        asm volatile("ds_read_b128 %0, %1 offset:2048" : "=v"(f.a[1]) : "v"(aa) : "memory");
        asm volatile("ds_read_b128 %0, %1 offset:2048" : "=v"(f.b[1]) : "v"(bb) : "memory");
        asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(f.b[2]) : "v"(bb) : "memory");
        if constexpr (NG == 4)
            asm volatile("ds_read_b128 %0, %1 offset:6144" : "=v"(f.b[3]) : "v"(bb) : "memory");
    };
    // all LDS reads issued so far have arrived; ties the fragments to the wait
    auto reads_done = [&](auto ng_tag, Frags &f) __attribute__((always_inline)) {
        constexpr int NG = decltype(ng_tag)::value;
        if constexpr (NG == 4)
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.b[0]), "+v"(f.b[1]), "+v"(f.b[2]), "+v"(f.b[3]));
        else
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.a[0]), "+v"(f.a[1]), "+v"(f.b[0]), "+v"(f.b[1]), "+v"(f.b[2]));
    };
    auto multiply = [&](auto ng_tag, const Frags &f) __attribute__((always_inline)) {
        constexpr int NG = decltype(ng_tag)::value;
#pragma unroll
        for (int m = 0; m < 2 * NG; ++m)
            mfma_step<T>(f.a[m / NG], f.b[m % NG], acc[m / NG][m % NG]);
    };
    // The same with the loads of stage s dealt out between the MFMAs, one after each: a
    // wave issues in order, and a burst of loads in front of the MFMAs would hold them back
    // until the memory pipeline has taken the loads of all waves of the CU.
    // (The condition wraps each load, not the MFMAs: accumulators that meet again after
    // a branch get copied.)
    auto multiply_and_issue = [&](auto ng_tag, const Frags &f, int s, int buf, bool wanted) __attribute__((always_inline)) {
        constexpr int NG = decltype(ng_tag)::value;
#pragma unroll
        for (int m = 0; m < 2 * NG; ++m) {
            mfma_step<T>(f.a[m / NG], f.b[m % NG], acc[m / NG][m % NG]);
            __builtin_amdgcn_sched_barrier(0);
            if (m < NLOAD && wanted) issue_one(s, buf, m);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    const std::integral_constant<int, NG_X> ngx;
    const std::integral_constant<int, NG_H> ngh;

    // One stage.  On entry P holds K group 0 of stage g (buffer cur).  The reads of K group 1
    // go out, K group 0 is multiplied; once those reads are back nobody needs buffer cur any
    // more, and after the barrier (which also publishes stage g+1) it takes the request for
    // stage g+3.  K group 0 of stage g+1 is then read while K group 1 of stage g is multiplied.
    // With two buffers (NBUF == 2) a stage's request follows the barrier that frees its buffer by one stage
    // instead of two: nothing younger is in flight at a barrier, and every wait is for all loads.
    static_assert(NBUF == 2 || NBUF == 3, "two or three stage buffers");
    Frags P, Q;
    int cur = 0;
    auto next_buf = [&]() __attribute__((always_inline)) { return cur == NBUF - 1 ? 0 : cur + 1; };
    auto step = [&](int g, auto ng_cur, auto ng_next, auto wait_tag) __attribute__((always_inline)) {
        constexpr int WAIT = NBUF == 2 ? 0 : decltype(wait_tag)::value;
        read_group(cur, 1, ng_cur, Q);
        __builtin_amdgcn_sched_barrier(0);
        multiply(ng_cur, P);
        __builtin_amdgcn_sched_barrier(0);
        reads_done(ng_cur, Q);
        dma_wait_barrier<WAIT>();
        read_group(next_buf(), 0, ng_next, P);
        __builtin_amdgcn_sched_barrier(0);
        multiply_and_issue(ng_cur, Q, g + NBUF, cur, g + NBUF < n_stages);
        __builtin_amdgcn_sched_barrier(0);
        reads_done(ng_next, P);
        cur = next_buf();
    };
    const std::integral_constant<int, NLOAD> w_more;   // a younger stage stays in flight
    const std::integral_constant<int, 0> w_none;

    // Warm L2 with the block's share of its A tile, one 4-byte load per 128-byte line (the
    // data goes to a sink): the stage loads further down the K loop then find their lines
    // in L2 instead of each waiting for HBM with only two stages of lookahead.  The blocks
    // of one column group of a row tile run side by side on one XCD and split the lines.
    // (A long reduction axis, as in the weight-gradient GEMMs, would ask for far more than L2
    // holds; there the stage loads take their chances.)
    if (MODE != MODE_PROJ && n_stages <= kWarmMaxStages) {
        char *sink_w = sink + wave * 256;
        const int n_lines = n_stages * (kDmaBM * kDmaStage / 128);
        const char *tile = static_cast<const char *>(a.stack) + (int64_t)tile_row0 * kDmaStage;
        const int left = a.n_col_tiles - (col_tile / kColGroup) * kColGroup;
        const int sharers = left < kColGroup ? left : kColGroup;
        for (int li = col_tile % kColGroup + sharers * t; li < n_lines; li += sharers * kDmaThreads) {
            const int slab = li >> 6, line = li & 63;
            __builtin_amdgcn_global_load_lds(JITDB_GLOBAL_PTR(tile + slab * a_stage + line * 128),
                                             JITDB_LDS_PTR(sink_w), 4, 0, 0);
        }
    }
    issue(0, 0);
    issue(1, 1);
    if (NBUF > 2 && n_stages > 2) issue(2, 2);
    after_first_requests();
    if (NBUF > 2 && n_stages > 2) dma_wait_barrier<2 * NLOAD>(); else dma_wait_barrier<NLOAD>();   // stage 0 is there
    int g = 0;
    if constexpr (MODE == MODE_PROJ) {
        read_group(0, 0, ngh, P);
        reads_done(ngh, P);
    } else {
        read_group(0, 0, ngx, P);
        reads_done(ngx, P);
        const int x_end = n_x - 1 < n_stages - 2 ? n_x - 1 : n_stages - 2;
        for (; g < x_end; ++g) step(g, ngx, ngx, w_more);
        if constexpr (MODE == MODE_INTERNAL) {   // n_h >= 2, so this stage is not among the last two
            step(g, ngx, ngh, w_more);
            ++g;
        }
    }
    if constexpr (MODE == MODE_LEAF) {
        step(g, ngx, ngx, w_none);
        read_group(cur, 1, ngx, Q);
        multiply(ngx, P);
        reads_done(ngx, Q);
        multiply(ngx, Q);
    } else {
        for (; g < n_stages - 2; ++g) step(g, ngh, ngh, w_more);
        step(g, ngh, ngh, w_none);
        read_group(cur, 1, ngh, Q);
        multiply(ngh, P);
        reads_done(ngh, Q);
        multiply(ngh, Q);
    }
    __builtin_amdgcn_sched_barrier(0);
    dma_wait_barrier<0>();       // every wave is done reading the stage buffers
}

// The bf16 leaf level's blocks spend more time getting started and in the cell update than in their short K loop
// (K = D only): there a block keeps two stage buffers instead of three and three blocks share a CU instead of
// two (its three gate tiles leave the registers for that).  (fp32 leaves, whose K loop is bound by the fp32
// matrix rate, lose 3 % that way and keep three buffers.)
template <typename T, int MODE> constexpr bool kLeafDense = MODE == MODE_LEAF && sizeof(T) == 2;
template <typename T, int MODE> constexpr int kLevelBufs = kLeafDense<T, MODE> ? 2 : kDmaBufs;
template <typename T, int MODE> constexpr int kLevelBlocksPerCu = kLeafDense<T, MODE> ? 3 : 2;
template <int MODE> constexpr int kEpiArrays = MODE == MODE_LEAF ? 2 : 3;      // i u and o; with children also W_f x + b_f

template <typename T, int MODE, bool SAVE = false, bool GROUPED = false>
__global__ void __launch_bounds__(kDmaThreads, (kLevelBlocksPerCu<T, MODE>))
level_kernel(const LevelArgs a_in) {
    LevelArgs a = a_in;
    constexpr int NBUF = kLevelBufs<T, MODE>;
    __shared__ __attribute__((aligned(1024))) char lds[NBUF * kDmaBuf];
    static_assert(4 * kEpiArrays<MODE> * 32 * kEpiStride * 4 <= NBUF * kDmaBuf, "epilogue regions must fit the stage buffers");
    static_assert(MODE != MODE_PROJ || 4 * 32 * kDmaProjStride * 4 <= NBUF * kDmaBuf, "projection regions must fit the stage buffers");
    __shared__ int row_node[kDmaBM];
    __shared__ int row_ar[kDmaBM];
    __shared__ int row_cb[kDmaBM];
    __shared__ int4 row_kid[kDmaBM];
    __shared__ __attribute__((aligned(256))) char sink[4 * 256];   // where the L2 warm-up loads end up

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    int row_tile, col_tile;
    if (!block_to_tile(blockIdx.x, a.n_row_tiles, a.n_col_tiles, row_tile, col_tile)) return;
    int tile_row0 = row_tile * kDmaBM;
    if constexpr (GROUPED) {     // the tile's slot: where its rows start and end, whose weights apply
        const int4 e = a.tiles[row_tile];
        tile_row0 = __builtin_amdgcn_readfirstlane(e.x);
        a.n_rows = __builtin_amdgcn_readfirstlane(e.y);
        const int sig = __builtin_amdgcn_readfirstlane(e.z);
        a.Bp = static_cast<const char *>(a.Bp) + sig * a.w_bytes;
        a.bp = a.bp + (int64_t)sig * a.NP;
    }

    int node_reg = -1;
    int4 rec0 = make_int4(-1, 0, 0, 0), rec1 = make_int4(-1, -1, -1, -1);
    if (t < kDmaBM && tile_row0 + t < a.n_rows) {
        if constexpr (MODE == MODE_INTERNAL) {
            rec0 = a.row_rec[2 * (int64_t)(tile_row0 + t)];
            rec1 = a.row_rec[2 * (int64_t)(tile_row0 + t) + 1];
        } else {
            node_reg = (MODE == MODE_PROJ && !GROUPED && a.proj_nodes) ? a.proj_nodes[tile_row0 + t]
                                                                     : a.row_rec[2 * (int64_t)(tile_row0 + t)].x;
        }
    }
    auto publish_rows = [&]() __attribute__((always_inline)) {
        if (t < kDmaBM) {
            if constexpr (MODE == MODE_INTERNAL) {
                row_node[t] = rec0.x;
                row_ar[t] = rec0.y;
                row_cb[t] = rec0.z;
                row_kid[t] = rec1;
            } else {
                row_node[t] = node_reg;
            }
        }
    };

    floatx16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][g][v] = 0.0f;

    CellBias bias = {};
    if constexpr (MODE == MODE_PROJ) {
        publish_rows();
        __syncthreads();
        dma_gemm<T, MODE, NBUF>(a, lds, row_node, tile_row0, col_tile, acc, sink, []() {});
    } else {
        bias = load_cell_bias<MODE>(a, col_tile * 2 + wn, lane);     // on its way while the GEMM runs
        dma_gemm<T, MODE, NBUF>(a, lds, row_node, tile_row0, col_tile, acc, sink, publish_rows);
    }

    if constexpr (MODE == MODE_PROJ) {
        // Each wave turns its 64 rows x 128 units around in a private LDS region, 32 rows at
        // a time, so that 16 lanes store one row's 128 units in 8-unit pieces.
        float *region = reinterpret_cast<float *>(lds) + wave * (32 * kDmaProjStride);
#pragma unroll
        for (int p = 0; p < 2; ++p)
            proj_pass<T>(a, acc[p], region, row_node + wm * 64 + p * 32, col_tile * 256 + wn * 128, lane);
    } else {
        float *region = reinterpret_cast<float *>(lds) + wave * (kEpiArrays<MODE> * 32 * kEpiStride);
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int r0 = wm * 64 + p * 32;
            cell_pass<T, MODE, SAVE>(a, acc[p], region, row_node + r0, row_ar + r0, row_cb + r0, row_kid + r0,
                               col_tile * 2 + wn, lane, bias);
        }
    }
}

// ---- the same GEMM core as a plain C = A B^T ------------------------------------------
// For the backward pass: both operands K-blocked, all four column groups multiplied in every
// stage, no cell update.  An output element goes to the epilogue named in the arguments.
// With a split reduction (splits > 1) the grid is one-dimensional and a block's K range
// decides its XCD: blocks are dealt to the eight XCDs round-robin, so block b runs on XCD
// b % 8, takes a split s with s % 8 == b % 8 and one of the output tiles of that split.  All
// tiles of a K range then share one L2, which reads that range of both operands once, and
// every XCD has work however few output tiles there are.
struct KbEpiArgs {
    int kind;
    void *out0; void *out1; const int32_t *node; int D; int H; int ldc;
    int M, N;
    int stages_total, stages_per_split, splits;
};

template <typename T>
__global__ void __launch_bounds__(kDmaThreads, 2)
gemm_kb_kernel(LevelArgs a, const KbEpiArgs e) {
    __shared__ __attribute__((aligned(1024))) char lds[kDmaBufs * kDmaBuf];
    __shared__ __attribute__((aligned(256))) char sink[4 * 256];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int hf = lane >> 5, l32 = lane & 31;
    int row_tile, col_tile, split = 0;
    if (e.splits > 1) {
        const int q = blockIdx.x >> 3, tiles = a.n_row_tiles * a.n_col_tiles;
        split = (blockIdx.x & 7) + 8 * (q / tiles);
        if (split >= e.splits) return;
        row_tile = (q % tiles) / a.n_col_tiles;
        col_tile = (q % tiles) % a.n_col_tiles;
    } else if (!block_to_tile(blockIdx.x, a.n_row_tiles, a.n_col_tiles, row_tile, col_tile)) {
        return;
    }
    const int tile_row0 = row_tile * kDmaBM;
    // this block's range of K stages
    const int s0 = split * e.stages_per_split;
    int n_st = e.stages_total - s0;
    if (n_st > e.stages_per_split) n_st = e.stages_per_split;
    a.stack = static_cast<const char *>(a.stack) + (int64_t)s0 * a.n_rows_alloc * kDmaStage;
    a.Bp = static_cast<const char *>(a.Bp) + (int64_t)s0 * a.NPU * kDmaStage;
    a.Dp = n_st * kDmaStage / (int)sizeof(T);
    a.Hp = 0;

    floatx16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][g][v] = 0.0f;
    // node ids of the tile's rows, fetched while the GEMM runs (the epilogue would otherwise
    // wait for one dependent load per output row)
    __shared__ int s_node[kDmaBM];
    if (e.kind == KB_EPI_DX_DHS && t < kDmaBM) s_node[t] = tile_row0 + t < e.M ? e.node[tile_row0 + t] : 0;
    dma_gemm<T, MODE_GENERIC>(a, lds, nullptr, tile_row0, col_tile, acc, sink, []() {});
    __syncthreads();

    if (e.kind == KB_EPI_ATOMIC_ACC) {
        float *out = static_cast<float *>(e.out0);
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = col_tile * kBN + wn * 128 + g * 32 + l32;
                if (col >= e.N) continue;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = tile_row0 + wm * 64 + i * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
                    if (row < e.M) atomicAdd(&out[(int64_t)row * e.ldc + col], acc[i][g][v]);
                }
            }
        return;
    }
    // Row-wise epilogues: a wave turns its 64 x 128 sub-tile, 32 rows at a time, through a
    // region of the (now free) stage buffers, so that a lane ends up with four consecutive
    // columns of one row and the wave stores whole 512-byte row segments.
    constexpr int kStride = 128 + 4;
    static_assert(4 * 32 * kStride * 4 <= kDmaBufs * kDmaBuf, "epilogue regions must fit the stage buffers");
    float *region = reinterpret_cast<float *>(lds) + wave * (32 * kStride);
    const int c4 = (lane & 31) * 4;
    const int col = col_tile * kBN + wn * 128 + c4;
    const bool vec_ok = (e.kind == KB_EPI_STORE || e.kind == KB_EPI_STORE_F32) ? (e.ldc & 3) == 0
                                                                               : ((e.D & 3) == 0 && (e.H & 3) == 0);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                region[((v >> 2) * 8 + hf * 4 + (v & 3)) * kStride + g * 32 + l32] = acc[i][g][v];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll 4
        for (int sweep = 0; sweep < 16; ++sweep) {
            const int rl = (lane >> 5) + 2 * sweep;
            const int row = tile_row0 + wm * 64 + i * 32 + rl;
            if (row >= e.M || col >= e.N) continue;
            const float4 q = *reinterpret_cast<const float4 *>(region + rl * kStride + c4);
            const float f[4] = {q.x, q.y, q.z, q.w};
            if (e.kind == KB_EPI_STORE_F32) {
                float *dst = static_cast<float *>(e.out0) + (int64_t)row * e.ldc + col;
                if (vec_ok && col + 4 <= e.N) {
                    *reinterpret_cast<float4 *>(dst) = q;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (col + j < e.N) dst[j] = f[j];
                }
            } else if (e.kind == KB_EPI_STORE) {
                T *dst = static_cast<T *>(e.out0) + (int64_t)row * e.ldc + col;
                if (vec_ok && col + 4 <= e.N) {
                    if constexpr (sizeof(T) == 4) {
                        *reinterpret_cast<float4 *>(dst) = q;
                    } else {
                        *reinterpret_cast<uint2 *>(dst) =
                            make_uint2((uint32_t)f32_to_bf16(f[0]) | ((uint32_t)f32_to_bf16(f[1]) << 16),
                                       (uint32_t)f32_to_bf16(f[2]) | ((uint32_t)f32_to_bf16(f[3]) << 16));
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (col + j < e.N) dst[j] = from_f32<T>(f[j]);
                }
            } else {   // KB_EPI_DX_DHS
                const int64_t nd = s_node[row - tile_row0];
                float *dx = static_cast<float *>(e.out0) + nd * e.D;
                T *dhs = static_cast<T *>(e.out1) + nd * e.H;
                if (vec_ok && col + 4 <= e.N) {        // D % 4 == 0: the four columns lie on one side of D
                    if (col < e.D) {
                        *reinterpret_cast<float4 *>(dx + col) = q;
                    } else if constexpr (sizeof(T) == 4) {
                        *reinterpret_cast<float4 *>(dhs + (col - e.D)) = q;
                    } else {
                        *reinterpret_cast<uint2 *>(dhs + (col - e.D)) =
                            make_uint2((uint32_t)f32_to_bf16(f[0]) | ((uint32_t)f32_to_bf16(f[1]) << 16),
                                       (uint32_t)f32_to_bf16(f[2]) | ((uint32_t)f32_to_bf16(f[3]) << 16));
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int cj = col + j;
                        if (cj >= e.N) continue;
                        if (cj < e.D) dx[cj] = f[j];
                        else dhs[cj - e.D] = from_f32<T>(f[j]);
                    }
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

// ---- a slot of N-ary Tree-LSTM nodes: contraction and cell update in one kernel -----------
// The same GEMM core on the slot's stacked rows [x | h_1 | ... | h_N] and the cell's weights packed like
// the child-sum cell's (nary_pack in cells.hip): row = unit tile * 128 + slot * 32 + u with the slots
// i, o, u, f_1, so a block's 256 columns are two unit tiles and every wave holds the four gates of its
// 64 rows x 32 units in its own accumulators.  The forget gates of the further child positions,
// f_2 .. f_N, are a plain GEMM of their own that runs before this kernel (no padding to whole slots that
// way) and leaves its pre-activations in F; the cell update reads them from there.  A slot of leaves
// runs the same kernel over the x part of K (the first slabs of the same packed weights) and uses i, o, u.
// Rows, child ids and arities come with the row records; outputs go out by node id, 32 lanes on 32
// consecutive units of a row, the c values of eight rows' children requested together.
struct NaryEpi {
    const int4 *row_rec; const float *bias; const float *cs; const float *F;
    float *c_out; void *h_out; void *hs_out; float *cs_out;
    int M, H, Hp, Hq, N;
};

template <typename T, bool LEAF>
__global__ void __launch_bounds__(kDmaThreads, 2)
nary_level_kernel(LevelArgs a, const NaryEpi e) {
    __shared__ __attribute__((aligned(1024))) char lds[kDmaBufs * kDmaBuf];
    __shared__ __attribute__((aligned(256))) char sink[4 * 256];
    __shared__ int s_node[kDmaBM];
    __shared__ int s_ar[kDmaBM];
    __shared__ int4 s_kid[kDmaBM];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int hf = lane >> 5, l32 = lane & 31;
    int row_tile, col_tile;
    if (!block_to_tile(blockIdx.x, a.n_row_tiles, a.n_col_tiles, row_tile, col_tile)) return;
    const int tile_row0 = row_tile * kDmaBM;

    floatx16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][g][v] = 0.0f;
    if (t < kDmaBM) {       // the tile's rows, fetched while the GEMM runs
        const int row = tile_row0 + t;
        const bool ok = row < e.M;
        const int4 r0 = e.row_rec[2 * (int64_t)(ok ? row : e.M - 1)];
        s_node[t] = ok ? r0.x : -1;
        if constexpr (!LEAF) {
            s_ar[t] = r0.y < e.N ? r0.y : e.N;
            s_kid[t] = e.row_rec[2 * (int64_t)(ok ? row : e.M - 1) + 1];
        }
    }
    dma_gemm<T, MODE_GENERIC>(a, lds, nullptr, tile_row0, col_tile, acc, sink, []() {});
    __syncthreads();

    const int unit = (col_tile * 2 + wn) * kUnit + l32;
    T *h_out = static_cast<T *>(e.h_out);
    T *hs_out = static_cast<T *>(e.hs_out);
    const bool separate_hs = hs_out != h_out;
    const bool separate_cs = e.cs_out != e.c_out;
    const int H = e.H;
    const bool live = unit < H;
    const int unit_ld = live ? unit : 0;
    const float bi = e.bias[unit_ld], bo = e.bias[H + unit_ld], bu = e.bias[2 * H + unit_ld];
    float bf[4] = {0.f, 0.f, 0.f, 0.f};
    if constexpr (!LEAF) {
#pragma unroll
        for (int l = 0; l < 4; ++l)
            if (l < e.N) bf[l] = e.bias[(3 + l) * H + unit_ld];
    }
    const int ldf = (e.N - 1) * H;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int vh = 0; vh < 2; ++vh) {
            int64_t node[8];
            float ck[8][4], fx[8][3];
            int m[8];
#pragma unroll
            for (int vv = 0; vv < 8; ++vv) {       // what eight rows need from memory first: loads in flight together
                const int v = vh * 8 + vv;
                const int lr = wm * 64 + i * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
                node[vv] = s_node[lr];
                m[vv] = 0;
#pragma unroll
                for (int l = 0; l < 4; ++l) ck[vv][l] = 0.0f;
#pragma unroll
                for (int l = 0; l < 3; ++l) fx[vv][l] = 0.0f;
                if constexpr (!LEAF) {
                    if (node[vv] >= 0) m[vv] = s_ar[lr];
                    const int4 k4 = s_kid[lr];
                    const int kid[4] = {k4.x, k4.y, k4.z, k4.w};
#pragma unroll
                    for (int l = 0; l < 4; ++l)
                        if (l < m[vv]) {
                            ck[vv][l] = e.cs[(int64_t)kid[l] * e.Hq + unit_ld];
                            if (l > 0) fx[vv][l - 1] = e.F[(int64_t)(tile_row0 + lr) * ldf + (l - 1) * H + unit_ld];
                        }
                }
            }
#pragma unroll
            for (int vv = 0; vv < 8; ++vv) {
                const int v = vh * 8 + vv;
                if (node[vv] < 0) continue;
                const int64_t nd = node[vv];
                if (!live) {                        // pad columns of the padded h copy
                    if (separate_hs && unit < e.Hp) hs_out[nd * e.Hp + unit] = T(0);
                    continue;
                }
                const float gi = sigmoid_t<T>(acc[i][0][v] + bi);
                const float go = sigmoid_t<T>(acc[i][1][v] + bo);
                const float gu = tanh_t<T>(acc[i][2][v] + bu);
                float c = gi * gu;
                if constexpr (!LEAF) {
#pragma unroll
                    for (int l = 0; l < 4; ++l)
                        if (l < m[vv]) c += sigmoid_t<T>((l == 0 ? acc[i][3][v] : fx[vv][l > 0 ? l - 1 : 0]) + bf[l]) * ck[vv][l];
                }
                const T hv = from_f32<T>(go * tanh_t<T>(c));
                e.c_out[nd * H + unit] = c;
                if (separate_cs) e.cs_out[nd * e.Hq + unit] = c;
                h_out[nd * H + unit] = hv;
                if (separate_hs) hs_out[nd * e.Hp + unit] = hv;
            }
        }
    }
}

// ---- thin levels ---------------------------------------------------------------------
// A level with a few thousand rows gives the 128 x 256 tiles too few blocks to fill 256
// CUs, and each block then runs a whole K loop back to back: the level costs that
// latency, not its work.  thin_kernel spreads such a level over many more waves.  A block
// of four waves owns one tile of 32 rows x 32 hidden units; wave g multiplies gate g (the
// projection: wave g one of four unit tiles of forget rows), taking its MFMA operands
// straight from global memory / L2 in fragment layout (16 bytes per lane, no LDS staging,
// kThinAhead K groups requested ahead), so the K loop of a tile is a quarter as long as
// with one wave per tile.  The gates meet in LDS and every wave finishes eight of the tile's
// rows (cell_rows).  One block barrier, none in the K loop.
constexpr int kThinWaves = 4;
constexpr int kThinMaxRows = 8192; // levels up to this many rows use the thin kernel
// ... and larger ones too, up to this size, if their nodes average kThinLongLists children or more: the thin
// kernel's cell update walks every row's own child list, the tiled kernel's makes 32 rows wait for the longest
constexpr int kThinMaxRowsLongLists = 16384;
constexpr int kThinLongLists = 5;
constexpr int kThinAhead = 8;      // K groups in flight per wave

template <typename T, int MODE, bool SAVE = false>
__device__ __forceinline__ void thin_body(const LevelArgs &a, int tile) {
    constexpr int ESZ = (int)sizeof(T);
    __shared__ __attribute__((aligned(16))) float smem[4 * 32 * kEpiStride];    // the four gates' pre-activations
    __shared__ int s_node[32];
    __shared__ int s_ar[32];
    __shared__ int s_cb[32];
    __shared__ int4 s_kid[32];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int hf = lane >> 5, l32 = lane & 31;
    const int row0 = (tile / a.n_col_tiles) * 32;
    const int col = tile % a.n_col_tiles;     // unit tile (gates) or group of four unit tiles (projection)
    // (leaves have no forget gate: its wave multiplies nothing, but takes its share of the cell update)
    if (MODE == MODE_PROJ && (col * 4 + wave) * kUnit >= a.Hu) return;            // past the last unit tile

    // ---- the tile's rows
    int my_row = row0 + l32;
    const bool row_ok = my_row < a.n_rows;
    if (!row_ok) my_row = a.n_rows - 1;       // computed twice, stored never
    int my_node;
    if constexpr (MODE == MODE_INTERNAL) {
        const int4 r0 = a.row_rec[2 * (int64_t)my_row];
        my_node = r0.x;
        if (wave == 0 && hf == 0) {
            const int4 r1 = a.row_rec[2 * (int64_t)my_row + 1];
            s_node[l32] = row_ok ? r0.x : -1;
            s_ar[l32] = row_ok ? r0.y : 0;
            s_cb[l32] = r0.z;
            s_kid[l32] = r1;
        }
    } else {
        my_node = a.row_rec[2 * (int64_t)my_row].x;
        if (wave == 0 && hf == 0) s_node[l32] = row_ok ? my_node : -1;
    }

    // ---- operand addresses: lane (l32, hf) supplies row l32, bytes [hf*16, +16) of each
    //      32-byte K group, for A and B alike.  K group g is bytes [32 g, 32 g + 32) of a
    //      row's K: half of slab g/2 in the K-blocked operands.
    const char *ap, *bp;
    int64_t a_pair, b_pair;                   // from K group g to g + 2
    int n_groups;                             // K groups this wave multiplies
    if constexpr (MODE == MODE_PROJ) {
        ap = static_cast<const char *>(a.hs) + (int64_t)my_node * a.Hp * ESZ + hf * 16;
        a_pair = 64;
        const int64_t row = (int64_t)(col * 4 + wave) * kGateTile + 3 * kUnit + l32;
        bp = static_cast<const char *>(a.Bp) + operand_offset(row, (int64_t)a.Dp * ESZ, a.NPU) + hf * 16;
        n_groups = a.Hp * ESZ / 32;
    } else {
        ap = static_cast<const char *>(a.stack) + operand_offset(my_row, 0, a.n_rows_alloc) + hf * 16;
        a_pair = (int64_t)a.n_rows_alloc * 64;
        const int64_t row = (int64_t)col * kGateTile + wave * kUnit + l32;
        bp = static_cast<const char *>(a.Bp) + operand_offset(row, 0, a.NPU) + hf * 16;
        // the forget rows take part in the x part only (U_f applies to each child's own h)
        n_groups = (a.Dp + (MODE == MODE_INTERNAL && wave != 3 ? a.Hp : 0)) * ESZ / 32;
        if (MODE == MODE_LEAF && wave == 3) n_groups = 0;
    }
    b_pair = (int64_t)a.NPU * 64;

    floatx16 acc[1];
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[0][v] = 0.0f;

    u32x4 fa[kThinAhead], fb[kThinAhead];
    auto request = [&](int g, int slot) __attribute__((always_inline)) {
        const int64_t ka = (int64_t)(g >> 1) * a_pair + (g & 1) * 32;
        const int64_t kb = (int64_t)(g >> 1) * b_pair + (g & 1) * 32;
        fa[slot] = *reinterpret_cast<const u32x4 *>(ap + ka);
        fb[slot] = *reinterpret_cast<const u32x4 *>(bp + kb);
    };
#pragma unroll
    for (int s = 0; s < kThinAhead; ++s)
        if (s < n_groups) request(s, s);
    for (int g0 = 0; g0 < n_groups; g0 += kThinAhead) {
#pragma unroll
        for (int s = 0; s < kThinAhead; ++s) {
            const int g = g0 + s;
            if (g < n_groups) {
                mfma_step<T>(fa[s], fb[s], acc[0]);
                if (g + kThinAhead < n_groups) request(g + kThinAhead, s);
            }
        }
    }

    if constexpr (MODE == MODE_PROJ) {
        T *P = static_cast<T *>(a.P);
        const int unit = (col * 4 + wave) * kUnit + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rl = (v >> 2) * 8 + hf * 4 + (v & 3);
            const int node = __shfl(my_node, rl, 64);      // lane rl holds the node of tile row rl (all lanes take part)
            if (unit < a.H && row0 + rl < a.n_rows) P[(int64_t)node * a.Hq + unit] = from_f32<T>(acc[0][v]);
        }
    } else {
        // the gates meet in LDS; every wave finishes eight of the tile's rows
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rl = (v >> 2) * 8 + hf * 4 + (v & 3);
            smem[wave * (32 * kEpiStride) + rl * kEpiStride + l32] = acc[0][v];
        }
        __syncthreads();
        cell_rows<T, MODE, SAVE>(a, smem, s_node, s_ar, s_cb, s_kid, col, wave, lane);
    }
}

template <typename T, int MODE, bool SAVE = false>
__global__ void __launch_bounds__(kThinWaves * 64, 2)
thin_kernel(const LevelArgs a) {
    thin_body<T, MODE, SAVE>(a, blockIdx.x);
}

// The projection of a thin slot and the stack step of the slot after it in one launch: both
// only need what the level kernel before them wrote, and a thin level costs its chain of
// launches, not its work.  Blocks [0, a.n_blocks) are projection tiles, the rest stack blocks.
template <typename T>
__global__ void __launch_bounds__(kThinWaves * 64, 2)
thin_proj_stack_kernel(const LevelArgs a, const StackArgs s) {
    static_assert(kThinWaves * 64 == kThreads, "both bodies use the same block size");
    if ((int)blockIdx.x < a.n_blocks)
        thin_body<T, MODE_PROJ>(a, blockIdx.x);
    else
        stack_body<T, true>(static_cast<const T *>(s.x), s.D, s.Dp, static_cast<const T *>(s.hs), s.Hp, s.row_rec,
                            s.child_idx, static_cast<T *>(s.A), s.n_rows, s.n_rows_alloc,
                            (int64_t)blockIdx.x - a.n_blocks);
}

// ---- chain levels ---------------------------------------------------------------------
// A level in which every node has exactly one child (sequences filed as chains, the long thin
// tail of a forest) needs neither the stack step nor the projection: the child sum is the
// child's h, read in place, and U_f h_k belongs to the same row, so the forget gate is a fourth
// full-K product like i, o and u.  One launch per level instead of two; such a level costs its
// chain of dependent launches and the memory latencies inside them, not its work, so the kernel
// is arranged to meet every latency once:
//
//   * tiles and waves as in thin_kernel (32 rows x 32 units, wave g = gate g);
//   * the four waves need the same A rows [x_j | h_child], so the block fetches the tile's whole
//     A (32 rows x K) once, all loads in flight together, 32 threads per row on consecutive
//     16-byte pieces (zero past D, past K and without a child), into LDS; one barrier;
//   * the K loop then has no barrier: A fragments from LDS (the next one read while this one is
//     multiplied), the wave's own weight rows from global memory / L2, kChainAhead K groups ahead,
//     the first turn requested before anything else in the kernel;
//   * the gates meet in LDS and each of the first four waves finishes eight of the tile's rows;
//   * KS > 1: 4 KS waves, wave w multiplies gate w % 4 over part w / 4 of K.  A level of a few hundred rows leaves
//     most SIMDs idle, and one wave per gate spends the level's time on its own chain of MFMAs (fp32: four
//     64-cycle MFMAs per 32 bytes of K); KS waves per gate cut that chain, and the weight loads and fragment
//     reads in it, KS-fold.  The parts' sums are added in the order of the parts.
//
// Needs D % 4 == 0 (an 8- / 16-byte piece of an x row is inside D or outside) and an A tile that
// fits LDS (chain_lds_bytes) beside the KS sets of pre-activations.
constexpr int kChainAhead = 16;                         // weight K groups in flight per wave
constexpr int kChainLdsTotal = 156 * 1024;              // LDS one block may take in all (static + dynamic)
constexpr int kChainStatic = 1024;                      // static LDS of chain_kernel beside its pre-activations (row ids), rounded up
__host__ __device__ constexpr int chain_zt_bytes(int ks) { return 4 * ks * 32 * kEpiStride * 4; }
// dynamic LDS chain_kernel<T, KS> may ask for
constexpr int chain_lds_max(int ks) { return kChainLdsTotal - kChainStatic - chain_zt_bytes(ks); }
// LDS pitch of an A row: K bytes + 16, so that 16 lanes' 16-byte reads of one K group fall in 64 different banks
__host__ __device__ inline int chain_row_pitch(int k_bytes) { return k_bytes + 16; }
inline size_t chain_lds_bytes(int k_bytes) { return (size_t)32 * chain_row_pitch(k_bytes); }

// Validity of the two halves of a 16-byte piece, K bytes [kb, kb + 16), of a chain row's A operand.
template <typename T>
__device__ __forceinline__ void chain_piece_ok(bool kid_ok, int kb, int x_bytes, int k_bytes, int D, bool &ok0, bool &ok1) {
    constexpr int ESZ = (int)sizeof(T);
    const bool in_x = kb < x_bytes;
    const int k0 = kb / ESZ;
    ok0 = in_x ? (k0 < D) : (kb < k_bytes && kid_ok);
    ok1 = (ESZ == 2 && in_x) ? (k0 + 4 < D) : ok0;       // bf16: the second four elements of the piece
}

template <typename T, int KS>
__global__ void __launch_bounds__(kThinWaves * 64 * KS, KS == 1 ? 2 : 1)
chain_kernel(const LevelArgs a) {
    constexpr int ESZ = (int)sizeof(T);
    extern __shared__ __attribute__((aligned(16))) char a_lds[];          // [32][chain_row_pitch]
    __shared__ __attribute__((aligned(16))) float zt[4 * KS][32 * kEpiStride];  // pre-activations, [part][gate][row][unit]
    __shared__ int s_node[32];
    __shared__ int s_kid[32];
    static_assert(sizeof(zt) == chain_zt_bytes(KS) && 2 * 32 * 4 <= kChainStatic, "chain_lds_max counts these");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int gate = wave & 3, part = wave >> 2;
    const int hf = lane >> 5, l32 = lane & 31;
    const int tile = blockIdx.x;
    const int row0 = (tile / a.n_col_tiles) * 32;
    const int col = tile % a.n_col_tiles;     // unit tile

    // ---- weights: lane (l32, hf) supplies row l32 of the wave's gate, bytes [hf*16, +16) of each 32-byte K
    //      group.  Every load of the ring is unconditional (a group index past the end is clamped to the
    //      last group, whose data is then not used): the number of loads between a request and its use is
    //      the same on every path, so the waits the compiler places are counted, not "all".
    const int x_bytes = a.Dp * ESZ;                      // K bytes of the x part
    const int k_bytes = x_bytes + a.Hp * ESZ;
    const int pitch = chain_row_pitch(k_bytes);
    const int n_all = k_bytes / 32;                      // K groups of a row (a multiple of four)
    // this wave's part of them, [g_begin, g_begin + n_groups): whole slabs (pairs of groups)
    const int per_part = ((n_all + KS - 1) / KS + 1) & ~1;
    const int g_begin = part * per_part < n_all ? part * per_part : n_all;
    const int n_groups = n_all - g_begin < per_part ? n_all - g_begin : per_part;
    const int last_group = n_groups > 0 ? g_begin + n_groups - 1 : n_all - 1;   // (a part without groups loads the row's last one, unused)
    const int64_t brow = (int64_t)col * kGateTile + gate * kUnit + l32;
    const char *bp = static_cast<const char *>(a.Bp) + operand_offset(brow, 0, a.NPU) + hf * 16;
    const int64_t b_pair = (int64_t)a.NPU * 64;
    u32x4 fb[kChainAhead];
    auto request = [&](int g, int slot) __attribute__((always_inline)) {
        fb[slot] = *reinterpret_cast<const u32x4 *>(bp + (int64_t)(g >> 1) * b_pair + (g & 1) * 32);
    };
#pragma unroll
    for (int s = 0; s < kChainAhead; ++s) request(g_begin + s < last_group ? g_begin + s : last_group, s);
    __builtin_amdgcn_sched_barrier(0);

    // ---- the tile's A: thread t moves pieces (t & 31) + 32 i of rows (t >> 5) + RPP j
    {
        constexpr int RPP = 8 * KS;           // rows per pass of the block's threads
        constexpr int NJ = 32 / RPP;
        const char *src_x[NJ], *src_h[NJ];
        bool kid_ok[NJ];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
            const int rl = (tid >> 5) + RPP * j;
            int r = row0 + rl;
            const bool ok = r < a.n_rows;
            if (!ok) r = a.n_rows - 1;                // computed twice, stored never
            const int4 r0 = a.row_rec[2 * (int64_t)r];
            const int4 r1 = a.row_rec[2 * (int64_t)r + 1];
            kid_ok[j] = r0.y >= 1;                    // always, in a level this kernel is launched for
            src_x[j] = static_cast<const char *>(a.x) + (int64_t)r0.x * a.D * ESZ;
            src_h[j] = static_cast<const char *>(a.hs) + (int64_t)(kid_ok[j] ? r1.x : 0) * a.Hp * ESZ;
            if ((tid & 31) == 0) {                    // the rows as the cell update wants them
                s_node[rl] = ok ? r0.x : -1;
                s_kid[rl] = (ok && kid_ok[j]) ? r1.x : -1;
            }
        }
        const int n_rounds = (k_bytes / 16 + 31) / 32;
#pragma unroll 4
        for (int i = 0; i < n_rounds; ++i) {
            const int kb = ((tid & 31) + 32 * i) * 16;
            if (kb >= k_bytes) break;
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                bool ok0, ok1;
                chain_piece_ok<T>(kid_ok[j], kb, x_bytes, k_bytes, a.D, ok0, ok1);
                // a piece that is not to be read comes from the start of the x row (always valid: D >= 4)
                // and is replaced by zero
                const char *p = kb < x_bytes ? src_x[j] + kb : src_h[j] + (kb - x_bytes);
                u32x4 v;
                if constexpr (ESZ == 4) {
                    v = *reinterpret_cast<const u32x4 *>(ok0 ? p : src_x[j]);
                } else {
                    const u32x2 q0 = *reinterpret_cast<const u32x2 *>(ok0 ? p : src_x[j]);
                    const u32x2 q1 = *reinterpret_cast<const u32x2 *>(ok1 ? p + 8 : src_x[j]);
                    v[0] = q0[0]; v[1] = q0[1]; v[2] = q1[0]; v[3] = q1[1];
                }
                v[0] = ok0 ? v[0] : 0u; v[1] = ok0 ? v[1] : 0u; v[2] = ok1 ? v[2] : 0u; v[3] = ok1 ? v[3] : 0u;
                *reinterpret_cast<u32x4 *>(a_lds + ((tid >> 5) + RPP * j) * pitch + kb) = v;
            }
        }
    }
    floatx16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
    __syncthreads();

    // ---- K loop: whole turns of the ring, then the rest (a multiple of 4 groups)
    const char *abuf = a_lds + l32 * pitch + hf * 16;    // this lane's A fragment, K group 0
    const int n_full = n_groups / kChainAhead;
    const int g_end = g_begin + n_groups;
    u32x4 fa = *reinterpret_cast<const u32x4 *>(abuf + (g_begin < n_all ? g_begin : n_all - 1) * 32);
    for (int c = 0; c < n_full; ++c) {
        const int g0 = g_begin + c * kChainAhead;
#pragma unroll
        for (int s = 0; s < kChainAhead; ++s) {
            // the next A fragment leaves LDS while this one is multiplied
            const int gnext = g0 + s + 1 < g_end ? g0 + s + 1 : last_group;
            const u32x4 fa_next = *reinterpret_cast<const u32x4 *>(abuf + gnext * 32);
            mfma_step<T>(fa, fb[s], acc);
            const int gn = g0 + s + kChainAhead;
            request(gn < last_group ? gn : last_group, s);
            __builtin_amdgcn_sched_barrier(0);      // the ring is refilled slot by slot, not in a burst at the end
            fa = fa_next;
        }
    }
    {
        const int g0 = g_begin + n_full * kChainAhead;
        const int tail = g_end - g0;
#pragma unroll
        for (int s = 0; s < kChainAhead; ++s)
            if (s < tail) {
                const int gnext = g0 + s + 1 < g_end ? g0 + s + 1 : last_group;
                const u32x4 fa_next = *reinterpret_cast<const u32x4 *>(abuf + gnext * 32);
                mfma_step<T>(fa, fb[s], acc);
                fa = fa_next;
            }
    }

    // ---- the gates meet in LDS; wave w < 4 finishes rows 8 w .. 8 w + 7: eight lanes per row, four units per lane
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int rl = (v >> 2) * 8 + hf * 4 + (v & 3);
        zt[wave][rl * kEpiStride + l32] = acc[v];
    }
    __syncthreads();
    if (wave >= 4) return;
    const int tr = wave * 8 + (lane >> 3);
    const int node = s_node[tr];
    if (node < 0) return;
    const int u4 = (lane & 7) * 4;
    const int unit0 = col * kUnit + u4;
    const int kid = s_kid[tr];
    const int unit_ld = unit0 < a.Hq ? unit0 : 0;        // unit groups past the padded width read the first group (and store nothing)
    float4 ck = make_float4(0.f, 0.f, 0.f, 0.f);
    if (kid >= 0) ck = *reinterpret_cast<const float4 *>(a.cs + (int64_t)kid * a.Hq + unit_ld);
    const float *bias = a.bp + col * kGateTile + u4;
    float z[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        float4 q = *reinterpret_cast<const float4 *>(&zt[g][tr * kEpiStride + u4]);
#pragma unroll
        for (int p = 1; p < KS; ++p) {
            const float4 qp = *reinterpret_cast<const float4 *>(&zt[4 * p + g][tr * kEpiStride + u4]);
            q.x += qp.x; q.y += qp.y; q.z += qp.z; q.w += qp.w;
        }
        const float4 bq = *reinterpret_cast<const float4 *>(bias + g * kUnit);
        z[g][0] = q.x + bq.x; z[g][1] = q.y + bq.y; z[g][2] = q.z + bq.z; z[g][3] = q.w + bq.w;
    }
    const float ckv[4] = {ck.x, ck.y, ck.z, ck.w};
    float cc[4], go[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float gi = sigmoid_t<T>(z[0][e]);
        go[e] = sigmoid_t<T>(z[1][e]);
        const float gu = tanh_t<T>(z[2][e]);
        const float gf = sigmoid_t<T>(z[3][e]);
        cc[e] = gi * gu + gf * ckv[e];
    }
    store_state<T>(a, node, unit0, make_float4(cc[0], cc[1], cc[2], cc[3]), make_float4(go[0], go[1], go[2], go[3]));
}

// ---- tile tables of a typed level --------------------------------------------------------
// One block.  bounds[e * stride] .. bounds[(e + 1) * stride], e < n_entries, are consecutive
// ranges of positions (the level's slots with stride = n_sig, its sub-slots with stride = 1);
// range e uses weight set e % n_sig when stride == 1 (a sub-slot is named by the parent's
// signature last), else e.  Entry i of the table describes the i-th 128-row tile when every
// range is cut into tiles of its own: (first row, end row of its range, weight set), rows
// relative to the level.
constexpr int kMaxTableEntries = JITDB_MAX_SIGNATURES * JITDB_MAX_SIGNATURES;
__global__ void __launch_bounds__(kThreads)
tile_table_kernel(const int32_t *__restrict__ bounds, int n_entries, int stride, int n_sig, int4 *__restrict__ tiles) {
    __shared__ int s_first[kMaxTableEntries + 1];      // tiles before entry e
    __shared__ int s_part[kThreads];
    // tiles per entry, then an exclusive scan: every thread owns a contiguous run of entries
    const int per = (n_entries + kThreads - 1) / kThreads;
    const int e0 = threadIdx.x * per, e1 = min(e0 + per, n_entries);
    int sum = 0;
    for (int e = e0; e < e1; ++e) {
        const int c = (bounds[(e + 1) * stride] - bounds[e * stride] + kDmaBM - 1) / kDmaBM;
        s_first[e] = sum;
        sum += c;
    }
    s_part[threadIdx.x] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int t = 0; t < kThreads; ++t) { const int v = s_part[t]; s_part[t] = run; run += v; }
        s_first[n_entries] = run;
    }
    __syncthreads();
    for (int e = e0; e < e1; ++e) s_first[e] += s_part[threadIdx.x];
    __syncthreads();
    const int base = bounds[0];
    for (int e = 0; e < n_entries; ++e) {
        const int n_t = s_first[e + 1] - s_first[e];
        if (n_t == 0) continue;
        const int lo = bounds[e * stride] - base, hi = bounds[(e + 1) * stride] - base;
        const int wset = stride == 1 ? e % n_sig : e;
        for (int j = threadIdx.x; j < n_t; j += kThreads)
            tiles[s_first[e] + j] = make_int4(lo + j * kDmaBM, hi, wset, 0);
    }
}

// ---- host side ---------------------------------------------------------------------
// Optional per-launch event pairs (see jitdb_profile_start in the header).
struct Profiler {
    bool on = false;
    int capacity = 0, used = 0;
    int64_t dropped = 0;
    hipEvent_t *begin = nullptr, *end = nullptr;
    int *cls = nullptr;
    int64_t *rows = nullptr;
    int64_t *edges = nullptr;
};
Profiler g_prof;

struct ScopedLaunchTimer {
    int slot = -1;
    hipStream_t st;
    // edges: children whose forget gates the launch computes in full (chain levels); else 0
    ScopedLaunchTimer(int kernel_class, int64_t rows, hipStream_t s, int64_t edges = 0) : st(s) {
        if (!g_prof.on) return;
        if (g_prof.used >= g_prof.capacity) { ++g_prof.dropped; return; }
        slot = g_prof.used++;
        g_prof.cls[slot] = kernel_class;
        g_prof.rows[slot] = rows;
        g_prof.edges[slot] = edges;
        (void)hipEventRecord(g_prof.begin[slot], st);
    }
    ~ScopedLaunchTimer() {
        if (slot >= 0) (void)hipEventRecord(g_prof.end[slot], st);
    }
};

struct ForwardWs {
    void *Bp;
    float *bp;
    void *Bf;     // fragment-major copy of the packed weights (bf16 with one cell), else nullptr
    void *stack;  // the current level's stacked input, (N + 256) rows of Dp + Hp
    int4 *row_rec; // row records of all level positions, two int4 each
    void *hs;     // nullptr when h_out can serve (H == Hp)
    void *P;
    float *cs;    // nullptr when c_out can serve (H == Hq)
    int4 *tiles;  // tile tables of one typed level: cell batches, then projection batches (nullptr with one cell)
    int64_t tiles_each;
    // tables that hold N-ary cells (jitdb_treelstm_forward_cells): one slot's stacked input and
    // pre-activations, each such cell's packed weights, the flag for nodes with too many children
    void *nary_A;
    float *nary_F;   // pre-activations of the forget gates of child positions 2 .. N of one slot
    void *nary_B[JITDB_MAX_SIGNATURES];
    int *nary_err;
    size_t bytes;
};

struct Dims {
    int D, H, Dp, Hp, Hu, NP;
    int Hq;       // H rounded up to 8: row stride of the side buffers (P, padded c)
    int NPU;      // rows of the packed U: padded so the projection's 8-unit-tile blocks stay inside
    size_t esz;
};

Dims make_dims(int D, int H, jitdb_dtype dtype) {
    Dims d;
    d.D = D; d.H = H;
    // K is padded to whole pipeline stages, so that only the last x stage can straddle D
    const int kpad = dtype == JITDB_F32 ? Traits<float>::BK : Traits<bf16_t>::BK;
    d.Dp = (int)round_up(D, kpad);
    d.Hp = (int)round_up(H, kpad);
    d.Hu = (int)round_up(H, 2 * kUnit);
    d.NP = 4 * d.Hu;
    d.Hq = (int)round_up(H, 8);
    d.NPU = (int)round_up(d.Hu / kUnit, 8) * kGateTile;
    d.esz = dtype == JITDB_F32 ? 4 : 2;
    return d;
}

// packed weights of one cell: bytes of Bp, floats of bp (one set per signature, back to back)
size_t packed_w_bytes(const Dims &d) { return (size_t)d.NPU * (d.Dp + d.Hp) * d.esz; }
// the 256 x 256 tile kernel (bf16, one cell) reads the weights in a second, fragment-major layout
bool has_fragment_copy(const Dims &d, int n_sig) { return d.esz == 2 && n_sig == 1; }

ForwardWs carve_forward_ws(int64_t n, int64_t e, const Dims &d, void *base, int n_sig = 1,
                           const jitdb_cell_t *cells = nullptr) {
    Carver c(base);
    ForwardWs w = {};
    (void)e;
    w.Bp = c.take<char>(packed_w_bytes(d) * n_sig);
    w.bp = c.take<float>((size_t)d.NP * n_sig);
    w.Bf = has_fragment_copy(d, n_sig) ? c.take<char>(packed_w_bytes(d)) : nullptr;
    // one level at a time; whole row tiles are read, hence the 256 spare rows
    w.stack = c.take<char>((size_t)(n + kRowPad) * (d.Dp + d.Hp) * d.esz);
    w.row_rec = c.take<int4>((size_t)2 * (n + kRowPad));   // every level position
    w.hs = (d.H == d.Hp) ? nullptr : c.take<char>((size_t)n * d.Hp * d.esz);
    w.P = c.take<char>((size_t)n * d.Hq * d.esz);
    w.cs = (d.H == d.Hq) ? nullptr : c.take<float>((size_t)n * d.Hq);
    w.tiles_each = n / kDmaBM + (int64_t)n_sig * n_sig + 1;
    w.tiles = n_sig > 1 ? c.take<int4>((size_t)(2 * w.tiles_each)) : nullptr;
    int n_max = 0;
    for (int t = 0; cells && t < n_sig; ++t)
        if (cells[t].kind == JITDB_CELL_NARY) {
            n_max = cells[t].arity > n_max ? cells[t].arity : n_max;
            w.nary_B[t] = c.take<char>(nary_packed_bytes(d.D, d.H, d.Dp, d.Hp, cells[t].arity, d.esz));
        }
    if (n_max > 0) {
        w.nary_A = c.take<char>((size_t)(n + kRowPad) * (d.Dp + (size_t)n_max * d.Hp) * d.esz);
        w.nary_F = n_max > 1 ? c.take<float>((size_t)n * (n_max - 1) * d.H) : nullptr;
        w.nary_err = c.take<int>(1);
    }
    w.bytes = c.off;
    return w;
}

bool dims_ok(int64_t n, int64_t e, int32_t D, int32_t H, int dtype) {
    if (n < 0 || n > JITDB_MAX_NODES || e < 0 || e > n) return false;
    if (D < 1 || D > (1 << 16)) return false;
    if (H < 1 || H > (1 << 14)) return false;
    if (dtype != JITDB_F32 && dtype != JITDB_BF16) return false;
    return true;
}

// One batched evaluation per slot of the table, levels in ascending order.  Without `slots` a
// level is one slot and there is one cell; with it, slot (l, t) is evaluated by cell t (its
// own packed weights), and the records keep every row inside its slot.
// With `cells` (one per signature) every signature names a cell of its own TYPE: child-sum cells
// take the path of this file, N-ary cells the three steps of cells.hip; W, U, b then come from the
// cells.
template <typename T, bool SAVE>
int run_forward(const void *x, const void *W, const void *U, const float *b, const Dims &d,
                const jitdb_schedule_t *s, const jitdb_slots_t *slots, const jitdb_cell_t *cells,
                void *h_out, float *c_out, void *gates, void *fgate,
                const ForwardWs &w_in, const void *packed, hipStream_t st) {
    // weights packed by an earlier jitdb_treelstm_pack are used where they lie
    ForwardWs w = w_in;
    const int n_sig_w = slots ? slots->n_sig : 1;
    if (packed) {
        w.Bp = const_cast<void *>(packed);
        w.bp = reinterpret_cast<float *>(static_cast<char *>(w.Bp) + round_up(packed_w_bytes(d) * n_sig_w, 256));
        w.Bf = has_fragment_copy(d, n_sig_w)
                   ? reinterpret_cast<char *>(w.bp) + round_up((int64_t)d.NP * n_sig_w * 4, 256) : nullptr;
    }
    const int L = s->n_levels;
    const int n_sig = slots ? slots->n_sig : 1;
    const int32_t *sp = slots ? slots->host_slot_ptr : s->host_level_ptr;
    const jitdb_dtype dtype = std::is_same<T, float>::value ? JITDB_F32 : JITDB_BF16;
    auto is_nary = [&](int t) { return cells != nullptr && t >= 0 && cells[t].kind == JITDB_CELL_NARY; };
    bool any_nary = false;
    for (int t = 0; t < n_sig; ++t) any_nary = any_nary || is_nary(t);

    {   // row records and packed weights (one launch; further cells' weights one launch each)
        const int64_t total = (int64_t)d.NPU * (d.Dp + d.Hp);
        const unsigned pack_grid = (unsigned)(ceil_div(total, kThreads) < 4096 ? ceil_div(total, kThreads) : 4096);
        auto pack_args = [&](int t) {
            PackArgs p;
            if (cells) {
                p.W = cells[t].W; p.U = cells[t].U; p.b = cells[t].b;
            } else {
                p.W = static_cast<const T *>(W) + (size_t)t * 4 * d.H * d.D;
                p.U = static_cast<const T *>(U) + (size_t)t * 4 * d.H * d.H;
                p.b = b + (size_t)t * 4 * d.H;
            }
            p.D = d.D; p.H = d.H; p.Dp = d.Dp; p.Hp = d.Hp; p.NP = d.NP; p.NPU = d.NPU;
            p.Bp = static_cast<char *>(w.Bp) + packed_w_bytes(d) * t;
            p.bp = w.bp + (size_t)d.NP * t;
            p.Bf = t == 0 ? w.Bf : nullptr;
            return p;
        };
        const bool large = s->n_nodes >= kRecLargeMinNodes;
        {
            ScopedLaunchTimer tm(JITDB_K_PACK, 0, st);
            const bool pack_here = !(packed || is_nary(0));
            if (large) {
                const int n_windows = (int)ceil_div(s->n_nodes, kRecWindowLarge);
                const unsigned pg = pack_here ? (unsigned)(ceil_div(total, kRecThreadsLarge) < 1024 ? ceil_div(total, kRecThreadsLarge) : 1024) : 0u;
                prepare_large_kernel<T><<<(unsigned)n_windows + pg, kRecThreadsLarge, 0, st>>>(
                    s->perm, slots ? slots->key : s->height, s->child_ptr, s->child_idx, w.row_rec, (int)s->n_nodes,
                    n_windows, pack_args(0));
            } else {
                const int n_windows = (int)ceil_div(s->n_nodes, kRecWindow);
                prepare_kernel<T><<<(unsigned)n_windows + (pack_here ? pack_grid : 0u), kThreads, 0, st>>>(
                    s->perm, slots ? slots->key : s->height, s->child_ptr, s->child_idx, w.row_rec, (int)s->n_nodes,
                    n_windows, pack_args(0));
            }
            JITDB_LAUNCH_CHECK();
        }
        for (int t = 1; t < n_sig && !packed; ++t) {
            if (is_nary(t)) continue;
            ScopedLaunchTimer tm(JITDB_K_PACK, 0, st);
            pack_weights_kernel<T><<<pack_grid, kThreads, 0, st>>>(pack_args(t));
            JITDB_LAUNCH_CHECK();
        }
        for (int t = 0; t < n_sig; ++t) {
            if (!is_nary(t)) continue;
            ScopedLaunchTimer tm(JITDB_K_PACK, 0, st);
            // (every such launch also clears the flag for nodes with too many children)
            const int rc = nary_pack(dtype, cells[t].W, cells[t].U, d.D, d.H, d.Dp, d.Hp, cells[t].arity, w.nary_B[t],
                                     w.nary_err, st);
            if (rc != JITDB_OK) return rc;
        }
    }

    LevelArgs a;
    a.proj_nodes = nullptr;
    a.stack = w.stack;
    a.Bf = w.Bf;
    // bf16 levels that are large enough run on 256 x 256 tiles (level256.hip); training and typed
    // tables keep the 128 x 256 kernel, which has those variants
    const bool may256 = std::is_same<T, bf16_t>::value && !SAVE && !slots && w.Bf != nullptr;
    a.hs = w.hs ? w.hs : h_out;
    a.x = x;
    a.child_idx = s->child_idx;

    a.P = w.P; a.c_out = c_out; a.h_out = h_out;
    a.cs = w.cs ? w.cs : c_out;
    a.Hq = d.Hq;
    a.hs_out = w.hs ? w.hs : h_out;
    a.gates = gates;
    a.fgate = fgate;
    a.D = d.D; a.Dp = d.Dp; a.H = d.H; a.Hp = d.Hp; a.Hu = d.Hu;
    a.NPU = d.NPU;

    // The table's ranges: slot (l, t) = the cell's batch = sub-slots (l, t, 0 .. n_sig-1); the
    // projection of sub-slot (l, t, p) uses the forget weights of cell p, the parent's.
    const int T2 = n_sig * n_sig;
    auto slot_begin = [&](int l, int t) { return sp[(l * n_sig + t) * (slots ? n_sig : 1)]; };
    auto sub_begin = [&](int l, int t, int p) { return sp[(l * n_sig + t) * n_sig + p]; };
    // The launches in order: one per non-empty slot, except that a level of a typed table that
    // is large enough for the tiled kernel runs all its slots in one grouped launch (sig = -1;
    // n_tiles / n_proj_tiles = 128-row tiles when every slot / sub-slot is cut into tiles of its own).
    struct Seg { int l, sig, begin, rows, n_tiles, n_proj_tiles; };
    std::vector<Seg> segs;
    segs.reserve((size_t)L * n_sig);
    for (int l = 0; l < L; ++l) {
        const int lvl_rows = slot_begin(l + 1, 0) - slot_begin(l, 0);
        int n_tiles = 0, n_proj_tiles = 0, used = 0;
        for (int t = 0; t < n_sig; ++t) {
            const int r = slot_begin(l, t + 1) - slot_begin(l, t);
            if (r < 0 || (r == 0 && !slots)) return JITDB_E_SCHEDULE;
            n_tiles += (int)ceil_div(r, kDmaBM);
            used += r > 0;
            if (slots)
                for (int p = 0; p < n_sig; ++p)
                    n_proj_tiles += (int)ceil_div(sub_begin(l, t, p + 1) - sub_begin(l, t, p), kDmaBM);
        }
        if (used > 1 && lvl_rows > kThinMaxRows && !any_nary) {
            segs.push_back({l, -1, slot_begin(l, 0), lvl_rows, n_tiles, n_proj_tiles});
        } else {
            for (int t = 0; t < n_sig; ++t) {
                const int r = slot_begin(l, t + 1) - slot_begin(l, t);
                if (r > 0) segs.push_back({l, t, slot_begin(l, t), r, 0, 0});
            }
        }
    }
    // stack: gather a slot's x rows and child sums into one dense matrix
    auto stack_args = [&](const Seg &g) {
        StackArgs sa;
        sa.x = x; sa.D = d.D; sa.Dp = d.Dp; sa.hs = a.hs; sa.Hp = d.Hp;
        sa.row_rec = w.row_rec + 2 * (int64_t)g.begin; sa.child_idx = s->child_idx;
        sa.A = w.stack; sa.n_rows = g.rows; sa.n_rows_alloc = (int)round_up(g.rows, kRowPad);
        return sa;
    };
    auto stack_blocks = [&](const Seg &g) {
        const int Kp = d.Dp + (g.l > 0 ? d.Hp : 0);
        return (unsigned)ceil_div((int64_t)g.rows * (Kp / Traits<T>::VEC), kThreads);
    };
    bool stacked_ahead = false;     // the slot's stack step already ran with the projection before it
    // Levels from chain_from on are thin and hold only nodes with exactly one child (the schedule says
    // how many children each level has): one launch each, no stack step, no projection.  A child
    // below chain_from whose parent is such a node needs no projection either, so the level right
    // below skips it too.
    int chain_from = L;
    const int chain_k_bytes = (d.Dp + d.Hp) * d.esz;
    const size_t chain_lds = chain_lds_bytes(chain_k_bytes);      // the tile's A rows live in LDS
    // waves per gate: fp32 (long MFMA chains) two if the LDS beside the A tile allows, bf16 one.  (Four measured
    // slower than two: blocks of 1024 threads start later than they finish earlier.)
    const int chain_ks = (sizeof(T) == 4 && chain_lds <= (size_t)chain_lds_max(2)) ? 2 : 1;
    if (!SAVE && !slots && s->host_level_kids && (d.D & 3) == 0 && chain_lds <= (size_t)chain_lds_max(chain_ks)) {
        for (int l = L - 1; l >= 1; --l) {
            const int rows = sp[l + 1] - sp[l];
            if (rows > kThinMaxRows || s->host_level_kids[l] != rows) break;
            chain_from = l;
        }
    }
    if (chain_from < L) {    // more dynamic LDS than a launch may ask for by default
        const void *fn = chain_ks == 2 ? reinterpret_cast<const void *>(&chain_kernel<T, 2>)
                                       : reinterpret_cast<const void *>(&chain_kernel<T, 1>);
        JITDB_HIP_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, chain_lds_max(chain_ks)));
    }
    const int n_unit_tiles = d.Hu / kUnit;
    a.w_bytes = (int64_t)packed_w_bytes(d);
    a.NP = d.NP;

    for (size_t i = 0; i < segs.size(); ++i) {
        const int l = segs[i].l, sig = segs[i].sig, n_rows = segs[i].rows;
        const bool grouped = sig < 0;
        a.Bp = static_cast<char *>(w.Bp) + packed_w_bytes(d) * (grouped ? 0 : sig);
        a.bp = w.bp + (size_t)d.NP * (grouped ? 0 : sig);
        a.row_rec = w.row_rec + 2 * (int64_t)segs[i].begin;
        a.n_rows = n_rows;
        a.n_rows_alloc = (int)round_up(n_rows, kRowPad);
        a.tiles = nullptr;
        const int row_tiles = grouped ? segs[i].n_tiles : (int)ceil_div(n_rows, kDmaBM);
        if (grouped) {      // both tile tables of the level: cell batches, projection batches
            const int32_t *lvl = slots->slot_ptr + (int64_t)l * T2;
            tile_table_kernel<<<1, kThreads, 0, st>>>(lvl, n_sig, n_sig, n_sig, w.tiles);
            JITDB_LAUNCH_CHECK();
            tile_table_kernel<<<1, kThreads, 0, st>>>(lvl, T2, 1, n_sig, w.tiles + w.tiles_each);
            JITDB_LAUNCH_CHECK();
            a.tiles = w.tiles;
        }
        if (l >= chain_from) {
            a.n_col_tiles = n_unit_tiles;
            a.n_tiles = (int)ceil_div(n_rows, 32) * a.n_col_tiles;
            a.n_blocks = a.n_tiles;
            ScopedLaunchTimer tm(JITDB_K_CHAIN, n_rows, st, s->host_level_kids[l]);
            if (chain_ks == 2) chain_kernel<T, 2><<<a.n_blocks, kThinWaves * 64 * 2, chain_lds, st>>>(a);
            else chain_kernel<T, 1><<<a.n_blocks, kThinWaves * 64, chain_lds, st>>>(a);
            JITDB_LAUNCH_CHECK();
            continue;
        }
        if (is_nary(sig)) {
            // a slot of N-ary nodes: stack, one contraction for all 3 + N gates, cell update (cells.hip)
            NarySlot ns;
            ns.x = x; ns.row_rec = a.row_rec; ns.A = w.nary_A; ns.Bn = w.nary_B[sig]; ns.b = cells[sig].b;
            ns.F = w.nary_F; ns.err = w.nary_err; ns.n_rows = n_rows; ns.N = cells[sig].arity; ns.leaves = l == 0;
            ScopedLaunchTimer tm(l == 0 ? JITDB_K_THIN_LEAF : JITDB_K_THIN_INTERNAL, n_rows, st);
            const int rc = run_nary_slot(dtype, a, ns, st);
            if (rc != JITDB_OK) return rc;
        } else {
            if (!stacked_ahead) {
                const StackArgs sa = stack_args(segs[i]);
                ScopedLaunchTimer tm(JITDB_K_STACK, n_rows, st);
                if (l == 0)
                    stack_kernel<T, false><<<stack_blocks(segs[i]), kThreads, 0, st>>>(
                        static_cast<const T *>(sa.x), sa.D, sa.Dp, static_cast<const T *>(sa.hs), sa.Hp, sa.row_rec,
                        sa.child_idx, static_cast<T *>(sa.A), sa.n_rows, sa.n_rows_alloc);
                else
                    stack_kernel<T, true><<<stack_blocks(segs[i]), kThreads, 0, st>>>(
                        static_cast<const T *>(sa.x), sa.D, sa.Dp, static_cast<const T *>(sa.hs), sa.Hp, sa.row_rec,
                        sa.child_idx, static_cast<T *>(sa.A), sa.n_rows, sa.n_rows_alloc);
                JITDB_LAUNCH_CHECK();
            }
            stacked_ahead = false;
            // Levels too small to give every CU a 256 x 256 tile go to the thin kernel.
            bool thin = n_rows <= kThinMaxRows;
            if (!thin && !SAVE && !slots && l > 0 && s->host_level_kids && n_rows <= kThinMaxRowsLongLists &&
                s->host_level_kids[l] >= (int64_t)kThinLongLists * n_rows)
                thin = true;
            if (thin) {
                a.n_col_tiles = n_unit_tiles;
                a.n_tiles = (int)ceil_div(n_rows, 32) * a.n_col_tiles;
                a.n_blocks = a.n_tiles;
            } else {
                a.n_col_tiles = d.NP / kBN;
                a.n_tiles = 0;
                a.n_row_tiles = row_tiles;
                a.n_blocks = 8 * (int)ceil_div(row_tiles, 8) * a.n_col_tiles;
            }
            {
                ScopedLaunchTimer tm(thin ? (l == 0 ? JITDB_K_THIN_LEAF : JITDB_K_THIN_INTERNAL)
                                          : (l == 0 ? JITDB_K_LEAF : JITDB_K_INTERNAL), n_rows, st);
                if (thin) {
                    if (l == 0)
                        thin_kernel<T, MODE_LEAF, SAVE><<<a.n_blocks, kThinWaves * 64, 0, st>>>(a);
                    else
                        thin_kernel<T, MODE_INTERNAL, SAVE><<<a.n_blocks, kThinWaves * 64, 0, st>>>(a);
                } else if (may256 && tile256_applies(l == 0 ? MODE_LEAF : MODE_INTERNAL, a)) {
                    const int rc = launch_tile256(l == 0 ? MODE_LEAF : MODE_INTERNAL, a, st);
                    if (rc != JITDB_OK) return rc;
                } else if (grouped) {
                    if (l == 0)
                        level_kernel<T, MODE_LEAF, false, true><<<a.n_blocks, kDmaThreads, 0, st>>>(a);
                    else
                        level_kernel<T, MODE_INTERNAL, false, true><<<a.n_blocks, kDmaThreads, 0, st>>>(a);
                } else {
                    if (l == 0)
                        level_kernel<T, MODE_LEAF, SAVE><<<a.n_blocks, kDmaThreads, 0, st>>>(a);
                    else
                        level_kernel<T, MODE_INTERNAL, SAVE><<<a.n_blocks, kDmaThreads, 0, st>>>(a);
                }
            }
            JITDB_LAUNCH_CHECK();
        }
        if (l + 1 >= L) continue;     // the top level has no parents to project for
        if (l + 1 >= chain_from) continue;   // every parent is a chain node: U_f h_k is part of its own launch

        // Forget projections of these nodes (roots' rows go unused), with the PARENT's weights.
        if (grouped) {
            ScopedLaunchTimer tm(JITDB_K_PROJ, n_rows, st);
            a.Bp = w.Bp; a.bp = w.bp;
            a.tiles = w.tiles + w.tiles_each;
            a.n_col_tiles = (int)ceil_div(n_unit_tiles, 8);
            a.n_row_tiles = segs[i].n_proj_tiles;
            a.n_blocks = 8 * (int)ceil_div(a.n_row_tiles, 8) * a.n_col_tiles;
            level_kernel<T, MODE_PROJ, false, true><<<a.n_blocks, kDmaThreads, 0, st>>>(a);
            JITDB_LAUNCH_CHECK();
            continue;
        }
        // one launch per non-empty sub-slot (a single one without a typed table)
        const int n_sub = slots ? n_sig : 1;
        int last_sub = -1;
        // (an N-ary parent needs no projection of its children: its forget gates are part of its own contraction)
        for (int p = 0; p < n_sub; ++p)
            if ((!slots || sub_begin(l, sig, p + 1) > sub_begin(l, sig, p)) && !is_nary(slots ? p : -1)) last_sub = p;
        for (int p = 0; p < n_sub; ++p) {
            const int begin = slots ? sub_begin(l, sig, p) : segs[i].begin;
            const int rows = slots ? sub_begin(l, sig, p + 1) - begin : n_rows;
            if (rows <= 0 || is_nary(slots ? p : -1)) continue;
            a.Bp = static_cast<char *>(w.Bp) + packed_w_bytes(d) * p;
            a.bp = w.bp + (size_t)d.NP * p;
            a.row_rec = w.row_rec + 2 * (int64_t)begin;
            a.proj_nodes = slots ? nullptr : s->perm + begin;
            a.n_rows = rows;
            const bool thin_p = rows <= kThinMaxRows;
            ScopedLaunchTimer tm(thin_p ? JITDB_K_THIN_PROJ : JITDB_K_PROJ, rows, st);
            if (thin_p) {
                a.n_col_tiles = (int)ceil_div(n_unit_tiles, 4);
                a.n_tiles = (int)ceil_div(rows, 32) * a.n_col_tiles;
                a.n_blocks = a.n_tiles;
                // the stack step of the next slot, if that is thin too, rides along with the slot's
                // last projection (the level kernel above was the stack buffer's only reader); its
                // rows are counted with this launch's class
                if (p == last_sub && i + 1 < segs.size() && segs[i + 1].l > 0 && segs[i + 1].rows <= kThinMaxRows &&
                    !is_nary(segs[i + 1].sig)) {
                    thin_proj_stack_kernel<T><<<a.n_blocks + stack_blocks(segs[i + 1]), kThinWaves * 64, 0, st>>>(
                        a, stack_args(segs[i + 1]));
                    stacked_ahead = true;
                } else {
                    thin_kernel<T, MODE_PROJ><<<a.n_blocks, kThinWaves * 64, 0, st>>>(a);
                }
            } else if (may256 && tile256_applies(MODE_PROJ, a)) {
                const int rc = launch_tile256(MODE_PROJ, a, st);
                if (rc != JITDB_OK) return rc;
            } else {
                a.n_col_tiles = (int)ceil_div(n_unit_tiles, 8);
                a.n_row_tiles = (int)ceil_div(rows, kDmaBM);
                a.n_blocks = 8 * (int)ceil_div(a.n_row_tiles, 8) * a.n_col_tiles;
                level_kernel<T, MODE_PROJ><<<a.n_blocks, kDmaThreads, 0, st>>>(a);
            }
            JITDB_LAUNCH_CHECK();
        }
    }
    return JITDB_OK;
}

}  // namespace

int launch_nary_level(jitdb_dtype dtype, const NaryLevel &g, hipStream_t st) {
    if (g.M <= 0) return JITDB_OK;
    if (g.k_bytes <= 0 || g.k_bytes % 128 != 0) return JITDB_E_BADARG;
    LevelArgs a = {};
    a.stack = g.A;
    a.n_rows_alloc = (int)g.a_rows_alloc;
    a.Bp = g.B;
    a.NPU = (int)g.b_rows_alloc;
    a.n_rows = g.M;
    a.Dp = (int)(g.k_bytes / (dtype == JITDB_F32 ? 4 : 2));
    a.Hp = 0;
    a.n_row_tiles = (int)ceil_div(g.M, kDmaBM);
    a.n_col_tiles = g.n_col_tiles;
    a.n_blocks = 8 * (int)ceil_div(a.n_row_tiles, 8) * a.n_col_tiles;
    NaryEpi e;
    e.row_rec = g.row_rec; e.bias = g.bias; e.cs = g.cs; e.F = g.F; e.c_out = g.c_out; e.h_out = g.h_out; e.hs_out = g.hs_out;
    e.cs_out = g.cs_out; e.M = g.M; e.H = g.H; e.Hp = g.Hp; e.Hq = g.Hq; e.N = g.N;
    dim3 grid((unsigned)a.n_blocks);
    if (dtype == JITDB_F32) {
        if (g.leaves) nary_level_kernel<float, true><<<grid, kDmaThreads, 0, st>>>(a, e);
        else nary_level_kernel<float, false><<<grid, kDmaThreads, 0, st>>>(a, e);
    } else {
        if (g.leaves) nary_level_kernel<bf16_t, true><<<grid, kDmaThreads, 0, st>>>(a, e);
        else nary_level_kernel<bf16_t, false><<<grid, kDmaThreads, 0, st>>>(a, e);
    }
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

int launch_kb_gemm(jitdb_dtype dtype, const KbGemm &g, hipStream_t st) {
    if (g.M <= 0 || g.N <= 0 || g.k_bytes <= 0) return JITDB_OK;
    if (g.k_bytes % 128 != 0) return JITDB_E_BADARG;
    LevelArgs a = {};
    a.stack = g.A;
    a.n_rows_alloc = (int)g.a_rows_alloc;
    a.Bp = g.B;
    a.NPU = (int)g.b_rows_alloc;
    a.n_rows = g.M;
    a.n_row_tiles = (int)ceil_div(g.M, kDmaBM);
    a.n_col_tiles = (int)ceil_div(g.N, kBN);
    a.n_blocks = 8 * (int)ceil_div(a.n_row_tiles, 8) * a.n_col_tiles;
    KbEpiArgs e;
    e.kind = g.epilogue; e.out0 = g.out0; e.out1 = g.out1; e.node = g.node; e.D = g.D; e.H = g.H; e.ldc = g.ldc;
    e.M = g.M; e.N = g.N;
    e.stages_total = (int)(g.k_bytes / kDmaStage);
    // ranges of at least two stages (the pipeline's minimum); the last one may be shorter but
    // not a single stage, in which case the ranges are made a stage longer
    int splits = g.k_splits < 1 ? 1 : g.k_splits;
    e.stages_per_split = (int)ceil_div(e.stages_total, splits);
    if (e.stages_per_split < 2) e.stages_per_split = 2;
    while (e.stages_per_split < e.stages_total && e.stages_total % e.stages_per_split == 1) ++e.stages_per_split;
    splits = (int)ceil_div(e.stages_total, e.stages_per_split);
    e.splits = splits;
    if (splits > 1) a.n_blocks = 8 * a.n_row_tiles * a.n_col_tiles * (int)ceil_div(splits, 8);
    dim3 grid((unsigned)a.n_blocks);
    if (dtype == JITDB_F32) gemm_kb_kernel<float><<<grid, kDmaThreads, 0, st>>>(a, e);
    else gemm_kb_kernel<bf16_t><<<grid, kDmaThreads, 0, st>>>(a, e);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

}  // namespace jitdb

using namespace jitdb;


namespace {
void profiler_release() {
    for (int i = 0; i < g_prof.capacity; ++i) {
        if (g_prof.begin && g_prof.begin[i]) (void)hipEventDestroy(g_prof.begin[i]);
        if (g_prof.end && g_prof.end[i]) (void)hipEventDestroy(g_prof.end[i]);
    }
    delete[] g_prof.begin; delete[] g_prof.end; delete[] g_prof.cls; delete[] g_prof.rows; delete[] g_prof.edges;
    g_prof = Profiler();
}
}  // namespace

extern "C" int jitdb_profile_start(int32_t capacity) {
    if (capacity < 1 || capacity > (1 << 20)) return JITDB_E_BADARG;
    if (g_prof.on) return JITDB_E_BADARG;
    // value-initialised arrays: an event handle that was never created stays null and is not destroyed
    g_prof.begin = new (std::nothrow) hipEvent_t[capacity]();
    g_prof.end = new (std::nothrow) hipEvent_t[capacity]();
    g_prof.cls = new (std::nothrow) int[capacity]();
    g_prof.rows = new (std::nothrow) int64_t[capacity]();
    g_prof.edges = new (std::nothrow) int64_t[capacity]();
    g_prof.capacity = capacity;
    if (!g_prof.begin || !g_prof.end || !g_prof.cls || !g_prof.rows || !g_prof.edges) {
        profiler_release();
        return JITDB_E_NOMEM;
    }
    for (int i = 0; i < capacity; ++i) {
        if (hipEventCreate(&g_prof.begin[i]) != hipSuccess || hipEventCreate(&g_prof.end[i]) != hipSuccess) {
            profiler_release();      // the events created so far go back
            return JITDB_E_HIP;
        }
    }
    g_prof.used = 0;
    g_prof.dropped = 0;
    g_prof.on = true;
    return JITDB_OK;
}

extern "C" int jitdb_profile_stop(jitdb_profile_t *out) {
    if (!out) return JITDB_E_NULL;
    if (!g_prof.on) return JITDB_E_BADARG;
    g_prof.on = false;
    int rc = JITDB_OK;
    for (int c = 0; c < JITDB_K_CLASSES; ++c) { out->ms[c] = 0.0; out->launches[c] = 0; out->rows[c] = 0; out->edges[c] = 0; }
    out->dropped = g_prof.dropped;
    for (int i = 0; i < g_prof.used; ++i) {
        float ms = 0.0f;
        if (hipEventSynchronize(g_prof.end[i]) != hipSuccess ||
            hipEventElapsedTime(&ms, g_prof.begin[i], g_prof.end[i]) != hipSuccess) {
            rc = JITDB_E_HIP;
            continue;
        }
        out->ms[g_prof.cls[i]] += ms;
        out->launches[g_prof.cls[i]] += 1;
        out->rows[g_prof.cls[i]] += g_prof.rows[i];
        out->edges[g_prof.cls[i]] += g_prof.edges[i];
    }
    profiler_release();
    return rc;
}

extern "C" size_t jitdb_treelstm_workspace_bytes(int64_t n_nodes, int64_t n_edges,
                                                 int32_t D, int32_t H, jitdb_dtype dtype) {
    if (!dims_ok(n_nodes, n_edges, D, H, (int)dtype)) return 0;
    const Dims d = make_dims(D, H, dtype);
    return carve_forward_ws(n_nodes, n_edges, d, nullptr).bytes;
}

namespace {
int forward_entry(const void *x, const void *W, const void *U, const float *b, int32_t D, int32_t H,
                  jitdb_dtype dtype, const jitdb_schedule_t *s, const jitdb_slots_t *slots,
                  void *h_out, float *c_out, void *gates, void *fgate, bool save,
                  void *workspace, size_t workspace_bytes, void *hip_stream, const void *packed = nullptr,
                  const jitdb_cell_t *cells = nullptr) {
    if (!s) return JITDB_E_NULL;
    const int n_sig = slots ? slots->n_sig : 1;
    if (n_sig < 1 || n_sig > JITDB_MAX_SIGNATURES) return JITDB_E_BADARG;
    for (int t = 0; cells && t < n_sig; ++t) {
        if (cells[t].kind != JITDB_CELL_CHILDSUM && cells[t].kind != JITDB_CELL_NARY) return JITDB_E_BADARG;
        if (cells[t].kind == JITDB_CELL_NARY && (cells[t].arity < 1 || cells[t].arity > JITDB_MAX_NARY)) return JITDB_E_BADARG;
        if (!cells[t].W || !cells[t].U || !cells[t].b) return JITDB_E_NULL;
    }
    drop_stale_hip_error();
    const int64_t n = s->n_nodes;
    if (!dims_ok(n, s->n_edges, D, H, (int)dtype)) return JITDB_E_BADARG;
    if (n == 0) return JITDB_OK;
    if (!x || !h_out || !c_out || !workspace) return JITDB_E_NULL;
    if (!packed && !cells && (!W || !U || !b)) return JITDB_E_NULL;
    if (packed && (reinterpret_cast<uintptr_t>(packed) & 255) != 0) return JITDB_E_BADARG;
    if (save && (!gates || !fgate)) return JITDB_E_NULL;
    if (!s->perm || !s->height || !s->child_ptr || !s->child_idx || !s->host_level_ptr) return JITDB_E_NULL;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return JITDB_E_BADARG;
    // rows are fetched in 16-byte pieces where their stride allows
    if ((reinterpret_cast<uintptr_t>(x) & 15) != 0) return JITDB_E_BADARG;
    if ((reinterpret_cast<uintptr_t>(h_out) & 15) != 0) return JITDB_E_BADARG;
    if ((reinterpret_cast<uintptr_t>(c_out) & 15) != 0) return JITDB_E_BADARG;
    const int L = s->n_levels;
    if (L < 1 || L > n) return JITDB_E_SCHEDULE;
    if (s->host_level_ptr[0] != 0 || s->host_level_ptr[L] != n) return JITDB_E_SCHEDULE;
    for (int l = 0; l < L; ++l)
        if (s->host_level_ptr[l + 1] <= s->host_level_ptr[l]) return JITDB_E_SCHEDULE;
    if (slots) {
        if (!slots->key || !slots->slot_ptr || !slots->host_slot_ptr) return JITDB_E_NULL;
        const int64_t T2 = (int64_t)n_sig * n_sig;
        if (slots->slot_capacity < L * T2 + 1) return JITDB_E_SCHEDULE;
        for (int64_t q = 0; q < L * T2; ++q)
            if (slots->host_slot_ptr[q + 1] < slots->host_slot_ptr[q]) return JITDB_E_SCHEDULE;
        for (int l = 0; l <= L; ++l)
            if (slots->host_slot_ptr[l * T2] != s->host_level_ptr[l]) return JITDB_E_SCHEDULE;
    }

    const Dims d = make_dims(D, H, dtype);
    const ForwardWs w = carve_forward_ws(n, s->n_edges, d, workspace, n_sig, cells);
    if (workspace_bytes < w.bytes) return JITDB_E_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    // run_forward keeps its list of launches in a std::vector: an allocation failure becomes a status
    JITDB_ABI_TRY
    if (dtype == JITDB_F32) {
        if (save) return run_forward<float, true>(x, W, U, b, d, s, slots, cells, h_out, c_out, gates, fgate, w, packed, st);
        return run_forward<float, false>(x, W, U, b, d, s, slots, cells, h_out, c_out, nullptr, nullptr, w, packed, st);
    }
    if (save) return run_forward<bf16_t, true>(x, W, U, b, d, s, slots, cells, h_out, c_out, gates, fgate, w, packed, st);
    return run_forward<bf16_t, false>(x, W, U, b, d, s, slots, cells, h_out, c_out, nullptr, nullptr, w, packed, st);
    JITDB_ABI_CATCH
}

size_t packed_total_bytes(const Dims &d, int n_sig) {
    return (size_t)round_up(packed_w_bytes(d) * n_sig, 256) + (size_t)round_up((int64_t)d.NP * n_sig * 4, 256) +
           (has_fragment_copy(d, n_sig) ? (size_t)round_up(packed_w_bytes(d), 256) : 0);
}
}  // namespace

extern "C" size_t jitdb_treelstm_packed_bytes(int32_t D, int32_t H, jitdb_dtype dtype, int32_t n_sig) {
    if (!dims_ok(0, 0, D, H, (int)dtype) || n_sig < 1 || n_sig > JITDB_MAX_SIGNATURES) return 0;
    return packed_total_bytes(make_dims(D, H, dtype), n_sig);
}

extern "C" int jitdb_treelstm_pack(const void *W, const void *U, const float *b, int32_t D, int32_t H,
                                   jitdb_dtype dtype, int32_t n_sig, void *packed, size_t packed_bytes,
                                   void *hip_stream) {
    if (!W || !U || !b || !packed) return JITDB_E_NULL;
    if (!dims_ok(0, 0, D, H, (int)dtype) || n_sig < 1 || n_sig > JITDB_MAX_SIGNATURES) return JITDB_E_BADARG;
    if ((reinterpret_cast<uintptr_t>(packed) & 255) != 0) return JITDB_E_BADARG;
    drop_stale_hip_error();
    const Dims d = make_dims(D, H, dtype);
    if (packed_bytes < packed_total_bytes(d, n_sig)) return JITDB_E_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t total = (int64_t)d.NPU * (d.Dp + d.Hp);
    const unsigned grid = (unsigned)(ceil_div(total, kThreads) < 4096 ? ceil_div(total, kThreads) : 4096);
    float *bp0 = reinterpret_cast<float *>(static_cast<char *>(packed) + round_up(packed_w_bytes(d) * n_sig, 256));
    for (int t = 0; t < n_sig; ++t) {
        PackArgs p;
        const size_t esz = d.esz;
        p.W = static_cast<const char *>(W) + (size_t)t * 4 * d.H * d.D * esz;
        p.U = static_cast<const char *>(U) + (size_t)t * 4 * d.H * d.H * esz;
        p.b = b + (size_t)t * 4 * d.H;
        p.D = d.D; p.H = d.H; p.Dp = d.Dp; p.Hp = d.Hp; p.NP = d.NP; p.NPU = d.NPU;
        p.Bp = static_cast<char *>(packed) + packed_w_bytes(d) * t;
        p.bp = bp0 + (size_t)d.NP * t;
        p.Bf = has_fragment_copy(d, n_sig) ? reinterpret_cast<char *>(bp0) + round_up((int64_t)d.NP * n_sig * 4, 256) : nullptr;
        if (dtype == JITDB_F32) pack_weights_kernel<float><<<grid, kThreads, 0, st>>>(p);
        else pack_weights_kernel<bf16_t><<<grid, kThreads, 0, st>>>(p);
        JITDB_LAUNCH_CHECK();
    }
    return JITDB_OK;
}

extern "C" int jitdb_treelstm_forward_packed(const void *x, const void *packed, int32_t D, int32_t H,
                                             jitdb_dtype dtype, const jitdb_schedule_t *s,
                                             const jitdb_slots_t *slots, void *h_out, float *c_out,
                                             void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!packed) return JITDB_E_NULL;
    return forward_entry(x, nullptr, nullptr, nullptr, D, H, dtype, s, slots, h_out, c_out, nullptr, nullptr, false,
                         workspace, workspace_bytes, hip_stream, packed);
}

extern "C" int jitdb_treelstm_forward(const void *x, const void *W, const void *U, const float *b,
                                      int32_t D, int32_t H, jitdb_dtype dtype,
                                      const jitdb_schedule_t *s, void *h_out, float *c_out,
                                      void *workspace, size_t workspace_bytes, void *hip_stream) {
    return forward_entry(x, W, U, b, D, H, dtype, s, nullptr, h_out, c_out, nullptr, nullptr, false,
                         workspace, workspace_bytes, hip_stream);
}

extern "C" size_t jitdb_treelstm_typed_workspace_bytes(int64_t n_nodes, int64_t n_edges, int32_t D, int32_t H,
                                                       jitdb_dtype dtype, int32_t n_sig) {
    if (!dims_ok(n_nodes, n_edges, D, H, (int)dtype) || n_sig < 1 || n_sig > JITDB_MAX_SIGNATURES) return 0;
    const Dims d = make_dims(D, H, dtype);
    return carve_forward_ws(n_nodes, n_edges, d, nullptr, n_sig).bytes;
}

extern "C" int jitdb_treelstm_forward_typed(const void *x, const void *W, const void *U, const float *b,
                                            int32_t D, int32_t H, jitdb_dtype dtype,
                                            const jitdb_schedule_t *s, const jitdb_slots_t *slots,
                                            void *h_out, float *c_out,
                                            void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!slots) return JITDB_E_NULL;
    return forward_entry(x, W, U, b, D, H, dtype, s, slots, h_out, c_out, nullptr, nullptr, false,
                         workspace, workspace_bytes, hip_stream);
}

extern "C" size_t jitdb_treelstm_cells_workspace_bytes(int64_t n_nodes, int64_t n_edges, int32_t D, int32_t H,
                                                       jitdb_dtype dtype, const jitdb_cell_t *cells, int32_t n_sig) {
    if (!cells || !dims_ok(n_nodes, n_edges, D, H, (int)dtype) || n_sig < 1 || n_sig > JITDB_MAX_SIGNATURES) return 0;
    for (int t = 0; t < n_sig; ++t)
        if (cells[t].kind == JITDB_CELL_NARY && (cells[t].arity < 1 || cells[t].arity > JITDB_MAX_NARY)) return 0;
    const Dims d = make_dims(D, H, dtype);
    return carve_forward_ws(n_nodes, n_edges, d, nullptr, n_sig, cells).bytes;
}

extern "C" int jitdb_treelstm_forward_cells(const void *x, const jitdb_cell_t *cells, int32_t n_sig,
                                            int32_t D, int32_t H, jitdb_dtype dtype,
                                            const jitdb_schedule_t *s, const jitdb_slots_t *slots,
                                            void *h_out, float *c_out,
                                            void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!slots || !cells) return JITDB_E_NULL;
    if (n_sig != slots->n_sig) return JITDB_E_BADARG;
    const int rc = forward_entry(x, nullptr, nullptr, nullptr, D, H, dtype, s, slots, h_out, c_out, nullptr, nullptr,
                                 false, workspace, workspace_bytes, hip_stream, nullptr, cells);
    if (rc != JITDB_OK || !s || s->n_nodes == 0) return rc;
    bool any_nary = false;
    for (int t = 0; t < n_sig; ++t) any_nary = any_nary || cells[t].kind == JITDB_CELL_NARY;
    if (!any_nary) return JITDB_OK;
    // a node with more children than its cell has positions: reported after the work has run
    const Dims d = make_dims(D, H, dtype);
    const ForwardWs w = carve_forward_ws(s->n_nodes, s->n_edges, d, workspace, n_sig, cells);
    int flag = 0;
    hipStream_t st = (hipStream_t)hip_stream;
    JITDB_HIP_CHECK(hipMemcpyAsync(&flag, w.nary_err, sizeof(int), hipMemcpyDeviceToHost, st));
    JITDB_HIP_CHECK(hipStreamSynchronize(st));
    return flag ? JITDB_E_ARITY : JITDB_OK;
}

extern "C" int jitdb_treelstm_forward_train(const void *x, const void *W, const void *U, const float *b,
                                            int32_t D, int32_t H, jitdb_dtype dtype,
                                            const jitdb_schedule_t *s, void *h_out, float *c_out,
                                            void *gates_out, void *fgate_out,
                                            void *workspace, size_t workspace_bytes, void *hip_stream) {
    return forward_entry(x, W, U, b, D, H, dtype, s, nullptr, h_out, c_out, gates_out, fgate_out, true,
                         workspace, workspace_bytes, hip_stream);
}

// ---- the forward for callers that cannot allocate ----------------------------------------
// Code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc have no
// workspace to hand over.  For them the workspace is this array, which every GPU the library
// runs on holds from the moment the code object is loaded until the process ends.  In host code
// the array's name is only a handle: the device address comes from hipGetSymbolAddress, once per
// device, and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[JITDB_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_lock;

int static_scratch_of_current_device(void **out) {
    int dev = -1;
    JITDB_HIP_CHECK(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return JITDB_E_BADARG;
    std::lock_guard<std::mutex> g(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        JITDB_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));    // this device's copy of the array
        if (!p) return JITDB_E_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return JITDB_OK;
}
}  // namespace

extern "C" int jitdb_treelstm_forward_static(const void *x, const void *W, const void *U, const float *b,
                                             int32_t D, int32_t H, jitdb_dtype dtype,
                                             const jitdb_schedule_t *s, void *h_out, float *c_out,
                                             void *hip_stream) {
    if (!s) return JITDB_E_NULL;
    if (!dims_ok(s->n_nodes, s->n_edges, D, H, (int)dtype)) return JITDB_E_BADARG;
    if (s->n_nodes == 0) return JITDB_OK;
    const size_t need = carve_forward_ws(s->n_nodes, s->n_edges, make_dims(D, H, dtype), nullptr).bytes;
    if (need > (size_t)JITDB_STATIC_SCRATCH_BYTES) return JITDB_E_WORKSPACE;
    drop_stale_hip_error();
    void *ws = nullptr;
    JITDB_ABI_TRY
    const int rc = static_scratch_of_current_device(&ws);
    if (rc != JITDB_OK) return rc;
    JITDB_ABI_CATCH
    // Nothing in the workspace has to start at zero: every region is written in full by this call
    // before anything reads it (packed weights, row records, the stacked level, P, padded copies).
    return forward_entry(x, W, U, b, D, H, dtype, s, nullptr, h_out, c_out, nullptr, nullptr, false,
                         ws, (size_t)JITDB_STATIC_SCRATCH_BYTES, hip_stream);
}
