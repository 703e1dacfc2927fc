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
//   level_kernel<GATES>   [x_j ; hs_j] x [W ; U]^T on MFMA with the whole cell
//                      fused into the epilogue: per-child forget gates from the
//                      precomputed P_k = U_f h_k, c_j and h_j written once
//   level_kernel<PROJ> P_k = U_f h_k for the nodes just produced, so that their
//                      parent reads one row per child (every non-root node is a
//                      child exactly once)
//
// "Stack" is the row gather through perm (level-major order) done by
// stack_kernel, "slice" is the scatter of rows back to node-id order in the
// epilogue.
//
// Weights are re-packed once per call: gate rows of 32 hidden units are
// interleaved (i|o|u|f blocks of 32 rows), so that one wave holds all four
// gates of a hidden unit in its own accumulators and the cell update needs no
// exchange between lanes; rows and K are zero padded to tile multiples.

#include "common.h"

#include <type_traits>

namespace jitdb {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t bf16_t;  // storage type of bfloat16 values
// Native vectors for data in flight (HIP's uint4 is a union-based struct, which the
// optimiser does not always break up into registers).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;     // small kernels
constexpr int kGemmThreads = 512; // level kernels: eight waves
constexpr int kBM = 256;        // rows (nodes) per block
constexpr int kBN = 256;        // packed columns per block = 2 unit tiles x 4 gates x 32
constexpr int kUnit = 32;       // hidden units per MFMA column tile
constexpr int kGateTile = 128;  // packed rows per unit tile (4 gates x 32 units)

constexpr int kEpiRows = 128;   // rows per pass of the projection's store epilogue
constexpr int kEpiStride = 40;  // floats per row of a wave's epilogue region: 32 units + 8; rows 4 apart fall 32 banks apart
constexpr int kProjStride = 264; // same for the projection's 256-unit rows
constexpr int kLdsStride = 144; // stage row (128 bytes) + 16: 128-bit LDS reads of 32 rows hit distinct banks

enum : int { MODE_LEAF = 0, MODE_INTERNAL = 1, MODE_PROJ = 2 };

template <typename T> struct Traits;
template <> struct Traits<float> {
    static constexpr int BK = 32;   // elements of K per stage (128 bytes)
    static constexpr int VEC = 4;   // elements per 16 bytes
};
template <> struct Traits<bf16_t> {
    static constexpr int BK = 64;
    static constexpr int VEC = 8;
};

// ---- scalar helpers ----------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {  // round to nearest even
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ T from_f32(float f);
template <> __device__ __forceinline__ float from_f32<float>(float f) { return f; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float f) { return f32_to_bf16(f); }

// fp32 path: library exp (about 1 ulp); bf16 path: the hardware exp2-based fast form.
template <typename T> __device__ __forceinline__ float exp_t(float z);
template <> __device__ __forceinline__ float exp_t<float>(float z) { return expf(z); }
template <> __device__ __forceinline__ float exp_t<bf16_t>(float z) { return __expf(z); }

// 1/(1+e) through the hardware reciprocal (1 ulp) instead of an IEEE division sequence.
template <typename T> __device__ __forceinline__ float sigmoid_t(float z) {
    return __builtin_amdgcn_rcpf(1.0f + exp_t<T>(-z));
}
template <typename T> __device__ __forceinline__ float tanh_t(float z) {
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + exp_t<T>(2.0f * z));
}

// ---- weight packing ----------------------------------------------------------------
// Packed row r = tile*128 + gate*32 + uu holds gate `gate` of hidden unit tile*32 + uu as
// [ W row (D values, zero padded to Dp) | U row (H values, zero padded to Hp) ].  There are
// NPU >= NP rows; rows of units >= H are zero.
template <typename T>
__global__ void __launch_bounds__(kThreads)
pack_weights_kernel(const T *__restrict__ W, const T *__restrict__ U, const float *__restrict__ b,
                    int D, int H, int Dp, int Hp, int NP, int NPU,
                    T *__restrict__ Bp, float *__restrict__ bp) {
    const int Kp = Dp + Hp;
    const int64_t total = (int64_t)NPU * Kp;
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * kThreads) {
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
        Bp[idx] = v;
        if (k == 0 && r < NP) bp[r] = row_ok ? b[src] : 0.0f;
    }
}

// ---- row records -------------------------------------------------------------------
// What the stack step and the cell update need to know about the node at level
// position p, in one 32-byte record: { node, arity, CSR start, - } { first four child
// ids (-1 where there is none) }.  Written once per forward for all positions, so that
// the per-level kernels start from one load instead of the chain perm -> child_ptr ->
// child_idx.
__global__ void __launch_bounds__(kThreads)
row_record_kernel(const int32_t *__restrict__ perm, const int32_t *__restrict__ child_ptr,
                  const int32_t *__restrict__ child_idx, int4 *__restrict__ row_rec, int n) {
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p >= n) return;
    const int node = perm[p];
    const int cb = child_ptr[node], ar = child_ptr[node + 1] - cb;
    int kid[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) kid[j] = j < ar ? child_idx[cb + j] : -1;
    row_rec[2 * p] = make_int4(node, ar, cb, 0);
    row_rec[2 * p + 1] = make_int4(kid[0], kid[1], kid[2], kid[3]);
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

template <typename T, bool WITH_H>
__global__ void __launch_bounds__(kThreads)
stack_kernel(const T *__restrict__ x, int D, int Dp, const T *__restrict__ hs, int Hp,
             const int4 *__restrict__ row_rec, const int32_t *__restrict__ child_idx,
             T *__restrict__ A, int n_rows) {
    constexpr int VEC = Traits<T>::VEC;
    const int Kp = Dp + (WITH_H ? Hp : 0);
    const int cpr = Kp / VEC;
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
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
    *reinterpret_cast<uint4 *>(A + row * Kp + k0) = o;
}

// ---- the level GEMM ----------------------------------------------------------------
struct LevelArgs {
    // A operands
    const void *stack;    // [n_rows, Dp (+ Hp)] the level's stacked input (leaf / internal)
    const void *hs;       // [N, Hp] rows by node id (projection)
    // B operand: packed [W | U], NPU rows of Dp + Hp
    const void *Bp;
    const float *bp;      // [NP] packed bias
    // schedule
    const int32_t *level_nodes;  // perm + level start: row -> node id
    const int4 *row_rec;         // two int4 per level row (this level's slice of the records)
    const int32_t *child_idx;
    // per-child forget projections U_f h_k, rows by node id, stride Hq, element type T
    // (bf16 in the bf16 path: it halves the largest stream of the forward)
    void *P;
    float *cs;            // [N, Hq] c with padded rows, or == c_out when H % 8 == 0
    // outputs
    float *c_out;         // [N, H]
    void *h_out;          // [N, H]
    void *hs_out;         // [N, Hp] or == h_out when H == Hp
    int D, Dp, H, Hp, Hu, Hq;
    int n_rows;
    int n_col_tiles;      // tiles along the column axis
    int n_tiles;          // thin kernel: number of wave tiles
    int n_blocks;
};

// Spread consecutive block ids (which the hardware deals round-robin to the 8
// XCDs) so that blocks sharing an A row tile land on the same XCD and L2.
__device__ __forceinline__ int xcd_remap(int b, int nb) {
    const int xcd = b & 7, idx = b >> 3;
    const int q = nb >> 3, r = nb & 7;
    return xcd * q + (xcd < r ? xcd : r) + idx;
}

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

// What one thread holds of a K stage on its way from global memory to LDS:
// 16 bytes of each of four A rows and four B rows.
struct StageRegs {
    u32x4 a[4];
    u32x4 b[4];
};

// The block GEMM: 256 rows x 256 packed columns per block of eight waves, each
// wave a 64 x 128 sub-tile (2 x 4 MFMA tiles of 32 x 32).  A is the level's
// stacked input [x | hsum] (row stride Kp = Dp + Hp), B the packed [W | U]
// with the same K layout; K runs over "stages" of 128 bytes per row (one cache
// line): n_x stages of the x part, then n_h of the h part, in which the forget
// gate is skipped (U_f applies to each child's own h, not to the sum).  The
// projection instead reads A rows from hs by node id and uses only the U part
// of the forget rows.  One software pipeline with two LDS buffers and one
// barrier per stage; in iteration g
//   - the registers holding stage g+1 (requested one iteration ago) go to the
//     idle LDS buffer; these writes drain through the 64-bytes-per-clock LDS
//     write port while the matrix cores work,
//   - stage g is multiplied out of the other buffer,
//   - half way through, stage g+2 is requested from global memory (by then
//     the LDS writes have released the registers).
//
// LDS layout: row r at r*kLdsStride, K contiguous, A rows 0-255 then B rows.
// In each 16-wide (bf16) or 8-wide (fp32) K group, lanes 0-31 take the first
// 16 bytes and lanes 32-63 the next 16 for A and B alike; since the same
// assignment is used on both operands any such split of K is a valid MFMA
// schedule.
//
// Staging map: eight consecutive lanes move the eight 16-byte pieces of one row
// (a whole line per row and load instruction); thread t handles piece t&7 of
// A rows t/8 + 64 i.  Of B it handles hidden unit (t/8)%32 of unit tile t/256,
// row group i being the gate (or, for the projection, unit tile 4*(t/256) + i),
// so whole gates can be skipped at compile time.
template <typename T, int MODE, typename Hook>
__device__ __forceinline__ void block_gemm(const LevelArgs &a, char *lds, const int *row_node,
                                           int tile_row0, int col_tile, floatx16 (&acc)[2][4],
                                           Hook &&after_first_requests) {
    constexpr int BK = Traits<T>::BK;
    constexpr int ESZ = (int)sizeof(T);
    constexpr int NG_X = (MODE == MODE_LEAF) ? 3 : 4;      // gate tiles multiplied in the x part
    constexpr int NG_H = (MODE == MODE_INTERNAL) ? 3 : 4;  // ... in the h part

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int hf = lane >> 5, l32 = lane & 31;

    const int n_x = (MODE == MODE_PROJ) ? 0 : a.Dp / BK;
    const int n_h = (MODE == MODE_LEAF) ? 0 : a.Hp / BK;
    const int n_stages = n_x + n_h;
    const int64_t b_row_bytes = (int64_t)(a.Dp + a.Hp) * ESZ;

    // ---- A source: rows tile_row0 + t/8 + 64 i of the stacked matrix (rows past the end
    //      of the level lie inside the buffer, hold anything and are never stored), or
    //      for the projection rows of hs by node id (clamped to the level's last row).
    const char *ap[MODE == MODE_PROJ ? 4 : 1];
    int64_t a_step = 0;
    if constexpr (MODE == MODE_PROJ) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int g = tile_row0 + (t >> 3) + 64 * i;
            if (g >= a.n_rows) g = a.n_rows - 1;
            ap[i] = static_cast<const char *>(a.hs) + (int64_t)row_node[g - tile_row0] * a.Hp * ESZ + (t & 7) * 16;
        }
    } else {
        const int64_t a_row_bytes = (int64_t)(a.Dp + (MODE == MODE_INTERNAL ? a.Hp : 0)) * ESZ;
        ap[0] = static_cast<const char *>(a.stack) + (int64_t)(tile_row0 + (t >> 3)) * a_row_bytes + (t & 7) * 16;
        a_step = 64 * a_row_bytes;
    }
    // ---- B source
    const int uu = (t >> 3) & 31, ut = t >> 8;
    const char *bp;
    int64_t b_step;
    if constexpr (MODE == MODE_PROJ) {
        const int64_t row = (int64_t)(col_tile * 8 + ut * 4) * kGateTile + 3 * kUnit + uu;
        bp = static_cast<const char *>(a.Bp) + row * b_row_bytes + (int64_t)a.Dp * ESZ + (t & 7) * 16;
        b_step = (int64_t)kGateTile * b_row_bytes;
    } else {
        const int64_t row = (int64_t)col_tile * kBN + ut * kGateTile + uu;
        bp = static_cast<const char *>(a.Bp) + row * b_row_bytes + (t & 7) * 16;
        b_step = (int64_t)kUnit * b_row_bytes;
    }
    const int a_wr = (t >> 3) * kLdsStride + (t & 7) * 16;
    const int b_wr = (kBM + ut * kGateTile + uu) * kLdsStride + (t & 7) * 16;
    const int a_rd = (wm * 64 + l32) * kLdsStride + hf * 16;
    const int b_rd = (kBM + wn * 128 + l32) * kLdsStride + hf * 16;

    auto ld16 = [](const char *p) __attribute__((always_inline)) { return *reinterpret_cast<const u32x4 *>(p); };

    // B row groups moved per stage.  The internal levels move the forget rows in the h
    // part too although they are not multiplied there: with x and h parts alike, every
    // iteration of the pipeline is one straight-line block that can be scheduled as a whole.
    constexpr int NG_F = (MODE == MODE_LEAF) ? 3 : 4;

    StageRegs r;
    // global -> registers, stage g
    auto fetch = [&](int g, StageRegs &r) __attribute__((always_inline)) {
        const int64_t kb = (int64_t)g * (BK * ESZ);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if constexpr (MODE == MODE_PROJ) r.a[i] = ld16(ap[i] + kb);
            else r.a[i] = ld16(ap[0] + i * a_step + kb);
        }
#pragma unroll
        for (int i = 0; i < NG_F; ++i) r.b[i] = ld16(bp + i * b_step + kb);
    };
    // registers -> LDS
    auto stash = [&](char *buf, const StageRegs &r) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4 *>(buf + a_wr + i * 64 * kLdsStride) = r.a[i];
#pragma unroll
        for (int i = 0; i < NG_F; ++i) *reinterpret_cast<u32x4 *>(buf + b_wr + i * 32 * kLdsStride) = r.b[i];
    };
    constexpr int kBufBytes = (kBM + kBN) * kLdsStride;
    const std::integral_constant<int, NG_X> ngx;
    const std::integral_constant<int, NG_H> ngh;
    const int last = n_stages - 1;

    // One iteration: stage g is multiplied out of buffer g&1 while stage g+1 moves from
    // the registers to the other buffer and stage g+2 from global memory to the registers.
    // The issue order is fixed by hand: per K group first its LDS reads, then its MFMAs
    // with one LDS write (K groups 0, 1) or one global load (K groups 2, 3) after every
    // quarter of them.  Left to itself the compiler issues all LDS writes first, and since
    // a wave issues in order its MFMAs then wait until the 64-bytes-per-clock write port
    // has taken the writes of all eight waves.  The last iterations repeat the stash /
    // fetch of the last stage (into the idle buffer, from addresses in range) instead of
    // branching around them.
    auto iteration = [&](int g, auto ng_tag) __attribute__((always_inline)) {
        constexpr int NG = decltype(ng_tag)::value;
        constexpr int M = 2 * NG;   // MFMA tiles per K group
        const char *sa = lds + (g & 1) * kBufBytes + a_rd;
        const char *sb = lds + (g & 1) * kBufBytes + b_rd;
        char *nxt = lds + ((g & 1) ^ 1) * kBufBytes;
        const int gf = g + 2 < last ? g + 2 : last;
        const int64_t kb = (int64_t)gf * (BK * ESZ);
        // Fragments are double buffered: the LDS reads of K group h+1 are issued ahead of
        // the MFMAs of K group h, so only the first group of a stage waits for LDS.
        u32x4 av[2][2], bv[2][NG];
        auto read_frags = [&](int h, int set) __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
                av[set][i] = *reinterpret_cast<const u32x4 *>(sa + i * 32 * kLdsStride + h * 32);
#pragma unroll
            for (int q = 0; q < NG; ++q)
                bv[set][q] = *reinterpret_cast<const u32x4 *>(sb + q * 32 * kLdsStride + h * 32);
        };
        read_frags(0, 0);
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            const int cur = h & 1;
            if (h < 3) read_frags(h + 1, cur ^ 1);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int m = j * M / 4; m < (j + 1) * M / 4; ++m)
                    mfma_step<T>(av[cur][m / NG], bv[cur][m % NG], acc[m / NG][m % NG]);
                __builtin_amdgcn_sched_barrier(0);
                const int o = (h & 1) * 4 + j;      // which of the eight moves of this half
                if (h < 2) {                         // registers -> LDS
                    if (o < 4)
                        *reinterpret_cast<u32x4 *>(nxt + a_wr + o * 64 * kLdsStride) = r.a[o];
                    else if (o - 4 < NG_F)
                        *reinterpret_cast<u32x4 *>(nxt + b_wr + (o - 4) * 32 * kLdsStride) = r.b[o - 4];
                } else {                             // global -> registers
                    if (o < 4) {
                        if constexpr (MODE == MODE_PROJ) r.a[o] = ld16(ap[o] + kb);
                        else r.a[o] = ld16(ap[0] + o * a_step + kb);
                    } else if (o - 4 < NG_F) {
                        r.b[o - 4] = ld16(bp + (o - 4) * b_step + kb);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
    };
    // Start-up: stages 0 and 1 are requested together (the accumulators are not live yet,
    // so a second register set is free), then the caller publishes its per-row data, whose
    // loads it issued before calling: one memory latency instead of three in a row.
    {
        StageRegs r_first;
        fetch(0, r_first);
        fetch(1 < last ? 1 : last, r);
        after_first_requests();
        stash(lds, r_first);
    }
    __syncthreads();
    for (int g = 0; g < n_x; ++g) iteration(g, ngx);
    for (int g = n_x; g < n_stages; ++g) iteration(g, ngh);
}

// ---- the cell update of one wave: 32 rows x 32 hidden units ---------------------------
// acc[g][v] holds the pre-activation (without bias) of gate g for row
// (v/4)*8 + hf*4 + v%4 and unit l32 of the wave's unit tile.  The wave writes i*u, o and
// the x part of the forget gate to its private LDS region and reads them back row-major,
// eight lanes per row and four consecutive units per lane: the rows of the children
// (P_k and c_k) are then fetched in 8- and 16-byte pieces, 64 / 128 contiguous bytes per
// row, with four rows in flight per lane.  rn / rar / rcb / rkid describe the 32 rows
// (node id or -1, arity, CSR start, first four child ids).  No block barrier inside.
template <typename T, int MODE>
__device__ __forceinline__ void cell_pass(const LevelArgs &a, const floatx16 (&acc)[4], float *region,
                                          const int *rn, const int *rar, const int *rcb,
                                          const int4 *rkid, int unit_tile, int lane) {
    const int hf = lane >> 5, l32 = lane & 31;
    const int pcol = unit_tile * kGateTile + l32;   // packed row of gate i for this unit
    const float bi = a.bp[pcol], bo = a.bp[pcol + kUnit], bu = a.bp[pcol + 2 * kUnit];
    float bf = 0.0f;
    if constexpr (MODE == MODE_INTERNAL) bf = a.bp[pcol + 3 * kUnit];
    float *s_iu = region;
    float *s_o = s_iu + 32 * kEpiStride;
    float *s_fx = s_o + 32 * kEpiStride;
    T *h_out = static_cast<T *>(a.h_out);
    T *hs_out = static_cast<T *>(a.hs_out);
    const bool separate_hs = (a.hs_out != a.h_out);
    const bool separate_cs = (a.cs != a.c_out);
    const bool vec_ok = (a.H & 3) == 0;
    const int unit0 = unit_tile * kUnit + (lane & 7) * 4;
    // unit groups past the padded width read the first group instead (and store nothing)
    const int unit_ld = unit0 < a.Hq ? unit0 : 0;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int rl = (v >> 2) * 8 + hf * 4 + (v & 3);   // 0..31
        const float gi = sigmoid_t<T>(acc[0][v] + bi);
        const float go = sigmoid_t<T>(acc[1][v] + bo);
        const float gu = tanh_t<T>(acc[2][v] + bu);
        s_iu[rl * kEpiStride + l32] = gi * gu;
        s_o[rl * kEpiStride + l32] = go;
        if constexpr (MODE == MODE_INTERNAL) s_fx[rl * kEpiStride + l32] = acc[3][v] + bf;
    }
    // the wave's own LDS writes are ordered before its reads; nothing else touches the region
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    float4 cc[4], go4[4], fx4[4];
    int node[4], tr[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        tr[q] = (lane >> 3) + 8 * q;
        node[q] = rn[tr[q]];
        const int so = tr[q] * kEpiStride + (lane & 7) * 4;
        cc[q] = *reinterpret_cast<const float4 *>(s_iu + so);
        go4[q] = *reinterpret_cast<const float4 *>(s_o + so);
        if constexpr (MODE == MODE_INTERNAL) fx4[q] = *reinterpret_cast<const float4 *>(s_fx + so);
    }
    if constexpr (MODE == MODE_INTERNAL) {
        // Children are taken two per row and round, for four rows at once: sixteen
        // independent 16-byte loads in flight per thread.  The first four child ids
        // of a row sit in LDS; longer lists (rare) continue from child_idx.  A slot
        // without a child re-reads the row's last child with weight zero, which
        // keeps every load unconditional.
        int ar[4];
        int max_ar = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            ar[q] = node[q] >= 0 ? rar[tr[q]] : 0;
            max_ar = max(max_ar, ar[q]);
        }
        int64_t last[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) last[q] = unit_ld;
        for (int c0 = 0; c0 < max_ar; c0 += 2) {
            int64_t ofs[4][2];
            float wgt[4][2];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int4 kids = make_int4(0, 0, 0, 0);
                if (c0 < 4) kids = rkid[tr[q]];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int c = c0 + j;
                    const bool has = c < ar[q];
                    int kid;
                    if (c0 == 0) kid = j ? kids.y : kids.x;
                    else if (c0 == 2) kid = j ? kids.w : kids.z;
                    else kid = has ? a.child_idx[rcb[tr[q]] + c] : 0;
                    if (has) last[q] = (int64_t)kid * a.Hq + unit_ld;
                    ofs[q][j] = last[q];
                    wgt[q][j] = has ? 1.0f : 0.0f;
                }
            }
            float4 pk[4][2], ck[4][2];
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if constexpr (sizeof(T) == 4) {
                        pk[q][j] = *reinterpret_cast<const float4 *>(static_cast<const float *>(a.P) + ofs[q][j]);
                    } else {
                        const uint2 w = *reinterpret_cast<const uint2 *>(static_cast<const bf16_t *>(a.P) + ofs[q][j]);
                        pk[q][j] = make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xFFFF0000u),
                                               __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xFFFF0000u));
                    }
                    ck[q][j] = *reinterpret_cast<const float4 *>(a.cs + ofs[q][j]);
                }
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    cc[q].x += wgt[q][j] * sigmoid_t<T>(fx4[q].x + pk[q][j].x) * ck[q][j].x;
                    cc[q].y += wgt[q][j] * sigmoid_t<T>(fx4[q].y + pk[q][j].y) * ck[q][j].y;
                    cc[q].z += wgt[q][j] * sigmoid_t<T>(fx4[q].z + pk[q][j].z) * ck[q][j].z;
                    cc[q].w += wgt[q][j] * sigmoid_t<T>(fx4[q].w + pk[q][j].w) * ck[q][j].w;
                }
        }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (node[q] < 0) continue;
        const float c4[4] = {cc[q].x, cc[q].y, cc[q].z, cc[q].w};
        const float o4[4] = {go4[q].x, go4[q].y, go4[q].z, go4[q].w};
        T hv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) hv[j] = from_f32<T>(o4[j] * tanh_t<T>(c4[j]));
        const int64_t nd = node[q];
        if (vec_ok) {
            if (unit0 < a.H) {
                *reinterpret_cast<float4 *>(a.c_out + nd * a.H + unit0) = cc[q];
                if (separate_cs) *reinterpret_cast<float4 *>(a.cs + nd * a.Hq + unit0) = cc[q];
                if constexpr (sizeof(T) == 4) {
                    const float4 h4 = make_float4(hv[0], hv[1], hv[2], hv[3]);
                    *reinterpret_cast<float4 *>(h_out + nd * a.H + unit0) = h4;
                    if (separate_hs) *reinterpret_cast<float4 *>(hs_out + nd * a.Hp + unit0) = h4;
                } else {
                    const uint2 h2 = make_uint2((uint32_t)hv[0] | ((uint32_t)hv[1] << 16),
                                                (uint32_t)hv[2] | ((uint32_t)hv[3] << 16));
                    *reinterpret_cast<uint2 *>(h_out + nd * a.H + unit0) = h2;
                    if (separate_hs) *reinterpret_cast<uint2 *>(hs_out + nd * a.Hp + unit0) = h2;
                }
            } else if (separate_hs && unit0 < a.Hp) {   // zero pad columns of the padded h copy
                if constexpr (sizeof(T) == 4)
                    *reinterpret_cast<float4 *>(hs_out + nd * a.Hp + unit0) = make_float4(0.f, 0.f, 0.f, 0.f);
                else
                    *reinterpret_cast<uint2 *>(hs_out + nd * a.Hp + unit0) = make_uint2(0u, 0u);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int unit = unit0 + j;
                if (unit < a.H) {
                    a.c_out[nd * a.H + unit] = c4[j];
                    if (separate_cs) a.cs[nd * a.Hq + unit] = c4[j];
                    h_out[nd * a.H + unit] = hv[j];
                    if (separate_hs) hs_out[nd * a.Hp + unit] = hv[j];
                } else if (separate_hs && unit < a.Hp) {
                    hs_out[nd * a.Hp + unit] = T(0);
                }
            }
        }
    }
}

template <typename T, int MODE>
__global__ void __launch_bounds__(kGemmThreads, 1)
level_kernel(const LevelArgs a) {
    __shared__ __attribute__((aligned(16))) char lds[2 * (kBM + kBN) * kLdsStride];
    static_assert(8 * 3 * 32 * kEpiStride * 4 <= 2 * (kBM + kBN) * kLdsStride, "epilogue regions must fit the staging buffers");
    static_assert(kEpiRows * kProjStride * 4 <= 2 * (kBM + kBN) * kLdsStride, "projection tile must fit the staging buffers");
    __shared__ int row_node[kBM];
    __shared__ int row_ar[kBM];     // number of children
    __shared__ int row_cb[kBM];     // start of the child list in child_idx
    __shared__ int4 row_kid[kBM];   // first four child ids

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int hf = lane >> 5, l32 = lane & 31;

    const int logical = xcd_remap(blockIdx.x, a.n_blocks);
    const int row_tile = logical / a.n_col_tiles;
    const int col_tile = logical % a.n_col_tiles;
    const int tile_row0 = row_tile * kBM;

    // Per-row data of the tile: requested now, written to LDS by publish_rows().
    int node_reg = -1;
    int4 rec0 = make_int4(-1, 0, 0, 0), rec1 = make_int4(-1, -1, -1, -1);
    if (t < kBM && tile_row0 + t < a.n_rows) {
        if constexpr (MODE == MODE_INTERNAL) {
            rec0 = a.row_rec[2 * (int64_t)(tile_row0 + t)];
            rec1 = a.row_rec[2 * (int64_t)(tile_row0 + t) + 1];
        } else {
            node_reg = a.level_nodes[tile_row0 + t];
        }
    }
    auto publish_rows = [&]() __attribute__((always_inline)) {
        if (t < kBM) {
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

    if constexpr (MODE == MODE_PROJ) {
        // the projection gathers its A rows by node id, so the ids must be in LDS first
        publish_rows();
        __syncthreads();
    }
    if constexpr (MODE == MODE_PROJ)
        block_gemm<T, MODE>(a, lds, row_node, tile_row0, col_tile, acc, []() {});
    else
        block_gemm<T, MODE>(a, lds, row_node, tile_row0, col_tile, acc, publish_rows);

    // ---- epilogue: accumulator element v of tile (i, g) is row
    //      wm*64 + i*32 + (v/4)*8 + hf*4 + v%4, column l32 of gate / unit tile g
    if constexpr (MODE == MODE_PROJ) {
        // P rows leave through LDS too (two passes of 128 rows, fp32 in LDS), so that a
        // thread stores eight consecutive units of one row: 32 lanes cover 256 units.
        float *sp = reinterpret_cast<float *>(lds);
        T *P = static_cast<T *>(a.P);
        const int u8 = (t & 31) * 8;
        const int unit0 = col_tile * 256 + u8;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            __syncthreads();
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rl = wm * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
                    sp[rl * kProjStride + wn * 128 + g * 32 + l32] = acc[p][g][v];
                }
            __syncthreads();
#pragma unroll
            for (int sweep = 0; sweep < 8; ++sweep) {
                const int rl = (t >> 5) + 16 * sweep;
                const int node = row_node[(rl >> 5) * 64 + p * 32 + (rl & 31)];
                if (node < 0 || unit0 >= a.H) continue;
                const float4 lo = *reinterpret_cast<const float4 *>(sp + rl * kProjStride + u8);
                const float4 hi = *reinterpret_cast<const float4 *>(sp + rl * kProjStride + u8 + 4);
                const float f[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                T *dst = P + (int64_t)node * a.Hq + unit0;
                if (unit0 + 8 <= a.H) {
                    if constexpr (sizeof(T) == 4) {
                        *reinterpret_cast<float4 *>(dst) = lo;
                        *reinterpret_cast<float4 *>(dst + 4) = hi;
                    } else {
                        uint4 o;
                        o.x = (uint32_t)f32_to_bf16(f[0]) | ((uint32_t)f32_to_bf16(f[1]) << 16);
                        o.y = (uint32_t)f32_to_bf16(f[2]) | ((uint32_t)f32_to_bf16(f[3]) << 16);
                        o.z = (uint32_t)f32_to_bf16(f[4]) | ((uint32_t)f32_to_bf16(f[5]) << 16);
                        o.w = (uint32_t)f32_to_bf16(f[6]) | ((uint32_t)f32_to_bf16(f[7]) << 16);
                        *reinterpret_cast<uint4 *>(dst) = o;
                    }
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (unit0 + j < a.H) dst[j] = from_f32<T>(f[j]);
                }
            }
        }
    } else {
        // The cell update runs wave by wave (cell_pass): each wave owns 64 rows x 32 units of
        // the tile and a private LDS region (the staging buffers are free now), and handles
        // them in two passes of 32 rows.  Apart from the one barrier that retires the main
        // loop the waves do not wait for each other, so the arithmetic of one overlaps the
        // memory latency of the others.
        float *region = reinterpret_cast<float *>(lds) + wave * (3 * 32 * kEpiStride);
        __syncthreads();   // every wave is done reading the staging buffers
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int r0 = wm * 64 + p * 32;
            cell_pass<T, MODE>(a, acc[p], region, row_node + r0, row_ar + r0, row_cb + r0, row_kid + r0,
                               col_tile * 2 + wn, lane);
        }
    }
}

// ---- thin levels ---------------------------------------------------------------------
// A level with a few thousand rows gives the 256 x 256 tiles too few blocks to fill 256
// CUs, and each block then runs one wave's whole K loop back to back: the level costs that
// latency, not its work.  thin_kernel spreads such a level over many more waves.  Every
// wave owns one tile of 32 rows x 32 hidden units (all four gates; the projection: 32 rows
// x 4 unit tiles of forget rows), takes its MFMA operands straight from global memory /
// L2 in fragment layout (16 bytes per lane, no LDS staging, four K groups requested
// ahead), and finishes with the same cell_pass.  Waves never wait for each other.
constexpr int kThinWaves = 4;     // waves (tiles) per block
#ifndef JITDB_THIN_MAX_ROWS
#define JITDB_THIN_MAX_ROWS 8192
#endif
constexpr int kThinMaxRows = JITDB_THIN_MAX_ROWS; // levels up to this many rows use the thin kernel
constexpr int kThinAhead = 4;     // K groups in flight per wave

template <typename T, int MODE>
__global__ void __launch_bounds__(kThinWaves * 64, 2)
thin_kernel(const LevelArgs a) {
    constexpr int ESZ = (int)sizeof(T);
    constexpr int NG_X = (MODE == MODE_LEAF) ? 3 : 4;
    __shared__ __attribute__((aligned(16))) float regions[kThinWaves][3 * 32 * kEpiStride];
    __shared__ int s_node[kThinWaves][32];
    __shared__ int s_ar[kThinWaves][32];
    __shared__ int s_cb[kThinWaves][32];
    __shared__ int4 s_kid[kThinWaves][32];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int hf = lane >> 5, l32 = lane & 31;
    const int tile = blockIdx.x * kThinWaves + wave;
    if (tile >= a.n_tiles) return;            // whole waves leave; there is no block barrier below
    const int row0 = (tile / a.n_col_tiles) * 32;
    const int col = tile % a.n_col_tiles;     // unit tile (gates) or group of four unit tiles (projection)

    // ---- the tile's rows
    int my_row = row0 + l32;
    const bool row_ok = my_row < a.n_rows;
    if (!row_ok) my_row = a.n_rows - 1;       // computed twice, stored never
    int my_node;
    if constexpr (MODE == MODE_INTERNAL) {
        const int4 r0 = a.row_rec[2 * (int64_t)my_row];
        const int4 r1 = a.row_rec[2 * (int64_t)my_row + 1];
        my_node = r0.x;
        if (hf == 0) {
            s_node[wave][l32] = row_ok ? r0.x : -1;
            s_ar[wave][l32] = row_ok ? r0.y : 0;
            s_cb[wave][l32] = r0.z;
            s_kid[wave][l32] = r1;
        }
    } else {
        my_node = a.level_nodes[my_row];
        if (hf == 0) s_node[wave][l32] = row_ok ? my_node : -1;
    }

    // ---- operand addresses: lane (l32, hf) supplies row l32, bytes [hf*16, +16) of each
    //      32-byte K group, for A and for every B row group alike
    const int64_t b_row_bytes = (int64_t)(a.Dp + a.Hp) * ESZ;
    const char *ap, *bp;
    int64_t b_step;
    int n_groups, n_groups_x;                 // K groups in total / with all four gates
    if constexpr (MODE == MODE_PROJ) {
        ap = static_cast<const char *>(a.hs) + (int64_t)my_node * a.Hp * ESZ + hf * 16;
        const int64_t row = (int64_t)(col * 4) * kGateTile + 3 * kUnit + l32;
        bp = static_cast<const char *>(a.Bp) + row * b_row_bytes + (int64_t)a.Dp * ESZ + hf * 16;
        b_step = (int64_t)kGateTile * b_row_bytes;
        n_groups = a.Hp * ESZ / 32;
        n_groups_x = n_groups;
    } else {
        const int64_t a_row_bytes = (int64_t)(a.Dp + (MODE == MODE_INTERNAL ? a.Hp : 0)) * ESZ;
        ap = static_cast<const char *>(a.stack) + (int64_t)my_row * a_row_bytes + hf * 16;
        const int64_t row = (int64_t)col * kGateTile + l32;
        bp = static_cast<const char *>(a.Bp) + row * b_row_bytes + hf * 16;
        b_step = (int64_t)kUnit * b_row_bytes;
        n_groups_x = a.Dp * ESZ / 32;
        n_groups = (int)(a_row_bytes / 32);
    }

    floatx16 acc[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[g][v] = 0.0f;

    u32x4 fa[kThinAhead], fb[kThinAhead][4];
    auto request = [&](int g, int slot) __attribute__((always_inline)) {
        const int64_t kb = (int64_t)g * 32;
        fa[slot] = *reinterpret_cast<const u32x4 *>(ap + kb);
#pragma unroll
        for (int q = 0; q < NG_X; ++q) fb[slot][q] = *reinterpret_cast<const u32x4 *>(bp + q * b_step + kb);
    };
#pragma unroll
    for (int s = 0; s < kThinAhead; ++s)
        if (s < n_groups) request(s, s);
    for (int g0 = 0; g0 < n_groups; g0 += kThinAhead) {
#pragma unroll
        for (int s = 0; s < kThinAhead; ++s) {
            const int g = g0 + s;
            if (g < n_groups) {
                mfma_step<T>(fa[s], fb[s][0], acc[0]);
                mfma_step<T>(fa[s], fb[s][1], acc[1]);
                mfma_step<T>(fa[s], fb[s][2], acc[2]);
                // the forget rows take part in the x part only (and in all of the projection)
                if (NG_X == 4 && (MODE != MODE_INTERNAL || g < n_groups_x)) mfma_step<T>(fa[s], fb[s][3], acc[3]);
                if (g + kThinAhead < n_groups) request(g + kThinAhead, s);
            }
        }
    }

    if constexpr (MODE == MODE_PROJ) {
        T *P = static_cast<T *>(a.P);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int unit = (col * 4 + q) * kUnit + l32;
            if (unit >= a.H) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = row0 + (v >> 2) * 8 + hf * 4 + (v & 3);
                if (r < a.n_rows) {
                    const int node = a.level_nodes[r];
                    P[(int64_t)node * a.Hq + unit] = from_f32<T>(acc[q][v]);
                }
            }
        }
    } else {
        // the row data written above is read by this wave only
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        cell_pass<T, MODE>(a, acc, regions[wave], s_node[wave], s_ar[wave], s_cb[wave], s_kid[wave], col, lane);
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
};
Profiler g_prof;

struct ScopedLaunchTimer {
    int slot = -1;
    hipStream_t st;
    ScopedLaunchTimer(int kernel_class, hipStream_t s) : st(s) {
        if (!g_prof.on) return;
        if (g_prof.used >= g_prof.capacity) { ++g_prof.dropped; return; }
        slot = g_prof.used++;
        g_prof.cls[slot] = kernel_class;
        (void)hipEventRecord(g_prof.begin[slot], st);
    }
    ~ScopedLaunchTimer() {
        if (slot >= 0) (void)hipEventRecord(g_prof.end[slot], st);
    }
};

struct ForwardWs {
    void *Bp;
    float *bp;
    void *stack;  // the current level's stacked input, (N + 256) rows of Dp + Hp
    int4 *row_rec; // row records of all level positions, two int4 each
    void *hs;     // nullptr when h_out can serve (H == Hp)
    void *P;
    float *cs;    // nullptr when c_out can serve (H == Hq)
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

ForwardWs carve_forward_ws(int64_t n, int64_t e, const Dims &d, void *base) {
    Carver c(base);
    ForwardWs w;
    (void)e;
    w.Bp = c.take<char>((size_t)d.NPU * (d.Dp + d.Hp) * d.esz);
    w.bp = c.take<float>(d.NP);
    // one level at a time; whole row tiles are read, hence the 256 spare rows
    w.stack = c.take<char>((size_t)(n + kBM) * (d.Dp + d.Hp) * d.esz);
    w.row_rec = c.take<int4>((size_t)2 * (n + kBM));   // every level position
    w.hs = (d.H == d.Hp) ? nullptr : c.take<char>((size_t)n * d.Hp * d.esz);
    w.P = c.take<char>((size_t)n * d.Hq * d.esz);
    w.cs = (d.H == d.Hq) ? nullptr : c.take<float>((size_t)n * d.Hq);
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

template <typename T>
int run_forward(const void *x, const void *W, const void *U, const float *b, const Dims &d,
                const jitdb_schedule_t *s, void *h_out, float *c_out, const ForwardWs &w,
                hipStream_t st) {
    const int L = s->n_levels;
    const int32_t *lp = s->host_level_ptr;

    {
        const int64_t total = (int64_t)d.NPU * (d.Dp + d.Hp);
        const unsigned grid = (unsigned)(ceil_div(total, kThreads) < 4096 ? ceil_div(total, kThreads) : 4096);
        ScopedLaunchTimer tm(JITDB_K_PACK, st);
        pack_weights_kernel<T><<<grid, kThreads, 0, st>>>(
            static_cast<const T *>(W), static_cast<const T *>(U), b, d.D, d.H, d.Dp, d.Hp, d.NP, d.NPU,
            static_cast<T *>(w.Bp), w.bp);
        JITDB_LAUNCH_CHECK();
    }

    {
        ScopedLaunchTimer tm(JITDB_K_PACK, st);
        row_record_kernel<<<(unsigned)ceil_div(s->n_nodes, kThreads), kThreads, 0, st>>>(
            s->perm, s->child_ptr, s->child_idx, w.row_rec, (int)s->n_nodes);
        JITDB_LAUNCH_CHECK();
    }

    LevelArgs a;
    a.stack = w.stack;
    a.hs = w.hs ? w.hs : h_out;
    a.Bp = w.Bp; a.bp = w.bp;
    a.child_idx = s->child_idx;

    a.P = w.P; a.c_out = c_out; a.h_out = h_out;
    a.cs = w.cs ? w.cs : c_out;
    a.Hq = d.Hq;
    a.hs_out = w.hs ? w.hs : h_out;
    a.D = d.D; a.Dp = d.Dp; a.H = d.H; a.Hp = d.Hp; a.Hu = d.Hu;

    for (int l = 0; l < L; ++l) {
        const int n_rows = lp[l + 1] - lp[l];
        if (n_rows <= 0) return JITDB_E_SCHEDULE;
        a.level_nodes = s->perm + lp[l];
        a.row_rec = w.row_rec + 2 * (int64_t)lp[l];
        a.n_rows = n_rows;
        const int row_tiles = (int)ceil_div(n_rows, kBM);
        {   // stack: gather the level's x rows and child sums into one dense matrix
            const int Kp = d.Dp + (l > 0 ? d.Hp : 0);
            const int64_t pieces = (int64_t)n_rows * (Kp / Traits<T>::VEC);
            const unsigned grid = (unsigned)ceil_div(pieces, kThreads);
            ScopedLaunchTimer tm(JITDB_K_STACK, st);
            if (l == 0)
                stack_kernel<T, false><<<grid, kThreads, 0, st>>>(
                    static_cast<const T *>(x), d.D, d.Dp, static_cast<const T *>(a.hs), d.Hp, a.row_rec,
                    s->child_idx, static_cast<T *>(w.stack), n_rows);
            else
                stack_kernel<T, true><<<grid, kThreads, 0, st>>>(
                    static_cast<const T *>(x), d.D, d.Dp, static_cast<const T *>(a.hs), d.Hp, a.row_rec,
                    s->child_idx, static_cast<T *>(w.stack), n_rows);
            JITDB_LAUNCH_CHECK();
        }
        // Levels too small to give every CU a 256 x 256 tile go to the thin kernel.
        const bool thin = n_rows <= kThinMaxRows;
        const int n_unit_tiles = d.Hu / kUnit;
        if (thin) {
            a.n_col_tiles = n_unit_tiles;
            a.n_tiles = (int)ceil_div(n_rows, 32) * a.n_col_tiles;
            a.n_blocks = (int)ceil_div(a.n_tiles, kThinWaves);
        } else {
            a.n_col_tiles = d.NP / kBN;
            a.n_tiles = 0;
            a.n_blocks = row_tiles * a.n_col_tiles;
        }
        {
            ScopedLaunchTimer tm(l == 0 ? JITDB_K_LEAF : JITDB_K_INTERNAL, st);
            if (thin) {
                if (l == 0)
                    thin_kernel<T, MODE_LEAF><<<a.n_blocks, kThinWaves * 64, 0, st>>>(a);
                else
                    thin_kernel<T, MODE_INTERNAL><<<a.n_blocks, kThinWaves * 64, 0, st>>>(a);
            } else {
                if (l == 0)
                    level_kernel<T, MODE_LEAF><<<a.n_blocks, kGemmThreads, 0, st>>>(a);
                else
                    level_kernel<T, MODE_INTERNAL><<<a.n_blocks, kGemmThreads, 0, st>>>(a);
            }
        }
        JITDB_LAUNCH_CHECK();
        if (l + 1 < L) {   // these nodes have parents (except roots, whose rows go unused)
            ScopedLaunchTimer tm(JITDB_K_PROJ, st);
            if (thin) {
                a.n_col_tiles = (int)ceil_div(n_unit_tiles, 4);
                a.n_tiles = (int)ceil_div(n_rows, 32) * a.n_col_tiles;
                a.n_blocks = (int)ceil_div(a.n_tiles, kThinWaves);
                thin_kernel<T, MODE_PROJ><<<a.n_blocks, kThinWaves * 64, 0, st>>>(a);
            } else {
                a.n_col_tiles = (int)ceil_div(n_unit_tiles, 8);
                a.n_blocks = row_tiles * a.n_col_tiles;
                level_kernel<T, MODE_PROJ><<<a.n_blocks, kGemmThreads, 0, st>>>(a);
            }
        }
        JITDB_LAUNCH_CHECK();
    }
    return JITDB_OK;
}

}  // namespace
}  // namespace jitdb

using namespace jitdb;

extern "C" int jitdb_profile_start(int32_t capacity) {
    if (capacity < 1 || capacity > (1 << 20)) return JITDB_E_BADARG;
    if (g_prof.on) return JITDB_E_BADARG;
    g_prof.begin = new hipEvent_t[capacity];
    g_prof.end = new hipEvent_t[capacity];
    g_prof.cls = new int[capacity];
    for (int i = 0; i < capacity; ++i) {
        if (hipEventCreate(&g_prof.begin[i]) != hipSuccess || hipEventCreate(&g_prof.end[i]) != hipSuccess)
            return JITDB_E_HIP;
    }
    g_prof.capacity = capacity;
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
    for (int c = 0; c < JITDB_K_CLASSES; ++c) { out->ms[c] = 0.0; out->launches[c] = 0; }
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
    }
    for (int i = 0; i < g_prof.capacity; ++i) {
        (void)hipEventDestroy(g_prof.begin[i]);
        (void)hipEventDestroy(g_prof.end[i]);
    }
    delete[] g_prof.begin; delete[] g_prof.end; delete[] g_prof.cls;
    g_prof = Profiler();
    return rc;
}

extern "C" size_t jitdb_treelstm_workspace_bytes(int64_t n_nodes, int64_t n_edges,
                                                 int32_t D, int32_t H, jitdb_dtype dtype) {
    if (!dims_ok(n_nodes, n_edges, D, H, (int)dtype)) return 0;
    const Dims d = make_dims(D, H, dtype);
    return carve_forward_ws(n_nodes, n_edges, d, nullptr).bytes;
}

extern "C" int jitdb_treelstm_forward(const void *x, const void *W, const void *U, const float *b,
                                      int32_t D, int32_t H, jitdb_dtype dtype,
                                      const jitdb_schedule_t *s, void *h_out, float *c_out,
                                      void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!s) return JITDB_E_NULL;
    drop_stale_hip_error();
    const int64_t n = s->n_nodes;
    if (!dims_ok(n, s->n_edges, D, H, (int)dtype)) return JITDB_E_BADARG;
    if (n == 0) return JITDB_OK;
    if (!x || !W || !U || !b || !h_out || !c_out || !workspace) return JITDB_E_NULL;
    if (!s->perm || !s->child_ptr || !s->child_idx || !s->host_level_ptr) return JITDB_E_NULL;
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

    const Dims d = make_dims(D, H, dtype);
    const ForwardWs w = carve_forward_ws(n, s->n_edges, d, workspace);
    if (workspace_bytes < w.bytes) return JITDB_E_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    if (dtype == JITDB_F32)
        return run_forward<float>(x, W, U, b, d, s, h_out, c_out, w, st);
    return run_forward<bf16_t>(x, W, U, b, d, s, h_out, c_out, w, st);
}
