// jitdb_treelstm_forward: the execution half of the method for gfx950.
//
// The paper runs the look-up table slot by slot in depth order; per slot it
// stacks the samples, runs the shared subgraph once and slices the results
// (section 4.3).  Here a slot is one height level of the forest and the
// subgraph is the Child-Sum Tree-LSTM cell (section 3).  Per level:
//
//   child_sum_kernel   hs_j = sum_k h_k over the child CSR (the arity-dependent
//                      operator; HBM-bound, 16-byte coalesced row pieces)
//   level_kernel<GATES>   [x_j ; hs_j] x [W ; U]^T on MFMA with the whole cell
//                      fused into the epilogue: per-child forget gates from the
//                      precomputed P_k = U_f h_k, c_j and h_j written once
//   level_kernel<PROJ> P_k = U_f h_k for the nodes just produced, so that their
//                      parent reads one row per child (every non-root node is a
//                      child exactly once)
//
// "Stack" is a row gather through perm (level-major order), "slice" is the
// scatter of rows back to node-id order in the epilogue.
//
// Weights are re-packed once per call: gate rows of 32 hidden units are
// interleaved (i|o|u|f blocks of 32 rows), so that one wave holds all four
// gates of a hidden unit in its own accumulators and the cell update needs no
// exchange between lanes; rows and K are zero padded to tile multiples.

#include "common.h"

namespace jitdb {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t bf16_t;  // storage type of bfloat16 values

constexpr int kThreads = 256;
constexpr int kBM = 128;        // rows (nodes) per block
constexpr int kBN = 256;        // packed columns per block = 2 unit tiles x 4 gates x 32
constexpr int kUnit = 32;       // hidden units per MFMA column tile
constexpr int kGateTile = 128;  // packed rows per unit tile (4 gates x 32 units)

constexpr int kLdsStride = 80;  // stage row + 16 bytes: 128-bit LDS reads of 32 rows hit distinct banks
constexpr int kKPad = 32;       // D and H are padded to multiples of this many elements

enum : int { MODE_LEAF = 0, MODE_INTERNAL = 1, MODE_PROJ = 2 };

template <typename T> struct Traits;
template <> struct Traits<float> {
    static constexpr int BK = 16;   // elements of K per stage
    static constexpr int VEC = 4;   // elements per 16 bytes
};
template <> struct Traits<bf16_t> {
    static constexpr int BK = 32;
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

template <typename T> __device__ __forceinline__ float sigmoid_t(float z) {
    return 1.0f / (1.0f + exp_t<T>(-z));
}
template <typename T> __device__ __forceinline__ float tanh_t(float z) {
    return 1.0f - 2.0f / (1.0f + exp_t<T>(2.0f * z));
}

// ---- weight packing ----------------------------------------------------------------
// Packed row r = tile*128 + gate*32 + uu holds gate `gate` of hidden unit tile*32 + uu.
template <typename T>
__global__ void __launch_bounds__(kThreads)
pack_weights_kernel(const T *__restrict__ W, const T *__restrict__ U, const float *__restrict__ b,
                    int D, int H, int Dp, int Hp, int NP,
                    T *__restrict__ Wp, T *__restrict__ Up, float *__restrict__ bp) {
    const int64_t total = (int64_t)NP * (Dp + Hp);
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * kThreads) {
        const int r = (int)(idx / (Dp + Hp));
        const int k = (int)(idx % (Dp + Hp));
        const int tile = r / kGateTile, gate = (r % kGateTile) / kUnit, uu = r % kUnit;
        const int unit = tile * kUnit + uu;
        const bool row_ok = unit < H;
        const int64_t src = (int64_t)gate * H + unit;
        if (k < Dp) {
            Wp[(int64_t)r * Dp + k] = (row_ok && k < D) ? W[src * D + k] : T(0);
        } else {
            const int kk = k - Dp;
            Up[(int64_t)r * Hp + kk] = (row_ok && kk < H) ? U[src * H + kk] : T(0);
        }
        if (k == 0) bp[r] = row_ok ? b[src] : 0.0f;
    }
}

// ---- child sum ---------------------------------------------------------------------
// hsum[row] = sum over children of hs[child]; one thread per 16-byte piece of a row.
// hs rows have stride Hp (pad columns are zero), rows indexed by node id.
template <typename T>
__global__ void __launch_bounds__(kThreads)
child_sum_kernel(const T *__restrict__ hs, int Hp, const int32_t *__restrict__ level_nodes,
                 const int32_t *__restrict__ child_ptr, const int32_t *__restrict__ child_idx,
                 T *__restrict__ hsum, int n_rows) {
    constexpr int VEC = Traits<T>::VEC;
    const int cpr = Hp / VEC;
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t row = gid / cpr;
    const int ch = (int)(gid % cpr);
    if (row >= n_rows) return;
    const int node = level_nodes[row];
    const int cb = child_ptr[node], ce = child_ptr[node + 1];
    float acc[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = 0.0f;
    for (int e = cb; e < ce; ++e) {
        const int k = child_idx[e];
        const uint4 v = *reinterpret_cast<const uint4 *>(hs + (int64_t)k * Hp + ch * VEC);
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
    uint4 o;
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
    *reinterpret_cast<uint4 *>(hsum + row * Hp + ch * VEC) = o;
}

// ---- the level GEMM ----------------------------------------------------------------
struct LevelArgs {
    // A operands
    const void *x;        // [N, D] rows by node id
    const void *hsum;     // [n_rows, Hp] level-local rows (MODE_INTERNAL)
    const void *hs;       // [N, Hp] rows by node id (MODE_PROJ)
    // B operands (packed)
    const void *Wp;       // [NP, Dp]
    const void *Up;       // [NP, Hp]
    const float *bp;      // [NP]
    // schedule
    const int32_t *level_nodes;  // perm + level start: row -> node id
    const int32_t *child_ptr;
    const int32_t *child_idx;
    // per-child forget projections, rows by node id, stride H
    float *P;
    // outputs
    float *c_out;         // [N, H]
    void *h_out;          // [N, H]
    void *hs_out;         // [N, Hp] or == h_out when H == Hp
    int D, Dp, H, Hp, Hu;
    int n_rows;
    int n_col_tiles;      // blocks along the packed-column axis
    int n_blocks;
};

// How a block's A rows are fetched for one K phase.
enum : int { A_X = 0, A_HSUM = 1, A_HS = 2 };


// Spread consecutive block ids (which the hardware deals round-robin to the 8
// XCDs) so that blocks sharing an A row tile land on the same XCD and L2.
__device__ __forceinline__ int xcd_remap(int b, int nb) {
    const int xcd = b & 7, idx = b >> 3;
    const int q = nb >> 3, r = nb & 7;
    return xcd * q + (xcd < r ? xcd : r) + idx;
}

template <typename T>
__device__ __forceinline__ void mfma_step(const uint4 &a, const uint4 &b, floatx16 &acc) {
    if constexpr (sizeof(T) == 2) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                      __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
    }
}

// One K phase of the block GEMM: acc[i][g] += A_tile x B_tile^T over k in [0, Kp).
//   A_KIND  where A rows come from (see above); B rows come from `Bsrc` (row stride Kp)
//   NG      number of 32-column tiles of B each wave multiplies (gate tiles 0..NG-1)
// LDS layout per stage: row r at r*kLdsStride, K contiguous.  In each 16-wide
// (bf16) or 8-wide (fp32) K group, lanes 0-31 take the first 16 bytes and
// lanes 32-63 the next 16 for A and B alike; since the same assignment is
// used on both operands any such split of K is a valid MFMA schedule.
template <typename T, int A_KIND, int NG>
__device__ __forceinline__ void gemm_phase(const LevelArgs &a, char *lds_a, char *lds_b,
                                           const int *row_node, int tile_row0, int Kp,
                                           const T *Bsrc, const int (&b_rows)[4], const bool (&b_need)[4],
                                           floatx16 (&acc)[2][4]) {
    constexpr int BK = Traits<T>::BK;
    constexpr int VEC = Traits<T>::VEC;
    // A chunks: X phase uses 4-element pieces (x rows are only 4-element aligned), others 16 bytes
    constexpr int A_CH_ELEMS = (A_KIND == A_X) ? 4 : VEC;
    constexpr int A_CH_BYTES = A_CH_ELEMS * (int)sizeof(T);
    constexpr int A_CPR = BK / A_CH_ELEMS;                 // chunks per row per stage
    constexpr int A_PER_THREAD = kBM * A_CPR / kThreads;   // 2 or 4
    constexpr int B_CPR = BK / VEC;                        // 4
    constexpr int B_PER_THREAD = kBN * B_CPR / kThreads;   // 4

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int hf = lane >> 5, l32 = lane & 31;

    // per-thread A sources
    const T *a_ptr[A_PER_THREAD];
    int a_lds[A_PER_THREAD];
    int a_k[A_PER_THREAD];
#pragma unroll
    for (int i = 0; i < A_PER_THREAD; ++i) {
        const int c = t + i * kThreads;
        const int r = c / A_CPR, ch = c % A_CPR;
        a_lds[i] = r * kLdsStride + ch * A_CH_BYTES;
        a_k[i] = ch * A_CH_ELEMS;
        const int grow = tile_row0 + r;
        if (grow < a.n_rows) {
            if constexpr (A_KIND == A_X)
                a_ptr[i] = static_cast<const T *>(a.x) + (int64_t)row_node[r] * a.D + a_k[i];
            else if constexpr (A_KIND == A_HSUM)
                a_ptr[i] = static_cast<const T *>(a.hsum) + (int64_t)grow * a.Hp + a_k[i];
            else
                a_ptr[i] = static_cast<const T *>(a.hs) + (int64_t)row_node[r] * a.Hp + a_k[i];
        } else {
            a_ptr[i] = nullptr;
        }
    }
    const T *b_ptr[B_PER_THREAD];
    int b_lds[B_PER_THREAD];
#pragma unroll
    for (int i = 0; i < B_PER_THREAD; ++i) {
        const int c = t + i * kThreads;
        const int r = c / B_CPR, ch = c % B_CPR;   // r = t/4 + 64 i
        b_lds[i] = r * kLdsStride + ch * 16;
        b_ptr[i] = Bsrc + (int64_t)b_rows[i] * Kp + ch * VEC;
    }

    uint4 a_reg[A_PER_THREAD];
    uint4 b_reg[B_PER_THREAD];
    const int k_limit = (A_KIND == A_X) ? a.D : Kp;

    auto load_global = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) {
            uint4 v = make_uint4(0, 0, 0, 0);
            if (a_ptr[i] != nullptr && (k0 + a_k[i]) < k_limit) {
                if constexpr (A_CH_BYTES == 16) {
                    v = *reinterpret_cast<const uint4 *>(a_ptr[i] + k0);
                } else {
                    const uint2 w = *reinterpret_cast<const uint2 *>(a_ptr[i] + k0);
                    v.x = w.x; v.y = w.y;
                }
            }
            a_reg[i] = v;
        }
#pragma unroll
        for (int i = 0; i < B_PER_THREAD; ++i)
            if (b_need[i]) b_reg[i] = *reinterpret_cast<const uint4 *>(b_ptr[i] + k0);
    };
    auto store_lds = [&](int buf) {
        char *sa = lds_a + buf * (kBM * kLdsStride);
        char *sb = lds_b + buf * (kBN * kLdsStride);
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) {
            if constexpr (A_CH_BYTES == 16)
                *reinterpret_cast<uint4 *>(sa + a_lds[i]) = a_reg[i];
            else
                *reinterpret_cast<uint2 *>(sa + a_lds[i]) = make_uint2(a_reg[i].x, a_reg[i].y);
        }
#pragma unroll
        for (int i = 0; i < B_PER_THREAD; ++i)
            if (b_need[i]) *reinterpret_cast<uint4 *>(sb + b_lds[i]) = b_reg[i];
    };

    const int a_rd = (wm * 64 + l32) * kLdsStride + hf * 16;
    const int b_rd = (wn * 128 + l32) * kLdsStride + hf * 16;
    auto compute = [&](int buf) {
        const char *sa = lds_a + buf * (kBM * kLdsStride) + a_rd;
        const char *sb = lds_b + buf * (kBN * kLdsStride) + b_rd;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            uint4 av[2], bv[NG];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                av[i] = *reinterpret_cast<const uint4 *>(sa + i * 32 * kLdsStride + s * 32);
#pragma unroll
            for (int g = 0; g < NG; ++g)
                bv[g] = *reinterpret_cast<const uint4 *>(sb + g * 32 * kLdsStride + s * 32);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int g = 0; g < NG; ++g) mfma_step<T>(av[i], bv[g], acc[i][g]);
        }
    };

    const int n_kt = Kp / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < n_kt; ++kt) {
        const bool more = (kt + 1) < n_kt;
        if (more) load_global((kt + 1) * BK);
        compute(kt & 1);
        if (more) store_lds((kt + 1) & 1);
        __syncthreads();
    }
}

template <typename T, int MODE>
__global__ void __launch_bounds__(kThreads, 2)
level_kernel(const LevelArgs a) {
    __shared__ __attribute__((aligned(16))) char lds_a[2 * kBM * kLdsStride];
    __shared__ __attribute__((aligned(16))) char lds_b[2 * kBN * kLdsStride];
    __shared__ int row_node[kBM];
    __shared__ int row_cb[kBM];
    __shared__ int row_ce[kBM];

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int hf = lane >> 5, l32 = lane & 31;

    const int logical = xcd_remap(blockIdx.x, a.n_blocks);
    const int row_tile = logical / a.n_col_tiles;
    const int col_tile = logical % a.n_col_tiles;
    const int tile_row0 = row_tile * kBM;

    if (t < kBM) {
        const int grow = tile_row0 + t;
        int node = -1, cb = 0, ce = 0;
        if (grow < a.n_rows) {
            node = a.level_nodes[grow];
            if constexpr (MODE == MODE_INTERNAL) {
                cb = a.child_ptr[node];
                ce = a.child_ptr[node + 1];
            }
        }
        row_node[t] = node;
        row_cb[t] = cb;
        row_ce[t] = ce;
    }
    __syncthreads();

    floatx16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][g][v] = 0.0f;

    // B rows this thread stages: LDS row r = t/4 + 64 i  ->  packed weight row
    int b_rows[4];
    bool need_all[4], need_iou[4];
    const int n_unit_tiles = a.Hu / kUnit;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = (t >> 2) + 64 * i;              // 0..255 within the block's column tile
        if constexpr (MODE == MODE_PROJ) {
            // eight unit tiles of forget rows side by side
            int ut = col_tile * 8 + (r >> 5);
            if (ut >= n_unit_tiles) ut = n_unit_tiles - 1;   // results of such columns are dropped
            b_rows[i] = ut * kGateTile + 3 * kUnit + (r & 31);
            need_all[i] = true;
            need_iou[i] = true;
        } else {
            b_rows[i] = col_tile * kBN + r;
            const bool is_f = (r & 127) >= 3 * kUnit;
            need_all[i] = (MODE == MODE_LEAF) ? !is_f : true;
            need_iou[i] = !is_f;
        }
    }

    if constexpr (MODE == MODE_LEAF) {
        gemm_phase<T, A_X, 3>(a, lds_a, lds_b, row_node, tile_row0, a.Dp,
                              static_cast<const T *>(a.Wp), b_rows, need_all, acc);
    } else if constexpr (MODE == MODE_INTERNAL) {
        gemm_phase<T, A_X, 4>(a, lds_a, lds_b, row_node, tile_row0, a.Dp,
                              static_cast<const T *>(a.Wp), b_rows, need_all, acc);
        gemm_phase<T, A_HSUM, 3>(a, lds_a, lds_b, row_node, tile_row0, a.Hp,
                                 static_cast<const T *>(a.Up), b_rows, need_iou, acc);
    } else {
        gemm_phase<T, A_HS, 4>(a, lds_a, lds_b, row_node, tile_row0, a.Hp,
                               static_cast<const T *>(a.Up), b_rows, need_all, acc);
    }

    // ---- epilogue: accumulator element v of tile (i, g) is row
    //      wm*64 + i*32 + (v/4)*8 + hf*4 + v%4, column l32 of gate / unit tile g
    if constexpr (MODE == MODE_PROJ) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int unit = (col_tile * 8 + wn * 4 + g) * kUnit + l32;
            if (unit >= a.H) continue;
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = wm * 64 + i * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
                    const int node = row_node[r];
                    if (node >= 0) a.P[(int64_t)node * a.H + unit] = acc[i][g][v];
                }
        }
    } else {
        const int unit = (col_tile * 2 + wn) * kUnit + l32;
        const int pcol = col_tile * kBN + wn * kGateTile + l32;   // packed row of gate i for this unit
        const float bi = a.bp[pcol], bo = a.bp[pcol + kUnit], bu = a.bp[pcol + 2 * kUnit];
        float bf = 0.0f;
        if constexpr (MODE == MODE_INTERNAL) bf = a.bp[pcol + 3 * kUnit];
        T *h_out = static_cast<T *>(a.h_out);
        T *hs_out = static_cast<T *>(a.hs_out);
        const bool separate_hs = (a.hs_out != a.h_out);
        if (unit < a.Hp) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int r = wm * 64 + i * 32 + (v >> 2) * 8 + hf * 4 + (v & 3);
                    const int node = row_node[r];
                    if (node < 0) continue;
                    if (unit >= a.H) {   // zero pad column of the padded h copy
                        if (separate_hs) hs_out[(int64_t)node * a.Hp + unit] = T(0);
                        continue;
                    }
                    const float gi = sigmoid_t<T>(acc[i][0][v] + bi);
                    const float go = sigmoid_t<T>(acc[i][1][v] + bo);
                    const float gu = tanh_t<T>(acc[i][2][v] + bu);
                    float cc = gi * gu;
                    if constexpr (MODE == MODE_INTERNAL) {
                        const float fx = acc[i][3][v] + bf;
                        const int cb = row_cb[r], ce = row_ce[r];
                        for (int e = cb; e < ce; ++e) {
                            const int64_t k = a.child_idx[e];
                            const float pk = a.P[k * a.H + unit];
                            const float ck = a.c_out[k * a.H + unit];
                            cc += sigmoid_t<T>(fx + pk) * ck;
                        }
                    }
                    const float hh = go * tanh_t<T>(cc);
                    a.c_out[(int64_t)node * a.H + unit] = cc;
                    const T hv = from_f32<T>(hh);
                    h_out[(int64_t)node * a.H + unit] = hv;
                    if (separate_hs) hs_out[(int64_t)node * a.Hp + unit] = hv;
                }
        }
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
    void *Wp, *Up;
    float *bp;
    void *hsum;
    void *hs;     // nullptr-sized when h_out can serve (H == Hp)
    float *P;
    size_t bytes;
};

struct Dims {
    int D, H, Dp, Hp, Hu, NP;
    size_t esz;
};

Dims make_dims(int D, int H, jitdb_dtype dtype) {
    Dims d;
    d.D = D; d.H = H;
    d.Dp = (int)round_up(D, kKPad);
    d.Hp = (int)round_up(H, kKPad);
    d.Hu = (int)round_up(H, 2 * kUnit);
    d.NP = 4 * d.Hu;
    d.esz = dtype == JITDB_F32 ? 4 : 2;
    return d;
}

ForwardWs carve_forward_ws(int64_t n, int64_t e, const Dims &d, void *base) {
    Carver c(base);
    ForwardWs w;
    const int64_t hsum_rows = e < n ? e : n;   // an internal node has at least one child
    w.Wp = c.take<char>((size_t)d.NP * d.Dp * d.esz);
    w.Up = c.take<char>((size_t)d.NP * d.Hp * d.esz);
    w.bp = c.take<float>(d.NP);
    w.hsum = c.take<char>((size_t)hsum_rows * d.Hp * d.esz);
    w.hs = (d.H == d.Hp) ? nullptr : c.take<char>((size_t)n * d.Hp * d.esz);
    if (d.H == d.Hp) c.take<char>(0);
    w.P = c.take<float>((size_t)n * d.H);
    w.bytes = c.off;
    return w;
}

bool dims_ok(int64_t n, int64_t e, int32_t D, int32_t H, int dtype) {
    if (n < 0 || n > JITDB_MAX_NODES || e < 0 || e > n) return false;
    if (D < 1 || D > (1 << 16) || (D % 4) != 0) return false;
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
        const int64_t total = (int64_t)d.NP * (d.Dp + d.Hp);
        const unsigned grid = (unsigned)(ceil_div(total, kThreads) < 4096 ? ceil_div(total, kThreads) : 4096);
        ScopedLaunchTimer tm(JITDB_K_PACK, st);
        pack_weights_kernel<T><<<grid, kThreads, 0, st>>>(
            static_cast<const T *>(W), static_cast<const T *>(U), b, d.D, d.H, d.Dp, d.Hp, d.NP,
            static_cast<T *>(w.Wp), static_cast<T *>(w.Up), w.bp);
        JITDB_LAUNCH_CHECK();
    }

    LevelArgs a;
    a.x = x; a.hsum = w.hsum;
    a.hs = w.hs ? w.hs : h_out;
    a.Wp = w.Wp; a.Up = w.Up; a.bp = w.bp;
    a.child_ptr = s->child_ptr; a.child_idx = s->child_idx;
    a.P = w.P; a.c_out = c_out; a.h_out = h_out;
    a.hs_out = w.hs ? w.hs : h_out;
    a.D = d.D; a.Dp = d.Dp; a.H = d.H; a.Hp = d.Hp; a.Hu = d.Hu;

    for (int l = 0; l < L; ++l) {
        const int n_rows = lp[l + 1] - lp[l];
        if (n_rows <= 0) return JITDB_E_SCHEDULE;
        a.level_nodes = s->perm + lp[l];
        a.n_rows = n_rows;
        const int row_tiles = (int)ceil_div(n_rows, kBM);
        if (l > 0) {
            const int64_t pieces = (int64_t)n_rows * (d.Hp / Traits<T>::VEC);
            ScopedLaunchTimer tm(JITDB_K_CHILD_SUM, st);
            child_sum_kernel<T><<<(unsigned)ceil_div(pieces, kThreads), kThreads, 0, st>>>(
                static_cast<const T *>(a.hs), d.Hp, a.level_nodes, s->child_ptr, s->child_idx,
                static_cast<T *>(w.hsum), n_rows);
            JITDB_LAUNCH_CHECK();
        }
        a.n_col_tiles = d.NP / kBN;
        a.n_blocks = row_tiles * a.n_col_tiles;
        {
            ScopedLaunchTimer tm(l == 0 ? JITDB_K_LEAF : JITDB_K_INTERNAL, st);
            if (l == 0)
                level_kernel<T, MODE_LEAF><<<a.n_blocks, kThreads, 0, st>>>(a);
            else
                level_kernel<T, MODE_INTERNAL><<<a.n_blocks, kThreads, 0, st>>>(a);
        }
        JITDB_LAUNCH_CHECK();
        if (l + 1 < L) {   // these nodes have parents (except roots, whose rows go unused)
            a.n_col_tiles = (int)ceil_div(d.Hu / kUnit, 8);
            a.n_blocks = row_tiles * a.n_col_tiles;
            {
                ScopedLaunchTimer tm(JITDB_K_PROJ, st);
                level_kernel<T, MODE_PROJ><<<a.n_blocks, kThreads, 0, st>>>(a);
            }
            JITDB_LAUNCH_CHECK();
        }
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
    const size_t esz = dtype == JITDB_F32 ? 4 : 2;
    // row pieces are fetched 4 elements at a time (x) and 16 bytes at a time (h when H is unpadded)
    if ((reinterpret_cast<uintptr_t>(x) % (4 * esz)) != 0) return JITDB_E_BADARG;
    if ((reinterpret_cast<uintptr_t>(h_out) & 15) != 0) return JITDB_E_BADARG;
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
