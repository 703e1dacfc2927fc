// Device-side pieces shared by the level kernels (forward.hip: 128 x 256 tiles, two blocks per CU,
// fp32 and bf16, training and typed variants; level256.hip: 256 x 256 tiles, one block per CU, bf16):
// operand types, the arguments of one level launch, and the fused cell update of one wave.
#pragma once

#include "common.h"

#include <type_traits>

namespace jitdb {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
// Native vectors for data in flight (HIP's uint4 is a union-based struct, which the
// optimiser does not always break up into registers).
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;     // small kernels
constexpr int kRowPad = 256;    // level row counts are rounded up to this for the stacked input
constexpr int kBN = 256;        // packed columns per block = 2 unit tiles x 4 gates x 32
constexpr int kUnit = 32;       // hidden units per MFMA column tile
constexpr int kGateTile = 128;  // packed rows per unit tile (4 gates x 32 units)

// Smallest level (rows) each kind of launch hands to the 256 x 256 tile kernel (level256.hip), by mode
// (leaf, internal, projection); INT32_MAX = never.  Measured on config 5: with one wave per SIMD nothing
// overlaps the cell update's activation arithmetic, so the leaf and internal launches (activation-heavy)
// are faster on 128 x 256 tiles with two blocks per CU; the projection has no activations.
constexpr int kTile256MinRows[3] = {INT32_MAX, INT32_MAX, INT32_MAX};

constexpr int kEpiStride = 40;  // floats per row of a wave's epilogue region: 32 units + 8; rows 4 apart fall 32 banks apart

enum : int { MODE_LEAF = 0, MODE_INTERNAL = 1, MODE_PROJ = 2, MODE_GENERIC = 3,   // GENERIC: plain C = A B^T
             MODE_CHAIN = 4 };   // internal rows with exactly one child: the forget gate's pre-activation is complete

template <typename T> struct Traits;
template <> struct Traits<float> {
    static constexpr int BK = 32;   // K is padded to multiples of this: 128 bytes, two pipeline stages
    static constexpr int VEC = 4;   // elements per 16 bytes
};
template <> struct Traits<bf16_t> {
    static constexpr int BK = 64;
    static constexpr int VEC = 8;
};

// ---- operand layout ----------------------------------------------------------------
// The two GEMM operands this file writes for itself (the stacked level input A and the
// packed weights B) are stored K-blocked: bytes [64 s, 64 s + 64) of every row form slab
// s, rows consecutive inside a slab.  A pipeline stage of the level kernel is 64 bytes of
// K per row, so the 16 rows x 64 bytes that one direct-to-LDS load instruction moves are
// 1 KB of consecutive memory, whole 128-byte lines.  (Fetching half a line now and the
// other half a stage later costs a full line transfer from L2 each time.)
// (operand_offset itself is in common.h: the backward pass writes operands in the same layout)

// ---- scalar helpers (bf16 conversions are in common.h) --------------------------------
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


}  // namespace

// ---- the arguments of one level launch (a named type: it crosses translation units) -----
struct LevelArgs {
    // A operands
    const void *stack;    // [n_rows, Dp (+ Hp)] the level's stacked input (leaf / internal)
    const void *hs;       // [N, Hp] rows by node id (projection)
    const void *x;        // [N, D] rows by node id (chain levels read them in place)
    // B operand: packed [W | U], NPU rows of Dp + Hp
    const void *Bp;
    const void *Bf;       // the same rows fragment-major (tile256_kernel), or null
    const float *bp;      // [NP] packed bias
    // schedule
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
    // training only: activations the backward pass needs
    void *gates;          // [N, 3H] of T: i | o | u after their non-linearities, rows by node id
    void *fgate;          // [N, H] of T: row k = forget gate the parent of k applied to k
    int D, Dp, H, Hp, Hu, Hq;
    int n_rows;
    int n_rows_alloc;     // rows per slab of the stacked input (n_rows rounded up to whole tiles)
    int NPU;              // rows per slab of the packed weights
    int n_row_tiles;      // level kernel: tiles along the row axis
    int n_col_tiles;      // tiles along the column axis
    int n_tiles;          // thin kernel: number of wave tiles
    int n_blocks;
    // grouped launch over the slots of one level (typed table): row tile i covers level rows
    // [tiles[i].x, min(tiles[i].x + 128, tiles[i].y)) and is evaluated by cell tiles[i].z
    const int4 *tiles;
    int64_t w_bytes;      // bytes between the packed weights of consecutive cells
    int NP;               // floats between their packed biases
    // tiled projection without a typed table: the level's node ids in position order (ascending ids, so the
    // gathered h rows are fetched front to back: 1.4 % off the projection), or nullptr: the ids come from the records
    const int32_t *proj_nodes;
};

namespace {



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

// ---- the cell update of one wave: 32 rows x 32 hidden units ---------------------------
// acc[g][v] holds the pre-activation (without bias) of gate g for row
// (v/4)*8 + hf*4 + v%4 and unit l32 of the wave's unit tile.  The wave writes i*u, o and
// the x part of the forget gate to its private LDS region and reads them back row-major,
// eight lanes per row and four consecutive units per lane: the rows of the children
// (P_k and c_k) are then fetched in 8- and 16-byte pieces, 64 / 128 contiguous bytes per
// row, with four rows in flight per lane.  rn / rar / rcb / rkid describe the 32 rows
// (node id or -1, arity, CSR start, first four child ids).  No block barrier inside.
// The packed bias of the wave's unit tile: gate g of unit l32 (lane & 31).  Loaded by the caller
// before its K loop, so that the cell update does not start with a trip to memory.
struct CellBias { float i, o, u, f; };
template <int MODE>
__device__ __forceinline__ CellBias load_cell_bias(const LevelArgs &a, int unit_tile, int lane) {
    const int pcol = unit_tile * kGateTile + (lane & 31);
    CellBias b;
    b.i = a.bp[pcol]; b.o = a.bp[pcol + kUnit]; b.u = a.bp[pcol + 2 * kUnit];
    b.f = (MODE == MODE_INTERNAL || MODE == MODE_CHAIN) ? a.bp[pcol + 3 * kUnit] : 0.0f;
    return b;
}

// c and h = o * tanh(c) of four consecutive units of node nd, to c_out / h_out and to their padded
// copies where those are separate arrays (pad columns of the padded h copy are zeroed).
template <typename T>
__device__ __forceinline__ void store_state(const LevelArgs &a, int64_t nd, int unit0, const float4 &cc, const float4 &go) {
    T *h_out = static_cast<T *>(a.h_out);
    T *hs_out = static_cast<T *>(a.hs_out);
    const bool separate_hs = (a.hs_out != a.h_out);
    const bool separate_cs = (a.cs != a.c_out);
    const float c4[4] = {cc.x, cc.y, cc.z, cc.w};
    const float o4[4] = {go.x, go.y, go.z, go.w};
    T hv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) hv[j] = from_f32<T>(o4[j] * tanh_t<T>(c4[j]));
    if ((a.H & 3) == 0) {
        if (unit0 < a.H) {
            *reinterpret_cast<float4 *>(a.c_out + nd * a.H + unit0) = cc;
            if (separate_cs) *reinterpret_cast<float4 *>(a.cs + nd * a.Hq + unit0) = cc;
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

template <typename T, int MODE, bool SAVE = false>
__device__ __forceinline__ void cell_pass(const LevelArgs &a, const floatx16 (&acc)[4], float *region,
                                          const int *rn, const int *rar, const int *rcb,
                                          const int4 *rkid, int unit_tile, int lane, const CellBias &bias) {
    constexpr bool KIDS = (MODE == MODE_INTERNAL || MODE == MODE_CHAIN);   // rows with children
    const int hf = lane >> 5, l32 = lane & 31;
    const float bi = bias.i, bo = bias.o, bu = bias.u, bf = bias.f;
    float *s_iu = region;
    float *s_o = s_iu + 32 * kEpiStride;
    float *s_fx = s_o + 32 * kEpiStride;
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
        if constexpr (KIDS) s_fx[rl * kEpiStride + l32] = acc[3][v] + bf;
        if constexpr (SAVE) {
            const int nd = rn[rl];
            const int unit = unit_tile * kUnit + l32;
            if (nd >= 0 && unit < a.H) {
                T *g = static_cast<T *>(a.gates) + (int64_t)nd * 3 * a.H + unit;
                g[0] = from_f32<T>(gi);
                g[a.H] = from_f32<T>(go);
                g[2 * a.H] = from_f32<T>(gu);
            }
        }
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
        if constexpr (KIDS) fx4[q] = *reinterpret_cast<const float4 *>(s_fx + so);
    }
    if constexpr (KIDS) {
        // Children are taken one per row and round, for four rows at once: eight independent loads in
        // flight per thread (two per row and round measured no faster: half of all parents have one
        // child, and the rows come sorted by arity).  The first four child ids of a row sit in LDS;
        // longer lists (rare) continue from child_idx.  A row without a further child re-reads its last
        // child with weight zero, which keeps every load unconditional.
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
        for (int c = 0; c < max_ar; ++c) {
            int64_t ofs[4];
            float wgt[4];
            int kidv[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int4 kids = make_int4(0, 0, 0, 0);
                if (c < 4) kids = rkid[tr[q]];
                const bool has = c < ar[q];
                int kid;
                if (c == 0) kid = kids.x;
                else if (c == 1) kid = kids.y;
                else if (c == 2) kid = kids.z;
                else if (c == 3) kid = kids.w;
                else kid = has ? a.child_idx[rcb[tr[q]] + c] : 0;
                if (has) last[q] = (int64_t)kid * a.Hq + unit_ld;
                ofs[q] = last[q];
                wgt[q] = has ? 1.0f : 0.0f;
                kidv[q] = has ? kid : -1;
            }
            float4 pk[4], ck[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if constexpr (MODE == MODE_CHAIN) {      // U_f h_k is in the accumulator already
                    pk[q] = make_float4(0.f, 0.f, 0.f, 0.f);
                } else if constexpr (sizeof(T) == 4) {
                    pk[q] = *reinterpret_cast<const float4 *>(static_cast<const float *>(a.P) + ofs[q]);
                } else {
                    const uint2 w = *reinterpret_cast<const uint2 *>(static_cast<const bf16_t *>(a.P) + ofs[q]);
                    pk[q] = make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xFFFF0000u),
                                        __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xFFFF0000u));
                }
                ck[q] = *reinterpret_cast<const float4 *>(a.cs + ofs[q]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float f0 = sigmoid_t<T>(fx4[q].x + pk[q].x), f1 = sigmoid_t<T>(fx4[q].y + pk[q].y);
                const float f2 = sigmoid_t<T>(fx4[q].z + pk[q].z), f3 = sigmoid_t<T>(fx4[q].w + pk[q].w);
                cc[q].x += wgt[q] * f0 * ck[q].x;
                cc[q].y += wgt[q] * f1 * ck[q].y;
                cc[q].z += wgt[q] * f2 * ck[q].z;
                cc[q].w += wgt[q] * f3 * ck[q].w;
                if constexpr (SAVE) {
                    if (kidv[q] >= 0) {
                        const float fv[4] = {f0, f1, f2, f3};
                        T *dst = static_cast<T *>(a.fgate) + (int64_t)kidv[q] * a.H + unit0;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (unit0 + e < a.H) dst[e] = from_f32<T>(fv[e]);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (node[q] < 0) continue;
        store_state<T>(a, node[q], unit0, cc[q], go4[q]);
    }
}

// ---- the cell update of a 32 x 32 tile by four waves: wave w finishes rows 8 w .. 8 w + 7 -------------
// For the kernels of small levels, where the tile's latency is what a level costs: zt holds the four
// gates' pre-activations (without bias) as [gate][row][unit] (kEpiStride floats per row); eight lanes
// share a row, four units each, and walk that row's own child list four children at a time (P_k and
// c_k of four children in flight per lane), in ascending child order.  With one wave for all 32 rows
// (cell_pass) every row waits for the tile's longest child list; here a wave waits for the longest
// of its eight rows, and four waves' loads are in flight together.  SAVE (training): the gates after
// their non-linearities and every child's forget gate are kept as well.
template <typename T, int MODE, bool SAVE = false>
__device__ __forceinline__ void cell_rows(const LevelArgs &a, const float *zt, const int *rn, const int *rar,
                                          const int *rcb, const int4 *rkid, int unit_tile, int wave, int lane) {
    const int tr = wave * 8 + (lane >> 3);
    const int node = rn[tr];
    if (node < 0) return;
    const int u4 = (lane & 7) * 4;
    const int unit0 = unit_tile * kUnit + u4;
    const float *bias = a.bp + unit_tile * kGateTile + u4;
    auto gate = [&](int g) __attribute__((always_inline)) {
        const float4 q = *reinterpret_cast<const float4 *>(zt + g * (32 * kEpiStride) + tr * kEpiStride + u4);
        const float4 bq = *reinterpret_cast<const float4 *>(bias + g * kUnit);
        return make_float4(q.x + bq.x, q.y + bq.y, q.z + bq.z, q.w + bq.w);
    };
    const float4 zi = gate(0), zo = gate(1), zu = gate(2);
    const float gi[4] = {sigmoid_t<T>(zi.x), sigmoid_t<T>(zi.y), sigmoid_t<T>(zi.z), sigmoid_t<T>(zi.w)};
    const float gu[4] = {tanh_t<T>(zu.x), tanh_t<T>(zu.y), tanh_t<T>(zu.z), tanh_t<T>(zu.w)};
    float4 cc = make_float4(gi[0] * gu[0], gi[1] * gu[1], gi[2] * gu[2], gi[3] * gu[3]);
    const float4 go = make_float4(sigmoid_t<T>(zo.x), sigmoid_t<T>(zo.y), sigmoid_t<T>(zo.z), sigmoid_t<T>(zo.w));
    if constexpr (SAVE) {      // training: the gates after their non-linearities, rows by node id
        const float o4[4] = {go.x, go.y, go.z, go.w};
        T *g = static_cast<T *>(a.gates) + (int64_t)node * 3 * a.H;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (unit0 + e < a.H) {
                g[unit0 + e] = from_f32<T>(gi[e]);
                g[a.H + unit0 + e] = from_f32<T>(o4[e]);
                g[2 * a.H + unit0 + e] = from_f32<T>(gu[e]);
            }
    }
    if constexpr (MODE == MODE_INTERNAL) {
        const float4 fx = gate(3);
        const int ar = rar[tr];
        const int cb = rcb[tr];
        const int4 k4 = rkid[tr];
        const int first[4] = {k4.x, k4.y, k4.z, k4.w};
        const int unit_ld = unit0 < a.Hq ? unit0 : 0;     // unit groups past the padded width read the first group (and store nothing)
        for (int c0 = 0; c0 < ar; c0 += 4) {
            bool has[4];
            int64_t ofs[4];
            int kidv[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = c0 + j;
                has[j] = c < ar;
                // a slot without a child re-reads the row's first child and is not added
                const int kid = !has[j] ? k4.x : (c0 == 0 ? first[j] : a.child_idx[cb + c]);
                kidv[j] = kid;
                ofs[j] = (int64_t)kid * a.Hq + unit_ld;
            }
            float4 pk[4], ck[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if constexpr (sizeof(T) == 4) {
                    pk[j] = *reinterpret_cast<const float4 *>(static_cast<const float *>(a.P) + ofs[j]);
                } else {
                    const uint2 w = *reinterpret_cast<const uint2 *>(static_cast<const bf16_t *>(a.P) + ofs[j]);
                    pk[j] = make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xFFFF0000u),
                                        __uint_as_float(w.y << 16), __uint_as_float(w.y & 0xFFFF0000u));
                }
                ck[j] = *reinterpret_cast<const float4 *>(a.cs + ofs[j]);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (has[j]) {
                    const float f[4] = {sigmoid_t<T>(fx.x + pk[j].x), sigmoid_t<T>(fx.y + pk[j].y),
                                        sigmoid_t<T>(fx.z + pk[j].z), sigmoid_t<T>(fx.w + pk[j].w)};
                    cc.x += f[0] * ck[j].x;
                    cc.y += f[1] * ck[j].y;
                    cc.z += f[2] * ck[j].z;
                    cc.w += f[3] * ck[j].w;
                    if constexpr (SAVE) {      // training: the forget gate this parent applied to child kidv[j]
                        T *dst = static_cast<T *>(a.fgate) + (int64_t)kidv[j] * a.H + unit0;
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (unit0 + e < a.H) dst[e] = from_f32<T>(f[e]);
                    }
                }
            }
        }
    }
    store_state<T>(a, node, unit0, cc, go);
}

// ---- the projection's store of one wave: 32 rows x 128 units ----------------------------
// acc[g][v] holds P = U_f h for row (v/4)*8 + hf*4 + v%4 and unit unit_base + g*32 + l32.  The wave
// turns the tile around in its private LDS region so that 16 lanes store one row's 128 units in
// 8-unit pieces (16 bytes of bf16).  rn: node ids of the 32 rows (-1: no such row).
constexpr int kDmaProjStride = 136; // floats per row of a wave's projection store region (128 units + 8)
template <typename T>
__device__ __forceinline__ void proj_pass(const LevelArgs &a, const floatx16 (&acc)[4], float *region,
                                          const int *rn, int unit_base, int lane) {
    const int hf = lane >> 5, l32 = lane & 31;
    T *P = static_cast<T *>(a.P);
    const int u8 = (lane & 15) * 8;
    const int unit0 = unit_base + u8;
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int rl = (v >> 2) * 8 + hf * 4 + (v & 3);
            region[rl * kDmaProjStride + g * 32 + l32] = acc[g][v];
        }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int sweep = 0; sweep < 8; ++sweep) {
        const int rl = (lane >> 4) + 4 * sweep;
        const int node = rn[rl];
        if (node < 0 || unit0 >= a.H) continue;
        const float4 lo = *reinterpret_cast<const float4 *>(region + rl * kDmaProjStride + u8);
        const float4 hi = *reinterpret_cast<const float4 *>(region + rl * kDmaProjStride + u8 + 4);
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
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

#define JITDB_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))
#define JITDB_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

}  // namespace

// cells.hip: the N-ary cell (second operator type of the table)
struct NarySlot {
    const void *x;          // [N, D] all nodes' inputs, rows by node id
    const int4 *row_rec;    // the slot's row records (two int4 per row)
    void *A;                // workspace: the slot's stacked input, K-blocked
    const void *Bn;         // the cell's packed weights (nary_pack): slots i, o, u, f_1 by unit tile, then the rows of f_2 .. f_N
    float *F;               // workspace: pre-activations of f_2 .. f_N, [n_rows, (N - 1) H]
    const float *b;         // the cell's bias [(3 + N) H]
    int *err;               // device flag: set when a node has more children than the cell has positions
    int n_rows, N;
    bool leaves;            // a slot of level 0: no children, so K is the x part alone and the forget gates are not needed
};
// The tiled GEMM with the N-ary cell update behind it (forward.hip): A [M rows] K-blocked, B packed by gate
// slot, outputs by node id.
struct NaryLevel {
    const void *A; int64_t a_rows_alloc; int M;
    const void *B; int64_t b_rows_alloc; int n_col_tiles;
    int64_t k_bytes;
    const int4 *row_rec; const float *bias; const float *cs; const float *F;
    float *c_out; void *h_out; void *hs_out; float *cs_out;
    int H, Hp, Hq, N;
    bool leaves;
};
int launch_nary_level(jitdb_dtype dtype, const NaryLevel &g, hipStream_t st);
size_t nary_packed_bytes(int D, int H, int Dp, int Hp, int N, size_t esz);
int nary_pack(jitdb_dtype dtype, const void *W, const void *U, int D, int H, int Dp, int Hp, int N, void *Bn,
              int *err_to_clear, hipStream_t st);
int run_nary_slot(jitdb_dtype dtype, const LevelArgs &a, const NarySlot &s, hipStream_t st);

// level256.hip
bool tile256_applies(int mode, const LevelArgs &a);
int launch_tile256(int mode, LevelArgs a, hipStream_t st);

}  // namespace jitdb
