// The second operator type of the table: the N-ary Tree-LSTM cell.
//
// The paper's look-up key holds the operator type next to the depth (sections 4.2, 4.3): nodes of
// different type never share a slot, each slot is one batched evaluation of its own subgraph.
// The child-sum cell is forward.hip.  The N-ary cell (at most N ordered children; every child
// position has weights of its own and every forget gate sees all children) needs no per-child
// projection and no child sum: with hc = [h_{k_1} ; ... ; h_{k_N}] (zero blocks for missing
// children) all of its 3 + N gates are one contraction
//
//     Z = [x | hc] [W | U]^T          rows: the slot's nodes, columns: i | o | u | f_1 | ... | f_N
//
// followed by an elementwise cell update.  Per slot:
//
//   nary_stack_kernel   the slot's dense input rows [x_j | h of child 1 | ... | h of child N], K-blocked
//                       (the "stack" of section 4.3; children by ascending id = position 1, 2, ...);
//                       a slot of leaves stacks x alone
//   launch_kb_gemm      for N > 1, internal nodes: the forget gates of positions 2 .. N as a plain GEMM
//                       (exactly (N - 1) H columns), pre-activations kept in fp32
//   nary_level_kernel   (forward.hip) the gates i, o, u, f_1 on the tiled MFMA core with the cell update as
//                       its epilogue: c = i u + sum_l f_l c_{k_l}, h = o tanh(c), rows written by node id
//                       (the "slice")
#include "level_common.h"

namespace jitdb {
namespace {

// ---- weights ---------------------------------------------------------------------------
// Two packed matrices, both K-blocked like every operand of the tiled GEMM, K = Dp + N Hp:
// [ W row (D, zero padded to Dp) | U columns of position 1 (H, padded to Hp) | ... | position N ].
//   main   row = unit tile * 128 + slot * 32 + u, slots i, o, u, f_1: the waves of one block hold all four
//          gates of a hidden unit (a slot of leaves multiplies the first slabs, the x part, of the same rows)
//   extra  the rows of f_2 .. f_N, gate-major ((N - 1) H rows): a plain GEMM of their own
__host__ __device__ inline int nary_rows_main(int H) { return ((((H + kUnit - 1) / kUnit) * 128 + 255) / 256) * 256; }
__host__ __device__ inline int nary_rows_extra(int H, int N) { return (((N - 1) * H + 255) / 256) * 256; }

template <typename T>
__global__ void __launch_bounds__(kThreads)
nary_pack_kernel(const T *__restrict__ W, const T *__restrict__ U, int D, int H, int Dp, int Hp, int N,
                 T *__restrict__ Bm, T *__restrict__ Bx, int *__restrict__ err_to_clear) {
    if (blockIdx.x == 0 && threadIdx.x == 0 && err_to_clear) *err_to_clear = 0;
    const int Kn = Dp + N * Hp;
    const int rows_m = nary_rows_main(H), rows_x = nary_rows_extra(H, N);
    const int64_t total_m = (int64_t)rows_m * Kn, total = total_m + (int64_t)rows_x * Kn;
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * kThreads) {
        const bool extra = idx >= total_m;
        const int64_t id = extra ? idx - total_m : idx;
        const int r = (int)(id / Kn), k = (int)(id % Kn);
        int64_t g = -1;                                          // row of W / U (gate-major), or none
        if (extra) {
            if (r < (N - 1) * H) g = (int64_t)4 * H + r;         // f_2 starts at gate row 4 H
        } else {
            const int slot = (r % 128) / kUnit, unit = (r / 128) * kUnit + r % kUnit;
            if (unit < H) g = (int64_t)slot * H + unit;
        }
        T v = T(0);
        if (g >= 0) {
            if (k < D) {
                v = W[g * D + k];
            } else if (k >= Dp) {
                const int l = (k - Dp) / Hp, j = (k - Dp) % Hp;
                if (j < H) v = U[g * N * H + l * H + j];
            }
        }
        T *dst = extra ? Bx : Bm;
        *reinterpret_cast<T *>(reinterpret_cast<char *>(dst) + operand_offset(r, (int64_t)k * sizeof(T), extra ? rows_x : rows_m)) = v;
    }
}

// ---- stack -----------------------------------------------------------------------------
// One thread per 16-byte piece of a row of A = [x_j | h_{k_1} | ... | h_{k_N}].  The child ids come
// with the row record (its first four children; N <= 4).  A node with more children than the cell
// has positions sets *err; the surplus children are left out.
template <typename T>
__global__ void __launch_bounds__(kThreads)
nary_stack_kernel(const T *__restrict__ x, int D, int Dp, const T *__restrict__ hs, int Hp, int N, int Nk,
                  const int4 *__restrict__ row_rec, T *__restrict__ A, int n_rows, int n_rows_alloc,
                  int *__restrict__ err) {
    // N: the cell's child positions; Nk <= N: positions stacked for this slot (0 for a slot of leaves)
    constexpr int VEC = Traits<T>::VEC;
    const int cpr = (Dp + Nk * Hp) / VEC;
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t row = gid / cpr;
    const int ch = (int)(gid % cpr);
    if (row >= n_rows) return;
    const int4 r0 = row_rec[2 * row];
    const int k0 = ch * VEC;
    uint4 o = make_uint4(0u, 0u, 0u, 0u);
    if (k0 < Dp) {
        const T *src = x + (int64_t)r0.x * D + k0;
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
        if (ch == 0 && r0.y > N) *err = 1;
    } else {
        const int l = (k0 - Dp) / Hp, kh = (k0 - Dp) % Hp;
        if (l < r0.y) {
            const int4 kids = row_rec[2 * row + 1];
            const int kid = l == 0 ? kids.x : l == 1 ? kids.y : l == 2 ? kids.z : kids.w;
            o = *reinterpret_cast<const uint4 *>(hs + (int64_t)kid * Hp + kh);   // pad columns of hs are zero
        }
    }
    *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(A) + operand_offset(row, (int64_t)k0 * sizeof(T), n_rows_alloc)) = o;
}

}  // namespace

static size_t nary_main_bytes(int H, int Dp, int Hp, int N, size_t esz) {
    return round_up((int64_t)nary_rows_main(H) * (size_t)(Dp + N * Hp) * esz, 256);
}
size_t nary_packed_bytes(int D, int H, int Dp, int Hp, int N, size_t esz) {
    (void)D;
    return nary_main_bytes(H, Dp, Hp, N, esz) + (size_t)nary_rows_extra(H, N) * (size_t)(Dp + N * Hp) * esz;
}

int nary_pack(jitdb_dtype dtype, const void *W, const void *U, int D, int H, int Dp, int Hp, int N, void *Bn,
              int *err_to_clear, hipStream_t st) {
    const size_t esz = dtype == JITDB_F32 ? 4 : 2;
    void *Bx = static_cast<char *>(Bn) + nary_main_bytes(H, Dp, Hp, N, esz);
    const int64_t total = (int64_t)(nary_rows_main(H) + nary_rows_extra(H, N)) * (Dp + N * Hp);
    const unsigned grid = (unsigned)(ceil_div(total, kThreads) < 4096 ? ceil_div(total, kThreads) : 4096);
    if (dtype == JITDB_F32)
        nary_pack_kernel<float><<<grid, kThreads, 0, st>>>(static_cast<const float *>(W), static_cast<const float *>(U),
                                                          D, H, Dp, Hp, N, static_cast<float *>(Bn),
                                                          static_cast<float *>(Bx), err_to_clear);
    else
        nary_pack_kernel<bf16_t><<<grid, kThreads, 0, st>>>(static_cast<const bf16_t *>(W), static_cast<const bf16_t *>(U),
                                                           D, H, Dp, Hp, N, static_cast<bf16_t *>(Bn),
                                                           static_cast<bf16_t *>(Bx), err_to_clear);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

// One slot of N-ary nodes: stack, (for N > 1 and internal nodes) the GEMM of the further forget gates,
// the level kernel.  a: the level arguments of the forward (x rows come through NarySlot, h and c of the
// children through a.hs / a.cs).
int run_nary_slot(jitdb_dtype dtype, const LevelArgs &a, const NarySlot &s, hipStream_t st) {
    if (s.n_rows <= 0) return JITDB_OK;
    const size_t esz = dtype == JITDB_F32 ? 4 : 2;
    const int vec = dtype == JITDB_F32 ? 4 : 8;
    const int Nk = s.leaves ? 0 : s.N;                       // child positions this slot stacks and multiplies
    const int Kn = a.Dp + Nk * a.Hp;
    const int rows_alloc = (int)round_up(s.n_rows, kRowPad);
    const unsigned sblocks = (unsigned)ceil_div((int64_t)s.n_rows * (Kn / vec), kThreads);
    if (dtype == JITDB_F32)
        nary_stack_kernel<float><<<sblocks, kThreads, 0, st>>>(static_cast<const float *>(s.x), a.D, a.Dp,
                                                              static_cast<const float *>(a.hs), a.Hp, s.N, Nk, s.row_rec,
                                                              static_cast<float *>(s.A), s.n_rows, rows_alloc, s.err);
    else
        nary_stack_kernel<bf16_t><<<sblocks, kThreads, 0, st>>>(static_cast<const bf16_t *>(s.x), a.D, a.Dp,
                                                               static_cast<const bf16_t *>(a.hs), a.Hp, s.N, Nk, s.row_rec,
                                                               static_cast<bf16_t *>(s.A), s.n_rows, rows_alloc, s.err);
    JITDB_LAUNCH_CHECK();
    if (!s.leaves && s.N > 1) {       // f_2 .. f_N of every row, before the kernel that uses them
        KbGemm x = {};
        x.A = s.A; x.a_rows_alloc = rows_alloc; x.M = s.n_rows;
        x.B = static_cast<const char *>(s.Bn) + nary_main_bytes(a.H, a.Dp, a.Hp, s.N, esz);
        x.b_rows_alloc = nary_rows_extra(a.H, s.N); x.N = (s.N - 1) * a.H;
        x.k_bytes = (int64_t)Kn * (int64_t)esz; x.k_splits = 1;
        x.epilogue = KB_EPI_STORE_F32; x.out0 = s.F; x.ldc = x.N;
        const int rc = launch_kb_gemm(dtype, x, st);
        if (rc != JITDB_OK) return rc;
    }
    NaryLevel g = {};
    g.A = s.A; g.a_rows_alloc = rows_alloc; g.M = s.n_rows;
    g.B = s.Bn; g.b_rows_alloc = nary_rows_main(a.H);
    g.n_col_tiles = (int)ceil_div(ceil_div(a.H, kUnit), 2);
    g.k_bytes = (int64_t)Kn * (int64_t)esz;
    g.row_rec = s.row_rec; g.bias = s.b; g.cs = a.cs; g.F = s.F;
    g.c_out = a.c_out; g.h_out = a.h_out; g.hs_out = a.hs_out; g.cs_out = a.cs;
    g.H = a.H; g.Hp = a.Hp; g.Hq = a.Hq; g.N = s.N; g.leaves = s.leaves;
    return launch_nary_level(dtype, g, st);
}

}  // namespace jitdb
