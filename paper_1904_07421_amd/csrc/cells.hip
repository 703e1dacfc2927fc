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
//                       (the "stack" of section 4.3; children by ascending id = position 1, 2, ...)
//   launch_kb_gemm      Z on the tiled MFMA core shared with the backward pass (fp32 out)
//   nary_cell_kernel    i, o, u, f_l, c = i u + sum_l f_l c_{k_l}, h = o tanh(c); rows written by node id
//                       (the "slice")
//
// This first version keeps the pre-activations in memory between the last two steps (the child-sum
// path fuses them); it is the slot's operator type that is new here, not its speed.
#include "level_common.h"

namespace jitdb {
namespace {

// ---- weights ---------------------------------------------------------------------------
// Bn: (3 + N) H rows (row = gate block * H + unit, padded to a multiple of 256), K = Dp + N Hp,
// K-blocked like every operand of the tiled GEMM: [ W row (D, zero padded to Dp) | U columns of
// position 1 (H, padded to Hp) | ... | position N ].
template <typename T>
__global__ void __launch_bounds__(kThreads)
nary_pack_kernel(const T *__restrict__ W, const T *__restrict__ U, int D, int H, int Dp, int Hp, int N,
                 int rows_alloc, T *__restrict__ Bn, int *__restrict__ err_to_clear) {
    if (blockIdx.x == 0 && threadIdx.x == 0 && err_to_clear) *err_to_clear = 0;
    const int Kn = Dp + N * Hp;
    const int G = 3 + N;
    const int64_t total = (int64_t)rows_alloc * Kn;
    for (int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * kThreads) {
        const int r = (int)(idx / Kn), k = (int)(idx % Kn);
        T v = T(0);
        if (r < G * H) {
            if (k < D) {
                v = W[(int64_t)r * D + k];
            } else if (k >= Dp) {
                const int l = (k - Dp) / Hp, j = (k - Dp) % Hp;
                if (j < H) v = U[(int64_t)r * N * H + l * H + j];
            }
        }
        *reinterpret_cast<T *>(reinterpret_cast<char *>(Bn) + operand_offset(r, (int64_t)k * sizeof(T), rows_alloc)) = v;
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

// ---- cell update -----------------------------------------------------------------------
// One thread per (row, unit) over the padded width Hp: units below H are computed, the pad
// columns of the padded h copy are zeroed.  Z [n_rows, (3 + N) H] fp32 without bias.
struct NaryCellArgs {
    const float *Z; const float *b; const int4 *row_rec; const float *cs;
    void *h_out; void *hs_out; float *c_out; float *cs_out;
    int n_rows, H, Hp, Hq, N;
};
template <typename T>
__global__ void __launch_bounds__(kThreads)
nary_cell_kernel(const NaryCellArgs a) {
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t row = gid / a.Hp;
    const int unit = (int)(gid % a.Hp);
    if (row >= a.n_rows) return;
    const int4 r0 = a.row_rec[2 * row];
    const int64_t nd = r0.x;
    T *h_out = static_cast<T *>(a.h_out), *hs_out = static_cast<T *>(a.hs_out);
    const bool separate_hs = hs_out != h_out;
    if (unit >= a.H) {
        if (separate_hs) hs_out[nd * a.Hp + unit] = T(0);
        return;
    }
    const int H = a.H, ldz = (3 + a.N) * H;
    const float *z = a.Z + row * ldz;
    const float gi = sigmoid_t<T>(z[unit] + a.b[unit]);
    const float go = sigmoid_t<T>(z[H + unit] + a.b[H + unit]);
    const float gu = tanh_t<T>(z[2 * H + unit] + a.b[2 * H + unit]);
    float c = gi * gu;
    const int m = r0.y < a.N ? r0.y : a.N;
    if (m > 0) {
        const int4 kids = a.row_rec[2 * row + 1];
        const int kid[4] = {kids.x, kids.y, kids.z, kids.w};
#pragma unroll
        for (int l = 0; l < 4; ++l)
            if (l < m) {
                const float f = sigmoid_t<T>(z[(3 + l) * H + unit] + a.b[(3 + l) * H + unit]);
                c += f * a.cs[(int64_t)kid[l] * a.Hq + unit];
            }
    }
    const T hv = from_f32<T>(go * tanh_t<T>(c));
    a.c_out[nd * H + unit] = c;
    if (a.cs_out != a.c_out) a.cs_out[nd * a.Hq + unit] = c;
    h_out[nd * H + unit] = hv;
    if (separate_hs) hs_out[nd * a.Hp + unit] = hv;
}

}  // namespace

size_t nary_packed_bytes(int D, int H, int Dp, int Hp, int N, size_t esz) {
    return (size_t)round_up((int64_t)(3 + N) * H, 256) * (size_t)(Dp + N * Hp) * esz;
}

int nary_pack(jitdb_dtype dtype, const void *W, const void *U, int D, int H, int Dp, int Hp, int N, void *Bn,
              int *err_to_clear, hipStream_t st) {
    const int rows_alloc = (int)round_up((int64_t)(3 + N) * H, 256);
    const int64_t total = (int64_t)rows_alloc * (Dp + N * Hp);
    const unsigned grid = (unsigned)(ceil_div(total, kThreads) < 4096 ? ceil_div(total, kThreads) : 4096);
    if (dtype == JITDB_F32)
        nary_pack_kernel<float><<<grid, kThreads, 0, st>>>(static_cast<const float *>(W), static_cast<const float *>(U),
                                                          D, H, Dp, Hp, N, rows_alloc, static_cast<float *>(Bn), err_to_clear);
    else
        nary_pack_kernel<bf16_t><<<grid, kThreads, 0, st>>>(static_cast<const bf16_t *>(W), static_cast<const bf16_t *>(U),
                                                           D, H, Dp, Hp, N, rows_alloc, static_cast<bf16_t *>(Bn), err_to_clear);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

// One slot of N-ary nodes: the three steps above.  a: the level arguments of the forward (x rows come
// through NarySlot, h and c of the children through a.hs / a.cs); rec: the slot's row records.
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
    KbGemm g = {};
    g.A = s.A; g.a_rows_alloc = rows_alloc; g.M = s.n_rows;
    // leaves: the gates i, o, u only (the first 3 H packed rows), over the x part of K (the first slabs)
    g.B = s.Bn; g.b_rows_alloc = round_up((int64_t)(3 + s.N) * a.H, 256); g.N = (3 + Nk) * a.H;
    g.k_bytes = (int64_t)Kn * (int64_t)esz; g.k_splits = 1;
    g.epilogue = KB_EPI_STORE_F32; g.out0 = s.Z; g.ldc = (3 + s.N) * a.H;
    const int rc = launch_kb_gemm(dtype, g, st);
    if (rc != JITDB_OK) return rc;
    NaryCellArgs c;
    c.Z = s.Z; c.b = s.b; c.row_rec = s.row_rec; c.cs = a.cs;
    c.h_out = a.h_out; c.hs_out = a.hs_out; c.c_out = a.c_out; c.cs_out = a.cs;
    c.n_rows = s.n_rows; c.H = a.H; c.Hp = a.Hp; c.Hq = a.Hq; c.N = s.N;
    const unsigned cblocks = (unsigned)ceil_div((int64_t)s.n_rows * a.Hp, kThreads);
    if (dtype == JITDB_F32) nary_cell_kernel<float><<<cblocks, kThreads, 0, st>>>(c);
    else nary_cell_kernel<bf16_t><<<cblocks, kThreads, 0, st>>>(c);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

}  // namespace jitdb
