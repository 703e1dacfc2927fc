// The level kernel for large bf16 levels: 256 x 256 tiles, one persistent block per CU.
//
// Same job as level_kernel in forward.hip (the batched execution of one slot of the paper's
// table, section 4.3: gate GEMM on the stacked rows with the cell update fused behind it, or the
// per-child forget projection), laid out for what bounds it on gfx950:
//
//   - A block of four waves owns 256 rows x 256 packed columns; each wave a 128 x 128 sub-tile,
//     4 x 4 MFMA tiles of 32 x 32 x 16 bf16, whose 256 accumulator registers live in the AGPR half
//     of the register file (one wave per SIMD, 512 registers).  A fragment then feeds four MFMAs:
//     per multiply a third fewer operand bytes than with 64 x 128 sub-tiles.
//   - B (the packed weights) never touches LDS: it is stored fragment-major, so that one 16-byte
//     load per lane IS an MFMA operand, and a wave fetches the four gate fragments of a K group
//     straight from L2 into registers, kPF K groups ahead.  LDS carries A only: reads and
//     direct-to-LDS writes together stay at about half of what the LDS port can move.
//   - A goes through a ring of kRing stage buffers (64 bytes of K per row each) filled by
//     direct-to-LDS loads; the ring is never drained: while a tile's last stages are multiplied and
//     while its cell update runs, the first stages of the block's next tile are already landing.
//   - Blocks are persistent (one per CU) and walk the tiles of their XCD's share of row tiles, so
//     the eight column tiles of a row tile run side by side on one L2.
//
// LDS reads of fragments and the loads of B are issued from inline asm and waited for by hand
// (s_waitcnt with counts derived below): the compiler waits for *everything* in flight as soon as
// direct-to-LDS loads and register loads are mixed.  The counts rely on loads completing in issue
// order and on every wave issuing the same fixed sequence of loads per stage; anything else a wave
// issues in between (the cell update's gathers and stores) only makes a wait stricter.
#include "level_common.h"

namespace jitdb {
namespace {

constexpr int kT256 = 256;                        // threads per block
constexpr int kBM256 = 256;                       // rows per tile
constexpr int kStage256 = 64;                     // bytes of K per row and stage
constexpr int kStageBytes = kBM256 * kStage256;   // 16 KB
constexpr int kRing = 5;                          // stage buffers
constexpr int kPF = 4;                            // K groups of B fragments in registers (= K groups per loop body)

template <int N>
__device__ __forceinline__ void wait_barrier256() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// Gate fragments multiplied per K group in the x part / the h part of K.
template <int MODE> struct Gates256 {
    static constexpr int X = (MODE == MODE_LEAF) ? 3 : 4;
    static constexpr int H = (MODE == MODE_INTERNAL) ? 3 : 4;
    // fewest loads any K group of this mode issues for B: the waits assume no more than this
    static constexpr int MIN = (MODE == MODE_PROJ) ? 4 : 3;
};

template <int MODE>
__global__ void __launch_bounds__(kT256, 1)
tile256_kernel(const LevelArgs a) {
    constexpr int kRegion = (MODE == MODE_PROJ) ? 32 * kDmaProjStride : 3 * 32 * kEpiStride;   // floats per wave
    __shared__ __attribute__((aligned(1024))) char ring[kRing * kStageBytes];
    __shared__ __attribute__((aligned(16))) float regions[4 * kRegion];
    __shared__ int row_node[kBM256];
    __shared__ int row_ar[MODE == MODE_INTERNAL ? kBM256 : 1];
    __shared__ int row_cb[MODE == MODE_INTERNAL ? kBM256 : 1];
    __shared__ int4 row_kid[MODE == MODE_INTERNAL ? kBM256 : 1];

    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int hf = lane >> 5, l32 = lane & 31;

    // ---- this block's tiles: XCD x owns row tiles x, x + 8, ...; its blocks deal out
    //      (row tile, column tile) pairs, column fastest
    const int xcd = blockIdx.x & 7, bi = blockIdx.x >> 3, per_xcd = gridDim.x >> 3;
    const int rows_x = (a.n_row_tiles - xcd + 7) >> 3;
    const int items = rows_x * a.n_col_tiles;
    if (bi >= items) return;

    // ---- K: groups of 32 bytes (one MFMA K step), two per stage
    const int nkg_x = (MODE == MODE_PROJ) ? 0 : a.Dp * 2 / 32;
    const int nkg_h = (MODE == MODE_LEAF) ? 0 : a.Hp * 2 / 32;
    const int nkg = nkg_x + nkg_h;               // multiple of 4
    const int nkg_all = (a.Dp + a.Hp) * 2 / 32;  // K groups of a packed row
    const int S = nkg >> 1;

    // ---- A fragments: lane (l32, hf) reads row l32 of a 32-row block, 16-byte piece 2h + hf of the
    //      stage's 64 bytes; piece p of row r sits in slot p ^ ((r >> 2) & 3)
    const uint32_t lds_base = (uint32_t)(uintptr_t)JITDB_LDS_PTR(ring);
    const int sw = (l32 >> 2) & 3;
    uint32_t a_rd[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) a_rd[h] = lds_base + (wm * 128 + l32) * kStage256 + (((2 * h + hf) ^ sw) * 16);
    struct Frags { u32x4 v[4]; };
    auto read_frags = [&](int slot, int h, Frags &f) __attribute__((always_inline)) {
        const uint32_t aa = a_rd[h] + slot * kStageBytes;
        asm volatile("ds_read_b128 %0, %1" : "=v"(f.v[0]) : "v"(aa) : "memory");
        asm volatile("ds_read_b128 %0, %1 offset:2048" : "=v"(f.v[1]) : "v"(aa) : "memory");
        asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(f.v[2]) : "v"(aa) : "memory");
        asm volatile("ds_read_b128 %0, %1 offset:6144" : "=v"(f.v[3]) : "v"(aa) : "memory");
    };
    auto reads_done = [&](Frags &f) __attribute__((always_inline)) {
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f.v[0]), "+v"(f.v[1]), "+v"(f.v[2]), "+v"(f.v[3]));
    };
    // ---- B fragments: 16 bytes per lane, fragment j of a K group 1 KB after fragment j - 1
    auto load_b = [&](u32x4 &dst, const char *p, int j) __attribute__((always_inline)) {
        if (j == 0) asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(p) : "memory");
        else if (j == 1) asm volatile("global_load_dwordx4 %0, %1, off offset:1024" : "=v"(dst) : "v"(p) : "memory");
        else if (j == 2) asm volatile("global_load_dwordx4 %0, %1, off offset:2048" : "=v"(dst) : "v"(p) : "memory");
        else asm volatile("global_load_dwordx4 %0, %1, off offset:3072" : "=v"(dst) : "v"(p) : "memory");
    };

    // ---- the mover: lane l fills slot l & 3 of row l >> 2 of each 16-row unit it is given; a wave
    //      moves units 4 wave .. 4 wave + 3 of every stage
    const int lrow = lane >> 2;
    const int piece16 = ((lane & 3) ^ ((lane >> 4) & 3)) * 16;
    const int64_t a_stage = (MODE == MODE_PROJ) ? kStage256 : (int64_t)a.n_rows_alloc * kStage256;

    // Where a tile's operands start.  A: the stacked matrix (K-blocked), or for the projection the
    // rows of h by node id.  B: the wave's four fragments per K group; gates i, o, u, f of one unit
    // tile lie 1 KB apart (pb[0] + j KB), the projection's four unit tiles a packed row block apart.
    struct TilePtrs {
        const char *pa[4];
        const char *pb[MODE == MODE_PROJ ? 4 : 1];
        int row0, col_tile;
    };
    auto tile_ptrs = [&](int q, TilePtrs &p) __attribute__((always_inline)) {
        const int row_tile = xcd + 8 * (q / a.n_col_tiles);
        p.col_tile = q % a.n_col_tiles;
        p.row0 = row_tile * kBM256;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = p.row0 + (wave * 4 + j) * 16 + lrow;
            if constexpr (MODE == MODE_PROJ) {
                const int g = r < a.n_rows ? r : a.n_rows - 1;     // rows past the end repeat the last one; never stored
                const int node = a.row_rec[2 * (int64_t)g].x;
                p.pa[j] = static_cast<const char *>(a.hs) + (int64_t)node * a.Hp * 2 + piece16;
            } else {
                p.pa[j] = static_cast<const char *>(a.stack) + (int64_t)r * kStage256 + piece16;
            }
        }
        if constexpr (MODE == MODE_PROJ) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                p.pb[j] = static_cast<const char *>(a.Bf) +
                          ((int64_t)(p.col_tile * 8 + wn * 4 + j) * nkg_all + (a.Dp * 2 / 32)) * 4096 + 3 * 1024 + lane * 16;
        } else {
            p.pb[0] = static_cast<const char *>(a.Bf) + (int64_t)(p.col_tile * 2 + wn) * nkg_all * 4096 + lane * 16;
        }
    };
    auto dma_unit = [&](const TilePtrs &p, int s, int slot, int j) __attribute__((always_inline)) {
        __builtin_amdgcn_global_load_lds(JITDB_GLOBAL_PTR(p.pa[j] + s * a_stage),
                                         JITDB_LDS_PTR(ring + slot * kStageBytes + (wave * 4 + j) * 1024), 16, 0, 0);
    };
    auto load_b_frag = [&](u32x4 &dst, const TilePtrs &p, int kg, int j) __attribute__((always_inline)) {
        if constexpr (MODE == MODE_PROJ) load_b(dst, p.pb[j] + (int64_t)kg * 4096, 0);
        else load_b(dst, p.pb[0] + (int64_t)kg * 4096, j);
    };

    // ---- fill the ring for the first tile (once per block; later tiles find their first stages
    //      requested by the tile before them)
    TilePtrs cur_t, next_t;
    tile_ptrs(bi, cur_t);
#pragma unroll
    for (int s = 0; s < kRing; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j) dma_unit(cur_t, s, s, j);
    int cur = 0;          // ring slot of the stage being multiplied

    // Waits.  Per stage a wave issues, in this order: the B loads of K group 2s + kPF (one after each
    // gate's MFMAs of K group 2s), then alternately a B load of K group 2s + 1 + kPF and one of its four
    // DMA units of stage s + kRing (after the MFMAs of K group 2s + 1), a DMA unit last.  NG below is the
    // fewest B loads a K group of this mode issues (more only makes a wait stricter).
    //   NWAIT: stage s + 1 has landed (asked at the barrier inside stage s).  Its last DMA unit was the
    //   last load of stage s + 1 - kRing; since then kRing - 2 whole stages and the first K group of stage s.
    //   BWAIT: the B fragments of a K group were requested kPF K groups earlier; since then kPF - 1 K
    //   groups of B loads and at least 2 kPF - 3 DMA units.
    // The last body of a tile requests no B fragments (the next tile asks for its own after the cell
    // update, so that no registers are held across it); its waits count what is really issued:
    //   K group nkg-4: as BWAIT.  nkg-3: two K groups of B loads, 5 DMA units.  nkg-2: one K group, 8 units.
    //   nkg-1: 5 units.  Barrier of stage S-2: kRing - 2 whole stages.  Barrier of stage S-1 (the next
    //   tile's stage 0): kRing - 3 whole stages and the 4 units of stage S-2.
    constexpr int NG = Gates256<MODE>::MIN;
    constexpr int NWAIT = (kRing - 2) * (2 * NG + 4) + NG;
    constexpr int BWAIT = (kPF - 1) * NG + 2 * kPF - 3;
    constexpr int NWAIT_T1 = (kRing - 2) * (2 * NG + 4);
    constexpr int NWAIT_T2 = (kRing - 3) * (2 * NG + 4) + 4;
    static_assert(kPF == 4 && kRing >= 4, "the tail's wait counts are written out for four K groups per body");
    static_assert(NWAIT < 64 && BWAIT < 64, "vmcnt is a 6-bit counter");

    for (int q = bi; q < items; q += per_xcd) {
        // the tile after this one; the block's last tile asks again for its own first stages (nobody reads them)
        const int qn = q + per_xcd < items ? q + per_xcd : q;
        tile_ptrs(q, cur_t);
        tile_ptrs(qn, next_t);

        // ---- the tile's first B fragments, and its rows for the cell update (everyone is done with
        //      the previous tile's)
        u32x4 Bs[kPF][4];
#pragma unroll
        for (int k = 0; k < kPF; ++k)
#pragma unroll
            for (int j = 0; j < (MODE == MODE_LEAF ? 3 : 4); ++j) load_b_frag(Bs[k][j], cur_t, k, j);
        CellBias bias = {};
        if constexpr (MODE != MODE_PROJ) bias = load_cell_bias<MODE>(a, cur_t.col_tile * 2 + wn, lane);
        __syncthreads();
        {
            const int r = cur_t.row0 + t;
            int4 rec0 = make_int4(-1, 0, 0, 0), rec1 = make_int4(-1, -1, -1, -1);
            if (r < a.n_rows) {
                rec0 = a.row_rec[2 * (int64_t)r];
                if constexpr (MODE == MODE_INTERNAL) rec1 = a.row_rec[2 * (int64_t)r + 1];
            }
            row_node[t] = rec0.x;
            if constexpr (MODE == MODE_INTERNAL) {
                row_ar[t] = rec0.y;
                row_cb[t] = rec0.z;
                row_kid[t] = rec1;
            }
        }
        // all of it has arrived (the fragments, and with them the stages requested before)
        if constexpr (MODE == MODE_LEAF)
            asm volatile("s_waitcnt vmcnt(0)"
                         : "+v"(Bs[0][0]), "+v"(Bs[0][1]), "+v"(Bs[0][2]), "+v"(Bs[1][0]), "+v"(Bs[1][1]), "+v"(Bs[1][2]),
                           "+v"(Bs[2][0]), "+v"(Bs[2][1]), "+v"(Bs[2][2]), "+v"(Bs[3][0]), "+v"(Bs[3][1]), "+v"(Bs[3][2]));
        else
            asm volatile("s_waitcnt vmcnt(0)"
                         : "+v"(Bs[0][0]), "+v"(Bs[0][1]), "+v"(Bs[0][2]), "+v"(Bs[0][3]), "+v"(Bs[1][0]), "+v"(Bs[1][1]),
                           "+v"(Bs[1][2]), "+v"(Bs[1][3]), "+v"(Bs[2][0]), "+v"(Bs[2][1]), "+v"(Bs[2][2]), "+v"(Bs[2][3]),
                           "+v"(Bs[3][0]), "+v"(Bs[3][1]), "+v"(Bs[3][2]), "+v"(Bs[3][3]));
        if (q == bi) wait_barrier256<0>();       // the first tile's stages were requested just above, by all waves
        Frags P, Q;
        read_frags(cur, 0, P);
        reads_done(P);

        floatx16 acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][g][v] = 0.0f;

        // MFMAs of one K group (NGC gate fragments from slot k) after waiting until at most BW younger
        // loads are outstanding; after each gate's four MFMAs the slot is refilled with the fragment of K
        // group kgn (NGT of them; none in a tile's last body), and in the second K group of a stage one
        // DMA unit of stage sn goes to the ring slot that the stage just released.
        auto half = [&](Frags &F, int k, auto ngc_tag, auto ngt_tag, auto bw_tag, int kgn, bool with_dma, int sn, int slot) __attribute__((always_inline)) {
            constexpr int NGC = decltype(ngc_tag)::value;
            constexpr int NGT = decltype(ngt_tag)::value;
            constexpr int BW = decltype(bw_tag)::value;
            if constexpr (NGC == 4)
                asm volatile("s_waitcnt vmcnt(%4)" : "+v"(Bs[k][0]), "+v"(Bs[k][1]), "+v"(Bs[k][2]), "+v"(Bs[k][3]) : "n"(BW));
            else
                asm volatile("s_waitcnt vmcnt(%3)" : "+v"(Bs[k][0]), "+v"(Bs[k][1]), "+v"(Bs[k][2]) : "n"(BW));
            const bool own_a = sn < S;
            const int64_t aofs = (int64_t)(own_a ? sn : sn - S) * a_stage;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (g < NGC) {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        acc[i][g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, F.v[i]),
                                                                           __builtin_bit_cast(bf16x8, Bs[k][g]), acc[i][g], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (g < NGT) load_b_frag(Bs[k][g], cur_t, kgn, g);
                // (the stage's source is chosen by selecting the pointer, not by branching)
                if (with_dma)
                    __builtin_amdgcn_global_load_lds(JITDB_GLOBAL_PTR((own_a ? cur_t.pa[g] : next_t.pa[g]) + aofs),
                                                     JITDB_LDS_PTR(ring + slot * kStageBytes + (wave * 4 + g) * 1024), 16, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        // Two stages = kPF K groups: the loop body.  NGT = 0 marks the tile's last body.
        auto body = [&](int s, auto ngc_tag, auto ngt_tag) __attribute__((always_inline)) {
            constexpr bool TAIL = decltype(ngt_tag)::value == 0;
            const std::integral_constant<int, BWAIT> w_steady;
            const std::integral_constant<int, 2 * NG + 5> w_t1;
            const std::integral_constant<int, NG + 8> w_t2;
            const std::integral_constant<int, 5> w_t3;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int ss = s + u;
                const int nxt = cur == kRing - 1 ? 0 : cur + 1;
                read_frags(cur, 1, Q);
                __builtin_amdgcn_sched_barrier(0);
                if (TAIL && u == 1) half(P, 2, ngc_tag, ngt_tag, w_t2, 2 * ss + kPF, false, 0, 0);
                else half(P, 2 * u, ngc_tag, ngt_tag, w_steady, 2 * ss + kPF, false, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                reads_done(Q);
                // stage ss + 1 has landed; everyone has read stage ss
                if (TAIL && u == 0) wait_barrier256<NWAIT_T1>();
                else if (TAIL) wait_barrier256<NWAIT_T2>();
                else wait_barrier256<NWAIT>();
                // (after a tile's last stage the next tile reads its own first fragments)
                if (!(TAIL && u == 1)) {
                    read_frags(nxt, 0, P);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (TAIL && u == 0) half(Q, 1, ngc_tag, ngt_tag, w_t1, 2 * ss + 1 + kPF, true, ss + kRing, cur);
                else if (TAIL) half(Q, 3, ngc_tag, ngt_tag, w_t3, 2 * ss + 1 + kPF, true, ss + kRing, cur);
                else half(Q, 2 * u + 1, ngc_tag, ngt_tag, w_steady, 2 * ss + 1 + kPF, true, ss + kRing, cur);
                __builtin_amdgcn_sched_barrier(0);
                if (!(TAIL && u == 1)) reads_done(P);
                cur = nxt;
            }
        };
        const std::integral_constant<int, Gates256<MODE>::X> ngx;
        const std::integral_constant<int, Gates256<MODE>::H> ngh;
        const std::integral_constant<int, 0> none;
        // the fragments requested in a body are multiplied one body later: in the last body of the
        // x part they belong to the h part
        if constexpr (MODE == MODE_LEAF) {
            int s = 0;
            for (; s < S - 2; s += 2) body(s, ngx, ngx);
            body(s, ngx, none);
        } else if constexpr (MODE == MODE_PROJ) {
            int s = 0;
            for (; s < S - 2; s += 2) body(s, ngh, ngh);
            body(s, ngh, none);
        } else {
            const int sx = nkg_x >> 1;
            int s = 0;
            for (; s < sx - 2; s += 2) body(s, ngx, ngx);
            body(s, ngx, ngh);
            s += 2;
            for (; s < S - 2; s += 2) body(s, ngh, ngh);
            body(s, ngh, none);
        }

        // ---- what the accumulators turn into: four passes of 32 rows.  The passes run as a real
        // loop over one copy of the code (the accumulators of pass i are moved to a fixed set of
        // registers first): unrolled, the compiler carries values of all four passes side by side
        // and runs out of registers.
        float *region = regions + wave * kRegion;
#pragma nounroll
        for (int i = 0; i < 4; ++i) {
            floatx16 pa4[4];
            switch (i) {
                case 0: pa4[0] = acc[0][0]; pa4[1] = acc[0][1]; pa4[2] = acc[0][2]; pa4[3] = acc[0][3]; break;
                case 1: pa4[0] = acc[1][0]; pa4[1] = acc[1][1]; pa4[2] = acc[1][2]; pa4[3] = acc[1][3]; break;
                case 2: pa4[0] = acc[2][0]; pa4[1] = acc[2][1]; pa4[2] = acc[2][2]; pa4[3] = acc[2][3]; break;
                default: pa4[0] = acc[3][0]; pa4[1] = acc[3][1]; pa4[2] = acc[3][2]; pa4[3] = acc[3][3]; break;
            }
            const int r0 = wm * 128 + i * 32;
            if constexpr (MODE == MODE_PROJ)
                proj_pass<bf16_t>(a, pa4, region, row_node + r0, cur_t.col_tile * 256 + wn * 128, lane);
            else
                cell_pass<bf16_t, MODE, false>(a, pa4, region, row_node + r0, row_ar + (MODE == MODE_INTERNAL ? r0 : 0),
                                               row_cb + (MODE == MODE_INTERNAL ? r0 : 0),
                                               row_kid + (MODE == MODE_INTERNAL ? r0 : 0), cur_t.col_tile * 2 + wn, lane, bias);
        }
    }
    wait_barrier256<0>();      // nothing is on its way to LDS when the block ends
}

}  // namespace

// Does the tile kernel take this launch?  bf16 levels large enough to give every CU several
// tiles, with a K loop long enough for the ring's pipeline (kRing stages ahead).
bool tile256_applies(int mode, const LevelArgs &a) {
    const int n_x = mode == MODE_PROJ ? 0 : a.Dp * 2 / kStage256;
    const int n_h = mode == MODE_LEAF ? 0 : a.Hp * 2 / kStage256;
    if (n_x + n_h < 8) return false;
    if (mode == MODE_INTERNAL && (n_x < 2 || n_h < 2)) return false;
    if (a.n_rows < kTile256MinRows[mode]) return false;
    return true;
}

// a.n_rows, a.n_rows_alloc (a multiple of 256), a.Bf and the usual level arguments are set by the caller.
int launch_tile256(int mode, LevelArgs a, hipStream_t st) {
    a.n_row_tiles = (int)ceil_div(a.n_rows, kBM256);
    const int n_unit_tiles = a.Hu / kUnit;
    a.n_col_tiles = mode == MODE_PROJ ? (int)ceil_div(n_unit_tiles, 8) : a.NP / kBN;
    const unsigned grid = 256;       // one block per CU; blocks without a tile return at once
    if (mode == MODE_LEAF) tile256_kernel<MODE_LEAF><<<grid, kT256, 0, st>>>(a);
    else if (mode == MODE_INTERNAL) tile256_kernel<MODE_INTERNAL><<<grid, kT256, 0, st>>>(a);
    else tile256_kernel<MODE_PROJ><<<grid, kT256, 0, st>>>(a);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

}  // namespace jitdb
