// jitdb_schedule: the analysis half of the method, as int32 HIP kernels for gfx950.
//
// The paper files each computation node in a table by its depth in the
// computation graph and batches the nodes of one depth (section 4.2, 4.3).
// For trees evaluated bottom-up that depth is the node height.  This file
// computes, entirely on the GPU:
//
//   child counts          one atomic add per node
//   child_ptr             exclusive scan of the counts
//   height                pointer jumping: in round k every node pushes
//                         height + 2^k to its 2^k-th ancestor (atomic max) and
//                         doubles its ancestor pointer; ceil(log2 N) rounds at
//                         most, rounds after the last live one return at once
//   level_ptr             histogram of heights + exclusive scan
//   perm / inv_perm       stable LSD radix sort of node ids by height
//   child_idx             stable LSD radix sort of node ids by parent
//
// jitdb_schedule_typed files by (height, signature, parent's signature) instead: the sort key
// and the histogram take that triple, everything else is the same code.  jitdb_schedule_append
// schedules arriving trees alone and merges the two tables in one linear pass.
//
// Stability of the radix passes is what gives the ascending-id order inside a
// level and inside a child list, so the result is unique and bit-reproducible.
// All atomics are integer add / max / or (order independent).

#include "common.h"

namespace jitdb {
namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;
constexpr int kWavesPerBlock = kThreads / kWave;

// ---- device-side bookkeeping words -------------------------------------------------
enum : int { META_ERR = 0, META_EDGES = 1, META_MAXH = 2, META_SIG = 3, META_LIVE = 8, META_WORDS = 64 };

// Thousands of waves updating ONE word with atomics serialise in L2 (about 10 ns each on
// MI355X, measured: 0.4 ms for one atomic per wave at 2.4 M nodes).  Flags are therefore set
// with a relaxed load-then-store (a benign race: every writer stores the same value), and
// reductions go through the block first.

// ---- exclusive scan (three phases, no inter-block waiting) -------------------------
constexpr int kScanItems = 16;
constexpr int kScanChunk = kThreads * kScanItems;  // 4096 elements per block

__device__ __forceinline__ int wave_inclusive_scan(int v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        int t = __shfl_up(v, d, kWave);
        if (lane >= d) v += t;
    }
    return v;
}

// Exclusive prefix of one value per thread over the block; *total gets the block sum.
__device__ __forceinline__ int block_exclusive_scan(int v, int *total) {
    __shared__ int wave_sum[kWavesPerBlock];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    int inc = wave_inclusive_scan(v);
    if (lane == kWave - 1) wave_sum[wave] = inc;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) {
        int s = wave_sum[w];
        if (w < wave) before += s;
        all += s;
    }
    __syncthreads();
    *total = all;
    return before + inc - v;
}

__global__ void __launch_bounds__(kThreads)
scan_reduce_kernel(const int32_t *__restrict__ in, int64_t n_in, int32_t *__restrict__ partial) {
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    int s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        int64_t idx = base + i;
        if (idx < n_in) s += in[idx];
    }
    int total;
    block_exclusive_scan(s, &total);
    if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

// One block turns the per-chunk sums into exclusive offsets, in place.
__global__ void __launch_bounds__(kThreads)
scan_partials_kernel(int32_t *partial, int n_partial) {
    int carry = 0;
    for (int base = 0; base < n_partial; base += kThreads) {
        int idx = base + threadIdx.x;
        int v = idx < n_partial ? partial[idx] : 0;
        int total;
        int ex = block_exclusive_scan(v, &total);
        if (idx < n_partial) partial[idx] = carry + ex;
        carry += total;
    }
}

// out[i] = sum of in[0..i) for i < n_out; in[i] counts as 0 for i >= n_in.  in == out is allowed.
__global__ void __launch_bounds__(kThreads)
scan_apply_kernel(const int32_t *in, int64_t n_in, int32_t *out, int64_t n_out,
                  const int32_t *__restrict__ partial) {
    const int64_t base = (int64_t)blockIdx.x * kScanChunk + (int64_t)threadIdx.x * kScanItems;
    int v[kScanItems];
    int s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        int64_t idx = base + i;
        v[i] = idx < n_in ? in[idx] : 0;
        s += v[i];
    }
    int total;
    int run = block_exclusive_scan(s, &total) + partial[blockIdx.x];
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        int64_t idx = base + i;
        if (idx < n_out) out[idx] = run;
        run += v[i];
    }
}

// The same scan by one block, chunk after chunk with a running carry: one launch instead of three where the
// array is short (the schedule of a small forest costs its number of launches, not its work).
constexpr int kScanOneBlockChunks = 4;
__global__ void __launch_bounds__(kThreads)
scan_one_block_kernel(const int32_t *in, int64_t n_in, int32_t *out, int64_t n_out) {
    int carry = 0;
    for (int64_t chunk = 0; chunk < n_out; chunk += kScanChunk) {
        const int64_t base = chunk + (int64_t)threadIdx.x * kScanItems;
        int v[kScanItems];
        int s = 0;
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            const int64_t idx = base + i;
            v[i] = idx < n_in ? in[idx] : 0;
            s += v[i];
        }
        int total;
        int run = block_exclusive_scan(s, &total) + carry;
#pragma unroll
        for (int i = 0; i < kScanItems; ++i) {
            const int64_t idx = base + i;
            if (idx < n_out) out[idx] = run;
            run += v[i];
        }
        carry += total;
    }
}

int launch_exclusive_scan(const int32_t *in, int64_t n_in, int32_t *out, int64_t n_out,
                          int32_t *partial, hipStream_t st) {
    if (n_out <= 0) return JITDB_OK;
    const int nb = (int)ceil_div(n_out, kScanChunk);
    if (nb <= kScanOneBlockChunks) {
        scan_one_block_kernel<<<1, kThreads, 0, st>>>(in, n_in, out, n_out);
        JITDB_LAUNCH_CHECK();
        return JITDB_OK;
    }
    scan_reduce_kernel<<<nb, kThreads, 0, st>>>(in, n_in, partial);
    JITDB_LAUNCH_CHECK();
    scan_partials_kernel<<<1, kThreads, 0, st>>>(partial, nb);
    JITDB_LAUNCH_CHECK();
    scan_apply_kernel<<<nb, kThreads, 0, st>>>(in, n_in, out, n_out, partial);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

// ---- small utilities ---------------------------------------------------------------
__global__ void __launch_bounds__(kThreads)
fill_kernel(int32_t *__restrict__ p, int64_t n, int32_t value) {
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = value;
}

int launch_fill(int32_t *p, int64_t n, int32_t value, hipStream_t st) {
    if (n <= 0) return JITDB_OK;
    fill_kernel<<<(unsigned)ceil_div(n, kThreads), kThreads, 0, st>>>(p, n, value);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}

// ---- child counts, validation, round-0 ancestor pointers ---------------------------
__global__ void __launch_bounds__(kThreads)
count_children_kernel(const int32_t *__restrict__ parent, int32_t n, int32_t *__restrict__ cnt,
                      int32_t *__restrict__ anc, int32_t *__restrict__ height,
                      int32_t *__restrict__ meta) {
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    bool bad = false;
    if (v < n) {
        int32_t p = parent[v];
        bad = (p < -1) || (p >= n) || (p == (int32_t)v);
        if (bad) p = -1;  // keeps every later access in bounds
        anc[v] = p;
        height[v] = 0;
        if (p >= 0) atomicAdd(&cnt[p], 1);
    }
    const unsigned long long bads = __ballot(bad);
    if (bads && (threadIdx.x & (kWave - 1)) == 0) atomicOr(&meta[META_ERR], 1);   // rare
}

// ---- signatures (the generic batcher's second key) ----------------------------------
// A signature must lie in [0, n_sig).
__global__ void __launch_bounds__(kThreads)
check_signatures_kernel(const int32_t *__restrict__ sig, int32_t n, int32_t n_sig, int32_t *__restrict__ meta) {
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    bool bad = false;
    if (v < n) {
        const int32_t t = sig[v];
        bad = t < 0 || t >= n_sig;
    }
    const unsigned long long bads = __ballot(bad);
    if (bads && (threadIdx.x & (kWave - 1)) == 0) atomicOr(&meta[META_SIG], 1);   // rare
}

// key = (height * n_sig + sig) * n_sig + psig, psig = the parent's signature (a root: its own).
// A node meets two sets of partners: its own cell batches it with its (height, sig), the forget
// projection of its parent's cell with its (height, psig); sorting by this key keeps both
// contiguous (the first as a run of n_sig sub-slots).  Runs after the parent array and the
// signatures have been validated.
__global__ void __launch_bounds__(kThreads)
slot_key_kernel(const int32_t *__restrict__ parent, const int32_t *__restrict__ height,
                const int32_t *__restrict__ sig, int32_t n, int32_t n_sig, int32_t *__restrict__ key) {
    const int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (v >= n) return;
    const int32_t p = parent[v];
    const int32_t t = sig[v];
    key[v] = (height[v] * n_sig + t) * n_sig + (p >= 0 ? sig[p] : t);
}

// level_ptr[l] = slot_ptr[l * stride], l = 0 .. n_levels
__global__ void __launch_bounds__(kThreads)
level_from_slots_kernel(const int32_t *__restrict__ slot_ptr, int32_t n_levels, int32_t stride,
                        int32_t *__restrict__ level_ptr) {
    const int64_t l = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (l <= n_levels) level_ptr[l] = slot_ptr[l * stride];
}

// Round k of pointer jumping.  anc_in[v] is the 2^k-th ancestor of v (or -1).
// Any value ever stored in height[] is the length of a real downward path, so
// reading a neighbour's height while it is still growing can only delay, never
// spoil, the result: after round k, height[a] >= the longest path shorter than
// 2^(k+1) below a.
__global__ void __launch_bounds__(kThreads)
jump_kernel(const int32_t *__restrict__ anc_in, int32_t *__restrict__ anc_out,
            int32_t *height, int32_t n, int k, int32_t *meta) {
    if (k > 0 && meta[META_LIVE + k - 1] == 0) return;  // uniform: nothing moved last round
    bool live = false;
    for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < n; v += (int64_t)gridDim.x * kThreads) {
        const int32_t a = anc_in[v];
        int32_t next = -1;
        if (a >= 0) {
            const int32_t hv = __atomic_load_n(&height[v], __ATOMIC_RELAXED);
            atomicMax(&height[a], hv + (1 << k));
            next = anc_in[a];
            live |= next >= 0;
        }
        anc_out[v] = next;
    }
    const unsigned long long any = __ballot(live);
    if (any && (threadIdx.x & (kWave - 1)) == 0 &&
        __atomic_load_n(&meta[META_LIVE + k], __ATOMIC_RELAXED) == 0)
        __atomic_store_n(&meta[META_LIVE + k], 1, __ATOMIC_RELAXED);
}

// Every round of the pointer jumping in one launch, by one block: for forests small enough that a round is a
// few passes of the block over the nodes.  The rounds are jump_kernel's (same reads, same atomic maxima, same
// flags in meta); a barrier stands where the next launch would, and the block stops after the first round in
// which no pointer moved.
constexpr int kJumpOneBlockThreads = 1024;
constexpr int kJumpOneBlockNodes = 8 * kJumpOneBlockThreads;
__global__ void __launch_bounds__(kJumpOneBlockThreads)
jump_one_block_kernel(int32_t *anc0, int32_t *anc1, int32_t *height, int32_t n, int rounds, int32_t *meta) {
    for (int k = 0; k < rounds; ++k) {
        const int32_t *anc_in = (k & 1) ? anc1 : anc0;
        int32_t *anc_out = (k & 1) ? anc0 : anc1;
        int live = 0;
        for (int v = threadIdx.x; v < n; v += kJumpOneBlockThreads) {
            const int32_t a = anc_in[v];
            int32_t next = -1;
            if (a >= 0) {
                const int32_t hv = __atomic_load_n(&height[v], __ATOMIC_RELAXED);
                atomicMax(&height[a], hv + (1 << k));
                next = anc_in[a];
                live |= next >= 0;
            }
            anc_out[v] = next;
        }
        const int any = __syncthreads_or(live);      // also: this round's stores and maxima before the next round's reads
        if (threadIdx.x == 0 && any) meta[META_LIVE + k] = 1;
        if (!any) break;
    }
}

__global__ void __launch_bounds__(kThreads)
max_height_kernel(const int32_t *__restrict__ height, int32_t n, const int32_t *__restrict__ child_ptr,
                  int32_t *__restrict__ meta) {
    __shared__ int wave_max[kWavesPerBlock];
    int m = 0;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * kThreads)
        m = max(m, height[i]);
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) m = max(m, __shfl_xor(m, d, kWave));
    if ((threadIdx.x & (kWave - 1)) == 0) wave_max[threadIdx.x / kWave] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) m = max(m, wave_max[w]);
        if (m > __atomic_load_n(&meta[META_MAXH], __ATOMIC_RELAXED)) atomicMax(&meta[META_MAXH], m);
        if (blockIdx.x == 0) meta[META_EDGES] = child_ptr[n];   // E = total number of children
    }
}

// ---- level histogram ---------------------------------------------------------------
constexpr int kLdsLevels = 2048;

__global__ void __launch_bounds__(kThreads)
level_hist_kernel(const int32_t *__restrict__ height, int32_t n, int32_t n_levels,
                  int32_t *__restrict__ level_cnt) {
    __shared__ int lds[kLdsLevels];
    const bool use_lds = n_levels <= kLdsLevels;
    if (use_lds) {
        for (int i = threadIdx.x; i < n_levels; i += kThreads) lds[i] = 0;
        __syncthreads();
    }
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * kThreads) {
        const int h = height[i];
        if (use_lds) atomicAdd(&lds[h], 1);
        else atomicAdd(&level_cnt[h], 1);
    }
    if (use_lds) {
        __syncthreads();
        for (int i = threadIdx.x; i < n_levels; i += kThreads) {
            const int c = lds[i];
            if (c) atomicAdd(&level_cnt[i], c);
        }
    }
}

// Children per level: every non-root node counts for the level of its parent.
__global__ void __launch_bounds__(kThreads)
level_kids_kernel(const int32_t *__restrict__ parent, const int32_t *__restrict__ height, int32_t n,
                  int32_t n_levels, int32_t *__restrict__ level_kids) {
    __shared__ int lds[kLdsLevels];
    const bool use_lds = n_levels <= kLdsLevels;
    if (use_lds) {
        for (int i = threadIdx.x; i < n_levels; i += kThreads) lds[i] = 0;
        __syncthreads();
    }
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * kThreads) {
        const int p = parent[i];
        if (p < 0) continue;
        const int h = height[p];
        if (use_lds) atomicAdd(&lds[h], 1);
        else atomicAdd(&level_kids[h], 1);
    }
    if (use_lds) {
        __syncthreads();
        for (int i = threadIdx.x; i < n_levels; i += kThreads) {
            const int c = lds[i];
            if (c) atomicAdd(&level_kids[i], c);
        }
    }
}

// ---- stable LSD radix sort of (key, node id) pairs, 8 bits per pass ----------------
constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kRadixItems = 8;                          // rounds of 64 keys per wave
constexpr int kWaveTile = kWave * kRadixItems;          // 512 consecutive keys per wave
constexpr int kBlockTile = kWaveTile * kWavesPerBlock;  // 2048 keys per block

// root_key >= 0: negative keys (roots of a parent array) sort as root_key, after every node id.
__device__ __forceinline__ int32_t load_key(const int32_t *keys, int64_t i, int32_t root_key) {
    int32_t k = keys[i];
    return (k < 0) ? root_key : k;
}

// block_hist is digit-major: [digit][block], so that its exclusive scan is the
// global start of every (digit, block) run.
__global__ void __launch_bounds__(kThreads)
radix_hist_kernel(const int32_t *__restrict__ keys, int32_t n, int shift, int32_t root_key,
                  int32_t *__restrict__ block_hist, int32_t n_blocks) {
    __shared__ int hist[kRadix];
    hist[threadIdx.x] = 0;  // kThreads == kRadix
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kBlockTile;
#pragma unroll
    for (int r = 0; r < kRadixItems; ++r) {
        const int64_t i = base + (int64_t)r * kThreads + threadIdx.x;
        if (i < n) atomicAdd(&hist[(load_key(keys, i, root_key) >> shift) & (kRadix - 1)], 1);
    }
    __syncthreads();
    block_hist[(int64_t)threadIdx.x * n_blocks + blockIdx.x] = hist[threadIdx.x];
}

// Each wave owns 512 consecutive keys and visits them 64 at a time, so the order
// (wave, round, lane) is the input order; ranks among equal digits follow it.
__global__ void __launch_bounds__(kThreads)
radix_scatter_kernel(const int32_t *__restrict__ keys, const int32_t *__restrict__ vals,
                     int32_t n, int shift, int32_t root_key,
                     const int32_t *__restrict__ block_ofs, int32_t n_blocks,
                     int32_t *__restrict__ keys_out, int32_t *__restrict__ vals_out) {
    __shared__ int wave_cnt[kWavesPerBlock][kRadix];
    __shared__ int wave_ofs[kWavesPerBlock][kRadix];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) wave_cnt[w][threadIdx.x] = 0;
    __syncthreads();

    const int64_t base = (int64_t)blockIdx.x * kBlockTile + (int64_t)wave * kWaveTile;
    const unsigned long long below = (1ull << lane) - 1ull;
    int32_t key[kRadixItems], val[kRadixItems], rank[kRadixItems];
#pragma unroll
    for (int r = 0; r < kRadixItems; ++r) {
        const int64_t i = base + (int64_t)r * kWave + lane;
        const bool valid = i < n;
        key[r] = valid ? load_key(keys, i, root_key) : 0;
        val[r] = valid ? (vals ? vals[i] : (int32_t)i) : 0;
        const int d = (key[r] >> shift) & (kRadix - 1);
        unsigned long long same = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kRadixBits; ++b) {
            const bool bit = (d >> b) & 1;
            const unsigned long long bal = __ballot(bit);
            same &= bit ? bal : ~bal;
        }
        if (!valid) same = 0;
        const int leader = same ? (__ffsll((long long)same) - 1) : 0;
        int prev = 0;
        if (valid && lane == leader) prev = atomicAdd(&wave_cnt[wave][d], (int)__popcll(same));
        prev = __shfl(prev, leader, kWave);
        rank[r] = prev + (int)__popcll(same & below);
    }
    __syncthreads();
    {
        const int d = threadIdx.x;
        int run = block_ofs[(int64_t)d * n_blocks + blockIdx.x];
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) {
            wave_ofs[w][d] = run;
            run += wave_cnt[w][d];
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRadixItems; ++r) {
        const int64_t i = base + (int64_t)r * kWave + lane;
        if (i < n) {
            const int d = (key[r] >> shift) & (kRadix - 1);
            const int pos = wave_ofs[wave][d] + rank[r];
            if (keys_out) keys_out[pos] = key[r];
            vals_out[pos] = val[r];
        }
    }
}

int bits_needed(int64_t max_value) {
    int b = 1;
    while (b < 31 && (int64_t(1) << b) <= max_value) ++b;
    return b;
}

struct SortScratch {
    int32_t *keys[2];
    int32_t *vals[2];
    int32_t *block_hist;
    int32_t *partial;
};

// vals_out[0..n) = node ids 0..n-1 stably sorted by key (negative keys last if root_key >= 0).
int radix_sort_ids(const int32_t *keys, int32_t n, int key_bits, int32_t root_key,
                   int32_t *vals_out, const SortScratch &sc, hipStream_t st) {
    const int passes = (key_bits + kRadixBits - 1) / kRadixBits;
    const int n_blocks = (int)ceil_div(n, kBlockTile);
    const int32_t *src_keys = keys;
    const int32_t *src_vals = nullptr;
    int32_t rk = root_key;
    for (int p = 0; p < passes; ++p) {
        const bool last = (p == passes - 1);
        int32_t *dst_keys = last ? nullptr : sc.keys[p & 1];
        int32_t *dst_vals = last ? vals_out : sc.vals[p & 1];
        const int shift = p * kRadixBits;
        radix_hist_kernel<<<n_blocks, kThreads, 0, st>>>(src_keys, n, shift, rk, sc.block_hist, n_blocks);
        JITDB_LAUNCH_CHECK();
        const int64_t m = (int64_t)kRadix * n_blocks;
        int rc = launch_exclusive_scan(sc.block_hist, m, sc.block_hist, m, sc.partial, st);
        if (rc != JITDB_OK) return rc;
        radix_scatter_kernel<<<n_blocks, kThreads, 0, st>>>(src_keys, src_vals, n, shift, rk,
                                                            sc.block_hist, n_blocks, dst_keys, dst_vals);
        JITDB_LAUNCH_CHECK();
        src_keys = dst_keys;
        src_vals = dst_vals;
        rk = -1;  // remapped keys were written out; later passes read them as they are
    }
    return JITDB_OK;
}

__global__ void __launch_bounds__(kThreads)
invert_perm_kernel(const int32_t *__restrict__ perm, int32_t n, int32_t *__restrict__ inv_perm) {
    const int64_t p = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (p < n) inv_perm[perm[p]] = (int32_t)p;
}

// ---- workspace ---------------------------------------------------------------------
struct ScheduleWs {
    int32_t *meta;
    int32_t *cnt;
    int32_t *anc[2];
    SortScratch sort;
    size_t bytes;
};

ScheduleWs carve_schedule_ws(int64_t n, void *base, int64_t n_keys = 1) {   // n_keys: sort keys per level
    Carver c(base);
    ScheduleWs w;
    const int64_t n_blocks = ceil_div(n > 0 ? n : 1, kBlockTile);
    const int64_t hist_len = (int64_t)kRadix * n_blocks;
    const int64_t scan_len = (hist_len > n * n_keys + 1 ? hist_len : n * n_keys + 1);   // longest array ever scanned
    w.meta = c.take<int32_t>(META_WORDS);
    w.cnt = c.take<int32_t>(n + 1);
    w.anc[0] = c.take<int32_t>(n);
    w.anc[1] = c.take<int32_t>(n);
    w.sort.keys[0] = c.take<int32_t>(n);
    w.sort.keys[1] = c.take<int32_t>(n);
    w.sort.vals[0] = c.take<int32_t>(n);
    w.sort.vals[1] = c.take<int32_t>(n);
    w.sort.block_hist = c.take<int32_t>(hist_len);
    w.sort.partial = c.take<int32_t>(ceil_div(scan_len, kScanChunk) + 1);
    w.bytes = c.off;
    return w;
}

// ---- appending trees to a schedule ---------------------------------------------------
// New nodes get ids n_a + v, so inside every level they sort after the old ones and inside
// every child list there is nothing to interleave (trees do not share nodes): the merged
// schedule is the old one with every level segment shifted by the number of new nodes in
// lower levels, and the new one shifted by the number of old nodes up to and including
// its level.  lpa / lpn are the two level_ptr arrays (valid up to la / ln).
__global__ void __launch_bounds__(kThreads)
append_merge_kernel(const int32_t *__restrict__ ha, const int32_t *__restrict__ perma,
                    const int32_t *__restrict__ cpa, const int32_t *__restrict__ cia,
                    const int32_t *__restrict__ lpa, int32_t na, int32_t ea, int32_t la,
                    const int32_t *__restrict__ hn, const int32_t *__restrict__ permn,
                    const int32_t *__restrict__ cpn, const int32_t *__restrict__ cin,
                    const int32_t *__restrict__ lpn, int32_t nn, int32_t en, int32_t ln,
                    int32_t *__restrict__ height, int32_t *__restrict__ level_ptr, int32_t *__restrict__ perm,
                    int32_t *__restrict__ inv_perm, int32_t *__restrict__ child_ptr,
                    int32_t *__restrict__ child_idx) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int32_t l_out = la > ln ? la : ln;
    if (i <= l_out) {
        const int32_t a = na > 0 ? lpa[i < la ? i : la] : 0;
        const int32_t b = nn > 0 ? lpn[i < ln ? i : ln] : 0;
        level_ptr[i] = a + b;
    }
    if (i < na) {
        height[i] = ha[i];
        const int32_t node = perma[i];
        const int32_t l = ha[node];
        const int32_t shift = nn > 0 ? lpn[l < ln ? l : ln] : 0;     // new nodes in lower levels
        perm[i + shift] = node;
        inv_perm[node] = (int32_t)i + shift;
        child_ptr[i] = cpa[i];
    }
    if (i < ea) child_idx[i] = cia[i];
    if (i < nn) {
        height[na + i] = hn[i];
        const int32_t v = permn[i];
        const int32_t l = hn[v];
        const int32_t shift = na > 0 ? lpa[l + 1 < la ? l + 1 : la] : 0;   // old nodes up to its level
        perm[i + shift] = na + v;
        inv_perm[na + v] = (int32_t)i + shift;
    }
    if (i <= nn) child_ptr[na + i] = ea + (nn > 0 ? cpn[i] : 0);
    if (i < en) child_idx[ea + i] = na + cin[i];
}

struct AppendWs {
    int32_t *height, *level_ptr, *perm, *inv_perm, *child_ptr, *child_idx;   // schedule of the new part
    void *sched_ws;
    size_t sched_ws_bytes;
    size_t bytes;
};

AppendWs carve_append_ws(int64_t n_new, void *base) {
    Carver c(base);
    AppendWs w;
    w.height = c.take<int32_t>(n_new);
    w.level_ptr = c.take<int32_t>(n_new + 1);
    w.perm = c.take<int32_t>(n_new);
    w.inv_perm = c.take<int32_t>(n_new);
    w.child_ptr = c.take<int32_t>(n_new + 1);
    w.child_idx = c.take<int32_t>(n_new);
    w.sched_ws_bytes = carve_schedule_ws(n_new, nullptr).bytes;
    w.sched_ws = c.take<char>(w.sched_ws_bytes);
    w.bytes = c.off;
    return w;
}

}  // namespace
}  // namespace jitdb

using namespace jitdb;

extern "C" size_t jitdb_schedule_workspace_bytes(int64_t n_nodes) {
    if (n_nodes < 0 || n_nodes > JITDB_MAX_NODES) return 0;
    return carve_schedule_ws(n_nodes, nullptr).bytes;
}

namespace {
// The analysis, plain (sig == nullptr: one slot per level) or filed by (depth, signature).
int schedule_impl(const int32_t *parent, const int32_t *sig, jitdb_slots_t *slots, jitdb_schedule_t *s,
                  void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!s) return JITDB_E_NULL;
    drop_stale_hip_error();
    const int32_t n_sig = slots ? slots->n_sig : 1;
    const int64_t n_keys = (int64_t)n_sig * n_sig;      // sub-slots per level
    if (slots) {
        if (n_sig < 1 || n_sig > JITDB_MAX_SIGNATURES) return JITDB_E_BADARG;
        if (s->n_nodes * n_keys >= (int64_t(1) << 31)) return JITDB_E_BADARG;
        if (!slots->host_slot_ptr) return JITDB_E_NULL;
        if (slots->slot_capacity < 1) return JITDB_E_BADARG;
        slots->host_slot_ptr[0] = 0;
    }
    const int64_t n64 = s->n_nodes;
    if (n64 < 0 || n64 > JITDB_MAX_NODES) return JITDB_E_BADARG;
    if (!s->host_level_ptr) return JITDB_E_NULL;
    s->n_levels = 0;
    s->n_edges = 0;
    if (n64 == 0) {
        s->host_level_ptr[0] = 0;
        if (s->host_level_kids) s->host_level_kids[0] = 0;
        if (slots && slots->slot_ptr) {
            int rc = launch_fill(slots->slot_ptr, 1, 0, (hipStream_t)hip_stream);
            if (rc != JITDB_OK) return rc;
        }
        if (s->level_ptr) {
            int rc = launch_fill(s->level_ptr, 1, 0, (hipStream_t)hip_stream);
            if (rc != JITDB_OK) return rc;
        }
        if (s->child_ptr) {
            int rc = launch_fill(s->child_ptr, 1, 0, (hipStream_t)hip_stream);
            if (rc != JITDB_OK) return rc;
        }
        return JITDB_OK;
    }
    if (!parent || !s->height || !s->level_ptr || !s->perm || !s->inv_perm || !s->child_ptr ||
        !s->child_idx || !workspace)
        return JITDB_E_NULL;
    if (slots && (!sig || !slots->key || !slots->slot_ptr)) return JITDB_E_NULL;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return JITDB_E_BADARG;
    ScheduleWs w = carve_schedule_ws(n64, workspace, n_keys);
    if (workspace_bytes < w.bytes) return JITDB_E_WORKSPACE;

    hipStream_t st = (hipStream_t)hip_stream;
    const int32_t n = (int32_t)n64;
    const unsigned grid = (unsigned)ceil_div(n64, kThreads);
    int rc;

    // 1. child counts + validation
    //    (the bookkeeping words and the counts lie back to back in the workspace: one fill)
    if ((rc = launch_fill(w.meta, (w.cnt - w.meta) + n64 + 1, 0, st)) != JITDB_OK) return rc;
    count_children_kernel<<<grid, kThreads, 0, st>>>(parent, n, w.cnt, w.anc[0], s->height, w.meta);
    JITDB_LAUNCH_CHECK();
    if (slots) {
        check_signatures_kernel<<<grid, kThreads, 0, st>>>(sig, n, n_sig, w.meta);
        JITDB_LAUNCH_CHECK();
    }

    // 2. child_ptr = exclusive scan of the counts (N + 1 entries, the last is E)
    if ((rc = launch_exclusive_scan(w.cnt, n64, s->child_ptr, n64 + 1, w.sort.partial, st)) != JITDB_OK)
        return rc;

    // 3. heights by pointer jumping: after round k the pointers are 2^(k+1)-th
    //    ancestors; in a forest they are all -1 once 2^rounds >= N.
    int rounds = 0;
    while ((int64_t(1) << rounds) < n64) ++rounds;
    // (a capped grid with a stride loop: the rounds after the last live one are launched all the
    //  same and should cost a few thousand blocks' worth of "return", not a block per 256 nodes)
    const unsigned jump_grid = grid < 4096 ? grid : 4096;
    if (n <= kJumpOneBlockNodes && rounds > 0) {      // a small forest: all rounds in one launch
        jump_one_block_kernel<<<1, kJumpOneBlockThreads, 0, st>>>(w.anc[0], w.anc[1], s->height, n, rounds, w.meta);
        JITDB_LAUNCH_CHECK();
    } else {
        for (int k = 0; k < rounds; ++k) {
            jump_kernel<<<jump_grid, kThreads, 0, st>>>(w.anc[k & 1], w.anc[(k + 1) & 1], s->height, n, k, w.meta);
            JITDB_LAUNCH_CHECK();
        }
    }
    {
        const unsigned g = (unsigned)(ceil_div(n64, kThreads) < 1024 ? ceil_div(n64, kThreads) : 1024);
        max_height_kernel<<<g, kThreads, 0, st>>>(s->height, n, s->child_ptr, w.meta);
        JITDB_LAUNCH_CHECK();
    }

    int32_t meta[META_WORDS];
    JITDB_HIP_CHECK(hipMemcpyAsync(meta, w.meta, sizeof(meta), hipMemcpyDeviceToHost, st));
    JITDB_HIP_CHECK(hipStreamSynchronize(st));
    if (meta[META_ERR] != 0) return JITDB_E_PARENT_RANGE;
    if (meta[META_SIG] != 0) return JITDB_E_SIGNATURE;
    if (rounds > 0 && meta[META_LIVE + rounds - 1] != 0) return JITDB_E_CYCLE;
    if (meta[META_EDGES] >= n) return JITDB_E_CYCLE;  // every node has a parent: no forest
    const int32_t L = meta[META_MAXH] + 1;
    if (L > n) return JITDB_E_CYCLE;
    s->n_levels = L;
    s->n_edges = meta[META_EDGES];

    // 4. the table's slot boundaries = exclusive scan of the key histogram; key = height (one
    //    slot per level) or (height * n_sig + sig) * n_sig + psig
    const int64_t S = (int64_t)L * n_keys;            // (sub-)slots, empty ones included
    const int32_t *key = s->height;
    int32_t *bounds = s->level_ptr;
    if (slots) {
        if (S + 1 > slots->slot_capacity) return JITDB_E_WORKSPACE;
        slot_key_kernel<<<grid, kThreads, 0, st>>>(parent, s->height, sig, n, n_sig, slots->key);
        JITDB_LAUNCH_CHECK();
        key = slots->key;
        bounds = slots->slot_ptr;
    }
    if ((rc = launch_fill(bounds, S + 1, 0, st)) != JITDB_OK) return rc;
    {
        const unsigned g = (unsigned)(ceil_div(n64, kThreads) < 1024 ? ceil_div(n64, kThreads) : 1024);
        level_hist_kernel<<<g, kThreads, 0, st>>>(key, n, (int32_t)S, bounds);
        JITDB_LAUNCH_CHECK();
    }
    if ((rc = launch_exclusive_scan(bounds, S, bounds, S + 1, w.sort.partial, st)) != JITDB_OK)
        return rc;
    if (slots) {
        level_from_slots_kernel<<<(unsigned)ceil_div((int64_t)L + 1, kThreads), kThreads, 0, st>>>(
            slots->slot_ptr, L, (int32_t)n_keys, s->level_ptr);
        JITDB_LAUNCH_CHECK();
    }

    // 5. perm: node ids sorted by (key, id); inv_perm its inverse
    if ((rc = radix_sort_ids(key, n, bits_needed(S - 1), -1, s->perm, w.sort, st)) != JITDB_OK) return rc;
    invert_perm_kernel<<<grid, kThreads, 0, st>>>(s->perm, n, s->inv_perm);
    JITDB_LAUNCH_CHECK();

    // 6. child_idx: node ids sorted by (parent, id); roots sort last and fall
    //    outside the first E entries
    if ((rc = radix_sort_ids(parent, n, bits_needed(n64), n, s->child_idx, w.sort, st)) != JITDB_OK) return rc;

    // 7. (optional) children per level, for the forward's choice of kernels; the child counts'
    //    array is free again by now
    if (s->host_level_kids) {
        if ((rc = launch_fill(w.cnt, L, 0, st)) != JITDB_OK) return rc;
        const unsigned g = (unsigned)(ceil_div(n64, kThreads) < 1024 ? ceil_div(n64, kThreads) : 1024);
        level_kids_kernel<<<g, kThreads, 0, st>>>(parent, s->height, n, L, w.cnt);
        JITDB_LAUNCH_CHECK();
        JITDB_HIP_CHECK(hipMemcpyAsync(s->host_level_kids, w.cnt, sizeof(int32_t) * (size_t)L, hipMemcpyDeviceToHost, st));
    }

    if (slots) {
        JITDB_HIP_CHECK(hipMemcpyAsync(slots->host_slot_ptr, slots->slot_ptr, sizeof(int32_t) * ((size_t)S + 1),
                                       hipMemcpyDeviceToHost, st));
        JITDB_HIP_CHECK(hipStreamSynchronize(st));
        for (int l = 0; l <= L; ++l) s->host_level_ptr[l] = slots->host_slot_ptr[(int64_t)l * n_keys];
    } else {
        JITDB_HIP_CHECK(hipMemcpyAsync(s->host_level_ptr, s->level_ptr, sizeof(int32_t) * ((size_t)L + 1),
                                       hipMemcpyDeviceToHost, st));
        JITDB_HIP_CHECK(hipStreamSynchronize(st));
    }
    if (s->host_level_ptr[0] != 0 || s->host_level_ptr[L] != n) return JITDB_E_CYCLE;
    return JITDB_OK;
}
}  // namespace

extern "C" int jitdb_schedule(const int32_t *parent, jitdb_schedule_t *s,
                              void *workspace, size_t workspace_bytes, void *hip_stream) {
    return schedule_impl(parent, nullptr, nullptr, s, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t jitdb_schedule_typed_workspace_bytes(int64_t n_nodes, int32_t n_sig) {
    if (n_nodes < 0 || n_nodes > JITDB_MAX_NODES || n_sig < 1 || n_sig > JITDB_MAX_SIGNATURES) return 0;
    if (n_nodes * (int64_t)n_sig * n_sig >= (int64_t(1) << 31)) return 0;
    return carve_schedule_ws(n_nodes, nullptr, (int64_t)n_sig * n_sig).bytes;
}

extern "C" int jitdb_schedule_typed(const int32_t *parent, const int32_t *sig, jitdb_schedule_t *s,
                                    jitdb_slots_t *slots, void *workspace, size_t workspace_bytes,
                                    void *hip_stream) {
    if (!slots) return JITDB_E_NULL;
    return schedule_impl(parent, sig, slots, s, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t jitdb_schedule_append_workspace_bytes(int64_t n_base, int64_t n_new) {
    if (n_base < 0 || n_new < 0 || n_base + n_new > JITDB_MAX_NODES) return 0;
    return carve_append_ws(n_new, nullptr).bytes;
}

extern "C" int jitdb_schedule_append(const jitdb_schedule_t *base, const int32_t *parent_new, int64_t n_new,
                                     jitdb_schedule_t *out, void *workspace, size_t workspace_bytes,
                                     void *hip_stream) {
    if (!base || !out) return JITDB_E_NULL;
    drop_stale_hip_error();
    const int64_t na = base->n_nodes;
    if (na < 0 || n_new < 0 || na + n_new > JITDB_MAX_NODES) return JITDB_E_BADARG;
    if (out->n_nodes != na + n_new) return JITDB_E_BADARG;
    if (!out->host_level_ptr || !base->host_level_ptr) return JITDB_E_NULL;
    const int64_t n_out = na + n_new;
    if (n_out > 0 && (!out->height || !out->level_ptr || !out->perm || !out->inv_perm || !out->child_ptr ||
                      !out->child_idx))
        return JITDB_E_NULL;
    if (na > 0) {
        if (!base->height || !base->level_ptr || !base->perm || !base->child_ptr || !base->child_idx)
            return JITDB_E_NULL;
        const int32_t la = base->n_levels;
        if (la < 1 || la > na || base->n_edges < 0 || base->n_edges >= na) return JITDB_E_SCHEDULE;
        if (base->host_level_ptr[0] != 0 || base->host_level_ptr[la] != na) return JITDB_E_SCHEDULE;
    }
    if (n_new > 0 && (!parent_new || !workspace)) return JITDB_E_NULL;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255) != 0) return JITDB_E_BADARG;
    const AppendWs w = carve_append_ws(n_new, workspace);
    if (n_new > 0 && workspace_bytes < w.bytes) return JITDB_E_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;

    // the arriving trees on their own; their host level_ptr lands in the tail of the
    // output's host array, which the merged one (written front to back below) never
    // overtakes: entry l of the merged array is written after entry l of the new one is read
    jitdb_schedule_t fresh;
    fresh.n_nodes = n_new;
    fresh.height = w.height; fresh.level_ptr = w.level_ptr; fresh.perm = w.perm; fresh.inv_perm = w.inv_perm;
    fresh.child_ptr = w.child_ptr; fresh.child_idx = w.child_idx;
    fresh.host_level_ptr = out->host_level_ptr + na;
    // children per level add up like the level sizes; known only if both parts know theirs
    const bool kids_known = out->host_level_kids && (na == 0 || base->host_level_kids);
    fresh.host_level_kids = kids_known ? out->host_level_kids + na : nullptr;
    fresh.n_levels = 0; fresh.n_edges = 0;
    if (n_new > 0) {
        const int rc = jitdb_schedule(parent_new, &fresh, w.sched_ws, w.sched_ws_bytes, hip_stream);
        if (rc != JITDB_OK) return rc;
    }
    const int32_t la = na > 0 ? base->n_levels : 0, ln = fresh.n_levels;
    const int32_t l_out = la > ln ? la : ln;
    const int64_t ea = na > 0 ? base->n_edges : 0, en = fresh.n_edges;
    for (int32_t l = 0; l <= l_out; ++l) {
        const int32_t b = n_new > 0 ? fresh.host_level_ptr[l < ln ? l : ln] : 0;
        const int32_t a = na > 0 ? base->host_level_ptr[l < la ? l : la] : 0;
        out->host_level_ptr[l] = a + b;
        if (out->host_level_kids && l < l_out) {
            const int32_t kb = (kids_known && l < ln) ? fresh.host_level_kids[l] : 0;
            const int32_t ka = (kids_known && l < la) ? base->host_level_kids[l] : 0;
            out->host_level_kids[l] = !kids_known || ka < 0 || kb < 0 ? -1 : ka + kb;
        }
    }
    out->n_levels = l_out;
    out->n_edges = ea + en;
    if (n_out == 0) return JITDB_OK;

    const int64_t span = (na > n_new ? na : n_new) + 1;
    append_merge_kernel<<<(unsigned)ceil_div(span, kThreads), kThreads, 0, st>>>(
        base->height, base->perm, base->child_ptr, base->child_idx, base->level_ptr, (int32_t)na, (int32_t)ea, la,
        w.height, w.perm, w.child_ptr, w.child_idx, w.level_ptr, (int32_t)n_new, (int32_t)en, ln,
        out->height, out->level_ptr, out->perm, out->inv_perm, out->child_ptr, out->child_idx);
    JITDB_LAUNCH_CHECK();
    return JITDB_OK;
}
