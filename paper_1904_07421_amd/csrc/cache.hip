// Schedule cache: a fingerprint of the parent array computed on the device, and a host-side
// least-recently-used table from (fingerprint, N) to a slot the caller keeps a schedule in.
//
// The paper rewrites the graph once and reuses the cached result when the same structure
// is seen again (section 4.3); with a fingerprint as the key a training loop that revisits
// its batches pays one read of the parent array instead of the analysis.

#include "common.h"

#include <list>
#include <mutex>
#include <new>
#include <unordered_map>

namespace jitdb {
namespace {

constexpr int kT = 256;
constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;
constexpr uint64_t kKey1 = 0xD1B54A32D192ED03ull;

// output function of SplitMix64
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ void __launch_bounds__(kT)
fingerprint_clear_kernel(unsigned long long *fp) {
    if (threadIdx.x < 2) fp[threadIdx.x] = 0ull;
}

// fp[0] += sum mix64(word_i + GOLDEN), fp[1] += sum mix64(word_i ^ KEY1), word_i = i << 32 | parent[i].
// Sums modulo 2^64 commute, so the order of the partial sums does not matter.
__global__ void __launch_bounds__(kT)
fingerprint_kernel(const int32_t *__restrict__ parent, int64_t n, unsigned long long *__restrict__ fp) {
    uint64_t s0 = 0, s1 = 0;
    for (int64_t i = (int64_t)blockIdx.x * kT + threadIdx.x; i < n; i += (int64_t)gridDim.x * kT) {
        const uint64_t word = ((uint64_t)i << 32) | (uint32_t)parent[i];
        s0 += mix64(word + kGolden);
        s1 += mix64(word ^ kKey1);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        s0 += __shfl_down((unsigned long long)s0, d, 64);
        s1 += __shfl_down((unsigned long long)s1, d, 64);
    }
    __shared__ unsigned long long part[2][kT / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { part[0][wave] = s0; part[1][wave] = s1; }
    __syncthreads();
    if (threadIdx.x < 2) {
        unsigned long long s = 0;
        for (int w = 0; w < kT / 64; ++w) s += part[threadIdx.x][w];
        atomicAdd(&fp[threadIdx.x], s);
    }
}

struct Key {
    uint64_t f0, f1;
    int64_t n;
    bool operator==(const Key &o) const { return f0 == o.f0 && f1 == o.f1 && n == o.n; }
};
struct KeyHash {
    size_t operator()(const Key &k) const { return (size_t)(k.f0 ^ (k.f1 * 0x9E3779B97F4A7C15ull) ^ (uint64_t)k.n); }
};

}  // namespace
}  // namespace jitdb

using namespace jitdb;

// Least recently used first in `order`; `where` finds a key's place in it.
struct jitdb_cache {
    int32_t capacity;
    std::mutex lock;
    std::list<std::pair<Key, int32_t>> order;
    std::unordered_map<Key, std::list<std::pair<Key, int32_t>>::iterator, KeyHash> where;
    int64_t hits = 0, misses = 0;
};

extern "C" int jitdb_forest_fingerprint(const int32_t *parent, int64_t n_nodes, uint64_t *fp_dev,
                                        uint64_t *fp_host, void *hip_stream) {
    if (!fp_dev) return JITDB_E_NULL;
    if (n_nodes < 0 || n_nodes > JITDB_MAX_NODES) return JITDB_E_BADARG;
    if (n_nodes > 0 && !parent) return JITDB_E_NULL;
    drop_stale_hip_error();
    hipStream_t st = (hipStream_t)hip_stream;
    unsigned long long *fp = reinterpret_cast<unsigned long long *>(fp_dev);
    fingerprint_clear_kernel<<<1, kT, 0, st>>>(fp);
    JITDB_LAUNCH_CHECK();
    if (n_nodes > 0) {
        int64_t blocks = ceil_div(n_nodes, (int64_t)kT * 4);
        if (blocks > 2048) blocks = 2048;
        fingerprint_kernel<<<(unsigned)blocks, kT, 0, st>>>(parent, n_nodes, fp);
        JITDB_LAUNCH_CHECK();
    }
    if (fp_host) {
        JITDB_HIP_CHECK(hipMemcpyAsync(fp_host, fp_dev, 2 * sizeof(uint64_t), hipMemcpyDeviceToHost, st));
        JITDB_HIP_CHECK(hipStreamSynchronize(st));
    }
    return JITDB_OK;
}

extern "C" int jitdb_cache_create(int32_t capacity, jitdb_cache_t **out) {
    if (!out) return JITDB_E_NULL;
    *out = nullptr;
    if (capacity < 1 || capacity > (1 << 20)) return JITDB_E_BADARG;
    jitdb_cache *c = new (std::nothrow) jitdb_cache;
    if (!c) return JITDB_E_NOMEM;
    c->capacity = capacity;
    *out = c;
    return JITDB_OK;
}

extern "C" void jitdb_cache_destroy(jitdb_cache_t *cache) { delete cache; }

extern "C" int32_t jitdb_cache_lookup(jitdb_cache_t *cache, const uint64_t *fp, int64_t n_nodes) {
    if (!cache || !fp) return -1;
    const Key k{fp[0], fp[1], n_nodes};
    std::lock_guard<std::mutex> g(cache->lock);
    auto it = cache->where.find(k);
    if (it == cache->where.end()) {
        ++cache->misses;
        return -1;
    }
    ++cache->hits;
    cache->order.splice(cache->order.end(), cache->order, it->second);   // most recent = back
    return it->second->second;
}

extern "C" int32_t jitdb_cache_insert(jitdb_cache_t *cache, const uint64_t *fp, int64_t n_nodes, int32_t *evicted) {
    if (evicted) *evicted = 0;
    if (!cache || !fp) return -1;
    const Key k{fp[0], fp[1], n_nodes};
    std::lock_guard<std::mutex> g(cache->lock);
    auto it = cache->where.find(k);
    if (it != cache->where.end()) {
        cache->order.splice(cache->order.end(), cache->order, it->second);
        return it->second->second;
    }
    // Everything that allocates happens before the table changes: a failure reports "no slot"
    // (-1) and leaves the table as it was.
    std::list<std::pair<Key, int32_t>> fresh;
    try {
        fresh.emplace_back(k, 0);
        cache->where.emplace(k, fresh.begin());
    } catch (...) {
        return -1;
    }
    int32_t slot;
    if ((int32_t)cache->order.size() < cache->capacity) {
        // lowest free slot: slots are handed out densely, and freed only by eviction, which
        // reuses the slot at once, so the next free one is the current size
        slot = (int32_t)cache->order.size();
    } else {
        slot = cache->order.front().second;
        cache->where.erase(cache->order.front().first);
        cache->order.pop_front();
        if (evicted) *evicted = 1;
    }
    fresh.front().second = slot;
    cache->order.splice(cache->order.end(), fresh);      // iterators stay valid across a splice
    return slot;
}

extern "C" void jitdb_cache_stats(const jitdb_cache_t *cache, int64_t *hits, int64_t *misses, int32_t *entries) {
    if (!cache) return;
    jitdb_cache *c = const_cast<jitdb_cache *>(cache);
    std::lock_guard<std::mutex> g(c->lock);
    if (hits) *hits = c->hits;
    if (misses) *misses = c->misses;
    if (entries) *entries = (int32_t)c->order.size();
}
