// The index of an HBM hot-row cache: one 16-byte entry per 64 table rows holding a
// presence bitmap and the number of cached rows that precede the entry.  The cached
// rows are stored in ascending row order, so the slot of a cached row is that count
// plus the population count of the lower bitmap bits: one 16-byte probe decides hit
// or miss and yields the slot, with no collisions and no search.
#pragma once
#include "emb_internal.h"
#include "gather.h"

struct CacheEntry {
    uint64_t bits;    // bit i set: row 64*e + i is cached
    uint32_t before;  // number of cached rows with a smaller row number
    uint32_t pad;
};
static_assert(sizeof(CacheEntry) == 16, "cache index entry must be 16 bytes");

// Slot of row r (0 <= r < num_rows) in the cache, or -1 if the row is not cached.
__device__ __forceinline__ int64_t cache_probe(const CacheEntry *__restrict__ index, uint64_t r, uint64_t num_hot)
{
    const uint4 raw = load_chunk(reinterpret_cast<const char *>(index + (r >> 6)));   // device memory
    const uint64_t bits = ((uint64_t)raw.y << 32) | raw.x;
    const int bit = (int)(r & 63);
    if ((bits >> bit) & 1ull) {
        const uint64_t slot = (uint64_t)raw.z + (uint64_t)__popcll(bits & ((1ull << bit) - 1ull));
        if (slot < num_hot) return (int64_t)slot;   // always true for an index built from a valid hot set
    }
    return -1;
}

// hit_miss[0] += hits, hit_miss[1] += misses, summed over the workgroup first: every thread of the
// workgroup calls this (uniformly), one thread then adds the two totals.  Thousands of wavefronts
// adding to the same two words are served one at a time by the L2 and cost more than a whole
// lookup over HBM takes; one pair of adds per workgroup is a quarter of that (256 threads).
__device__ __forceinline__ void cache_add_hit_miss(uint32_t hits, uint32_t misses, unsigned long long *hit_miss)
{
    if (!hit_miss) return;   // uniform: a kernel argument
    __shared__ uint32_t s_hm[2];
    if (threadIdx.x == 0) s_hm[0] = s_hm[1] = 0;
    __syncthreads();
#pragma unroll
    for (int d = EMB_WAVE >> 1; d >= 1; d >>= 1) {
        hits += __shfl_xor(hits, d, EMB_WAVE);
        misses += __shfl_xor(misses, d, EMB_WAVE);
    }
    if ((threadIdx.x & (EMB_WAVE - 1)) == 0) {
        if (hits) atomicAdd(&s_hm[0], hits);
        if (misses) atomicAdd(&s_hm[1], misses);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (s_hm[0]) atomicAdd(&hit_miss[0], (unsigned long long)s_hm[0]);
        if (s_hm[1]) atomicAdd(&hit_miss[1], (unsigned long long)s_hm[1]);
    }
}
