// Stable LSD radix sort of (key, payload) records, 8 bits per pass, as three
// launches per pass: per-tile digit histogram, scan, stable scatter.
#pragma once
#include "bwd_common.h"
#include "scan.h"

// Digit totals are accumulated into TOTAL_SLOTS slots per digit (tile b adds to
// slot b % TOTAL_SLOTS) so that hundreds of tiles do not queue on one address.
template <typename KeyT>
__global__ __launch_bounds__(SORT_BLOCK) void sort_hist_kernel(const KeyT *__restrict__ keys, uint32_t n, int shift,
                                                               uint32_t *__restrict__ hist /*[RADIX][tiles]*/,
                                                               uint32_t tiles,
                                                               uint32_t *__restrict__ totals /*[RADIX][TOTAL_SLOTS]*/,
                                                               const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    __shared__ uint32_t h[RADIX];
    h[threadIdx.x] = 0;  // SORT_BLOCK == RADIX
    __syncthreads();
    const uint32_t base = blockIdx.x * SORT_TILE;
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        uint32_t i = base + k * SORT_BLOCK + threadIdx.x;
        if (i < n) atomicAdd(&h[(uint32_t)(keys[i] >> shift) & (RADIX - 1)], 1u);
    }
    __syncthreads();
    const uint32_t c = h[threadIdx.x];
    hist[threadIdx.x * tiles + blockIdx.x] = c;
    if (c) atomicAdd(&totals[threadIdx.x * TOTAL_SLOTS + (blockIdx.x % TOTAL_SLOTS)], c);
}
static_assert(SORT_BLOCK == RADIX, "histogram kernels map one thread to one digit");

// One workgroup per digit: exclusive scan of that digit's per-tile counts,
// offset by the number of records with a smaller digit.
__global__ __launch_bounds__(1024) void sort_scan_kernel(uint32_t *__restrict__ hist, uint32_t tiles,
                                                          const uint32_t *__restrict__ totals,
                                                          const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    __shared__ uint32_t wave_sums[1024 / EMB_WAVE];
    const uint32_t d = blockIdx.x;
    uint32_t below = 0;
    for (uint32_t i = threadIdx.x; i < d * TOTAL_SLOTS; i += 1024) below += totals[i];
    uint32_t carry;
    block_inclusive_scan<uint32_t, 1024>(below, wave_sums, carry);
    uint32_t *row = hist + (size_t)d * tiles;
    for (uint32_t b0 = 0; b0 < tiles; b0 += 1024) {
        const uint32_t b = b0 + threadIdx.x;
        const uint32_t v = b < tiles ? row[b] : 0u;
        uint32_t total;
        const uint32_t inc = block_inclusive_scan<uint32_t, 1024>(v, wave_sums, total);
        if (b < tiles) row[b] = carry + inc - v;
        carry += total;
    }
}

template <typename KeyT>
__global__ __launch_bounds__(SORT_BLOCK) void sort_scatter_kernel(const KeyT *__restrict__ keys_in,
                                                                  const uint32_t *__restrict__ pay_in,
                                                                  KeyT *__restrict__ keys_out,
                                                                  uint32_t *__restrict__ pay_out, uint32_t n, int shift,
                                                                  const uint32_t *__restrict__ hist, uint32_t tiles,
                                                                  const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    // per-wave digit counters, then per-wave destination bases
    __shared__ uint32_t cnt[SORT_WAVES][RADIX];
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const int wave = threadIdx.x / EMB_WAVE;
#pragma unroll
    for (int w = 0; w < SORT_WAVES; ++w) cnt[w][threadIdx.x] = 0;
    __syncthreads();

    // wave `wave` owns records [base + wave*1024, +1024) and walks them 64 at a
    // time in ascending order, which makes the ranking stable
    const uint32_t wbase = blockIdx.x * SORT_TILE + wave * (SORT_TILE / SORT_WAVES);
    KeyT key[SORT_ITEMS];
    uint32_t rank[SORT_ITEMS];
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        const bool live = i < n;
        key[k] = live ? keys_in[i] : (KeyT)0;
        const uint32_t digit = (uint32_t)(key[k] >> shift) & (RADIX - 1);
        // lanes holding the same digit (dead lanes match nobody)
        uint64_t peers = __ballot(live);
#pragma unroll
        for (int bit = 0; bit < RADIX_BITS; ++bit) {
            const bool set = (digit >> bit) & 1u;
            const uint64_t m = __ballot(set);
            peers &= set ? m : ~m;
        }
        const uint32_t before = __popcll(peers & lt_mask);
        uint32_t prev = 0;
        if (live && before == 0) {  // lowest lane of each digit group updates the wave's counter
            prev = cnt[wave][digit];
            cnt[wave][digit] = prev + (uint32_t)__popcll(peers);
        }
        const int leader = live ? (__ffsll((unsigned long long)peers) - 1) : lane;
        prev = __shfl(prev, leader, EMB_WAVE);
        rank[k] = prev + before;
    }
    __syncthreads();

    // thread d turns the per-wave counts of digit d into destination bases
    {
        const uint32_t d = threadIdx.x;
        uint32_t run = hist[(size_t)d * tiles + blockIdx.x];
#pragma unroll
        for (int w = 0; w < SORT_WAVES; ++w) {
            const uint32_t c = cnt[w][d];
            cnt[w][d] = run;
            run += c;
        }
    }
    __syncthreads();

#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        if (i < n) {
            const uint32_t digit = (uint32_t)(key[k] >> shift) & (RADIX - 1);
            const uint32_t dst = cnt[wave][digit] + rank[k];
            keys_out[dst] = key[k];
            pay_out[dst] = pay_in[i];
        }
    }
}
