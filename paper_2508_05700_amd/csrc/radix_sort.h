// Stable LSD radix sort of (key, payload) records, 8 bits per pass, as three
// launches per pass: per-tile digit histogram, scan, stable scatter.
//
// The sort is segmented: the records of one table are contiguous before the sort
// (bags are table-major) and stay in the table's range, so the keys sorted are
// row numbers inside the table and the passes cover the bits of the largest
// table, not of the sum of all tables.  A tile holds records of one table only
// (SortTile); the last pass turns the keys into positions in the concatenation
// of the tables, which is what the stages after the sort work on.
#pragma once
#include "bwd_common.h"
#include "scan.h"

struct SortTile {
    uint32_t start, count;  // records [start, start + count); count == 0: tile not in use
    uint32_t first, next;   // first tile of this tile's table, first tile of the next table
    uint32_t seg_start;     // first record of the table
    uint32_t table;
    uint32_t pad[2];
};
static_assert(sizeof(SortTile) == 32, "tile descriptors are read as two 16-byte loads");

// Stable rank of every record of a wavefront's share of a tile among the records
// of the same digit, and the wavefront's digit counts.  A wavefront walks its
// share 64 records at a time in ascending order; lanes holding the same digit
// are matched with one ballot per digit bit (every lane collects the lanes whose
// bit differs from its own: what is left are its peers), the lowest of them bumps
// the wavefront's private LDS counter, so there are no LDS atomics and no
// same-address serialisation when many records share a digit (the hot rows of
// a skewed batch, or the table bits of the key).
template <typename KeyT, bool WANT_RANK>
__device__ __forceinline__ void wave_rank_digits(const KeyT (&key)[SORT_ITEMS], uint32_t wbase, uint32_t n, int shift,
                                                 uint32_t *cnt /*LDS [RADIX], this wavefront's, zeroed*/,
                                                 uint32_t (&rank)[SORT_ITEMS])
{
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        const bool live = i < n;
        rank[k] = 0;
        const uint64_t lv = __ballot(live);
        if (lv == 0) continue;            // uniform: the share ends before this step
        const uint32_t digit = (uint32_t)(key[k] >> shift) & (RADIX - 1);
        // (kept as two 32-bit halves: a lane's own bit, spread over a word, serves both)
        uint32_t differ_lo = 0, differ_hi = 0;
#pragma unroll
        for (int bit = 0; bit < RADIX_BITS; ++bit) {
            const uint32_t set = digit & (1u << bit);
            const uint64_t with = __ballot(set != 0);
            const uint32_t mine = set ? 0xFFFFFFFFu : 0u;   // all ones if my bit is set
            differ_lo |= (uint32_t)with ^ mine;
            differ_hi |= (uint32_t)(with >> 32) ^ mine;
        }
        const uint64_t peers = lv & ~(((uint64_t)differ_hi << 32) | differ_lo);   // dead lanes match nobody
        const uint32_t before = __popcll(peers & lt_mask);
        uint32_t prev = 0;
        if (live && before == 0) {  // lowest lane of each digit group updates the wavefront's counter
            prev = cnt[digit];
            cnt[digit] = prev + (uint32_t)__popcll(peers);
        }
        if (WANT_RANK) {
            const int leader = live ? (__ffsll((unsigned long long)peers) - 1) : lane;
            prev = __shfl(prev, leader, EMB_WAVE);
            rank[k] = prev + before;
        }
    }
}

// hist is [RADIX][tiles + 1]: row d holds digit d's count in every tile and, in
// its last column (written by the scan), the digit's count over all tiles.
template <typename KeyT>
__global__ __launch_bounds__(SORT_BLOCK) void sort_hist_kernel(const KeyT *__restrict__ keys,
                                                               const SortTile *__restrict__ desc, int shift,
                                                               uint32_t *__restrict__ hist, uint32_t tiles,
                                                               const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    __shared__ uint32_t cnt[SORT_WAVES][RADIX];
    const SortTile tile = desc[blockIdx.x];
    const bool owner = threadIdx.x < RADIX;   // thread d < RADIX reports digit d
    uint32_t *slot = hist + (size_t)(owner ? threadIdx.x : 0) * (tiles + 1) + blockIdx.x;
    if (tile.count == 0) {   // uniform over the workgroup
        if (owner) *slot = 0;
        return;
    }
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const int wave = threadIdx.x / EMB_WAVE;
    for (int i = threadIdx.x; i < SORT_WAVES * RADIX; i += SORT_BLOCK) (&cnt[0][0])[i] = 0;
    __syncthreads();
    const uint32_t end = tile.start + tile.count;
    const uint32_t wbase = tile.start + wave * (SORT_TILE / SORT_WAVES);
    KeyT key[SORT_ITEMS];
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        key[k] = i < end ? keys[i] : (KeyT)0;
    }
    // Counting needs no ranks: one LDS add per record into the wavefront's own counters.  Lanes
    // that share a digit are serialised by the LDS, which is cheaper than matching them by ballots
    // unless all 64 hold the same digit (the records of one hot row, once an earlier pass has made
    // them adjacent): that case is one add by one lane.
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        const bool live = i < end;
        const uint32_t digit = (uint32_t)(key[k] >> shift) & (RADIX - 1);
        const uint64_t lv = __ballot(live);
        if (lv == 0) continue;                                     // uniform
        const int first = __ffsll((unsigned long long)lv) - 1;
        const uint32_t d0 = (uint32_t)__shfl((int)digit, first, EMB_WAVE);
        if (__ballot(live && digit == d0) == lv) {                 // uniform
            if (lane == first) cnt[wave][d0] += (uint32_t)__popcll(lv);
        } else if (live) {
            atomicAdd(&cnt[wave][digit], 1u);
        }
    }
    __syncthreads();
    if (owner) {
        uint32_t c = 0;
#pragma unroll
        for (int w = 0; w < SORT_WAVES; ++w) c += cnt[w][threadIdx.x];
        *slot = c;
    }
}
static_assert(SORT_BLOCK >= RADIX && SORT_BLOCK % RADIX == 0, "the first RADIX threads of a workgroup own one digit each");

// One workgroup per digit: exclusive scan of that digit's per-tile counts in
// place; the digit's total goes to the row's last column.
__global__ __launch_bounds__(1024) void sort_scan_kernel(uint32_t *__restrict__ hist, uint32_t tiles,
                                                          const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    __shared__ uint32_t wave_sums[1024 / EMB_WAVE];
    uint32_t *row = hist + (size_t)blockIdx.x * (tiles + 1);
    uint32_t carry = 0;
    for (uint32_t b0 = 0; b0 < tiles; b0 += 1024) {
        const uint32_t b = b0 + threadIdx.x;
        const uint32_t v = b < tiles ? row[b] : 0u;
        uint32_t total;
        const uint32_t inc = block_inclusive_scan<uint32_t, 1024>(v, wave_sums, total);
        if (b < tiles) row[b] = carry + inc - v;
        carry += total;
    }
    if (threadIdx.x == 0) row[tiles] = carry;
}

// Stable scatter of one tile.  After ranking, the tile's records are first put in
// digit order in LDS; the copy-out then walks that order, so the lanes of a store
// instruction write consecutive addresses within each digit's run (about
// SORT_TILE / RADIX records long) instead of 64 unrelated ones.
//
// A record's destination is: start of its table's range + records of the table
// with a smaller digit + records of the table with the same digit in earlier
// tiles + its rank among the tile's records of that digit.  The scanned
// histogram P (exclusive over all tiles, total in the last column) gives the two
// middle terms as differences against the column of the table's first tile.
//
// LAST: the final pass writes the key's position in the concatenation of the
// tables (row + row_base), and the marker of an invalid row (`local_sentinel`,
// which sorts last inside its table) as `global_sentinel`.
template <typename KeyT, bool LAST>
__global__ __launch_bounds__(SORT_BLOCK) void sort_scatter_kernel(const KeyT *__restrict__ keys_in,
                                                                  const uint32_t *__restrict__ pay_in,
                                                                  KeyT *__restrict__ keys_out,
                                                                  uint32_t *__restrict__ pay_out,
                                                                  const SortTile *__restrict__ desc, int shift,
                                                                  const uint32_t *__restrict__ hist /*scanned*/,
                                                                  uint32_t tiles, const emb_table *__restrict__ tables,
                                                                  KeyT local_sentinel, KeyT global_sentinel,
                                                                  const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    __shared__ uint32_t cnt[SORT_WAVES][RADIX];  // per-wavefront digit counts, then offsets inside the tile
    __shared__ uint32_t delta[RADIX];            // global position minus tile position, per digit
    __shared__ unsigned long long wave_sums[SORT_WAVES];
    __shared__ KeyT sk[SORT_TILE];
    __shared__ uint32_t sp[SORT_TILE];
    const SortTile tile = desc[blockIdx.x];
    if (tile.count == 0) return;   // uniform over the workgroup
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const int wave = threadIdx.x / EMB_WAVE;
    // thread d's three entries of the scanned histogram do not depend on the records: they are
    // asked for together with them, not after the ranking
    const bool owner = threadIdx.x < RADIX;   // thread d < RADIX looks after digit d
    const uint32_t *hrow = hist + (size_t)(owner ? threadIdx.x : 0) * (tiles + 1);
    const uint32_t p_first = hrow[tile.first], p_next = hrow[tile.next], p_mine = hrow[blockIdx.x];
    for (int i = threadIdx.x; i < SORT_WAVES * RADIX; i += SORT_BLOCK) (&cnt[0][0])[i] = 0;
    __syncthreads();

    const uint32_t end = tile.start + tile.count;
    const uint32_t wbase = tile.start + wave * (SORT_TILE / SORT_WAVES);
    KeyT key[SORT_ITEMS];
    uint32_t pay[SORT_ITEMS];
    uint32_t rank[SORT_ITEMS];
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        key[k] = i < end ? keys_in[i] : (KeyT)0;
        pay[k] = i < end ? pay_in[i] : 0u;
    }
    wave_rank_digits<KeyT, true>(key, wbase, end, shift, cnt[wave], rank);
    __syncthreads();

    // thread d: digit d's count in the tile, its start inside the tile and the number of the
    // table's records with a smaller digit (one scan over the digits of both, packed: the tile
    // counts add up to at most SORT_TILE, so the low half never carries), the wavefronts'
    // offsets within it, and the shift to global positions
    {
        const uint32_t d = owner ? threadIdx.x : 0;
        const uint32_t digit_total = owner ? p_next - p_first : 0;   // in this table
        const uint32_t before_in_digit = p_mine - p_first;           // in this table's earlier tiles
        uint32_t c[SORT_WAVES], total = 0;
        if (owner) {
#pragma unroll
            for (int w = 0; w < SORT_WAVES; ++w) {
                c[w] = cnt[w][d];
                total += c[w];
            }
        }
        unsigned long long all;
        const unsigned long long inc = block_inclusive_scan<unsigned long long, SORT_BLOCK>(
            ((unsigned long long)digit_total << 32) | total, wave_sums, all);
        if (owner) {
            const uint32_t start = (uint32_t)inc - total;
            const uint32_t below = (uint32_t)(inc >> 32) - digit_total;
            uint32_t run = start;
#pragma unroll
            for (int w = 0; w < SORT_WAVES; ++w) {
                cnt[w][d] = run;
                run += c[w];
            }
            delta[d] = tile.seg_start + below + before_in_digit - start;
        }
    }
    __syncthreads();

#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        if (i < end) {
            const uint32_t digit = (uint32_t)(key[k] >> shift) & (RADIX - 1);
            const uint32_t at = cnt[wave][digit] + rank[k];
            sk[at] = key[k];
            sp[at] = pay[k];
        }
    }
    __syncthreads();

    KeyT row_base = 0;
    if (LAST) row_base = (KeyT)tables[tile.table].row_base;
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t at = k * SORT_BLOCK + threadIdx.x;
        if (at < tile.count) {
            const KeyT kk = sk[at];
            const uint32_t dst = delta[(uint32_t)(kk >> shift) & (RADIX - 1)] + at;
            keys_out[dst] = LAST ? (kk == local_sentinel ? global_sentinel : (KeyT)(kk + row_base)) : kk;
            pay_out[dst] = sp[at];
        }
    }
}
