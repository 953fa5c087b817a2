// Stable LSD radix sort of (key, payload) records, 8 bits per pass, in one of two
// forms the host chooses between (run_sort).  By exchange: one launch counts the
// digits of every pass per tile (up to four passes per launch), one scans all
// those counts, then every pass is one stable scatter.  Pass by pass: a counting
// launch, a scan and a scatter for each pass.
//
// What a scatter needs besides the ranks inside its tile: how many records of its
// table hold a smaller digit (the same whatever the order of the records, so
// counts taken before the first pass serve every pass) and how many records with
// the same digit lie in earlier tiles of the table.  The latter depends on the
// order the previous pass left: a pass that has just been counted has it from the
// scanned counts (the first pass always, every pass in the pass-by-pass form); the
// later passes of the exchange form pass it between the workgroups of the scatter
// itself (sort_lookback_walk).
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

// hist is [passes][tiles + 1][RADIX]: entry (p, t, d) holds the count of digit d of pass p in
// tile t (the tiles as they are before the first pass); the scan turns the counts of a digit
// into their exclusive prefix sums over the tiles and writes the count over all tiles as entry
// (p, tiles, d).  The RADIX counts of a tile lie together: the workgroup that counts a tile
// writes them with consecutive lanes, and the scatter reads what it needs of them the same way.  One launch counts the digits of passes
// [first_pass, first_pass + NP).  flags (optional): the scatters' exchange words (sort_lookback_walk) of the passes after the
// first, [flag_passes][tiles][RADIX]; every tile in use clears its own.  list_flags (optional):
// [list_tiles] words; workgroup b < list_tiles clears word b.
template <typename KeyT, int NP>
__global__ __launch_bounds__(SORT_BLOCK) void sort_hist_kernel(const KeyT *__restrict__ keys,
                                                               const SortTile *__restrict__ desc, int first_pass,
                                                               uint32_t *__restrict__ hist, uint32_t tiles,
                                                               unsigned long long *__restrict__ flags, int flag_passes,
                                                               unsigned long long *__restrict__ list_flags,
                                                               uint32_t list_tiles, const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    // (optional) the exchange word per tile of the kernel that lists the distinct rows after the sort
    if (list_flags && blockIdx.x < list_tiles && threadIdx.x == 0) list_flags[blockIdx.x] = 0ull;
    __shared__ uint32_t cnt[SORT_WAVES][NP][RADIX];
    const SortTile tile = desc[blockIdx.x];
    const bool owner = threadIdx.x < RADIX;   // thread d < RADIX reports digit d
    uint32_t *slot = hist + ((size_t)first_pass * (tiles + 1) + blockIdx.x) * RADIX + (owner ? threadIdx.x : 0);
    const size_t pass_stride = (size_t)RADIX * (tiles + 1);
    if (tile.count == 0) {   // uniform over the workgroup
        if (owner) {
#pragma unroll
            for (int q = 0; q < NP; ++q) slot[q * pass_stride] = 0;
        }
        return;
    }
    if (flags && owner) {
        for (int f = 0; f < flag_passes; ++f) flags[((size_t)f * tiles + blockIdx.x) * RADIX + threadIdx.x] = 0ull;
    }
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const int wave = threadIdx.x / EMB_WAVE;
    for (int i = threadIdx.x; i < SORT_WAVES * NP * RADIX; i += SORT_BLOCK) (&cnt[0][0][0])[i] = 0;
    __syncthreads();
    const uint32_t end = tile.start + tile.count;
    const uint32_t wbase = tile.start + wave * (SORT_TILE / SORT_WAVES);
    KeyT key[SORT_ITEMS];
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        key[k] = i < end ? keys[i] : (KeyT)0;
    }
    // Counting needs no ranks: one LDS add per record and digit into the wavefront's own counters.
    // Lanes that share a digit are serialised by the LDS, which is cheaper than matching them by
    // ballots unless all 64 hold the same digit (the records of one hot row, which share every
    // digit): that case is one add by one lane.
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        const bool live = i < end;
        const uint64_t lv = __ballot(live);
        if (lv == 0) continue;                                     // uniform
        const int first = __ffsll((unsigned long long)lv) - 1;
#pragma unroll
        for (int q = 0; q < NP; ++q) {
            const uint32_t digit = (uint32_t)(key[k] >> ((first_pass + q) * RADIX_BITS)) & (RADIX - 1);
            const uint32_t d0 = (uint32_t)__shfl((int)digit, first, EMB_WAVE);
            if (__ballot(live && digit == d0) == lv) {             // uniform
                if (lane == first) cnt[wave][q][d0] += (uint32_t)__popcll(lv);
            } else if (live) {
                atomicAdd(&cnt[wave][q][digit], 1u);
            }
        }
    }
    __syncthreads();
    if (owner) {
#pragma unroll
        for (int q = 0; q < NP; ++q) {
            uint32_t c = 0;
#pragma unroll
            for (int w = 0; w < SORT_WAVES; ++w) c += cnt[w][q][threadIdx.x];
            slot[q * pass_stride] = c;
        }
    }
}
static_assert(SORT_BLOCK >= RADIX && SORT_BLOCK % RADIX == 0, "the first RADIX threads of a workgroup own one digit each");

// One wavefront per pass and group of SCAN_DIGITS digits: exclusive scan, over the tiles, of those
// digits' counts, in place; the totals go to the entry after the last tile.  No LDS and no barrier: in
// a round a lane takes SCAN_TILES_PER_LANE consecutive tiles (their SCAN_DIGITS counts are one 16-byte
// load each, all requested together), sums them, and the lanes' sums are scanned by shuffles.
constexpr int SCAN_DIGITS = 4;
constexpr int SCAN_TILES_PER_LANE = 16;
constexpr int SCAN_BLOCK_THREADS = 256;
__global__ __launch_bounds__(SCAN_BLOCK_THREADS) void sort_scan_kernel(uint32_t *__restrict__ hist, uint32_t tiles,
                                                                        const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    static_assert(SCAN_DIGITS == 4 && RADIX % (SCAN_DIGITS * (SCAN_BLOCK_THREADS / EMB_WAVE)) == 0,
                  "one uint4 per tile and digit group, whole workgroups per pass");
    constexpr uint32_t GROUPS = RADIX / SCAN_DIGITS;   // digit groups (= wavefronts) per pass
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const uint32_t wave = blockIdx.x * (SCAN_BLOCK_THREADS / EMB_WAVE) + threadIdx.x / EMB_WAVE;
    const uint32_t pass = wave / GROUPS, d0 = (wave % GROUPS) * SCAN_DIGITS;
    uint32_t *base = hist + (size_t)pass * (tiles + 1) * RADIX + d0;
    uint4 carry = make_uint4(0u, 0u, 0u, 0u);   // a count over all tiles is below 2^32
    constexpr uint32_t ROUND = EMB_WAVE * SCAN_TILES_PER_LANE;
    for (uint32_t b0 = 0; b0 < tiles; b0 += ROUND) {
        const uint32_t first = b0 + lane * SCAN_TILES_PER_LANE;
        uint4 v[SCAN_TILES_PER_LANE];
#pragma unroll
        for (int i = 0; i < SCAN_TILES_PER_LANE; ++i) {
            v[i] = make_uint4(0u, 0u, 0u, 0u);
            if (first + i < tiles) v[i] = *reinterpret_cast<const uint4 *>(base + (size_t)(first + i) * RADIX);
        }
        uint4 mine = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int i = 0; i < SCAN_TILES_PER_LANE; ++i) {
            mine.x += v[i].x; mine.y += v[i].y; mine.z += v[i].z; mine.w += v[i].w;
        }
        uint4 inc;
        inc.x = wave_inclusive_scan(mine.x);
        inc.y = wave_inclusive_scan(mine.y);
        inc.z = wave_inclusive_scan(mine.z);
        inc.w = wave_inclusive_scan(mine.w);
        uint4 run = make_uint4(carry.x + inc.x - mine.x, carry.y + inc.y - mine.y, carry.z + inc.z - mine.z,
                               carry.w + inc.w - mine.w);
#pragma unroll
        for (int i = 0; i < SCAN_TILES_PER_LANE; ++i) {
            if (first + i < tiles) *reinterpret_cast<uint4 *>(base + (size_t)(first + i) * RADIX) = run;
            run.x += v[i].x; run.y += v[i].y; run.z += v[i].z; run.w += v[i].w;
        }
        carry.x += (uint32_t)__shfl((int)inc.x, EMB_WAVE - 1, EMB_WAVE);
        carry.y += (uint32_t)__shfl((int)inc.y, EMB_WAVE - 1, EMB_WAVE);
        carry.z += (uint32_t)__shfl((int)inc.z, EMB_WAVE - 1, EMB_WAVE);
        carry.w += (uint32_t)__shfl((int)inc.w, EMB_WAVE - 1, EMB_WAVE);
    }
    if (lane == 0) *reinterpret_cast<uint4 *>(base + (size_t)tiles * RADIX) = carry;
}

// How the workgroups of one scatter tell each other their digit counts (the scheme of a single-pass
// scan with decoupled look-back, Merrill and Garland 2016, applied per digit).  Every tile owns one 64-bit
// word per digit, cleared before the pass: the top two bits say what the low 32 hold: nothing yet,
// the tile's own count (SORT_FLAG_COUNT), or the count of the table's tiles up to and including this
// one (SORT_FLAG_PREFIX).  Count and state travel in one word, written and read with relaxed
// device-scope atomics, so no fence is needed.  A tile publishes its count as soon as it has ranked
// its records, then walks back over the earlier tiles of its table, adding counts until it meets a
// prefix or the table's first tile, and publishes its own prefix.
//
// A tile only ever waits for tiles with a smaller number.  Workgroups are started in the order of
// their numbers, so the unfinished tile with the smallest number is running and waits for nobody:
// the waits end.  They are bounded all the same: after poll_limit polls of one word the tile gives
// up and publishes SORT_FLAG_FAILED, every tile that meets that word does the same at once, and the
// kernel sets the backward's abort flag: the sort is abandoned, no row is updated, and the caller
// finds EMB_STATUS_SORT_ABANDONED in the status word.  poll_limit == 0 makes every wait fail at
// once (used to test that path).
constexpr unsigned long long SORT_FLAG_COUNT = 1ull << 62, SORT_FLAG_PREFIX = 2ull << 62, SORT_FLAG_FAILED = 3ull << 62;
constexpr int SORT_LOOKBACK_BATCH = 4;   // words requested together (2, 4, 8 measure the same; 16 costs registers)

__device__ __forceinline__ unsigned long long sort_flag_load(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void sort_flag_store(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// For the thread that owns digit `d` of tile `me`: the tile's own count goes out as soon as it is known ...
__device__ __forceinline__ void sort_lookback_publish(unsigned long long *flags /*[tiles][RADIX]*/, uint32_t me, uint32_t d,
                                                      uint32_t count)
{
    sort_flag_store(flags + (size_t)me * RADIX + d, SORT_FLAG_COUNT | count);
}

// ... and the walk follows once the scatter has done the work that does not depend on other tiles (by
// then most of the words it needs have been published).  Returns in `before` the number of records with
// this digit in tiles [first, me) and publishes the prefix; false if a wait ran out or met a failed tile.
__device__ __forceinline__ bool sort_lookback_walk(unsigned long long *flags, uint32_t first, uint32_t me, uint32_t d,
                                                   uint32_t count, uint32_t poll_limit, uint32_t &before)
{
    uint32_t sum = 0;
    bool ok = true, done = false;
    for (int64_t t = (int64_t)me - 1; t >= (int64_t)first && !done; t -= SORT_LOOKBACK_BATCH) {
        unsigned long long v[SORT_LOOKBACK_BATCH];
#pragma unroll
        for (int i = 0; i < SORT_LOOKBACK_BATCH; ++i) {
            const int64_t tt = t - i;
            v[i] = tt >= (int64_t)first ? sort_flag_load(flags + (size_t)tt * RADIX + d) : SORT_FLAG_PREFIX;
        }
#pragma unroll
        for (int i = 0; i < SORT_LOOKBACK_BATCH; ++i) {
            if (done) break;
            const int64_t tt = t - i;
            if (tt < (int64_t)first) {
                done = true;
                break;
            }
            unsigned long long x = v[i];
            uint32_t polls = 0;
            while ((x >> 62) == 0) {            // not published yet
                if (polls >= poll_limit) {
                    x = SORT_FLAG_FAILED;
                    break;
                }
                ++polls;
                __builtin_amdgcn_s_sleep(2);
                x = sort_flag_load(flags + (size_t)tt * RADIX + d);
            }
            if (poll_limit == 0) x = SORT_FLAG_FAILED;
            const unsigned long long state = x & SORT_FLAG_FAILED;
            if (state == SORT_FLAG_FAILED) {
                ok = false;
                done = true;
                break;
            }
            sum += (uint32_t)x;
            if (state == SORT_FLAG_PREFIX) done = true;
        }
    }
    sort_flag_store(flags + (size_t)me * RADIX + d, ok ? (SORT_FLAG_PREFIX | (uint32_t)(sum + count)) : SORT_FLAG_FAILED);
    before = sum;
    return ok;
}

// Stable scatter of one tile.  After ranking, the tile's records are first put in
// digit order in LDS; the copy-out then walks that order, so the lanes of a store
// instruction write consecutive addresses within each digit's run (about
// SORT_TILE / RADIX records long) instead of 64 unrelated ones.
//
// A record's destination is: start of its table's range + records of the table
// with a smaller digit + records of the table with the same digit in earlier
// tiles + its rank among the tile's records of that digit.  The scanned counts P
// of this pass's digit (exclusive over all tiles, total in the last column) give
// the first middle term as a difference between the columns of the table's first
// tile and of the next table's, whatever order the records are in.  The second:
// LOOKBACK false (the first pass: the records are in the order they were counted
// in) from P as well; LOOKBACK true from the other workgroups (sort_lookback_walk).
//
// LAST: the final pass writes the key's position in the concatenation of the
// tables (row + row_base), and the marker of an invalid row (`local_sentinel`,
// which sorts last inside its table) as `global_sentinel`.
template <typename KeyT, bool LAST, bool LOOKBACK>
__global__ __launch_bounds__(SORT_BLOCK) void sort_scatter_kernel(const KeyT *__restrict__ keys_in,
                                                                  const uint32_t *__restrict__ pay_in,
                                                                  KeyT *__restrict__ keys_out,
                                                                  uint32_t *__restrict__ pay_out,
                                                                  const SortTile *__restrict__ desc, int shift,
                                                                  const uint32_t *__restrict__ hist /*scanned*/,
                                                                  uint32_t tiles, const emb_table *__restrict__ tables,
                                                                  KeyT local_sentinel, KeyT global_sentinel,
                                                                  BwdCtrl *ctrl, unsigned long long *flags,
                                                                  uint32_t poll_limit, uint32_t *status)
{
    if (ctrl->abort) {   // uniform; nobody is to wait for this tile
        if (LOOKBACK && threadIdx.x < RADIX) sort_flag_store(flags + (size_t)blockIdx.x * RADIX + threadIdx.x, SORT_FLAG_FAILED);
        return;
    }
    __shared__ uint32_t lookback_failed;
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
    const uint32_t *hcol = hist + (owner ? threadIdx.x : 0);
    const uint32_t p_first = hcol[(size_t)tile.first * RADIX], p_next = hcol[(size_t)tile.next * RADIX];
    const uint32_t p_mine = LOOKBACK ? 0u : hcol[(size_t)blockIdx.x * RADIX];
    for (int i = threadIdx.x; i < SORT_WAVES * RADIX; i += SORT_BLOCK) (&cnt[0][0])[i] = 0;
    if (threadIdx.x == 0) lookback_failed = 0;
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
    const uint32_t d = owner ? threadIdx.x : 0;
    const uint32_t digit_total = owner ? p_next - p_first : 0;   // in this table
    uint32_t total = 0, dshift = 0;                              // dshift: delta[d] but for the earlier tiles' share
    {
        uint32_t c[SORT_WAVES];
        if (owner) {
#pragma unroll
            for (int w = 0; w < SORT_WAVES; ++w) {
                c[w] = cnt[w][d];
                total += c[w];
            }
            if (LOOKBACK) sort_lookback_publish(flags, blockIdx.x, d, total);
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
            dshift = tile.seg_start + below - start;
            if (!LOOKBACK) delta[d] = dshift + (p_mine - p_first);   // + the digit's records in the table's earlier tiles
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
    if (LOOKBACK && owner) {   // the other tiles have had the time of the step above to publish their counts
        uint32_t before_in_digit = 0;
        if (!sort_lookback_walk(flags, tile.first, blockIdx.x, d, total, poll_limit, before_in_digit))
            lookback_failed = 1;
        delta[d] = dshift + before_in_digit;
    }
    __syncthreads();
    if (LOOKBACK && lookback_failed) {   // uniform: positions unknown, nothing is written
        if (threadIdx.x == 0) {
            ctrl->abort = 1;
            emb_flag(status, EMB_STATUS_SORT_ABANDONED);
        }
        return;
    }

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
