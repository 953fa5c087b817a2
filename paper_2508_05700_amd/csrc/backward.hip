// Exact sparse backward of the pooled lookup plus one row-wise Adagrad step
// (fine-tuning of table rows, paper Section 3.1).
//
// Stages, all on the caller's stream, all in caller-provided workspace:
//   keys     one (key, bag) record per lookup; key = the row inside its table,
//            or a marker for an out-of-range row; offsets are validated
//   sort     stable LSD radix sort of the records by key, 8 bits per pass,
//            table by table (the records of a table are contiguous), only as
//            many passes as the largest table needs; leaves keys row_base + row,
//            the marker as the sentinel total_rows               (radix_sort.h)
//   update   runs of equal keys are found on the fly; each run's gradients are
//            summed in a fixed order (ascending record order for runs of up to
//            UPD_SHORT_MAX records; longer runs are cut into chunks, each summed
//            by a wavefront as a fixed tree, and the chunk sums added in chunk
//            order) and Adagrad is applied once to its row              (update.h)
//   runs     only when the caller asks for the list of distinct rows: head
//            flags, scan and compaction into unique keys and counts
// The payload carried through the sort is the bag number: lookups of one row
// are then ordered by bag, which is ascending lookup order except between
// duplicates inside one bag, whose gradient terms are identical.  Every sum is
// taken in a fixed order, so results are bit-identical from run to run.
#include "bwd_common.h"
#include "gather.h"
#include "radix_sort.h"
#include "scan.h"
#include "update.h"
#include "u64mod.h"

namespace {

// ---------------------------------------------------------------------------
// workspace
// ---------------------------------------------------------------------------
struct BwdLayout {
    size_t ctrl, keys_a, keys_b, pay_a, pay_b, bag_scale, first_tile, tile_desc, hist, sort_flags, tile_heads, seg_start, seg_real,
        local_offsets, tile_prefix,
        queue, queue_end, span_head, wave_heads, segs, multi_list, chunk_tasks, partials, total;
    int key_bytes;
    int lpr, cpl;       // lanes per row and chunks per lane of the update kernels
    int64_t tiles;      // tiles of the sort: none straddles two tables
    int64_t flat_tiles; // tiles of the run-length kernels, which cut [0, nnz) evenly
    int64_t slots;      // wavefronts of the short-run kernel
    int64_t qslots;     // queue slots
    int64_t upd_blocks; // its grid
    int64_t chunk_cap;
};

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Lanes per row / chunks per lane for the update: two 16-byte chunks per lane while
// that leaves at least 4 lanes (64 contiguous bytes per row and load instruction);
// measured best on 256-byte rows (8 lanes x 2 chunks: 8 rows per wavefront
// instruction) against 4 x 4 and 16 x 1.
inline void upd_row_split(int chunks, int &lpr, int &cpl)
{
    int want = (chunks + 1) / 2;
    if (want < 4) want = chunks < 4 ? chunks : 4;
    lpr = 1;
    while (lpr < want && lpr < 64) lpr <<= 1;
    int need = (chunks + lpr - 1) / lpr;
    cpl = 1;
    while (cpl < need) cpl <<= 1;
}

inline BwdLayout bwd_layout(int32_t T, int64_t B, int64_t nnz, int64_t total_rows, int32_t D, int32_t dtype)
{
    BwdLayout L;
    L.key_bytes = ((uint64_t)total_rows < 0xFFFFFFFFull) ? 4 : 8;
    L.flat_tiles = (nnz + SORT_TILE - 1) / SORT_TILE;
    if (L.flat_tiles < 1) L.flat_tiles = 1;
    L.tiles = nnz / SORT_TILE + (T > 0 ? T : 1);   // sum over tables of ceil(n_t / SORT_TILE) is at most this
    const int esz = dtype == EMB_BF16 ? 2 : 4;
    upd_row_split((int)(((int64_t)D * esz + 15) / 16), L.lpr, L.cpl);
    L.slots = (nnz + UPD_SPAN - 1) / UPD_SPAN;
    if (L.slots < 1) L.slots = 1;
    const int64_t waves = UPD_BLOCK / EMB_WAVE;
    L.upd_blocks = emb_round_up_xcds((L.slots + waves - 1) / waves);
    L.qslots = L.slots * UPD_QSLOTS;
    // every queued run has at least one chunk
    L.chunk_cap = nnz / LONG_CHUNK + L.qslots + 2;
    const size_t n = (size_t)(nnz > 0 ? nnz : 1);
    const size_t np = n + SORT_PAD;
    size_t off = 0;
    L.ctrl = off;        off += align256(sizeof(BwdCtrl));
    L.keys_a = off;      off += align256(np * L.key_bytes);
    L.keys_b = off;      off += align256(np * L.key_bytes);
    L.pay_a = off;       off += align256(np * 4);
    L.pay_b = off;       off += align256(np * 4);
    L.bag_scale = off;   off += align256((size_t)T * (size_t)B * 4 + 4);
    L.first_tile = off;  off += align256(((size_t)T + 1) * 4);
    L.tile_desc = off;   off += align256((size_t)L.tiles * sizeof(SortTile));
    // the digit counts of every pass, and the words the scatters of the passes after the first exchange
    const int max_passes = L.key_bytes * 8 / RADIX_BITS;
    L.hist = off;        off += align256((size_t)max_passes * (L.tiles + 1) * RADIX * 4);
    L.sort_flags = off;  off += align256((size_t)(max_passes - 1) * L.tiles * RADIX * 8);
    L.tile_heads = off;  off += align256((size_t)L.flat_tiles * 8);    // one exchange word per tile (runs_list_kernel)
    L.seg_start = off;   off += align256((n + 1) * 4);
    L.seg_real = off;    off += align256(n * 4);
    L.queue = off;       off += align256((size_t)L.qslots * 4);
    L.queue_end = off;   off += align256((size_t)L.qslots * 4);
    L.span_head = off;   off += align256((size_t)L.slots * 4);
    L.wave_heads = off;  off += align256((size_t)L.upd_blocks * (UPD_BLOCK / EMB_WAVE) * 4);
    L.segs = off;        off += align256((size_t)L.qslots * sizeof(LongSeg));
    L.multi_list = off;  off += align256((size_t)L.qslots * 4);
    L.chunk_tasks = off; off += align256((size_t)L.chunk_cap * sizeof(uint2));
    L.partials = off;    off += align256((size_t)L.chunk_cap * (size_t)D * 4);   // one chunk-sum slot per task
    // emb_bag_forward_train_lengths: the offsets as sums within tiles, and the tiles' prefix sums
    const size_t bags = (size_t)T * (size_t)B;
    L.local_offsets = off; off += align256((bags + 1) * 8);
    L.tile_prefix = off;   off += align256((bags / EMB_OFFSETS_TILE + 2) * 8);
    L.total = off;
    return L;
}

// ---------------------------------------------------------------------------
// init + key build
// ---------------------------------------------------------------------------
// One workgroup: clears the control block, checks that the tables' record ranges
// [offsets[t*B], offsets[(t+1)*B]) partition [0, nnz) in order, numbers the
// tiles of the sort (first_tile[t] = tiles of the tables before t; T + 1 entries)
// and writes their descriptors.
// T == 0 is passed when there are no records and the offsets are not to be read.
// tile_prefix != NULL: `offsets` holds sums within tiles of EMB_OFFSETS_TILE lengths (emb_offsets_tile_sums);
// the kernel first writes the exclusive prefix sums of the tile totals there (one entry per tile of the
// T_all * B lengths, whatever T says) and reads every offset through emb_offset_at.
__global__ __launch_bounds__(1024) void bwd_init_kernel(BwdCtrl *ctrl, const int64_t *__restrict__ offsets, int32_t T,
                                                         int64_t B, int64_t nnz, uint32_t *__restrict__ first_tile,
                                                         SortTile *__restrict__ desc, uint32_t tiles,
                                                         int64_t *num_unique_out, uint32_t *status,
                                                         int64_t *__restrict__ tile_prefix = nullptr,
                                                         int64_t n_lengths = 0)
{
    __shared__ uint32_t wave_sums[1024 / EMB_WAVE];
    __shared__ int64_t wave_sums64[1024 / EMB_WAVE];
    __shared__ uint32_t bad;
    const int i = threadIdx.x;
    if (i == 0) bad = 0;
    if (tile_prefix) {
        const int64_t n_tiles = (n_lengths + EMB_OFFSETS_TILE - 1) / EMB_OFFSETS_TILE;
        int64_t carry64 = 0;
        for (int64_t k0 = 0; k0 < n_tiles; k0 += 1024) {
            const int64_t k = k0 + i;
            int64_t end = (k + 1) * EMB_OFFSETS_TILE;
            if (end > n_lengths) end = n_lengths;
            const int64_t v = k < n_tiles ? offsets[end] : 0;   // the tile's total stands at its end
            int64_t total;
            const int64_t inc = block_inclusive_scan<int64_t, 1024>(v, wave_sums64, total);
            if (k < n_tiles) tile_prefix[k] = carry64 + inc - v;
            carry64 += total;
        }
    }
    __syncthreads();   // tile_prefix[] was written by this workgroup: visible to all of it now
    uint32_t carry = 0;
    for (int32_t t0 = 0; t0 < T; t0 += 1024) {
        const int32_t t = t0 + i;
        uint32_t c = 0;
        if (t < T) {
            const int64_t s = emb_offset_at(offsets, tile_prefix, (int64_t)t * B);
            const int64_t e = emb_offset_at(offsets, tile_prefix, (int64_t)(t + 1) * B);
            const bool ok = s >= 0 && s <= e && e <= nnz && (t > 0 || s == 0) && (t < T - 1 || e == nnz);
            if (ok) c = (uint32_t)((e - s + SORT_TILE - 1) / SORT_TILE);
            else bad = 1;
        }
        uint32_t total;
        const uint32_t inc = block_inclusive_scan<uint32_t, 1024>(c, wave_sums, total);
        if (t < T) first_tile[t] = carry + inc - c;
        carry += total;
    }
    __syncthreads();
    if (i < 64) reinterpret_cast<uint32_t *>(ctrl)[i] = (i == 0) ? bad : 0u;   // word 0 is `abort`
    if (i == 0) {
        first_tile[T] = carry;
        if (bad) emb_flag(status, EMB_STATUS_BAD_OFFSETS);
        if (num_unique_out) *num_unique_out = 0;
    }
    if (bad) return;          // uniform; the record ranges are not to be trusted and nothing will read the tiles
    __syncthreads();          // first_tile[] was written by this workgroup: visible to all of it now

    // which table every tile of the sort belongs to and which records it holds
    for (uint32_t b = (uint32_t)i; b < tiles; b += 1024) {
        SortTile d = {0, 0, 0, 0, 0, 0, {0, 0}};
        if (b < carry) {
            // the table with first_tile[t] <= b < first_tile[t + 1]; tables without records own no tile
            int32_t lo = 0, hi = T;
            while (hi - lo > 1) {
                const int32_t mid = lo + (hi - lo) / 2;
                if (first_tile[mid] <= b) lo = mid;
                else hi = mid;
            }
            const int64_t s = emb_offset_at(offsets, tile_prefix, (int64_t)lo * B);
            const int64_t e = emb_offset_at(offsets, tile_prefix, (int64_t)(lo + 1) * B);
            const int64_t start = s + (int64_t)(b - first_tile[lo]) * SORT_TILE;
            const int64_t left = e - start;
            d.start = (uint32_t)start;
            d.count = (uint32_t)(left < SORT_TILE ? left : SORT_TILE);
            d.first = first_tile[lo];
            d.next = first_tile[lo + 1];
            d.seg_start = (uint32_t)s;
            d.table = (uint32_t)lo;
        }
        desc[b] = d;
    }
}
static_assert(offsetof(BwdCtrl, abort) == 0, "bwd_init_kernel writes abort as word 0");

constexpr int KEY_LANES = 16;  // lanes that share one bag in the key build

template <typename KeyT>
__global__ __launch_bounds__(256) void bwd_keys_kernel(const emb_table *__restrict__ tables, int32_t T, int64_t B,
                                                       int64_t nnz, const int64_t *__restrict__ rows,
                                                       const int64_t *__restrict__ offsets, int32_t mode,
                                                       KeyT local_sentinel, KeyT *__restrict__ keys,
                                                       uint32_t *__restrict__ pay, float *__restrict__ bag_scale,
                                                       BwdCtrl *ctrl, uint32_t *status)
{
    const int t = blockIdx.y;
    const int g = threadIdx.x / KEY_LANES;
    const int l = threadIdx.x % KEY_LANES;
    const int64_t b = (int64_t)blockIdx.x * (256 / KEY_LANES) + g;
    if (b >= B) return;
    const emb_table tb = tables[t];
    const int64_t bag = (int64_t)t * B + b;
    const int64_t s = offsets[bag], e = offsets[bag + 1];
    if (s < 0 || e < s || e > nnz) {
        if (l == 0) {
            atomicOr(&ctrl->abort, 1u);
            emb_flag(status, EMB_STATUS_BAD_OFFSETS);
        }
        return;
    }
    if (l == 0) bag_scale[bag] = (mode == EMB_POOL_MEAN && e > s) ? 1.0f / (float)(e - s) : 1.0f;
    for (int64_t j = s + l; j < e; j += KEY_LANES) {
        const int64_t r = rows[j];
        KeyT k;
        if ((uint64_t)r < (uint64_t)tb.num_rows) {
            k = (KeyT)r;
        } else {
            k = local_sentinel;   // sorts after every row of the table
            emb_flag(status, EMB_STATUS_BAD_INDEX);
        }
        keys[j] = k;
        pay[j] = (uint32_t)bag;
    }
}

// ---------------------------------------------------------------------------
// run-length boundaries of the sorted keys
// ---------------------------------------------------------------------------
// Invalid rows leave sentinel records at the end of their table's range, i.e.
// between the runs of two tables.  Every change of key starts a run; runs of the
// sentinel are numbered with the others (their start ends the run before them)
// but are not rows: seg_real maps a run to its place in the list of distinct rows.
// One launch numbers the runs.  A tile (SORT_TILE records of the sorted array, whatever table they belong
// to) counts its run starts and row starts, and learns how many lie in the tiles before it from those tiles
// themselves: the exchange of the sort's scatters (radix_sort.h: a count, then a prefix, in one flagged word;
// bounded waits for tiles with smaller numbers only).  Here a tile has one word that holds both numbers
// (31 bits each: there are fewer than 2^31 records), and the tile's first wavefront walks back
// RUNS_WINDOWS * 64 tiles per round trip to memory: lane l requests the words of tiles t - l, t - 64 - l, ...
// together, then the windows are added up nearest first until one holds a tile that knows its prefix.
// flags: [tiles], cleared by the sort's first counting launch.
constexpr int RUNS_WINDOWS = 4;
__device__ __forceinline__ unsigned long long runs_pack(uint32_t runs, uint32_t rows)
{
    return ((unsigned long long)runs << 31) | rows;
}
__device__ __forceinline__ bool runs_lookback(unsigned long long *flags, uint32_t me, uint32_t count_runs,
                                              uint32_t count_rows, uint32_t poll_limit, uint32_t &before_runs,
                                              uint32_t &before_rows)
{
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    if (lane == 0) sort_flag_store(flags + me, SORT_FLAG_COUNT | runs_pack(count_runs, count_rows));
    uint32_t sum_runs = 0, sum_rows = 0;
    bool done = false, ok = true;   // the same in all lanes
    for (int64_t t = (int64_t)me - 1; !done; t -= RUNS_WINDOWS * EMB_WAVE) {
        unsigned long long x[RUNS_WINDOWS];
#pragma unroll
        for (int w = 0; w < RUNS_WINDOWS; ++w) {
            const int64_t tt = t - w * EMB_WAVE - lane;
            x[w] = tt >= 0 ? sort_flag_load(flags + tt) : SORT_FLAG_PREFIX;   // before the first tile: a prefix of nothing
        }
#pragma unroll
        for (int w = 0; w < RUNS_WINDOWS; ++w) {
            if (done) break;   // uniform
            const int64_t tt = t - w * EMB_WAVE - lane;
            unsigned long long v = x[w];
            uint32_t polls = 0;
            while ((v >> 62) == 0) {            // not published yet
                if (polls >= poll_limit) {
                    v = SORT_FLAG_FAILED;
                    break;
                }
                ++polls;
                __builtin_amdgcn_s_sleep(2);
                v = sort_flag_load(flags + tt);
            }
            if (poll_limit == 0 && tt >= 0) v = SORT_FLAG_FAILED;
            const unsigned long long state = v & SORT_FLAG_FAILED;
            const uint64_t prefix = __ballot(state == SORT_FLAG_PREFIX);
            const int stop = prefix ? __ffsll((unsigned long long)prefix) - 1 : EMB_WAVE;   // the nearest tile that knows its prefix
            if (__ballot(state == SORT_FLAG_FAILED && lane <= stop) != 0) {
                ok = false;
                done = true;
                break;
            }
            uint32_t r = lane <= stop ? (uint32_t)((v >> 31) & 0x7FFFFFFFu) : 0u;
            uint32_t q = lane <= stop ? (uint32_t)(v & 0x7FFFFFFFu) : 0u;
#pragma unroll
            for (int d = EMB_WAVE >> 1; d >= 1; d >>= 1) {
                r += (uint32_t)__shfl_xor((int)r, d, EMB_WAVE);
                q += (uint32_t)__shfl_xor((int)q, d, EMB_WAVE);
            }
            sum_runs += r;
            sum_rows += q;
            if (prefix) done = true;
        }
    }
    if (lane == 0)
        sort_flag_store(flags + me, ok ? (SORT_FLAG_PREFIX | runs_pack(sum_runs + count_runs, sum_rows + count_rows))
                                       : SORT_FLAG_FAILED);
    before_runs = sum_runs;
    before_rows = sum_rows;
    return ok;
}

template <typename KeyT>
__global__ __launch_bounds__(SORT_BLOCK) void runs_list_kernel(const KeyT *__restrict__ keys, uint32_t n, KeyT sentinel,
                                                               unsigned long long *__restrict__ flags, uint32_t tiles,
                                                               uint32_t *__restrict__ seg_start,
                                                               uint32_t *__restrict__ seg_real,
                                                               int64_t *__restrict__ unique_keys_out, BwdCtrl *ctrl,
                                                               int64_t *num_unique_out, uint32_t poll_limit,
                                                               uint32_t *status)
{
    if (ctrl->abort) {   // uniform; nobody is to wait for this tile
        if (threadIdx.x == 0) sort_flag_store(flags + blockIdx.x, SORT_FLAG_FAILED);
        return;
    }
    __shared__ unsigned long long wave_sums[SORT_WAVES];
    __shared__ unsigned long long tile_before;   // runs in the high half, rows in the low half
    __shared__ uint32_t lookback_failed;
    // the tile's runs in order: where each starts, and its place among the rows (NO_ROW: the marker's run)
    __shared__ uint32_t run_pos[SORT_TILE];
    __shared__ uint32_t run_row[SORT_TILE];
    constexpr uint32_t NO_ROW = 0xFFFFFFFFu;
    // a thread looks at SORT_ITEMS consecutive records (the arrays carry SORT_PAD records of slack; what
    // lies past n is not looked at) and at the record before them
    const uint32_t base = blockIdx.x * SORT_TILE + threadIdx.x * SORT_ITEMS;
    KeyT k[SORT_ITEMS];
    KeyT prev = sentinel;
    if (base < n) {
        load_records<KeyT, SORT_ITEMS>(keys + base, k);
        if (base > 0) prev = keys[base - 1];
    }
    unsigned long long f[SORT_ITEMS], c = 0;
#pragma unroll
    for (int e = 0; e < SORT_ITEMS; ++e) {
        const uint32_t i = base + e;
        f[e] = 0ull;
        if (i < n && (i == 0 || k[e] != (e == 0 ? prev : k[e - 1])))
            f[e] = (1ull << 32) | (k[e] != sentinel ? 1ull : 0ull);   // high half: runs, low half: rows
        c += f[e];
    }
    unsigned long long total;
    const unsigned long long inc = block_inclusive_scan<unsigned long long, SORT_BLOCK>(c, wave_sums, total);
    // the tile's runs go to LDS in order while the first wavefront asks the earlier tiles
    {
        unsigned long long at = inc - c;
        uint32_t v = (uint32_t)(at >> 32), u = (uint32_t)at;
#pragma unroll
        for (int e = 0; e < SORT_ITEMS; ++e) {
            if (f[e]) {
                const bool real = (f[e] & 1ull) != 0;
                run_pos[v] = base + e;
                run_row[v] = real ? u : NO_ROW;
                u += real ? 1u : 0u;
                ++v;
            }
        }
    }
    if (threadIdx.x < EMB_WAVE) {
        uint32_t runs_before = 0, rows_before = 0;
        const bool ok = runs_lookback(flags, blockIdx.x, (uint32_t)(total >> 32), (uint32_t)total, poll_limit,
                                      runs_before, rows_before);
        if (threadIdx.x == 0) {
            tile_before = ((unsigned long long)runs_before << 32) | rows_before;
            lookback_failed = ok ? 0u : 1u;
        }
    }
    __syncthreads();
    if (lookback_failed) {   // uniform: the numbering is unknown, nothing is written
        if (threadIdx.x == 0) {
            ctrl->abort = 1;
            emb_flag(status, EMB_STATUS_SORT_ABANDONED);
        }
        return;
    }
    const uint32_t v0 = (uint32_t)(tile_before >> 32), u0 = (uint32_t)tile_before;
    const uint32_t tile_runs = (uint32_t)(total >> 32);
    for (uint32_t i = threadIdx.x; i < tile_runs; i += SORT_BLOCK) {   // consecutive lanes, consecutive entries
        const uint32_t pos = run_pos[i], row = run_row[i];
        seg_start[v0 + i] = pos;
        seg_real[v0 + i] = row == NO_ROW ? NO_ROW : u0 + row;
        if (row != NO_ROW && unique_keys_out) unique_keys_out[u0 + row] = (int64_t)keys[pos];
    }
    if (blockIdx.x == tiles - 1 && threadIdx.x == 0) {   // the last tile knows the totals
        const unsigned long long all = tile_before + total;
        const uint32_t runs = (uint32_t)(all >> 32);
        ctrl->num_runs = runs;
        seg_start[runs] = n;   // the last run ends with the records
        if (num_unique_out) *num_unique_out = (int64_t)(uint32_t)all;
    }
}

__global__ __launch_bounds__(256) void runs_counts_kernel(const uint32_t *__restrict__ seg_start,
                                                          const uint32_t *__restrict__ seg_real,
                                                          int32_t *__restrict__ unique_counts_out,
                                                          const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    const uint32_t runs = ctrl->num_runs;
    for (uint32_t v = blockIdx.x * 256 + threadIdx.x; v < runs; v += gridDim.x * 256) {
        const uint32_t u = seg_real[v];
        if (u != 0xFFFFFFFFu) unique_counts_out[u] = (int32_t)(seg_start[v + 1] - seg_start[v]);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct BwdArgs {
    const emb_table *tables_dev = nullptr;
    int32_t T = 0, D = 0, dtype = 0, mode = 0;
    const int64_t *rows = nullptr, *offsets = nullptr;
    bool from_lengths = false;           // emb_bag_forward_train_lengths: the offsets are made on the way
    const int32_t *lengths = nullptr;    // ... from these (NULL when there are no bags)
    int64_t *offsets_out = nullptr;      // ... and written here
    int64_t B = 0, nnz = 0, total_rows = 0, max_rows = 0;
    int passes = 1;   // of the sort: enough for the bits of max_rows, the value that marks an invalid row
    const float *dout = nullptr;
    float lr = 0.f, eps = 0.f;
    char *ws = nullptr;
    int64_t *unique_keys_out = nullptr;
    int32_t *unique_counts_out = nullptr;
    int64_t *num_unique_out = nullptr;
    uint32_t *status = nullptr;
    void *const *events = nullptr;
    const emb_side_stream *side = nullptr;   // NULL: everything on `stream`
    const emb_side_stream *after = nullptr;  // emb_bag_forward_train_lengths_after: wait for its join event before the tables are read
    hipStream_t stream = nullptr;
    // record stage event i, if the caller asked for stage timing
    int mark(int i) const
    {
        if (events && events[i] && hipEventRecord(reinterpret_cast<hipEvent_t>(events[i]), stream) != hipSuccess)
            return EMB_ERR_HIP;
        return EMB_OK;
    }
};
#define EMB_MARK(a, i) do { if ((a).mark(i) != EMB_OK) return EMB_ERR_HIP; } while (0)

template <typename KeyT, int LPR, int CPL, int EU, bool BF16>
int launch_update(const BwdArgs &a, const BwdLayout &L, const KeyT *keys, const uint32_t *pay, int chunks)
{
    BwdCtrl *ctrl = reinterpret_cast<BwdCtrl *>(a.ws + L.ctrl);
    float *bag_scale = reinterpret_cast<float *>(a.ws + L.bag_scale);
    uint32_t *queue = reinterpret_cast<uint32_t *>(a.ws + L.queue);
    uint32_t *queue_end = reinterpret_cast<uint32_t *>(a.ws + L.queue_end);
    uint32_t *span_head = reinterpret_cast<uint32_t *>(a.ws + L.span_head);
    uint32_t *wave_heads = reinterpret_cast<uint32_t *>(a.ws + L.wave_heads);
    LongSeg *segs = reinterpret_cast<LongSeg *>(a.ws + L.segs);
    uint32_t *multi_list = reinterpret_cast<uint32_t *>(a.ws + L.multi_list);
    uint2 *chunk_tasks = reinterpret_cast<uint2 *>(a.ws + L.chunk_tasks);
    float *partials = reinterpret_cast<float *>(a.ws + L.partials);
    const uint32_t n = (uint32_t)a.nnz;
    const KeyT sentinel = (KeyT)a.total_rows;
    const float inv_D = 1.0f / (float)a.D;
    BagDiv bdiv;
    bdiv.B = (uint32_t)a.B;
    bdiv.magic = 0xFFFFFFFFu / (uint32_t)a.B;

    // Runs of up to UPD_SHORT_MAX records are updated by update_kernel, the longer ones by
    // detect -> prepare -> reduce -> combine.  The two paths touch different rows and only read the
    // sorted records, so with a side stream they run beside each other (fork after the sort, join
    // at the end); without one they run one after the other on the caller's stream.
    hipStream_t ls = a.stream;
    if (a.side) {
        ls = reinterpret_cast<hipStream_t>(a.side->stream);
        hipEvent_t fork = reinterpret_cast<hipEvent_t>(a.side->fork_event);
        if (hipEventRecord(fork, a.stream) != hipSuccess || hipStreamWaitEvent(ls, fork, 0) != hipSuccess)
            return EMB_ERR_HIP;
    }
    constexpr int DWAVES = 256 / EMB_WAVE;
    hipLaunchKernelGGL(long_detect_kernel<KeyT>, dim3((unsigned)((L.slots + DWAVES - 1) / DWAVES)), dim3(256), 0, ls,
                       keys, n, sentinel, ctrl, queue, queue_end, span_head, wave_heads, (uint32_t)L.slots);
    EMB_RETURN_IF_LAUNCH_FAILED();

    if (a.T <= UPD_LDS_TABLES)
        hipLaunchKernelGGL((update_kernel<KeyT, LPR, CPL, EU, BF16, true>), dim3((unsigned)L.upd_blocks), dim3(UPD_BLOCK),
                           0, a.stream, a.tables_dev, a.T, keys, pay, n, sentinel, bag_scale, a.dout, chunks, a.D, inv_D,
                           a.lr, a.eps, bdiv, ctrl);
    else
        hipLaunchKernelGGL((update_kernel<KeyT, LPR, CPL, EU, BF16, false>), dim3((unsigned)L.upd_blocks), dim3(UPD_BLOCK),
                           0, a.stream, a.tables_dev, a.T, keys, pay, n, sentinel, bag_scale, a.dout, chunks, a.D, inv_D,
                           a.lr, a.eps, bdiv, ctrl);
    EMB_RETURN_IF_LAUNCH_FAILED();
    EMB_MARK(a, 4);

    const int64_t pthreads = L.qslots > L.slots ? L.qslots : L.slots;
    hipLaunchKernelGGL(long_prepare_kernel, dim3((unsigned)((pthreads + PREP_BLOCK - 1) / PREP_BLOCK)), dim3(PREP_BLOCK),
                       0, ls, n, ctrl, queue, queue_end, (uint32_t)L.qslots, span_head, wave_heads, (uint32_t)L.slots, segs,
                       multi_list, chunk_tasks, (uint32_t)L.chunk_cap);
    EMB_RETURN_IF_LAUNCH_FAILED();

    // one wavefront per task; enough workgroups to fill the chip, tasks beyond that are strided over
    int64_t want = (L.chunk_cap + (UPD_BLOCK / EMB_WAVE) - 1) / (UPD_BLOCK / EMB_WAVE);
    const unsigned lgrid = (unsigned)emb_round_up_xcds(want < 4096 ? want : 4096);
    hipLaunchKernelGGL((long_reduce_kernel<KeyT, LPR, CPL, EU, BF16>), dim3(lgrid), dim3(UPD_BLOCK), 0, ls,
                       a.tables_dev, a.T, keys, pay, bag_scale, a.dout, chunks, a.D, inv_D, a.lr, a.eps, bdiv, ctrl,
                       segs, chunk_tasks, (uint32_t)L.chunk_cap, partials);
    EMB_RETURN_IF_LAUNCH_FAILED();

    // runs of several chunks: at most nnz / LONG_CHUNK of them
    const int64_t multi_max = a.nnz / LONG_CHUNK + 1;
    constexpr int CWAVES = UPD_BLOCK / EMB_WAVE;
    int64_t cwant = (multi_max + CWAVES - 1) / CWAVES;
    const unsigned cgrid = (unsigned)(cwant < 1024 ? cwant : 1024);
    hipLaunchKernelGGL((long_combine_kernel<KeyT, LPR, CPL, BF16>), dim3(cgrid), dim3(UPD_BLOCK), 0, ls,
                       a.tables_dev, a.T, keys, pay, chunks, inv_D, a.lr, a.eps, bdiv, ctrl, segs, multi_list,
                       (uint32_t)L.qslots, partials, a.num_unique_out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    if (a.side) {
        // (with defer_join the caller makes its stream wait later: emb_side_stream_join, or the next
        // step's emb_bag_forward_train_lengths_after)
        hipEvent_t join = reinterpret_cast<hipEvent_t>(a.side->join_event);
        if (hipEventRecord(join, ls) != hipSuccess) return EMB_ERR_HIP;
        if (!a.side->defer_join && hipStreamWaitEvent(a.stream, join, 0) != hipSuccess) return EMB_ERR_HIP;
    }
    EMB_MARK(a, 5);
    return EMB_OK;
}

// How often a scatter of the sort polls one word of another workgroup before it gives the sort up
// (sort_lookback_walk, radix_sort.h); emb_debug_sort_poll_limit changes it.
static constexpr uint32_t SORT_POLL_LIMIT_DEFAULT = 1u << 20;
static constexpr int SORT_SCAN_BLOCKS = RADIX / SCAN_DIGITS / (SCAN_BLOCK_THREADS / EMB_WAVE);   // workgroups of the scan, per pass
static constexpr int SORT_EXCHANGE_MAX_TILES = 64;   // per table, on average: above it every pass counts and scans
static uint32_t sort_poll_limit = SORT_POLL_LIMIT_DEFAULT;

extern "C" void emb_debug_sort_poll_limit(int64_t polls)
{
    sort_poll_limit = polls < 0 ? SORT_POLL_LIMIT_DEFAULT : (polls > 0xFFFFFFFFll ? 0xFFFFFFFFu : (uint32_t)polls);
}

// Keys, sort and the optional list of distinct rows: everything that needs the indices only.
// prepared: the control block, the tile descriptors and the records are in the workspace already
// (emb_bag_forward_train put them there), so only the passes and the optional list run.
template <typename KeyT>
int run_sort(const BwdArgs &a, const BwdLayout &L, bool prepared = false)
{
    BwdCtrl *ctrl = reinterpret_cast<BwdCtrl *>(a.ws + L.ctrl);
    KeyT *keys_a = reinterpret_cast<KeyT *>(a.ws + L.keys_a);
    KeyT *keys_b = reinterpret_cast<KeyT *>(a.ws + L.keys_b);
    uint32_t *pay_a = reinterpret_cast<uint32_t *>(a.ws + L.pay_a);
    uint32_t *pay_b = reinterpret_cast<uint32_t *>(a.ws + L.pay_b);
    float *bag_scale = reinterpret_cast<float *>(a.ws + L.bag_scale);
    uint32_t *first_tile = reinterpret_cast<uint32_t *>(a.ws + L.first_tile);
    SortTile *tile_desc = reinterpret_cast<SortTile *>(a.ws + L.tile_desc);
    uint32_t *hist = reinterpret_cast<uint32_t *>(a.ws + L.hist);
    unsigned long long *sort_flags = reinterpret_cast<unsigned long long *>(a.ws + L.sort_flags);
    unsigned long long *tile_heads = reinterpret_cast<unsigned long long *>(a.ws + L.tile_heads);
    uint32_t *seg_start = reinterpret_cast<uint32_t *>(a.ws + L.seg_start);
    uint32_t *seg_real = reinterpret_cast<uint32_t *>(a.ws + L.seg_real);
    const KeyT sentinel = (KeyT)a.total_rows;       // after the sort
    const KeyT local_sentinel = (KeyT)a.max_rows;   // during it
    const uint32_t n = (uint32_t)a.nnz;
    const uint32_t tiles = (uint32_t)L.tiles;
    const uint32_t flat_tiles = (uint32_t)L.flat_tiles;
    hipStream_t s = a.stream;

    EMB_MARK(a, 0);
    if (!prepared) {
        hipLaunchKernelGGL(bwd_init_kernel, dim3(1), dim3(1024), 0, s, ctrl, a.offsets, a.nnz > 0 ? a.T : 0, a.B, a.nnz,
                           first_tile, tile_desc, a.nnz > 0 ? tiles : 0u, a.num_unique_out, a.status);
        EMB_RETURN_IF_LAUNCH_FAILED();
    }
    if (a.nnz == 0) {
        for (int i = 1; i <= 3; ++i) EMB_MARK(a, i);
        return EMB_OK;
    }

    if (!prepared) {
        constexpr int BAGS = 256 / KEY_LANES;
        dim3 grid((unsigned)((a.B + BAGS - 1) / BAGS), (unsigned)a.T);
        hipLaunchKernelGGL(bwd_keys_kernel<KeyT>, grid, dim3(256), 0, s, a.tables_dev, a.T, a.B, a.nnz, a.rows,
                           a.offsets, a.mode, local_sentinel, keys_a, pay_a, bag_scale, ctrl, a.status);
        EMB_RETURN_IF_LAUNCH_FAILED();
    }
    EMB_MARK(a, 1);

    KeyT *kin = keys_a, *kout = keys_b;
    uint32_t *pin = pay_a, *pout = pay_b;
    // Two ways through the passes (radix_sort.h).  Tables of up to SORT_EXCHANGE_MAX_TILES tiles of records
    // each (all the host can know is the average): the digits of all passes are counted by one launch
    // and scanned by one, and the scatters of the later passes exchange their counts.  Larger tables: a
    // counting launch and a scan per pass, because a scatter's walk back over its table's earlier tiles
    // grows with their number (a table of 640 tiles sorts 12 % slower by exchange, one of 40 tiles 11 %
    // faster).
    // the optional list of distinct rows exchanges counts between tiles too; its words are cleared by the
    // first counting launch
    const bool want_list = a.unique_keys_out || a.unique_counts_out;
    unsigned long long *list_flags = want_list ? tile_heads : nullptr;
    const bool exchange = a.nnz <= (int64_t)SORT_EXCHANGE_MAX_TILES * SORT_TILE * (a.T > 0 ? a.T : 1);
    const uint32_t poll_limit = sort_poll_limit;
    if (exchange) {
        for (int p0 = 0; p0 < a.passes; p0 += 4) {
            unsigned long long *fl = p0 == 0 ? sort_flags : nullptr;   // the first launch clears the scatters' words
            const int np = a.passes - p0 < 4 ? a.passes - p0 : 4;
#define EMB_SORT_HIST(NP)                                                                                          \
    hipLaunchKernelGGL((sort_hist_kernel<KeyT, NP>), dim3(tiles), dim3(SORT_BLOCK), 0, s, kin, tile_desc, p0, hist, \
                       tiles, fl, a.passes - 1, p0 == 0 ? list_flags : nullptr, flat_tiles, ctrl)
            switch (np) {
                case 1: EMB_SORT_HIST(1); break;
                case 2: EMB_SORT_HIST(2); break;
                case 3: EMB_SORT_HIST(3); break;
                default: EMB_SORT_HIST(4); break;
            }
#undef EMB_SORT_HIST
            EMB_RETURN_IF_LAUNCH_FAILED();
        }
        hipLaunchKernelGGL(sort_scan_kernel, dim3(SORT_SCAN_BLOCKS * a.passes), dim3(SCAN_BLOCK_THREADS), 0, s, hist, tiles,
                           ctrl);
        EMB_RETURN_IF_LAUNCH_FAILED();
    }
    for (int p = 0; p < a.passes; ++p) {
        const int shift = p * RADIX_BITS;
        uint32_t *hp = hist + (size_t)p * RADIX * (tiles + 1);
        const bool lookback = exchange && p > 0;
        unsigned long long *fl = lookback ? sort_flags + (size_t)(p - 1) * tiles * RADIX : nullptr;
        const bool last = p == a.passes - 1;
        if (!exchange) {
            hipLaunchKernelGGL((sort_hist_kernel<KeyT, 1>), dim3(tiles), dim3(SORT_BLOCK), 0, s, kin, tile_desc, p, hist,
                               tiles, (unsigned long long *)nullptr, 0, p == 0 ? list_flags : nullptr, flat_tiles, ctrl);
            EMB_RETURN_IF_LAUNCH_FAILED();
            hipLaunchKernelGGL(sort_scan_kernel, dim3(SORT_SCAN_BLOCKS), dim3(SCAN_BLOCK_THREADS), 0, s, hp, tiles, ctrl);
            EMB_RETURN_IF_LAUNCH_FAILED();
        }
#define EMB_SORT_SCATTER(LAST, LOOKBACK)                                                                            \
    hipLaunchKernelGGL((sort_scatter_kernel<KeyT, LAST, LOOKBACK>), dim3(tiles), dim3(SORT_BLOCK), 0, s, kin, pin, \
                       kout, pout, tile_desc, shift, hp, tiles, a.tables_dev, local_sentinel, sentinel, ctrl, fl,   \
                       poll_limit, a.status)
        if (!lookback) {
            if (last) EMB_SORT_SCATTER(true, false);
            else EMB_SORT_SCATTER(false, false);
        } else {
            if (last) EMB_SORT_SCATTER(true, true);
            else EMB_SORT_SCATTER(false, true);
        }
#undef EMB_SORT_SCATTER
        EMB_RETURN_IF_LAUNCH_FAILED();
        KeyT *tk = kin; kin = kout; kout = tk;
        uint32_t *tp = pin; pin = pout; pout = tp;
    }
    // sorted records are now in (kin, pin)
    EMB_MARK(a, 2);

    if (want_list) {
        // (the update counts the distinct rows again on its own: ctrl->num_unique is not touched here)
        hipLaunchKernelGGL(runs_list_kernel<KeyT>, dim3(flat_tiles), dim3(SORT_BLOCK), 0, s, kin, n, sentinel, tile_heads,
                           flat_tiles, seg_start, seg_real, a.unique_keys_out, ctrl, a.num_unique_out, poll_limit,
                           a.status);
        EMB_RETURN_IF_LAUNCH_FAILED();
        if (a.unique_counts_out) {
            const unsigned cgrid = (unsigned)(flat_tiles < 1024 ? flat_tiles : 1024);
            hipLaunchKernelGGL(runs_counts_kernel, dim3(cgrid), dim3(256), 0, s, seg_start, seg_real,
                               a.unique_counts_out, ctrl);
            EMB_RETURN_IF_LAUNCH_FAILED();
        }
    }

    EMB_MARK(a, 3);
    return EMB_OK;
}

// Segment reduce + Adagrad over the records run_sort left in the workspace.
template <typename KeyT>
int run_update(const BwdArgs &a, const BwdLayout &L)
{
    // an odd number of passes leaves the sorted records in the second pair of arrays
    const bool in_b = (a.passes & 1) != 0;
    const KeyT *kin = reinterpret_cast<const KeyT *>(a.ws + (in_b ? L.keys_b : L.keys_a));
    const uint32_t *pin = reinterpret_cast<const uint32_t *>(a.ws + (in_b ? L.pay_b : L.pay_a));
    EMB_MARK(a, 3);
    if (a.nnz == 0) {
        EMB_MARK(a, 4);
        EMB_MARK(a, 5);
        return EMB_OK;
    }
    const int chunks = a.D * emb_elem_size(a.dtype) / 16;
    const bool bf16 = a.dtype == EMB_BF16;
#define EMB_UPD(LL, C, EU)                                                                   \
    return bf16 ? launch_update<KeyT, LL, C, EU, true>(a, L, kin, pin, chunks)               \
                : launch_update<KeyT, LL, C, EU, false>(a, L, kin, pin, chunks)
    switch (L.lpr * 100 + L.cpl) {
        case 101: EMB_UPD(1, 1, 4);
        case 201: EMB_UPD(2, 1, 4);
        case 401: EMB_UPD(4, 1, 4);
        case 402: EMB_UPD(4, 2, 4);
        case 802: EMB_UPD(8, 2, 4);
        case 1602: EMB_UPD(16, 2, 4);
        case 3202: EMB_UPD(32, 2, 4);
        case 6402: EMB_UPD(64, 2, 4);
        case 6404: EMB_UPD(64, 4, 2);
        case 6408: EMB_UPD(64, 8, 1);
        case 6416: EMB_UPD(64, 16, 1);
        default: return EMB_ERR_UNSUPPORTED;
    }
#undef EMB_UPD
}

}  // namespace

extern "C" size_t emb_bag_backward_workspace_bytes(int32_t T, int64_t B, int64_t nnz, int64_t total_rows, int32_t D,
                                                   int32_t dtype)
{
    if (T < 0 || B < 0 || nnz < 0 || total_rows < 0) return 0;
    if (emb_check_row_shape(D, dtype) != EMB_OK) return 0;
    return bwd_layout(T, B, nnz, total_rows, D, dtype).total;
}

namespace {

// ---------------------------------------------------------------------------
// training forward: the pooled lookup of a batch that will be followed by its backward
// ---------------------------------------------------------------------------
// The lookup hashes the raw IDs itself (as emb_bag_forward_hashed) and, having the row number
// and the bag of every lookup in hand, writes the backward's (row, bag) record and the bag's
// gradient scale while it is there: the backward then needs no pass over the indices.
template <typename KeyT>
struct TrainSource {
    const char *weights;
    uint64_t num_rows, salt, magic;
    int64_t row_bytes;
    int64_t *rows_out;   // nullable
    KeyT *keys;
    uint32_t *pay;
    uint32_t bag;
    __device__ __forceinline__ uint64_t resolve(int64_t raw, int64_t j) const
    {
        const uint64_t r = emb_fast_mod(emb_splitmix64((uint64_t)raw ^ salt), num_rows, magic);
        if (rows_out) rows_out[j] = (int64_t)r;
        keys[j] = (KeyT)r;
        pay[j] = bag;
        return reinterpret_cast<uint64_t>(weights + (int64_t)r * row_bytes);
    }
};

constexpr int TRAIN_BLOCK = 256;

template <int LPR, int CPL, int UNROLL, bool BF16, typename KeyT>
__global__ __launch_bounds__(TRAIN_BLOCK) void bag_forward_train_kernel(
    const emb_table *__restrict__ tables, int32_t T, int64_t B, uint32_t blocks_per_table, int64_t nnz,
    const int64_t *__restrict__ raw, const int64_t *__restrict__ offsets, int32_t chunks_per_row, int32_t mode,
    float *__restrict__ out, int64_t *__restrict__ rows_out, KeyT *__restrict__ keys, uint32_t *__restrict__ pay,
    float *__restrict__ bag_scale, BwdCtrl *ctrl, uint32_t *status, const int64_t *__restrict__ tile_prefix,
    int64_t *__restrict__ offsets_out)
{
    // tile_prefix != NULL: `offsets` are sums within tiles (emb_offset_at) and the final offsets go to offsets_out
    constexpr int GROUPS = TRAIN_BLOCK / LPR;
    constexpr int F = ChunkAcc<BF16>::FLOATS;
    const uint32_t lb = emb_xcd_block(blockIdx.x, gridDim.x);
    const uint32_t t_raw = lb / blocks_per_table;
    const bool tail = t_raw >= (uint32_t)T;          // the grid is rounded up to whole dies
    const int t = tail ? T - 1 : (int)t_raw;
    const int l = threadIdx.x % LPR;
    const int64_t b = tail ? B : (int64_t)(lb % blocks_per_table) * GROUPS + threadIdx.x / LPR;
    const bool live = b < B;
    const int64_t bag = (int64_t)t * B + b;
    const emb_table tb = tables[t];
    if (live && l == 0) {
        // what bwd_keys_kernel does per bag: the scale of its gradient, or the abort of the backward
        int64_t s, e;
        emb_bag_bounds(offsets, tile_prefix, bag, s, e);
        if (s < 0 || e < s || e > nnz) atomicOr(&ctrl->abort, 1u);   // the lookup below flags the status word
        else bag_scale[bag] = (mode == EMB_POOL_MEAN && e > s) ? 1.0f / (float)(e - s) : 1.0f;
        if (offsets_out) {
            offsets_out[bag + 1] = e;
            if (bag == 0) offsets_out[0] = 0;
        }
    }
    TrainSource<KeyT> src{reinterpret_cast<const char *>(tb.weights), (uint64_t)tb.num_rows, tb.salt, tb.mod_magic,
                          (int64_t)chunks_per_row * 16, rows_out, keys, pay, (uint32_t)bag};
    gather_pool_bag<LPR, CPL, UNROLL, BF16>(src, live, bag, l, nnz, raw, offsets, chunks_per_row, mode,
                                            out + bag * ((int64_t)chunks_per_row * F), status, tile_prefix);
}

template <typename KeyT, int LPR, int CPL, int UNROLL>
int launch_train(bool bf16, const BwdArgs &a, const BwdLayout &L, const int64_t *raw, float *out, int64_t *rows_out,
                 int chunks)
{
    constexpr int GROUPS = TRAIN_BLOCK / LPR;
    const int64_t per_table = (a.B + GROUPS - 1) / GROUPS;
    const int64_t blocks = emb_round_up_xcds(per_table * a.T);
    if (blocks > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    BwdCtrl *ctrl = reinterpret_cast<BwdCtrl *>(a.ws + L.ctrl);
    KeyT *keys = reinterpret_cast<KeyT *>(a.ws + L.keys_a);
    uint32_t *pay = reinterpret_cast<uint32_t *>(a.ws + L.pay_a);
    float *bag_scale = reinterpret_cast<float *>(a.ws + L.bag_scale);
    // made from lengths: the offsets are the sums within tiles in the workspace plus the tiles' prefix sums
    const int64_t *offsets = a.from_lengths ? reinterpret_cast<const int64_t *>(a.ws + L.local_offsets) : a.offsets;
    const int64_t *tile_prefix = a.from_lengths ? reinterpret_cast<const int64_t *>(a.ws + L.tile_prefix) : nullptr;
    if (bf16)
        hipLaunchKernelGGL((bag_forward_train_kernel<LPR, CPL, UNROLL, true, KeyT>), dim3((unsigned)blocks),
                           dim3(TRAIN_BLOCK), 0, a.stream, a.tables_dev, a.T, a.B, (uint32_t)per_table, a.nnz, raw,
                           offsets, chunks, a.mode, out, rows_out, keys, pay, bag_scale, ctrl, a.status, tile_prefix,
                           a.offsets_out);
    else
        hipLaunchKernelGGL((bag_forward_train_kernel<LPR, CPL, UNROLL, false, KeyT>), dim3((unsigned)blocks),
                           dim3(TRAIN_BLOCK), 0, a.stream, a.tables_dev, a.T, a.B, (uint32_t)per_table, a.nnz, raw,
                           offsets, chunks, a.mode, out, rows_out, keys, pay, bag_scale, ctrl, a.status, tile_prefix,
                           a.offsets_out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

template <typename KeyT>
int run_train_forward(const BwdArgs &a, const BwdLayout &L, const int64_t *raw, float *out, int64_t *rows_out)
{
    BwdCtrl *ctrl = reinterpret_cast<BwdCtrl *>(a.ws + L.ctrl);
    uint32_t *first_tile = reinterpret_cast<uint32_t *>(a.ws + L.first_tile);
    SortTile *tile_desc = reinterpret_cast<SortTile *>(a.ws + L.tile_desc);
    if (a.from_lengths) {
        // bag offsets on the way: sums within tiles by one launch; the tiles' prefix sums by the
        // single workgroup of bwd_init_kernel; the lookup adds the two (and writes the offsets out)
        const int64_t n_lengths = (int64_t)a.T * a.B;
        // (no bags: the offsets are the single entry 0, which the tile sums then write straight to the caller)
        int64_t *local = n_lengths == 0 ? a.offsets_out : reinterpret_cast<int64_t *>(a.ws + L.local_offsets);
        int64_t *tile_prefix = reinterpret_cast<int64_t *>(a.ws + L.tile_prefix);
        const int rc = emb_offsets_tile_sums(a.lengths, n_lengths, local, a.status, a.stream);
        if (rc != EMB_OK) return rc;
        hipLaunchKernelGGL(bwd_init_kernel, dim3(1), dim3(1024), 0, a.stream, ctrl, local, a.nnz > 0 ? a.T : 0, a.B, a.nnz,
                           first_tile, tile_desc, a.nnz > 0 ? (uint32_t)L.tiles : 0u, a.num_unique_out, a.status,
                           tile_prefix, n_lengths);
    } else {
        hipLaunchKernelGGL(bwd_init_kernel, dim3(1), dim3(1024), 0, a.stream, ctrl, a.offsets, a.nnz > 0 ? a.T : 0, a.B,
                           a.nnz, first_tile, tile_desc, a.nnz > 0 ? (uint32_t)L.tiles : 0u, a.num_unique_out, a.status);
    }
    EMB_RETURN_IF_LAUNCH_FAILED();
    // Work of an earlier backward that still runs on its side stream changes table rows: the lookup
    // waits for it; the two launches above read neither tables nor that backward's workspace.
    if (a.after && hipStreamWaitEvent(a.stream, reinterpret_cast<hipEvent_t>(a.after->join_event), 0) != hipSuccess)
        return EMB_ERR_HIP;
    if (a.T == 0 || a.B == 0) return EMB_OK;
    const int chunks = a.D * emb_elem_size(a.dtype) / 16;
    int lpr, cpl;
    emb_row_split(chunks, lpr, cpl);
    const bool bf16 = a.dtype == EMB_BF16;
#define EMB_TR(LL, C, U) return launch_train<KeyT, LL, C, U>(bf16, a, L, raw, out, rows_out, chunks)
    if (cpl == 1) {
        switch (lpr) {
            case 1: EMB_TR(1, 1, 8);
            case 2: EMB_TR(2, 1, 8);
            case 4: EMB_TR(4, 1, 8);
            case 8: EMB_TR(8, 1, 8);
            case 16: EMB_TR(16, 1, 8);
            case 32: EMB_TR(32, 1, 8);
            default: EMB_TR(64, 1, 8);
        }
    }
    switch (cpl) {
        case 2: EMB_TR(64, 2, 4);
        case 4: EMB_TR(64, 4, 2);
        case 8: EMB_TR(64, 8, 1);
        default: EMB_TR(64, 16, 1);
    }
#undef EMB_TR
}

// Host-side checks and the workspace layout shared by the backward entry points.
int bwd_plan(const emb_table *tables_host, const emb_table *tables_dev, int32_t T, int32_t D, int32_t dtype, int64_t B,
             int64_t nnz, void *workspace_dev, size_t workspace_bytes, void *stream, BwdArgs &a, BwdLayout &L)
{
    if (B < 0 || nnz < 0) return EMB_ERR_INVALID_ARG;
    int rc = emb_check_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    rc = emb_check_tables(tables_host, tables_dev, T, true);
    if (rc != EMB_OK) return rc;
    if (T > 65535) return EMB_ERR_UNSUPPORTED;
    if ((T == 0 || B == 0) && nnz != 0) return EMB_ERR_INVALID_ARG;
    if (nnz >= ((int64_t)1 << 31)) return EMB_ERR_UNSUPPORTED;
    if (B > 0 && (int64_t)T > ((int64_t)0xFFFFFFFE) / B) return EMB_ERR_UNSUPPORTED;
    if (B > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;

    int64_t total_rows = 0, max_rows = 0;
    for (int32_t t = 0; t < T; ++t) {
        total_rows += tables_host[t].num_rows;
        if (tables_host[t].num_rows > max_rows) max_rows = tables_host[t].num_rows;
    }
    L = bwd_layout(T, B, nnz, total_rows, D, dtype);
    if (!workspace_dev || !emb_aligned(workspace_dev, 256) || workspace_bytes < L.total) return EMB_ERR_WORKSPACE;
    int bits = 0;
    for (uint64_t v = (uint64_t)max_rows; v; v >>= 1) ++bits;
    int passes = (bits + RADIX_BITS - 1) / RADIX_BITS;
    if (passes < 1) passes = 1;

    a = BwdArgs();
    a.tables_dev = tables_dev;
    a.T = T; a.D = D; a.dtype = dtype;
    a.B = B; a.nnz = nnz; a.total_rows = total_rows; a.max_rows = max_rows;
    a.passes = passes;
    a.ws = reinterpret_cast<char *>(workspace_dev);
    a.stream = emb_stream(stream);
    return EMB_OK;
}

}  // namespace

extern "C" int emb_bag_backward_sort(const emb_table *tables_host, const emb_table *tables_dev, int32_t T, int32_t D,
                                     int32_t dtype, const int64_t *rows_dev, const int64_t *offsets_dev, int64_t B,
                                     int64_t nnz, int32_t mode, void *workspace_dev, size_t workspace_bytes,
                                     int64_t *unique_keys_out_dev, int32_t *unique_counts_out_dev,
                                     int64_t *num_unique_out_dev, uint32_t *status_dev, void *const *stage_events,
                                     void *stream)
{
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    BwdArgs a;
    BwdLayout L;
    const int rc = bwd_plan(tables_host, tables_dev, T, D, dtype, B, nnz, workspace_dev, workspace_bytes, stream, a, L);
    if (rc != EMB_OK) return rc;
    if (nnz > 0 && (!rows_dev || !offsets_dev)) return EMB_ERR_INVALID_ARG;
    a.mode = mode;
    a.rows = rows_dev; a.offsets = offsets_dev;
    a.unique_keys_out = unique_keys_out_dev;
    a.unique_counts_out = unique_counts_out_dev;
    a.num_unique_out = num_unique_out_dev;
    a.status = status_dev;
    a.events = stage_events;
    return L.key_bytes == 4 ? run_sort<uint32_t>(a, L) : run_sort<uint64_t>(a, L);
}

extern "C" int emb_bag_forward_train(const emb_table *tables_host, const emb_table *tables_dev, int32_t T, int32_t D,
                                     int32_t dtype, const uint64_t *raw_dev, const int64_t *offsets_dev, int64_t B,
                                     int64_t nnz, int32_t mode, float *out_dev, int64_t *rows_out_dev,
                                     void *workspace_dev, size_t workspace_bytes, int64_t *num_unique_out_dev,
                                     uint32_t *status_dev, void *stream)
{
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    BwdArgs a;
    BwdLayout L;
    const int rc = bwd_plan(tables_host, tables_dev, T, D, dtype, B, nnz, workspace_dev, workspace_bytes, stream, a, L);
    if (rc != EMB_OK) return rc;
    if (T > 0 && B > 0) {
        if (!offsets_dev || !out_dev || (nnz > 0 && !raw_dev)) return EMB_ERR_INVALID_ARG;
        if (!emb_aligned(out_dev, 16)) return EMB_ERR_INVALID_ARG;
    }
    a.mode = mode;
    a.offsets = offsets_dev;
    a.num_unique_out = num_unique_out_dev;
    a.status = status_dev;
    const int64_t *raw = reinterpret_cast<const int64_t *>(raw_dev);
    return L.key_bytes == 4 ? run_train_forward<uint32_t>(a, L, raw, out_dev, rows_out_dev)
                            : run_train_forward<uint64_t>(a, L, raw, out_dev, rows_out_dev);
}

static int train_forward_from_lengths(const emb_table *tables_host, const emb_table *tables_dev, int32_t T, int32_t D,
                                      int32_t dtype, const uint64_t *raw_dev, const int32_t *lengths_dev, int64_t B,
                                      int64_t nnz, int32_t mode, float *out_dev, int64_t *offsets_out_dev,
                                      int64_t *rows_out_dev, void *workspace_dev, size_t workspace_bytes,
                                      int64_t *num_unique_out_dev, uint32_t *status_dev,
                                      const emb_side_stream *after, void *stream)
{
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    if (after && (!after->join_event || after->stream == stream)) return EMB_ERR_INVALID_ARG;
    BwdArgs a;
    BwdLayout L;
    const int rc = bwd_plan(tables_host, tables_dev, T, D, dtype, B, nnz, workspace_dev, workspace_bytes, stream, a, L);
    if (rc != EMB_OK) return rc;
    if (!offsets_out_dev) return EMB_ERR_INVALID_ARG;
    if (T > 0 && B > 0) {
        if (!lengths_dev || !out_dev || (nnz > 0 && !raw_dev)) return EMB_ERR_INVALID_ARG;
        if (!emb_aligned(out_dev, 16)) return EMB_ERR_INVALID_ARG;
    }
    a.mode = mode;
    a.after = after;
    a.from_lengths = true;
    a.lengths = lengths_dev;
    a.offsets_out = offsets_out_dev;
    a.num_unique_out = num_unique_out_dev;
    a.status = status_dev;
    const int64_t *raw = reinterpret_cast<const int64_t *>(raw_dev);
    return L.key_bytes == 4 ? run_train_forward<uint32_t>(a, L, raw, out_dev, rows_out_dev)
                            : run_train_forward<uint64_t>(a, L, raw, out_dev, rows_out_dev);
}

extern "C" int emb_bag_forward_train_lengths(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                                             int32_t D, int32_t dtype, const uint64_t *raw_dev,
                                             const int32_t *lengths_dev, int64_t B, int64_t nnz, int32_t mode,
                                             float *out_dev, int64_t *offsets_out_dev, int64_t *rows_out_dev,
                                             void *workspace_dev, size_t workspace_bytes, int64_t *num_unique_out_dev,
                                             uint32_t *status_dev, void *stream)
{
    return train_forward_from_lengths(tables_host, tables_dev, T, D, dtype, raw_dev, lengths_dev, B, nnz, mode, out_dev,
                                      offsets_out_dev, rows_out_dev, workspace_dev, workspace_bytes, num_unique_out_dev,
                                      status_dev, nullptr, stream);
}

extern "C" int emb_bag_forward_train_lengths_after(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                                                   int32_t D, int32_t dtype, const uint64_t *raw_dev,
                                                   const int32_t *lengths_dev, int64_t B, int64_t nnz, int32_t mode,
                                                   float *out_dev, int64_t *offsets_out_dev, int64_t *rows_out_dev,
                                                   void *workspace_dev, size_t workspace_bytes,
                                                   int64_t *num_unique_out_dev, uint32_t *status_dev,
                                                   const emb_side_stream *after, void *stream)
{
    return train_forward_from_lengths(tables_host, tables_dev, T, D, dtype, raw_dev, lengths_dev, B, nnz, mode, out_dev,
                                      offsets_out_dev, rows_out_dev, workspace_dev, workspace_bytes, num_unique_out_dev,
                                      status_dev, after, stream);
}

extern "C" int emb_bag_backward_sort_prepared(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                                              int32_t D, int32_t dtype, int64_t B, int64_t nnz, void *workspace_dev,
                                              size_t workspace_bytes, int64_t *unique_keys_out_dev,
                                              int32_t *unique_counts_out_dev, int64_t *num_unique_out_dev,
                                              uint32_t *status_dev, void *const *stage_events, void *stream)
{
    BwdArgs a;
    BwdLayout L;
    const int rc = bwd_plan(tables_host, tables_dev, T, D, dtype, B, nnz, workspace_dev, workspace_bytes, stream, a, L);
    if (rc != EMB_OK) return rc;
    a.unique_keys_out = unique_keys_out_dev;
    a.unique_counts_out = unique_counts_out_dev;
    a.num_unique_out = num_unique_out_dev;
    a.status = status_dev;
    a.events = stage_events;
    return L.key_bytes == 4 ? run_sort<uint32_t>(a, L, true) : run_sort<uint64_t>(a, L, true);
}

extern "C" int emb_bag_backward_update(const emb_table *tables_host, const emb_table *tables_dev, int32_t T, int32_t D,
                                       int32_t dtype, int64_t B, int64_t nnz, const float *dout_dev, float lr,
                                       float eps, void *workspace_dev, size_t workspace_bytes,
                                       int64_t *num_unique_out_dev, void *const *stage_events,
                                       const emb_side_stream *side, void *stream)
{
    BwdArgs a;
    BwdLayout L;
    const int rc = bwd_plan(tables_host, tables_dev, T, D, dtype, B, nnz, workspace_dev, workspace_bytes, stream, a, L);
    if (rc != EMB_OK) return rc;
    if (nnz > 0 && (!dout_dev || !emb_aligned(dout_dev, 16))) return EMB_ERR_INVALID_ARG;
    if (side && (!side->stream || !side->fork_event || !side->join_event || side->stream == stream))
        return EMB_ERR_INVALID_ARG;
    a.dout = dout_dev;
    a.lr = lr; a.eps = eps;
    a.num_unique_out = num_unique_out_dev;
    a.events = stage_events;
    a.side = side;
    return L.key_bytes == 4 ? run_update<uint32_t>(a, L) : run_update<uint64_t>(a, L);
}

extern "C" int emb_bag_backward_rowwise_adagrad(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                                                int32_t D, int32_t dtype, const int64_t *rows_dev,
                                                const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode,
                                                const float *dout_dev, float lr, float eps, void *workspace_dev,
                                                size_t workspace_bytes, int64_t *unique_keys_out_dev,
                                                int32_t *unique_counts_out_dev, int64_t *num_unique_out_dev,
                                                uint32_t *status_dev, void *const *stage_events,
                                                const emb_side_stream *side, void *stream)
{
    // every argument of the second half is checked before the first half is enqueued
    if (nnz > 0 && (!dout_dev || !emb_aligned(dout_dev, 16))) return EMB_ERR_INVALID_ARG;
    if (side && (!side->stream || !side->fork_event || !side->join_event || side->stream == stream))
        return EMB_ERR_INVALID_ARG;
    const int rc = emb_bag_backward_sort(tables_host, tables_dev, T, D, dtype, rows_dev, offsets_dev, B, nnz, mode,
                                         workspace_dev, workspace_bytes, unique_keys_out_dev, unique_counts_out_dev,
                                         num_unique_out_dev, status_dev, stage_events, stream);
    if (rc != EMB_OK) return rc;
    return emb_bag_backward_update(tables_host, tables_dev, T, D, dtype, B, nnz, dout_dev, lr, eps, workspace_dev,
                                   workspace_bytes, num_unique_out_dev, stage_events, side, stream);
}
